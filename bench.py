"""Benchmark of the population step on one MI355X.

A "step" is one pass of the whole hot path over one mini-batch per member: fetch, forward, loss,
backward, optimiser update for all P members, plus `eval` and exploit/explore at the workload's
cadence (every `ready_interval` steps).  Workload: the wide bf16 MLP population (P = 64,
256-1024-1024-10, batch 128, Adam).  All inputs are synthetic and resident in HBM before the
timed region.  Prints one JSON line."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published

# HBM bytes per launch from the FETCH_SIZE / WRITE_SIZE counters, scaled by what the same counters read
# for a copy of known size (profiles/population_step_<workload>_hbm_counters.md), by (workload, kernel
# class).  An entry is only valid for the kernel as it was when the counters were taken; remove it when
# the kernel changes.
MEASURED_TRAFFIC_BYTES = {(2, "optimizer"): 2.541e9, (2, "gemm_wgrad_fused"): 1.1187e9, (4, "optimizer"): 10.115e9}


def cpu_baseline(workload, wl, seed, budget_s=15.0):
    """The oracle as it stands, timed on the host cores over a bounded sample of the workload:
    member-steps of the first population step(s), member after member, until the budget is used."""
    import numpy as np
    from paper_1711_09846_amd import workloads
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    H = workloads.initial_hypers(wl, 6)
    oc = {k: float(np.float32(v)) for k, v in wl.opt_const.items()}
    if workload == 2:
        from oracle import classifier as o
        from tests.harness import oracle_spec
        (tx, ty), _ = workloads.classifier_data(wl)
        spec = oracle_spec(wl, seed)
        weights = workloads.initial_mlp_weights(wl.dims, wl.P, 5)
        pop = [o.new_member(spec, weights[i], H[i], i) for i in range(wl.P)]
        step = lambda m, i, s: o.step(spec, m, i, s, tx, ty)
    elif workload == 3:
        from oracle import gan as o
        tx, _ = workloads.gan_data(wl)
        spec = o.GanSpec(wl.dims, wl.dims2, wl.batch, seed, roles=wl.roles, beta1=oc["beta1"], beta2=oc["beta2"], eps=oc["eps"], bf16_storage=True)
        weights = workloads.initial_gan_weights(wl, wl.P, 5)
        pop = [o.new_member(spec, weights[i][0], weights[i][1], H[i], i) for i in range(wl.P)]
        step = lambda m, i, s: o.step(spec, m, i, s, tx)
    elif workload == 4:
        from oracle import transformer as o
        pool, _ = workloads.zipf_bigram_sequences(wl)
        spec = o.TransformerSpec(wl.vocab, wl.d_model, wl.heads, wl.d_ff, wl.n_blocks, wl.seq, wl.batch, seed, roles=wl.roles,
                                 beta1=oc["beta1"], beta2=oc["beta2"], eps=oc["eps"], bf16_storage=True)
        weights = workloads.initial_transformer_weights(wl, 2, 5)
        pop = [o.new_member(spec, weights[i], H[i], i) for i in range(2)]
        step = lambda m, i, s: o.step(spec, m, i, s, pool)
    else:
        from oracle import a2c as o
        obs, act, rew = workloads.trajectory_pool(wl)
        spec = o.A2CSpec(wl.dims[:-1], wl.n_actions, wl.batch, wl.unroll, seed, roles=wl.roles, gamma=float(np.float32(wl.gamma)),
                         value_cost=float(np.float32(wl.value_cost)), rho=oc["rho"], rms_eps=oc["eps"], hidden_act=wl.act, bf16_storage=True)
        weights = workloads.initial_mlp_weights(wl.dims, wl.P, 5)
        pop = [o.new_member(spec, weights[i], H[i], i) for i in range(wl.P)]
        step = lambda m, i, s: o.step(spec, m, i, s, obs, act, rew)
    done, s, t0 = 0, 0, time.perf_counter()
    while time.perf_counter() - t0 < budget_s and s < 32:
        for i, m in enumerate(pop):
            step(m, i, s)
            done += 1
            if time.perf_counter() - t0 >= budget_s:
                break
        s += 1
    dt = time.perf_counter() - t0
    return {"value": done / dt, "unit": "member-steps/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d member-steps of %s (step only, numpy float64 with bf16 storage rounding where the workload has it)" % (done, wl.name)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="default 400 (30 for the transformer workload)")
    ap.add_argument("--warmup", type=int, default=None, help="default 20 (3 for the transformer workload)")
    ap.add_argument("--kernel", default=None, help="kernel class whose roofline is reported (default: the dominant one)")
    ap.add_argument("--fused", type=int, default=None, choices=[0, 1],
                    help="1 = optimiser applied inside the weight-gradient GEMMs (default for workload 2, where it is "
                         "the faster of the two as measured), 0 = separate streaming optimiser pass (default otherwise)")
    ap.add_argument("--workload", type=int, default=2, choices=[2, 3, 4, 5],
                    help="2 = wide bf16 MLP classifiers (default, the headline workload), 3 = MLP GAN pairs, "
                         "4 = decoder-only transformers, 5 = actor-critic")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (no sharding, no collectives); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    if args.fused is None:
        args.fused = 1 if args.workload == 2 else 0
    if args.steps is None:
        args.steps = 30 if args.workload == 4 else 400
    if args.warmup is None:
        args.warmup = 3 if args.workload == 4 else 20

    import numpy as np
    import torch
    from paper_1711_09846_amd import binding, workloads

    wl = workloads.WORKLOADS[args.workload]
    seed = workloads.POPULATION_SEED
    cfg = binding.make_config(wl, seed, fuse_optimizer=args.fused)
    pop = binding.Population(cfg)
    dev = pop.device
    if args.kernel is None:
        args.kernel = "gemm_fwd" if args.workload == 4 else "gemm_wgrad" if args.fused else "optimizer"
    data = None
    if args.workload == 2:
        data = workloads.classifier_data(wl)
        (tx, ty), (ex, ey) = data
        pop.set_members(workloads.initial_mlp_weights(wl.dims, wl.P, 5), workloads.initial_hypers(wl, 6))
        d_train = [torch.from_numpy(tx).to(dev), torch.from_numpy(ty).to(dev)]
        d_eval = [torch.from_numpy(ex).to(dev), torch.from_numpy(ey).to(dev)]
    elif args.workload == 3:
        tx, ex = workloads.gan_data(wl)
        pop.set_members([list(g) + list(d) for g, d in workloads.initial_gan_weights(wl, wl.P, 5)], workloads.initial_hypers(wl, 6))
        d_train, d_eval = [torch.from_numpy(tx).to(dev)], [torch.from_numpy(ex).to(dev)]
    elif args.workload == 4:
        pool, held_out = workloads.zipf_bigram_sequences(wl)
        weights = workloads.initial_transformer_weights(wl, wl.P, 5)
        pop.set(binding.ARR_W32, np.stack([binding.pack_segments(pop.layout, a) for a in weights]))
        pop.set(binding.ARR_HYPER, workloads.initial_hypers(wl, 6))
        d_train, d_eval = [torch.from_numpy(pool).to(dev)], [torch.from_numpy(held_out).to(dev)]
    else:
        obs, act, rew = workloads.trajectory_pool(wl)
        pop.set_members(workloads.initial_mlp_weights(wl.dims, wl.P, 5), workloads.initial_hypers(wl, 6))
        d_train, d_eval = [torch.from_numpy(obs).to(dev), torch.from_numpy(act).to(dev), torch.from_numpy(rew).to(dev)], []

    klass = {"optimizer": binding.K_OPTIMIZER, "gemm_fwd": binding.K_GEMM_FWD, "gemm_wgrad": binding.K_GEMM_WGRAD,
             "gemm_dgrad": binding.K_GEMM_DGRAD, "copy": binding.K_COPY, "head": binding.K_HEAD,
             "fetch": binding.K_FETCH, "bias_grad": binding.K_BIAS_GRAD}[args.kernel]

    def run(first, n, rnd):
        for s in range(first, first + n):
            pop.step(d_train, s)
            if (s + 1) % wl.ready_interval == 0:
                pop.eval(d_eval)
                pop.exploit_explore(rnd)
                rnd += 1
        return rnd

    rnd = run(0, args.warmup, 0)
    # the warm-up also exercises eval + exploit once so that nothing is first-touched in the timed region
    pop.eval(d_eval)
    pop.exploit_explore(1 << 20)
    torch.cuda.synchronize()
    # an event pair costs the stream a few microseconds around the launch it brackets (the wide MLP step lost
    # 3 % to them): every 7th launch of the class is recorded, which over the timed region still visits each
    # of the class's launches of a step equally often
    pop.timing_enable(klass, 8 * args.steps + 64)
    pop.timing_stride(7 if args.steps >= 100 else 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # step indices continue from the warm-up so that the cadence (eval + exploit every
    # ready_interval steps) falls inside the timed region as it does in a real run
    run(args.warmup, args.steps, rnd)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    k_ms, k_n = pop.timing_read()
    pop.timing_enable(binding.K_NONE, 0)
    n_rounds = (args.warmup + args.steps) // wl.ready_interval - args.warmup // wl.ready_interval

    n = pop.layout.n_params
    L = len(wl.dims) - 1
    flops_fwd = sum(2.0 * wl.batch * wl.dims[l] * wl.dims[l + 1] for l in range(L - 1)) * wl.P
    state_bytes = {2: 14.0, 3: 14.0, 4: 14.0, 5: 10.0}[args.workload]      # fp32 theta + optimiser state (+ bf16 shadow) per parameter
    if args.workload == 4:
        # dense layers of one forward pass: per block QKV, attention output, two feed-forward matrices; the vocabulary head
        rows, d, f = wl.batch * wl.seq, wl.d_model, wl.d_ff
        dense = 2.0 * rows * (wl.n_blocks * (3 * d * d + d * d + 2 * d * f) + d * wl.vocab) * wl.P
        n_dense = 4 * wl.n_blocks + 1
        per_launch = {"optimizer": ("hbm", 30.0 * n * wl.P), "copy": ("hbm", 2.0 * state_bytes * n * wl.n_trunc),
                      "gemm_fwd": ("mfma", dense / n_dense), "gemm_wgrad": ("mfma", dense / n_dense),
                      "gemm_dgrad": ("mfma", dense / n_dense)}.get(args.kernel)
    else:
      per_launch = {
        # Adam: read theta, g, m, v (16 B), write theta, m, v (12 B) and the bf16 shadow (2 B) per parameter
        # (RMSProp: theta, g, one state array read, theta, state and the shadow written: 22 B; the GAN step has two
        # launches, one over the discriminator's and one over the generator's parameters: mean of the two)
        "optimizer": ("hbm", {2: 30.0, 3: 15.0, 5: 22.0}[args.workload] * n * wl.P),
        # read + write of every array of the n_trunc copied members: fp32 theta, optimiser state, bf16 shadow
        "copy": ("hbm", 2.0 * state_bytes * n * wl.n_trunc),
        "gemm_fwd": ("mfma", flops_fwd / (L - 1)) if args.workload == 2 else None,
        # fused: per hidden matrix read theta, m, v (12 B) and write theta, m, v and the bf16 shadow (14 B) per
        # parameter, plus the bf16 operands X and dZ; averaged over the launches of one step (one per matrix)
        "gemm_wgrad": (("hbm", (26.0 * sum(wl.dims[l] * wl.dims[l + 1] for l in range(L - 1))
                                + 2.0 * wl.batch * sum(wl.dims[l] + wl.dims[l + 1] for l in range(L - 1))) * wl.P / (L - 1))
                       if args.fused else ("mfma", flops_fwd / (L - 1))) if args.workload == 2 else None,
        "gemm_dgrad": ("mfma", 2.0 * wl.batch * wl.dims[1] * wl.dims[2] * wl.P) if args.workload == 2 else None,
      }.get(args.kernel)
    roofline = None
    if per_launch and k_n:
        bound, work = per_launch
        avg_s = k_ms / k_n * 1e-3
        if bound == "hbm":
            ach, peak, unit = work / avg_s / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, peak, unit = work / avg_s / 1e12, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"
        roofline = {"kernel": args.kernel, "bound": bound, "achieved": ach, "peak": peak, "unit": unit,
                    "frac": ach / peak, "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, args.kernel + ("_fused" if args.fused and args.kernel == "gemm_wgrad" else ""))), "avg_launch_us": avg_s * 1e6, "launches": k_n,
                    "work_per_launch": work}

    out = {
        "metric": "population member-steps/sec at 1 MI355X", "value": wl.P * args.steps / dt, "unit": "member-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "fused_optimizer": bool(args.fused), "P": wl.P,
                   "dims": wl.dims or {"blocks": wl.n_blocks, "d_model": wl.d_model, "heads": wl.heads, "d_ff": wl.d_ff, "seq": wl.seq, "vocab": wl.vocab},
                   "batch": wl.batch,
                   "optimizer": {0: "sgd_momentum", 1: "adam", 2: "rmsprop"}[wl.optimizer],
                   "ready_interval": wl.ready_interval, "n_trunc": wl.n_trunc, "eval_rows": wl.n_eval,
                   "exploit_rounds_in_timed_region": n_rounds},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload, wl, seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
