"""Benchmark of the PBT population step on one MI355X.

A "step" is one pass of the whole hot path over one mini-batch per member: fetch, forward, loss,
backward, optimiser update for all P members; `eval` and exploit/explore run every `ready_interval`
steps.  All inputs are synthetic and resident in HBM before any timed region.

The top-level record is the largest workload, `transformer_bf16` (P = 16 decoder-only transformers,
4 blocks, d_model 512, 8 heads, FFN 2048, 128 positions, vocabulary 8192, 32 sequences per member and
step): `--steps` population steps are timed after `--warmup` untimed ones, then one `eval` and one
exploit/explore pass are timed on their own, and `value` is the member-steps per second of a run at the
workload's cadence (ready_interval steps + one eval + one exploit/explore); `step_only` gives the rate
of the steps alone.  While the steps are timed, HIP events on the kernels' own stream bracket a sample
of the launches of the GEMM, optimiser and copy kernel classes; `rooflines` holds one entry per class
(`roofline` repeats the dominant one).  `workloads` holds the same record for each of the five workloads
(`--workload N` runs only that one, as the top-level record).  `cpu_baseline` is the float64 oracle timed
on the host cores over a bounded sample of the same workload.  Prints one JSON line."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published
ALU_FP32_PEAK_TFLOPS = 78.6      # 256 CU x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz, no packed math
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file, scaled by what the same counters
# read for the exploit copy (a plain copy of known size): keyed by (workload, fused optimiser, variant) and kernel class.
# They describe the kernels as they were when the counters were taken; a kernel that changes loses its entry.
_W4 = "profiles/population_step_transformer_bf16_hbm_counters.md"
_W2 = "profiles/population_step_mlp_wide_bf16_hbm_counters.md"
TRAFFIC = {
    (4, False, None): {"optimizer": (10.115e9, _W4), "copy": (1.770e9, _W4), "gemm": (0.481e9, _W4)},
    (2, True, None): {"gemm_wgrad": (1.1188e9, _W2), "copy": (0.4446e9, _W2)},
}
TARGET = {"mfma": 0.5, "hbm": 0.7}   # the fractions aimed at for the GEMMs and for the optimiser / exploit copy

# steps timed for the workloads that are not the top-level record (their own warm-up in brackets)
SUB_STEPS = {1: (1000, 100), 2: (200, 20), 3: (200, 20), 4: (10, 2), 5: (200, 20)}


def _workload(key, variant):
    """Workload 5 acts on-policy (unrolls generated on the device from each member's current policy); variant "pool"
    is the same agents on pre-recorded trajectories.  Workload 3 is the logistic GAN; variant "wgan_gp" is the
    paper's own step (5 critic updates on the WGAN-GP objective per generator update)."""
    from paper_1711_09846_amd import workloads
    if key == 5:
        return workloads.A2C_MLP if variant == "pool" else workloads.A2C_MLP_ON_POLICY
    if key == 3 and variant == "wgan_gp":
        return workloads.GAN_MLP_WGAN_GP
    return workloads.WORKLOADS[key]


def _oracle_setup(key, wl, seed):
    """(members, step function) of the oracle for one workload; inputs from the seeded generators."""
    import numpy as np
    from paper_1711_09846_amd import workloads
    H = workloads.initial_hypers(wl, 6)
    oc = {k: float(np.float32(v)) for k, v in wl.opt_const.items()}
    bf16 = wl.dtype == workloads.DTYPE_BF16
    if key in (1, 2):
        from oracle import classifier as o
        (tx, ty), _ = workloads.classifier_data(wl)
        spec = o.ClassifierSpec(wl.dims, wl.act, wl.optimizer, wl.batch, wl.roles, seed,
                                momentum=oc.get("momentum", float(np.float32(0.9))), beta1=oc.get("beta1", float(np.float32(0.9))),
                                beta2=oc.get("beta2", 0.999), eps=oc.get("eps", 1e-8), wd=oc.get("wd", 0.0), bf16_storage=bf16)
        weights = workloads.initial_mlp_weights(wl.dims, wl.P, 5)
        pop = [o.new_member(spec, weights[i], H[i], i) for i in range(wl.P)]
        return pop, lambda m, i, s: o.step(spec, m, i, s, tx, ty)
    if key == 3:
        from oracle import gan as o
        tx, _ = workloads.gan_data(wl)
        spec = o.GanSpec(wl.dims, wl.dims2, wl.batch, seed, roles=wl.roles, beta1=oc["beta1"], beta2=oc["beta2"], eps=oc["eps"], bf16_storage=True,
                         objective=getattr(wl, "objective", "logistic"), n_critic=getattr(wl, "n_critic", 1),
                         gp_weight=float(np.float32(getattr(wl, "gp_weight", 10.0))))
        weights = workloads.initial_gan_weights(wl, wl.P, 5)
        pop = [o.new_member(spec, weights[i][0], weights[i][1], H[i], i) for i in range(wl.P)]
        return pop, lambda m, i, s: o.step(spec, m, i, s, tx)
    if key == 4:
        from oracle import transformer as o
        pool, _ = workloads.zipf_bigram_sequences(wl)
        spec = o.TransformerSpec(wl.vocab, wl.d_model, wl.heads, wl.d_ff, wl.n_blocks, wl.seq, wl.batch, seed, roles=wl.roles,
                                 beta1=oc["beta1"], beta2=oc["beta2"], eps=oc["eps"], bf16_storage=True)
        weights = workloads.initial_transformer_weights(wl, 2, 5)
        pop = [o.new_member(spec, weights[i], H[i], i) for i in range(2)]
        return pop, lambda m, i, s: o.step(spec, m, i, s, pool)
    from oracle import a2c as o
    if getattr(wl, "on_policy", 0):
        from oracle import a2c_env
        env = a2c_env.Environment(*workloads.latent_system(wl))
    else:
        obs, act, rew = workloads.trajectory_pool(wl)
    spec = o.A2CSpec(wl.dims[:-1], wl.n_actions, wl.batch, wl.unroll, seed, roles=wl.roles, gamma=float(np.float32(wl.gamma)),
                     value_cost=float(np.float32(wl.value_cost)), rho=oc["rho"], rms_eps=oc["eps"], hidden_act=wl.act, bf16_storage=True)
    weights = workloads.initial_mlp_weights(wl.dims, wl.P, 5)
    pop = [o.new_member(spec, weights[i], H[i], i) for i in range(wl.P)]
    if getattr(wl, "on_policy", 0):
        return pop, lambda m, i, s: o.step_on_policy(spec, env, m, i, s)
    return pop, lambda m, i, s: o.step(spec, m, i, s, obs, act, rew)


def cpu_baseline(key, wl, seed, budget_s):
    """The oracle as it stands, timed on the host cores over a bounded sample of the workload: member-steps
    of the first population step(s), member after member, until the budget is used (at least one)."""
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    pop, step = _oracle_setup(key, wl, seed)
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
            "sample": "%d member-steps of %s (step only; numpy float64%s)" % (done, wl.name, ", bf16 rounding model" if wl.dtype else "")}


def _setup_gpu(key, wl, seed, fused):
    """Population on the GPU with uploaded initial state, and its resident inputs."""
    import numpy as np
    import torch
    from paper_1711_09846_amd import binding, workloads
    pop = binding.Population(binding.make_config(wl, seed, fuse_optimizer=fused))
    dev = pop.device
    to = lambda a: torch.from_numpy(a).to(dev)
    H = workloads.initial_hypers(wl, 6)
    if key in (1, 2):
        (tx, ty), (ex, ey) = workloads.classifier_data(wl)
        pop.set_members(workloads.initial_mlp_weights(wl.dims, wl.P, 5), H)
        return pop, [to(tx), to(ty)], [to(ex), to(ey)]
    if key == 3:
        tx, ex = workloads.gan_data(wl)
        pop.set_members([list(g) + list(d) for g, d in workloads.initial_gan_weights(wl, wl.P, 5)], H)
        return pop, [to(tx)], [to(ex)]
    if key == 4:
        pool, held_out = workloads.zipf_bigram_sequences(wl)
        weights = workloads.initial_transformer_weights(wl, wl.P, 5)
        pop.set(binding.ARR_W32, np.stack([binding.pack_segments(pop.layout, a) for a in weights]))
        pop.set(binding.ARR_HYPER, H)
        return pop, [to(pool)], [to(held_out)]
    pop.set_members(workloads.initial_mlp_weights(wl.dims, wl.P, 5), H)
    if getattr(wl, "on_policy", 0):
        A, Bm, Cm, w = workloads.latent_system(wl)
        noise = np.array([1.0, 0.1, 0.1])      # observation, reward and transition noise scales of the latent system
        return pop, [to(np.ascontiguousarray(a, dtype=np.float64)) for a in (A, Bm, Cm, w, noise)], []
    obs, act, rew = workloads.trajectory_pool(wl)
    return pop, [to(obs), to(act), to(rew)], []


def _work_per_step(key, wl, n, fused):
    """Algorithmic work of one population step per kernel class: {class: (bound, work, launches per step)};
    work in flop (mfma / alu) or bytes (hbm)."""
    P = wl.P
    state_bytes = {1: 8.0, 2: 14.0, 3: 14.0, 4: 14.0, 5: 10.0}[key]   # fp32 theta + optimiser state (+ bf16 shadow) per parameter
    out = {"copy": ("hbm", 2.0 * state_bytes * n * wl.n_trunc, 1)}      # per exploit: every copied byte is read once and written once
    if key == 1:
        L = len(wl.dims) - 1
        # forward, input-gradient and weight-gradient products of every layer, for the steps of one launch
        out["fused_step"] = ("alu", 6.0 * wl.batch * sum(wl.dims[l] * wl.dims[l + 1] for l in range(L)) * P * wl.ready_interval, 1)
        return out
    if key == 4:
        rows, d, f = wl.batch * wl.seq, wl.d_model, wl.d_ff
        dense = 2.0 * rows * (wl.n_blocks * (3 * d * d + d * d + 2 * d * f) + d * wl.vocab) * P    # one pass over every dense layer
        n_dense = 4 * wl.n_blocks + 1
        out.update(gemm_fwd=("mfma", dense, n_dense), gemm_dgrad=("mfma", dense, n_dense), gemm_wgrad=("mfma", dense, n_dense),
                   optimizer=("hbm", 30.0 * n * P, 1))
        return out
    if key == 2:
        mats = list(zip(wl.dims[:-1], wl.dims[1:]))[:-1]                # the two hidden matrices (the output layer has its own kernels)
        flops = sum(2.0 * wl.batch * a * b for a, b in mats) * P
        out["gemm_fwd"] = ("mfma", flops, len(mats))
        out["gemm_dgrad"] = ("mfma", 2.0 * wl.batch * wl.dims[1] * wl.dims[2] * P, 1)
        if fused:
            # per hidden matrix read theta, m, v (12 B) and write theta, m, v and the bf16 shadow (14 B) per parameter, plus the
            # bf16 operands X and dZ
            out["gemm_wgrad"] = ("hbm", (26.0 * sum(a * b for a, b in mats) + 2.0 * wl.batch * sum(a + b for a, b in mats)) * P, len(mats))
        else:
            out["gemm_wgrad"] = ("mfma", flops, len(mats))
            out["optimizer"] = ("hbm", 30.0 * n * P, 1)
    elif key == 3:
        # Adam, one launch per network update (discriminator's, then generator's parameters): 30 B per parameter
        n_d = sum(a * b + b for a, b in zip(wl.dims2[:-1], wl.dims2[1:]))
        k = getattr(wl, "n_critic", 1)
        out["optimizer"] = ("hbm", 30.0 * (n + (k - 1) * n_d) * P, 1 + k)
    else:
        # RMSProp: theta, g and one state array read, theta, state and the bf16 shadow written: 22 B per parameter
        out["optimizer"] = ("hbm", 22.0 * n * P, 1)
    return out


def run_workload(key, steps, warmup, fused, baseline_budget_s, variant=None):
    import torch
    from paper_1711_09846_amd import binding, workloads
    wl = _workload(key, variant)
    seed = workloads.POPULATION_SEED
    pop, d_train, d_eval = _setup_gpu(key, wl, seed, fused)
    K = {"gemm_fwd": binding.K_GEMM_FWD, "gemm_wgrad": binding.K_GEMM_WGRAD, "gemm_dgrad": binding.K_GEMM_DGRAD,
         "optimizer": binding.K_OPTIMIZER, "copy": binding.K_COPY, "fused_step": binding.K_FUSED_STEP}
    work = _work_per_step(key, wl, pop.layout.n_params, fused)

    # the fp32 workload runs a whole ready interval per launch (its weights stay in LDS between the steps)
    chunk = wl.ready_interval if key == 1 else 1
    steps, warmup = max(chunk, steps // chunk * chunk), (warmup + chunk - 1) // chunk * chunk
    for s in range(0, warmup, chunk):
        pop.step(d_train, s, n_steps=chunk)
    # the warm-up also runs eval + exploit once so that nothing is first-touched in a timed region
    pop.eval(d_eval)
    pop.exploit_explore(1 << 20)
    torch.cuda.synchronize()
    # an event pair costs the stream a few microseconds around the launch it brackets, so only every third launch
    # of a class is recorded (an odd stride visits the launches of a step in turn)
    per_step = sum(w[2] for name, w in work.items() if name != "copy")
    stride = 3 if steps // chunk >= 9 else 1
    pop.timing_enable_classes([K[name] for name in work if name != "copy"], per_step * steps // chunk // stride + steps + 16)
    pop.timing_stride(stride)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(warmup, warmup + steps, chunk):
        pop.step(d_train, s, n_steps=chunk)
    torch.cuda.synchronize()
    dt_steps = time.perf_counter() - t0
    timed = {name: pop.timing_read_class(K[name]) for name in work if name != "copy"}
    pop.timing_enable_classes([K["copy"]], 8)
    pop.timing_stride(1)
    t0 = time.perf_counter()
    pop.eval(d_eval)
    torch.cuda.synchronize()
    dt_eval = time.perf_counter() - t0
    t0 = time.perf_counter()
    pop.exploit_explore(0)
    torch.cuda.synchronize()
    dt_exploit = time.perf_counter() - t0
    # (two more rounds outside every clock above: the scores have not changed, so the same members copy again; a
    # single launch of the copy kernel is too noisy a sample for its roofline entry)
    for rnd in (1, 2):
        pop.exploit_explore(rnd)
    torch.cuda.synchronize()

    timed["copy"] = pop.timing_read_class(K["copy"])
    rooflines = []
    measured = TRAFFIC.get((key, bool(fused), variant), {})
    for name, (bound, w, launches) in work.items():
        ms, n_rec = timed[name]
        if not n_rec:
            continue
        avg_s = ms / n_rec * 1e-3
        per_launch = w / launches
        if bound == "hbm":
            ach, peak, unit = per_launch / avg_s / 1e9, HBM_PEAK_GBS, "GB/s"
        elif bound == "mfma":
            ach, peak, unit = per_launch / avg_s / 1e12, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"
        else:
            ach, peak, unit = per_launch / avg_s / 1e12, ALU_FP32_PEAK_TFLOPS, "TFLOP/s"
        r = {"kernel": name, "bound": bound, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
             "traffic": None, "avg_launch_us": avg_s * 1e6, "launches_timed": n_rec, "launches_per_step": launches,
             "work_per_launch": per_launch}
        if name in measured:
            r["traffic"], r["traffic_source"] = measured[name]
        if bound in TARGET:
            r["target_frac"] = TARGET[bound]
            r["meets_target"] = bool(ach / peak >= TARGET[bound])
        rooflines.append(r)
    pop.timing_enable(binding.K_NONE, 0)
    # the GEMM classes together, when the workload's step is bound by them
    gemms = [r for r in rooflines if r["kernel"].startswith("gemm") and r["bound"] == "mfma"]
    if key == 4 and gemms:
        t_all = sum(r["avg_launch_us"] * r["launches_per_step"] for r in gemms)
        w_all = sum(r["work_per_launch"] * r["launches_per_step"] for r in gemms)
        n_all = sum(r["launches_per_step"] for r in gemms)
        ach = w_all / (t_all * 1e-6) / 1e12
        rooflines.insert(0, {"kernel": "gemm (forward, input-gradient and weight-gradient classes together)", "bound": "mfma",
                             "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS,
                             "traffic": None, "avg_launch_us": t_all / n_all, "launches_timed": sum(r["launches_timed"] for r in gemms),
                             "launches_per_step": n_all, "work_per_launch": w_all / n_all, "target_frac": TARGET["mfma"],
                             "meets_target": bool(ach / MFMA_BF16_PEAK_TFLOPS >= TARGET["mfma"])})
        if "gemm" in measured:
            rooflines[0]["traffic"], rooflines[0]["traffic_source"] = measured["gemm"]
    dominant = {1: "fused_step", 2: "gemm_wgrad" if fused else "optimizer", 3: "optimizer", 4: "gemm (", 5: "optimizer"}[key]
    roofline = next((r for r in rooflines if r["kernel"].startswith(dominant)), None)

    ms_step = dt_steps / steps * 1e3
    ms_cadence = (wl.ready_interval * ms_step + (dt_eval + dt_exploit) * 1e3) / wl.ready_interval
    rec = {
        "metric": "population member-steps/sec at 1 MI355X", "value": wl.P / (ms_cadence * 1e-3), "unit": "member-steps/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_cadence,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == workloads.DTYPE_BF16 else "f32", "data": "synthetic",
        "step_only": {"value": wl.P / (ms_step * 1e-3), "ms_per_step": ms_step},
        "eval_ms": dt_eval * 1e3, "exploit_explore_ms": dt_exploit * 1e3,
        "config": {"workload": wl.name + (" (%s)" % variant if variant else ""), "P": wl.P,
                   "dims": wl.dims or {"blocks": wl.n_blocks, "d_model": wl.d_model, "heads": wl.heads, "d_ff": wl.d_ff, "seq": wl.seq, "vocab": wl.vocab},
                   "batch": wl.batch, "optimizer": {0: "sgd_momentum", 1: "adam", 2: "rmsprop"}[wl.optimizer],
                   "fused_optimizer": bool(fused), "steps_per_launch": chunk, "ready_interval": wl.ready_interval, "n_trunc": wl.n_trunc, "eval_rows": wl.n_eval,
                   "cadence": "value = P * ready_interval / (ready_interval timed steps + one timed eval + one timed exploit/explore)"},
        "roofline": roofline, "rooflines": rooflines,
    }
    pop.close()
    del pop, d_train, d_eval
    torch.cuda.empty_cache()
    if baseline_budget_s > 0:
        rec["cpu_baseline"] = cpu_baseline(key, wl, seed, baseline_budget_s)
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps of the top-level workload (default 20; 400 for workloads 2, 3, 5; 2000 for 1)")
    ap.add_argument("--warmup", type=int, default=None, help="default 5")
    ap.add_argument("--workload", type=int, default=0, choices=[0, 1, 2, 3, 4, 5],
                    help="0 (default) = transformer_bf16 as the top-level record plus one record per workload; "
                         "1 = mlp_small_fp32, 2 = mlp_wide_bf16, 3 = gan_mlp_bf16, 4 = transformer_bf16, 5 = a2c_mlp_bf16 alone")
    ap.add_argument("--fused", type=int, default=None, choices=[0, 1],
                    help="1 = optimiser applied inside the weight-gradient GEMMs (default for workload 2, where it is the "
                         "faster of the two as measured), 0 = separate streaming optimiser pass (default otherwise)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (no sharding, no collectives); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)
    top = args.workload or 4
    steps = args.steps if args.steps is not None else {1: 2000, 4: 20}.get(top, 400)
    warmup = args.warmup if args.warmup is not None else 5
    fused = lambda key: args.fused if args.fused is not None and key == top else (1 if key == 2 else 0)
    out = run_workload(top, steps, warmup, fused(top), 0 if args.no_cpu_baseline else 20.0)
    if args.workload == 0:
        subs = []
        for key in (1, 2, 3, 5):
            k_steps, k_warm = SUB_STEPS[key]
            subs.append(run_workload(key, k_steps, k_warm, fused(key), 0 if args.no_cpu_baseline else 5.0))
        top_copy = {k: v for k, v in out.items()}
        subs.insert(3, top_copy)
        # the same networks under the other step definitions that are built
        subs.append(run_workload(3, 100, 10, 0, 0, variant="wgan_gp"))
        subs.append(run_workload(5, 200, 20, 0, 0, variant="pool"))
        out["workloads"] = subs
    print(json.dumps(out))


if __name__ == "__main__":
    main()
