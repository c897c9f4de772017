"""Shared plumbing of the GPU parity tests: builds the same population on the
GPU library and in the oracle from one set of seeded inputs, and measures the
distance between the two."""
import numpy as np

from oracle import classifier as oc, pbt as opbt, nets as onets
from paper_1711_09846_amd import binding, workloads


def exploit_variant(wl):
    """The oracle's keyword arguments for the exploit / explore variant a workload description selects."""
    return dict(mode=("truncation", "tournament", "ttest")[getattr(wl, "exploit_mode", 0)],
                ttest_alpha=float(np.float32(getattr(wl, "ttest_alpha", 0.05))),
                copy_weights=not getattr(wl, "keep_weights", 0), copy_hypers=not getattr(wl, "keep_hypers", 0),
                explore="resample" if getattr(wl, "explore_mode", 0) else "perturb",
                resample_prob=float(np.float32(getattr(wl, "resample_prob", 0.0))), priors=wl.priors)


def oracle_spec(wl, seed):
    # optimiser constants cross the C ABI as float32; the oracle widens those exact values
    oc_ = {k: float(np.float32(v)) for k, v in wl.opt_const.items()}
    return oc.ClassifierSpec(wl.dims, wl.act, wl.optimizer, wl.batch, wl.roles, seed,
                             momentum=oc_.get("momentum", float(np.float32(0.9))), beta1=oc_.get("beta1", float(np.float32(0.9))),
                             beta2=oc_.get("beta2", 0.999), eps=oc_.get("eps", 1e-8), wd=oc_.get("wd", 0.0),
                             rho=oc_.get("rho", 0.99), rms_eps=oc_.get("eps", 1e-5),
                             bf16_storage=wl.dtype == workloads.DTYPE_BF16)


class Pair:
    """One population on the GPU and its twin in the oracle."""

    def __init__(self, wl, seed=workloads.POPULATION_SEED, init_seed=5, data=None, eval_chunk=0, ref_members=None,
                 fuse_optimizer=0):
        import torch
        self.torch = torch
        self.wl = wl
        self.seed = seed
        (self.train_x, self.train_y), (self.eval_x, self.eval_y) = data or workloads.classifier_data(wl)
        self.cfg = binding.make_config(wl, seed, eval_chunk=eval_chunk, fuse_optimizer=fuse_optimizer)
        self.gpu = binding.Population(self.cfg)
        weights = workloads.initial_mlp_weights(wl.dims, wl.P, init_seed)
        H = workloads.initial_hypers(wl, init_seed + 1)
        self.gpu.set_members(weights, H)
        self.spec = oracle_spec(wl, seed)
        # the oracle twin of every member, or only of the listed ones (members are independent
        # between exploit points, so a sample can be followed one by one)
        self.ref_ids = list(range(wl.P)) if ref_members is None else list(ref_members)
        self.ref = {i: oc.new_member(self.spec, weights[i], H[i], i) for i in self.ref_ids}
        if ref_members is None:
            self.ref = [self.ref[i] for i in range(wl.P)]
        dev = self.gpu.device
        self.d_train = [torch.from_numpy(self.train_x).to(dev), torch.from_numpy(self.train_y).to(dev)]
        self.d_eval = [torch.from_numpy(self.eval_x).to(dev), torch.from_numpy(self.eval_y).to(dev)]

    # -- one step / eval / exploit on both sides ------------------------------------------------
    def _members(self):
        return [(i, self.ref[i]) for i in self.ref_ids]

    def step_ref(self, s):
        return np.array([oc.step(self.spec, m, i, s, self.train_x, self.train_y) for i, m in self._members()])

    def eval_ref(self):
        return np.array([oc.evaluate(self.spec, m, self.eval_x, self.eval_y) for _, m in self._members()])

    def sync_ref_from_gpu(self, i):
        """Oracle member i takes over the GPU's weights, optimiser state, update count and
        hyperparameters (float32 values widen exactly)."""
        m = self.ref[i]
        lay, dims = self.gpu.layout, self.wl.dims
        n_state = len(m.opt)
        for what, which in [("theta", binding.ARR_W32), ("s0", binding.ARR_OPT0), ("s1", binding.ARR_OPT1)][:1 + n_state]:
            flat = self.gpu.get(which, i).astype(np.float64)
            arrs = m.theta if what == "theta" else m.opt[what]
            for l in range(len(dims) - 1):
                arrs[2 * l] = flat[lay.w_off[l]:lay.w_off[l] + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1]).copy()
                arrs[2 * l + 1] = flat[lay.b_off[l]:lay.b_off[l] + dims[l + 1]].copy()
        m.t = int(self.gpu.get(binding.ARR_T, i)[0])
        m.h = self.gpu.get(binding.ARR_HYPER, i).copy()

    def member_errors(self, i, which, what, flat_ref=None, rms_floor=0.0):
        """(worst per-array, whole-vector) relative L2 distance of member i's `which` array.
        rms_floor: arrays whose reference rms is below it are compared at that scale."""
        g = self.gpu.get(which, i).astype(np.float64)
        r = self.ref_flat(i, what) if flat_ref is None else flat_ref
        lay, dims = self.gpu.layout, self.wl.dims
        worst = 0.0
        for l in range(len(dims) - 1):
            for off, n in ((lay.w_off[l], dims[l] * dims[l + 1]), (lay.b_off[l], dims[l + 1])):
                den = max(np.linalg.norm(r[off:off + n]), rms_floor * np.sqrt(n), 1e-12)
                worst = max(worst, np.linalg.norm(g[off:off + n] - r[off:off + n]) / den)
        return worst, np.linalg.norm(g - r) / max(np.linalg.norm(r), rms_floor * np.sqrt(len(r)), 1e-12)

    def exploit_ref(self, rnd, scores):
        wl = self.wl
        return opbt.exploit_explore(self.ref, rnd, self.seed, wl.n_trunc, wl.perturb[0], wl.perturb[1], wl.h_max,
                                    scores=scores, **exploit_variant(wl))

    # -- distances -----------------------------------------------------------------------------
    def ref_flat(self, member, what):
        """Oracle arrays of one member in the library's flat layout (float64)."""
        m = self.ref[member]
        arrs = m.theta if what == "theta" else m.opt[what]
        layers = [(arrs[2 * l], arrs[2 * l + 1]) for l in range(len(arrs) // 2)]
        lay = self.gpu.layout
        flat = np.zeros(lay.stride)
        for l, (W, b) in enumerate(layers):
            flat[lay.w_off[l]:lay.w_off[l] + W.size] = W.ravel()
            flat[lay.b_off[l]:lay.b_off[l] + b.size] = b.ravel()
        return flat

    def tensor_errors(self, which, what):
        """max over members and parameter arrays of ||gpu - ref||_2 / max(||ref||_2, 1e-12)."""
        G = self.gpu.get(which).astype(np.float64)
        lay, dims = self.gpu.layout, self.wl.dims
        worst = 0.0
        for i in range(self.wl.P):
            R = self.ref_flat(i, what)
            for l in range(len(dims) - 1):
                for off, n in ((lay.w_off[l], dims[l] * dims[l + 1]), (lay.b_off[l], dims[l + 1])):
                    g, r = G[i, off:off + n], R[off:off + n]
                    worst = max(worst, np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-12))
        return worst

    @staticmethod
    def scalar_errors(gpu, ref, floor):
        """max |gpu - ref| / max(|ref|, floor) over members (losses, scores)."""
        gpu, ref = np.asarray(gpu, dtype=np.float64), np.asarray(ref, dtype=np.float64)
        return float(np.max(np.abs(gpu - ref) / np.maximum(np.abs(ref), floor)))


class GanPair:
    """A GAN population on the GPU and its oracle twin (all members or a sample)."""

    def __init__(self, wl, seed=workloads.POPULATION_SEED, init_seed=5, ref_members=None, fuse_optimizer=0):
        import torch
        from oracle import gan as og
        self.og, self.wl, self.seed = og, wl, seed
        self.train_x, self.eval_x = workloads.gan_data(wl)
        self.cfg = binding.make_config(wl, seed, fuse_optimizer=fuse_optimizer)
        self.gpu = binding.Population(self.cfg)
        weights = workloads.initial_gan_weights(wl, wl.P, init_seed)
        H = workloads.initial_hypers(wl, init_seed + 1)
        self.gpu.set_members([list(g) + list(d) for g, d in weights], H)
        oc_ = {k: float(np.float32(v)) for k, v in wl.opt_const.items()}
        self.spec = og.GanSpec(wl.dims, wl.dims2, wl.batch, seed, roles=wl.roles, g_hidden=wl.act, g_out=wl.act_out,
                               d_hidden=wl.act2, beta1=oc_["beta1"], beta2=oc_["beta2"], eps=oc_["eps"],
                               bf16_storage=wl.dtype == workloads.DTYPE_BF16, objective=getattr(wl, "objective", "logistic"),
                               n_critic=getattr(wl, "n_critic", 1), gp_weight=float(np.float32(getattr(wl, "gp_weight", 10.0))))
        self.ref_ids = list(range(wl.P)) if ref_members is None else list(ref_members)
        self.ref = {i: og.new_member(self.spec, weights[i][0], weights[i][1], H[i], i) for i in self.ref_ids}
        dev = self.gpu.device
        self.d_train = [torch.from_numpy(self.train_x).to(dev)]
        self.d_eval = [torch.from_numpy(self.eval_x).to(dev)]

    def step_ref(self, s):
        return np.array([self.og.step(self.spec, self.ref[i], i, s, self.train_x) for i in self.ref_ids])

    def eval_ref(self):
        return np.array([self.og.evaluate(self.spec, self.ref[i], i, self.eval_x) for i in self.ref_ids])

    def ref_flat(self, i, what):
        m = self.ref[i]
        arrs = m.theta if what == "theta" else m.opt[what]
        lay = self.gpu.layout
        flat = np.zeros(lay.stride)
        for l in range(len(arrs) // 2):
            W, b = arrs[2 * l], arrs[2 * l + 1]
            flat[lay.w_off[l]:lay.w_off[l] + W.size] = W.ravel()
            flat[lay.b_off[l]:lay.b_off[l] + b.size] = b.ravel()
        return flat

    def sync_ref_from_gpu(self, i):
        m = self.ref[i]
        lay, shapes = self.gpu.layout, self.gpu.layer_shapes
        for what, which in (("theta", binding.ARR_W32), ("s0", binding.ARR_OPT0), ("s1", binding.ARR_OPT1)):
            flat = self.gpu.get(which, i).astype(np.float64)
            arrs = m.theta if what == "theta" else m.opt[what]
            for l, (fi, fo) in enumerate(shapes):
                arrs[2 * l] = flat[lay.w_off[l]:lay.w_off[l] + fi * fo].reshape(fi, fo).copy()
                arrs[2 * l + 1] = flat[lay.b_off[l]:lay.b_off[l] + fo].copy()
        m.t = int(self.gpu.get(binding.ARR_T, i)[0])
        m.h = self.gpu.get(binding.ARR_HYPER, i).copy()

    def member_errors(self, i, which, what):
        """(worst per-array, whole-vector) relative L2 distance of member i's array."""
        g = self.gpu.get(which, i).astype(np.float64)
        r = self.ref_flat(i, what)
        lay = self.gpu.layout
        worst = 0.0
        for l, (fi, fo) in enumerate(self.gpu.layer_shapes):
            for off, n in ((lay.w_off[l], fi * fo), (lay.b_off[l], fo)):
                worst = max(worst, np.linalg.norm(g[off:off + n] - r[off:off + n]) / max(np.linalg.norm(r[off:off + n]), 1e-12))
        return worst, np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-12)

    def exploit_ref(self, rnd, scores):
        wl = self.wl
        pop = [self.ref[i] for i in range(wl.P)]
        return opbt.exploit_explore(pop, rnd, self.seed, wl.n_trunc, wl.perturb[0], wl.perturb[1], wl.h_max, scores=scores,
                                    **exploit_variant(wl))


class A2CPair:
    """An actor-critic population on the GPU and its oracle twin (all members or a sample)."""

    def __init__(self, wl, seed=workloads.POPULATION_SEED, init_seed=5, ref_members=None, fuse_optimizer=0):
        import torch
        from oracle import a2c as oa
        self.oa, self.wl, self.seed = oa, wl, seed
        self.on_policy = bool(getattr(wl, "on_policy", 0))
        if self.on_policy:
            from oracle import a2c_env
            self.env_mod = a2c_env
            self.env = a2c_env.Environment(*workloads.latent_system(wl))
        else:
            self.obs, self.actions, self.rewards = workloads.trajectory_pool(wl)
        self.cfg = binding.make_config(wl, seed, fuse_optimizer=fuse_optimizer)
        self.gpu = binding.Population(self.cfg)
        weights = workloads.initial_mlp_weights(wl.dims, wl.P, init_seed)
        H = workloads.initial_hypers(wl, init_seed + 1)
        self.gpu.set_members(weights, H)
        oc_ = {k: float(np.float32(v)) for k, v in wl.opt_const.items()}
        self.spec = oa.A2CSpec(wl.dims[:-1], wl.n_actions, wl.batch, wl.unroll, seed, roles=wl.roles,
                               gamma=float(np.float32(wl.gamma)), value_cost=float(np.float32(wl.value_cost)),
                               rho=oc_["rho"], rms_eps=oc_["eps"], hidden_act=wl.act,
                               bf16_storage=wl.dtype == workloads.DTYPE_BF16)
        self.ref_ids = list(range(wl.P)) if ref_members is None else list(ref_members)
        self.ref = {i: oa.new_member(self.spec, weights[i], H[i], i) for i in self.ref_ids}
        dev = self.gpu.device
        if self.on_policy:
            e = self.env
            noise = np.array([e.obs_noise, e.reward_noise, e.trans_noise])
            self.d_pool = [torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64)).to(dev) for a in (e.A, e.B, e.C, e.w, noise)]
        else:
            self.d_pool = [torch.from_numpy(self.obs).to(dev), torch.from_numpy(self.actions).to(dev),
                           torch.from_numpy(self.rewards).to(dev)]

    def gpu_unroll(self, i):
        """The unroll member i's last step was taken on, as the GPU holds it: (obs float64 [B][T+1][d] of bf16
        values, actions [B][T], rewards float32 [B][T])."""
        wl = self.wl
        obs = (self.gpu.get(binding.ARR_TRAJ_OBS, i).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        return (obs.reshape(wl.batch, wl.unroll + 1, wl.dims[0]), self.gpu.get(binding.ARR_TRAJ_ACT, i).reshape(wl.batch, wl.unroll),
                self.gpu.get(binding.ARR_TRAJ_REW, i).reshape(wl.batch, wl.unroll))

    def step_ref(self, s):
        if self.on_policy:      # the oracle takes its step on the unroll the GPU generated
            return np.array([self.oa.step_on_policy(self.spec, self.env, self.ref[i], i, s, batch=self.gpu_unroll(i))[0] for i in self.ref_ids])
        return np.array([self.oa.step(self.spec, self.ref[i], i, s, self.obs, self.actions, self.rewards) for i in self.ref_ids])

    def eval_ref(self):
        return np.array([self.oa.evaluate(self.spec, self.ref[i]) for i in self.ref_ids], dtype=np.float32)

    ref_flat = GanPair.ref_flat
    member_errors = GanPair.member_errors

    def sync_ref_from_gpu(self, i):
        m = self.ref[i]
        lay, shapes = self.gpu.layout, self.gpu.layer_shapes
        for what, which in (("theta", binding.ARR_W32), ("s0", binding.ARR_OPT0)):
            flat = self.gpu.get(which, i).astype(np.float64)
            arrs = m.theta if what == "theta" else m.opt[what]
            for l, (fi, fo) in enumerate(shapes):
                arrs[2 * l] = flat[lay.w_off[l]:lay.w_off[l] + fi * fo].reshape(fi, fo).copy()
                arrs[2 * l + 1] = flat[lay.b_off[l]:lay.b_off[l] + fo].copy()
        m.t = int(self.gpu.get(binding.ARR_T, i)[0])
        m.h = self.gpu.get(binding.ARR_HYPER, i).copy()
        m.hist = [np.float32(v) for v in self.gpu.history()[i]]

    def exploit_ref(self, rnd, scores):
        wl = self.wl
        pop = [self.ref[i] for i in range(wl.P)]
        return opbt.exploit_explore(pop, rnd, self.seed, wl.n_trunc, wl.perturb[0], wl.perturb[1], wl.h_max, scores=scores,
                                    **exploit_variant(wl))


class TransformerPair:
    """A transformer population on the GPU and its oracle twin (all members or a sample)."""

    def __init__(self, wl, seed=workloads.POPULATION_SEED, init_seed=5, ref_members=None, H=None):
        import torch
        from oracle import transformer as ot
        self.ot, self.wl, self.seed = ot, wl, seed
        self.pool, self.eval_seqs = workloads.zipf_bigram_sequences(wl)
        self.cfg = binding.make_config(wl, seed)
        self.gpu = binding.Population(self.cfg)
        self.shapes = workloads.transformer_shapes(wl)
        weights = workloads.initial_transformer_weights(wl, wl.P, init_seed)
        H = workloads.initial_hypers(wl, init_seed + 1) if H is None else np.asarray(H, dtype=np.float32)
        self.gpu.set(binding.ARR_W32, np.stack([binding.pack_segments(self.gpu.layout, a) for a in weights]))
        self.gpu.set(binding.ARR_HYPER, H)
        oc_ = {k: float(np.float32(v)) for k, v in wl.opt_const.items()}
        self.spec = ot.TransformerSpec(wl.vocab, wl.d_model, wl.heads, wl.d_ff, wl.n_blocks, wl.seq, wl.batch, seed,
                                       roles=wl.roles, beta1=oc_["beta1"], beta2=oc_["beta2"], eps=oc_["eps"],
                                       bf16_storage=True)
        assert [s for _, s in self.spec.param_shapes()] == self.shapes
        self.ref_ids = list(range(wl.P)) if ref_members is None else list(ref_members)
        self.ref = {i: ot.new_member(self.spec, weights[i], H[i], i) for i in self.ref_ids}
        dev = self.gpu.device
        self.d_pool = [torch.from_numpy(self.pool).to(dev)]
        self.d_eval = [torch.from_numpy(self.eval_seqs).to(dev)]

    def step_ref(self, s):
        return np.array([self.ot.step(self.spec, self.ref[i], i, s, self.pool) for i in self.ref_ids])

    def eval_ref(self):
        return np.array([self.ot.evaluate(self.spec, self.ref[i], self.eval_seqs, chunk=self.wl.batch) for i in self.ref_ids])

    def ref_arrays(self, i, what):
        m = self.ref[i]
        return m.theta if what == "theta" else m.opt[what]

    def gpu_arrays(self, i, which):
        return binding.unpack_segments(self.gpu.layout, self.shapes, self.gpu.get(which, i).astype(np.float64))

    def array_errors(self, i, which, ref_arrays, rms_floor=0.0, skip_key_bias=False):
        """Per parameter array: relative L2 distance between the GPU's and the given reference arrays.

        skip_key_bias leaves the key third of every bqkv out.  Adding a constant to all keys shifts each
        row of scores by a constant, which the softmax removes: the network does not depend on the key
        bias and its exact gradient is zero.  What reaches Adam is rounding noise, which Adam's
        normalisation turns into steps of the full learning rate with random signs, so the value of
        that bias (and its moment estimates) is not a reproducible quantity."""
        d = self.wl.d_model
        out = []
        for (name, _), g, r in zip(self.spec.param_shapes(), self.gpu_arrays(i, which), ref_arrays):
            if skip_key_bias and name.startswith("bqkv"):
                g, r = np.delete(g, np.s_[d:2 * d]), np.delete(r, np.s_[d:2 * d])
            den = max(np.linalg.norm(r), rms_floor * np.sqrt(r.size), 1e-30)
            out.append(np.linalg.norm(g - r) / den)
        return np.array(out)

    def sync_ref_from_gpu(self, i):
        m = self.ref[i]
        for what, which in (("theta", binding.ARR_W32), ("s0", binding.ARR_OPT0), ("s1", binding.ARR_OPT1)):
            arrs = self.gpu_arrays(i, which)
            if what == "theta":
                m.theta = arrs
            else:
                m.opt[what] = arrs
        m.t = int(self.gpu.get(binding.ARR_T, i)[0])
        m.h = self.gpu.get(binding.ARR_HYPER, i).copy()

    def exploit_ref(self, rnd, scores):
        wl = self.wl
        pop = [self.ref[i] for i in range(wl.P)]
        return opbt.exploit_explore(pop, rnd, self.seed, wl.n_trunc, wl.perturb[0], wl.perturb[1], wl.h_max, scores=scores,
                                    **exploit_variant(wl))


# ---- helpers shared by the window tests: any pair, any oracle member (not only pair.ref) ----------------

def gpu_arrays(pair, i, which):
    """Member i's `which` array of the population store as float64 parameter arrays in the oracle's order."""
    if isinstance(pair, TransformerPair):
        return pair.gpu_arrays(i, which)
    flat = pair.gpu.get(which, i).astype(np.float64)
    lay, out = pair.gpu.layout, []
    for l, (fi, fo) in enumerate(pair.gpu.layer_shapes):
        out.append(flat[lay.w_off[l]:lay.w_off[l] + fi * fo].reshape(fi, fo).copy())
        out.append(flat[lay.b_off[l]:lay.b_off[l] + fo].copy())
    return out


def sync_member(pair, m, i):
    """Oracle member m takes over GPU member i's weights, optimiser state, update count, hyperparameters
    (and return history): float32 values widen exactly."""
    m.theta = gpu_arrays(pair, i, binding.ARR_W32)
    for what, which in (("s0", binding.ARR_OPT0), ("s1", binding.ARR_OPT1)):
        if what in m.opt:
            m.opt[what] = gpu_arrays(pair, i, which)
    m.t = int(pair.gpu.get(binding.ARR_T, i)[0])
    m.h = pair.gpu.get(binding.ARR_HYPER, i).copy()
    if isinstance(pair, A2CPair):
        m.hist = [np.float32(v) for v in pair.gpu.history()[i]]


def oracle_step(pair, m, i, s, spec=None):
    """One `step` of oracle member m as population member i; returns the loss(es) as a float array."""
    spec = spec or pair.spec
    if isinstance(pair, TransformerPair):
        return np.array([pair.ot.step(spec, m, i, s, pair.pool)])
    if isinstance(pair, GanPair):
        return np.array(pair.og.step(spec, m, i, s, pair.train_x))
    if isinstance(pair, A2CPair):
        if pair.on_policy:
            return np.array([pair.oa.step_on_policy(spec, pair.env, m, i, s, batch=pair.gpu_unroll(i))[0]])
        return np.array([pair.oa.step(spec, m, i, s, pair.obs, pair.actions, pair.rewards)])
    return np.array([oc.step(spec, m, i, s, pair.train_x, pair.train_y)])


def oracle_eval(pair, m, i, spec=None):
    spec = spec or pair.spec
    if isinstance(pair, TransformerPair):
        return float(pair.ot.evaluate(spec, m, pair.eval_seqs, chunk=pair.wl.batch))
    if isinstance(pair, GanPair):
        return float(pair.og.evaluate(spec, m, i, pair.eval_x))
    if isinstance(pair, A2CPair):
        return float(pair.oa.evaluate(spec, m))
    return float(oc.evaluate(spec, m, pair.eval_x, pair.eval_y))


def train_inputs(pair):
    return pair.d_pool if hasattr(pair, "d_pool") else pair.d_train


def eval_inputs(pair):
    return [] if isinstance(pair, A2CPair) else pair.d_eval


def exact_spec(pair):
    """The pair's oracle specification without the bf16 rounding model: plain float64 everywhere."""
    import copy
    spec = copy.copy(pair.spec)
    spec.q = onets.identity
    return spec


def array_distances(pair, got, ref, bias_floor=0.0):
    """(per-array relative L2 distances, whole-vector relative L2 distance) between two lists of parameter
    arrays.  The transformer's key biases are left out (the network does not depend on them: softmax removes
    a constant added to all keys, so their gradient is rounding noise).  bias_floor: one-dimensional arrays
    (biases, which start at or near zero) are compared at no smaller scale than an rms of bias_floor."""
    d = pair.wl.d_model if isinstance(pair, TransformerPair) else 0
    names = [n for n, _ in pair.spec.param_shapes()] if d else [""] * len(ref)
    per, num, den = [], 0.0, 0.0
    for name, g, r in zip(names, got, ref):
        g, r = np.asarray(g, dtype=np.float64), np.asarray(r, dtype=np.float64)
        if name.startswith("bqkv"):
            g, r = np.delete(g, np.s_[d:2 * d]), np.delete(r, np.s_[d:2 * d])
        floor = bias_floor * np.sqrt(r.size) if r.ndim == 1 else 0.0
        per.append(np.linalg.norm(g - r) / max(np.linalg.norm(r), floor, 1e-30))
        num += float(np.sum((g - r) ** 2))
        den += float(np.sum(r ** 2))
    return np.array(per), float(np.sqrt(num / max(den, 1e-300)))
