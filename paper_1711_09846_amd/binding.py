"""ctypes binding of the C-ABI library `libpbt.so` (declared in include/pbt.h).

Argument marshalling only: every step of the population pass runs in the
library's HIP kernels.  PyTorch supplies device memory (`torch.empty` on
`cuda`) and the current HIP stream.  If the library has not been built the
import of a symbol fails loudly; there is no fallback path.
"""
import ctypes as C
import math
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpbt.so")

PBT_MAX_DIMS, PBT_MAX_HYPER, PBT_MAX_SEGMENTS = 16, 8, 96
(ARR_W32, ARR_OPT0, ARR_OPT1, ARR_W16, ARR_GRAD, ARR_HYPER, ARR_SCORE, ARR_LOSS, ARR_T, ARR_ORDER, ARR_DONOR,
 ARR_PARENT, ARR_HIST, ARR_TRAJ_OBS, ARR_TRAJ_ACT, ARR_TRAJ_REW) = range(16)
_ARR_DTYPE = {ARR_W32: np.float32, ARR_OPT0: np.float32, ARR_OPT1: np.float32, ARR_W16: np.uint16,
              ARR_GRAD: np.float32, ARR_HYPER: np.float32, ARR_SCORE: np.float32, ARR_LOSS: np.float32,
              ARR_T: np.int32, ARR_ORDER: np.int32, ARR_DONOR: np.int32, ARR_PARENT: np.int32, ARR_HIST: np.float32,
              ARR_TRAJ_OBS: np.uint16, ARR_TRAJ_ACT: np.int32, ARR_TRAJ_REW: np.float32}

EXPORTS = ["pbt_query_sizes", "pbt_init", "pbt_step", "pbt_eval", "pbt_exploit_explore", "pbt_get_state",
           "pbt_set_state", "pbt_state_ptr", "pbt_destroy", "pbt_last_error", "pbt_batched_gemm_bf16",
           "pbt_timing_enable", "pbt_timing_stride", "pbt_timing_read", "pbt_init_population", "pbt_set_priors",
           "pbt_step_static", "pbt_timing_enable_classes", "pbt_timing_read_class"]
STATIC_SCRATCH_BYTES = 8 << 20
(K_NONE, K_FETCH, K_GEMM_FWD, K_HEAD, K_GEMM_WGRAD, K_GEMM_DGRAD, K_BIAS_GRAD, K_OPTIMIZER, K_RANK, K_COPY,
 K_FUSED_STEP) = range(-1, 10)


class PbtConfig(C.Structure):
    _fields_ = [("workload", C.c_int32), ("P", C.c_int32), ("batch", C.c_int32), ("n_layers", C.c_int32),
                ("dims", C.c_int32 * PBT_MAX_DIMS), ("act", C.c_int32), ("optimizer", C.c_int32),
                ("compute_dtype", C.c_int32), ("n_hyper", C.c_int32), ("hyper_role", C.c_int32 * PBT_MAX_HYPER),
                ("hyper_max", C.c_float * PBT_MAX_HYPER), ("n_trunc", C.c_int32), ("perturb_lo", C.c_float),
                ("perturb_hi", C.c_float), ("opt_const", C.c_float * 4), ("act_out", C.c_int32),
                ("n_layers2", C.c_int32), ("dims2", C.c_int32 * PBT_MAX_DIMS), ("act2", C.c_int32), ("unroll", C.c_int32),
                ("gamma", C.c_float), ("value_cost", C.c_float), ("tf_vocab", C.c_int32), ("tf_d_model", C.c_int32),
                ("tf_heads", C.c_int32), ("tf_d_ff", C.c_int32), ("tf_seq", C.c_int32), ("n_train", C.c_int32),
                ("n_eval", C.c_int32), ("eval_chunk", C.c_int32), ("fuse_optimizer", C.c_int32), ("exploit_mode", C.c_int32),
                ("explore_mode", C.c_int32), ("resample_prob", C.c_float), ("keep_weights", C.c_int32), ("keep_hypers", C.c_int32),
                ("ttest_alpha", C.c_float), ("on_policy", C.c_int32), ("latent_dim", C.c_int32),
                ("gan_objective", C.c_int32), ("n_critic", C.c_int32), ("gp_weight", C.c_float),
                ("seed", C.c_uint64)]


class PbtLayout(C.Structure):
    _fields_ = [("stride", C.c_int64), ("n_params", C.c_int64), ("w_off", C.c_int64 * PBT_MAX_DIMS),
                ("b_off", C.c_int64 * PBT_MAX_DIMS), ("n_seg", C.c_int32), ("seg_off", C.c_int64 * PBT_MAX_SEGMENTS),
                ("seg_len", C.c_int64 * PBT_MAX_SEGMENTS)]


class PbtPrior(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lo", C.c_double), ("hi", C.c_double)]


class PbtError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("pbt status %d: %s" % (status, message))
        self.status = status


_lib = None


def lib():
    """Opens libpbt.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: build it with `python -m paper_1711_09846_amd.build`" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        L.pbt_query_sizes.argtypes = [C.POINTER(PbtConfig), C.POINTER(sz), C.POINTER(sz), C.POINTER(PbtLayout)]
        L.pbt_init.argtypes = [C.POINTER(PbtConfig), vp, sz, vp, sz, vp, C.POINTER(vp)]
        L.pbt_step.argtypes = [vp, C.POINTER(vp), i32, i64, i32, vp]
        L.pbt_step_static.argtypes = [vp, C.POINTER(vp), i32, i64, i32, vp]
        L.pbt_eval.argtypes = [vp, C.POINTER(vp), i32, vp]
        L.pbt_exploit_explore.argtypes = [vp, i64, vp, vp]
        L.pbt_get_state.argtypes = [vp, i32, i32, vp, sz, vp]
        L.pbt_set_state.argtypes = [vp, i32, i32, vp, sz, vp]
        L.pbt_state_ptr.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(sz)]
        L.pbt_destroy.argtypes = [vp]
        L.pbt_last_error.argtypes = [vp]
        L.pbt_last_error.restype = C.c_char_p
        L.pbt_batched_gemm_bf16.argtypes = [vp, i64, i64, i32, vp, i64, i64, i32, vp, i64, i64, i32, i32, i32, i32, i32, vp]
        L.pbt_init_population.argtypes = [vp, C.POINTER(PbtPrior), vp]
        L.pbt_set_priors.argtypes = [vp, C.POINTER(PbtPrior)]
        L.pbt_timing_enable.argtypes = [vp, i32, i32]
        L.pbt_timing_stride.argtypes = [vp, i32]
        L.pbt_timing_enable_classes.argtypes = [vp, C.c_uint32, i32]
        L.pbt_timing_read_class.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(i64)]
        L.pbt_timing_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
        for name in EXPORTS:
            if name != "pbt_last_error":
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def make_config(wl, seed, P=None, n_trunc=None, eval_chunk=0, fuse_optimizer=0):
    """PbtConfig from a workloads.Workload description."""
    c = PbtConfig()
    c.workload = wl.kind
    c.P = wl.P if P is None else P
    c.batch = wl.batch
    if wl.kind == 4:                                    # transformer: n_layers counts blocks
        c.n_layers = wl.n_blocks
        c.tf_vocab, c.tf_d_model, c.tf_heads, c.tf_d_ff, c.tf_seq = wl.vocab, wl.d_model, wl.heads, wl.d_ff, wl.seq
    else:
        c.n_layers = len(wl.dims) - 1
        for k, d in enumerate(wl.dims):
            c.dims[k] = d
    c.act, c.optimizer, c.compute_dtype = wl.act, wl.optimizer, wl.dtype
    c.n_hyper = len(wl.roles)
    for k, r in enumerate(wl.roles):
        c.hyper_role[k] = r
        c.hyper_max[k] = wl.h_max[k]
    c.n_trunc = wl.n_trunc if n_trunc is None else n_trunc
    c.perturb_lo, c.perturb_hi = wl.perturb
    oc = wl.opt_const
    if wl.optimizer == 0:
        vals = [oc.get("momentum", 0.9), 0, 0, 0]
    elif wl.optimizer == 1:
        vals = [oc.get("beta1", 0.9), oc.get("beta2", 0.999), oc.get("eps", 1e-8), oc.get("wd", 0.0)]
    else:
        vals = [oc.get("rho", 0.99), oc.get("eps", 1e-5), 0, 0]
    for k, v in enumerate(vals):
        c.opt_const[k] = v
    if getattr(wl, "dims2", None):                      # two-network workloads (GAN): generator, then discriminator
        c.act_out, c.act2, c.n_layers2 = wl.act_out, wl.act2, len(wl.dims2) - 1
        for k, d in enumerate(wl.dims2):
            c.dims2[k] = d
    if getattr(wl, "unroll", None):                     # actor-critic
        c.unroll, c.gamma, c.value_cost = wl.unroll, wl.gamma, wl.value_cost
    c.n_train, c.n_eval, c.eval_chunk = wl.n_train, wl.n_eval, eval_chunk
    c.fuse_optimizer = fuse_optimizer
    # variants of exploit / explore (Sections 4.3.1, 4.4, 4.1.1 Explore (b)); all default to 0
    c.exploit_mode = getattr(wl, "exploit_mode", 0)
    c.explore_mode = getattr(wl, "explore_mode", 0)
    c.resample_prob = getattr(wl, "resample_prob", 0.0)
    c.keep_weights = getattr(wl, "keep_weights", 0)
    c.keep_hypers = getattr(wl, "keep_hypers", 0)
    c.ttest_alpha = getattr(wl, "ttest_alpha", 0.0)
    c.on_policy = getattr(wl, "on_policy", 0)
    c.latent_dim = getattr(wl, "latent", 0) if wl.kind == 5 else 0
    c.gan_objective = 1 if getattr(wl, "objective", "logistic") == "wgan_gp" else 0
    c.n_critic = getattr(wl, "n_critic", 1)
    c.gp_weight = getattr(wl, "gp_weight", 10.0)
    c.seed = seed
    return c


def query_sizes(cfg):
    st, sc, lay = C.c_size_t(), C.c_size_t(), PbtLayout()
    rc = lib().pbt_query_sizes(C.byref(cfg), C.byref(st), C.byref(sc), C.byref(lay))
    if rc != 0:
        raise PbtError(rc, lib().pbt_last_error(None).decode())
    return st.value, sc.value, lay


def pack_params(lay, layers):
    """[(W[fan_in][fan_out], b[fan_out]), ...] -> flat float32 vector of one member (padding = 0)."""
    flat = np.zeros(lay.stride, dtype=np.float32)
    for l, (W, b) in enumerate(layers):
        flat[lay.w_off[l]:lay.w_off[l] + W.size] = np.asarray(W, dtype=np.float32).ravel()
        flat[lay.b_off[l]:lay.b_off[l] + b.size] = np.asarray(b, dtype=np.float32).ravel()
    return flat


def pack_segments(lay, arrays):
    """Parameter arrays in layout order -> flat float32 vector of one member (padding = 0)."""
    assert len(arrays) == lay.n_seg
    flat = np.zeros(lay.stride, dtype=np.float32)
    for j, a in enumerate(arrays):
        assert a.size == lay.seg_len[j]
        flat[lay.seg_off[j]:lay.seg_off[j] + a.size] = np.asarray(a, dtype=np.float32).ravel()
    return flat


def unpack_segments(lay, shapes, flat):
    """Inverse of pack_segments; shapes in layout order."""
    return [np.array(flat[lay.seg_off[j]:lay.seg_off[j] + int(np.prod(sh))]).reshape(sh) for j, sh in enumerate(shapes)]


def unpack_params(lay, dims, flat):
    """dims: widths of one MLP, or a list of (fan_in, fan_out) pairs in layout order."""
    shapes = dims if dims and isinstance(dims[0], tuple) else list(zip(dims[:-1], dims[1:]))
    out = []
    for l, (fi, fo) in enumerate(shapes):
        W = np.array(flat[lay.w_off[l]:lay.w_off[l] + fi * fo]).reshape(fi, fo)
        b = np.array(flat[lay.b_off[l]:lay.b_off[l] + fo])
        out.append((W, b))
    return out


class Population:
    """Owns the device buffers (through torch) and a library handle."""

    def __init__(self, cfg, device="cuda:0"):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        state_bytes, scratch_bytes, self.layout = query_sizes(cfg)
        self.state = torch.empty(state_bytes, dtype=torch.uint8, device=self.device)
        self.scratch = torch.empty(scratch_bytes, dtype=torch.uint8, device=self.device)
        self._h = C.c_void_p()
        with torch.cuda.device(self.device):
            rc = lib().pbt_init(C.byref(cfg), self.state.data_ptr(), state_bytes, self.scratch.data_ptr(),
                                scratch_bytes, self._stream(), C.byref(self._h))
        if rc != 0:
            raise PbtError(rc, lib().pbt_last_error(None).decode())
        self.dims = [cfg.dims[k] for k in range(cfg.n_layers + 1)]
        self.n_loss = 2 if cfg.workload == 3 else 1
        # (fan_in, fan_out) of every dense layer in layout order
        self.layer_shapes = list(zip(self.dims[:-1], self.dims[1:]))
        if cfg.n_layers2:
            d2 = [cfg.dims2[k] for k in range(cfg.n_layers2 + 1)]
            self.layer_shapes += list(zip(d2[:-1], d2[1:]))

    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def _check(self, rc):
        if rc != 0:
            raise PbtError(rc, lib().pbt_last_error(self._h).decode())

    @staticmethod
    def _ptrs(tensors):
        arr = (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
        return arr

    def step(self, inputs, step_index, n_steps=1):
        self._check(lib().pbt_step(self._h, self._ptrs(inputs), len(inputs), step_index, n_steps, self._stream()))

    def step_static(self, inputs, step_index, n_steps=1):
        """pbt_step with the library's static working memory (no buffer of the caller's is used as scratch)."""
        self._check(lib().pbt_step_static(self._h, self._ptrs(inputs), len(inputs), step_index, n_steps, self._stream()))

    def eval(self, inputs=()):
        ptrs = self._ptrs(inputs) if len(inputs) else None
        self._check(lib().pbt_eval(self._h, ptrs, len(inputs), self._stream()))

    def history(self):
        """Actor-critic: per member the unroll returns still in the ring, oldest first."""
        raw = self.get(ARR_HIST)
        out = []
        for row in raw:
            n = int(row[10:11].view(np.int32)[0])
            m = min(n, 10)
            out.append([row[(n - m + k) % 10] for k in range(m)])
        return out

    def exploit_explore(self, round_index, scores_override=None):
        p = None if scores_override is None else C.c_void_p(scores_override.data_ptr())
        self._check(lib().pbt_exploit_explore(self._h, round_index, p, self._stream()))

    def init_population(self, priors):
        """priors: [("uniform" | "log", lo, hi), ...], one per hyperparameter column."""
        arr = (PbtPrior * len(priors))(*[PbtPrior(1 if k == "log" else 0, lo, hi) for k, lo, hi in priors])
        self._check(lib().pbt_init_population(self._h, arr, self._stream()))

    def set_priors(self, priors):
        """priors as in init_population; used by resample explore."""
        arr = (PbtPrior * len(priors))(*[PbtPrior(1 if k == "log" else 0, lo, hi) for k, lo, hi in priors])
        self._check(lib().pbt_set_priors(self._h, arr))

    def timing_enable(self, kernel_class, max_launches=1):
        self._check(lib().pbt_timing_enable(self._h, kernel_class, max_launches))

    def timing_enable_classes(self, classes, max_launches):
        """Brackets every launch of the listed kernel classes (K_* constants) with HIP events."""
        mask = 0
        for k in classes:
            mask |= 1 << k
        self._check(lib().pbt_timing_enable_classes(self._h, mask, max_launches))

    def timing_read_class(self, kernel_class):
        """(summed device milliseconds, recorded launches) of one class; does not rearm."""
        ms, n = C.c_double(), C.c_int64()
        self._check(lib().pbt_timing_read_class(self._h, kernel_class, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def timing_stride(self, stride):
        self._check(lib().pbt_timing_stride(self._h, stride))

    def timing_read(self):
        ms, n = C.c_double(), C.c_int64()
        self._check(lib().pbt_timing_read(self._h, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def _shape(self, which):
        P = self.cfg.P
        if which in (ARR_W32, ARR_OPT0, ARR_OPT1, ARR_W16, ARR_GRAD):
            return (P, self.layout.stride)
        if which == ARR_HYPER:
            return (P, self.cfg.n_hyper)
        if which == ARR_HIST:
            return (P, 12)
        if which == ARR_TRAJ_OBS:
            return (P, self.cfg.batch * (self.cfg.unroll + 1), self.cfg.dims[0])
        if which in (ARR_TRAJ_ACT, ARR_TRAJ_REW):
            return (P, self.cfg.batch * self.cfg.unroll)
        if which == ARR_LOSS and self.n_loss > 1:
            return (P, self.n_loss)
        return (P,)

    def get(self, which, member=-1):
        shape = self._shape(which)
        if member >= 0:
            shape = shape[1:] if len(shape) > 1 else (1,)
        out = np.empty(shape, dtype=_ARR_DTYPE[which])
        self._check(lib().pbt_get_state(self._h, which, member, out.ctypes.data, out.nbytes, self._stream()))
        return out

    def set(self, which, values, member=-1):
        a = np.ascontiguousarray(values, dtype=_ARR_DTYPE[which])
        self._check(lib().pbt_set_state(self._h, which, member, a.ctypes.data, a.nbytes, self._stream()))

    def device_view(self, which):
        """Zero-copy torch view of one array of the store."""
        ptr, nbytes = C.c_void_p(), C.c_size_t()
        self._check(lib().pbt_state_ptr(self._h, which, C.byref(ptr), C.byref(nbytes)))
        base = self.state if self.state.data_ptr() <= ptr.value < self.state.data_ptr() + self.state.numel() else self.scratch
        off = ptr.value - base.data_ptr()
        tdt = {np.float32: self.torch.float32, np.int32: self.torch.int32, np.uint16: self.torch.int16}[_ARR_DTYPE[which]]
        return base[off:off + nbytes.value].view(tdt).view(self._shape(which))

    def set_members(self, layers_per_member, H):
        """Uploads initial weights ([(W, b), ...] per member) and hyperparameters [P][n_h]."""
        flat = np.stack([pack_params(self.layout, m) for m in layers_per_member])
        self.set(ARR_W32, flat)
        self.set(ARR_HYPER, np.asarray(H, dtype=np.float32))

    def member_params(self, member, which=ARR_W32):
        return unpack_params(self.layout, self.layer_shapes, self.get(which, member))

    def close(self):
        if self._h:
            lib().pbt_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def batched_gemm_bf16(a, b, c, M, N, K, batch, lda, sa, a_m_contig, ldb, sb, b_k_contig, ldc, sc):
    """c (torch float32 or bfloat16), a, b (torch bfloat16) on the device."""
    import torch
    rc = lib().pbt_batched_gemm_bf16(a.data_ptr(), lda, sa, int(a_m_contig), b.data_ptr(), ldb, sb, int(b_k_contig),
                                     c.data_ptr(), ldc, sc, int(c.dtype == torch.bfloat16), M, N, K, batch,
                                     C.c_void_p(torch.cuda.current_stream(a.device).cuda_stream))
    if rc != 0:
        raise PbtError(rc, lib().pbt_last_error(None).decode())
