// Instantiations of the population-batched bf16 MFMA GEMM for the epilogues the step uses.
#include "gemm_bf16.h"
#include "gemm_nt_lds.h"
#include "internal.h"

namespace pbt {

template <class E>
static hipError_t run(const GemmOperands& o, const E& e, hipStream_t s) {
  // long contractions of two K-contiguous operands (input gradients) take the direct-to-LDS kernel
  if constexpr (std::is_same_v<E, EpiStoreBF16> || std::is_same_v<E, EpiDgradAct>) {
    GemmArgs g;
    g.A = o.A; g.lda = o.lda; g.sa = o.sa;
    g.B = o.B; g.ldb = o.ldb; g.sb = o.sb;
    g.M = o.M; g.N = o.N; g.K = o.K; g.batch = o.batch;
    g.tiles_m = g.tiles_n = 0;
    g.inner = o.inner < 1 ? 1 : o.inner; g.sa_in = o.sa_in; g.sb_in = o.sb_in;
    if (!o.colsum && nt_lds_applies(g, o.a_m_contig, o.b_k_contig)) return launch_gemm_nt_lds(g, e, s);
  }
  return launch_gemm_bf16<E>(o.A, o.lda, o.sa, o.a_m_contig, o.B, o.ldb, o.sb, o.b_k_contig, o.M, o.N, o.K, o.batch, e, s, o.inner,
                             o.sa_in, o.sb_in, o.colsum, o.colsum_stride, o.colsum_k);
}

hipError_t gemm_store_f32(const GemmOperands& o, float* C, int64_t ldc, int64_t sc, hipStream_t s) {
  return run(o, EpiStoreF32{C, ldc, sc}, s);
}
hipError_t gemm_store_bf16(const GemmOperands& o, bf16_t* C, int64_t ldc, int64_t sc, hipStream_t s) {
  return run(o, EpiStoreBF16{C, ldc, sc}, s);
}
hipError_t gemm_store_bf16_heads(const GemmOperands& o, bf16_t* C, int64_t ldc, int64_t sc, int64_t sc_in, hipStream_t s) {
  return run(o, EpiStoreBF16{C, ldc, sc, o.inner, sc_in}, s);
}
hipError_t gemm_bias_f32(const GemmOperands& o, const float* bias, int64_t sbias, float* C, int64_t ldc, int64_t sc, hipStream_t s) {
  return run(o, EpiBiasF32{bias, sbias, C, ldc, sc}, s);
}
hipError_t gemm_bias_act(const GemmOperands& o, const float* bias, int64_t sbias, bf16_t* Z, bf16_t* Aout, int64_t ld,
                         int64_t so, int act, hipStream_t s, const DropSite& site) {
  if (!site.record) return run(o, EpiBiasAct{bias, sbias, Z, Aout, ld, so, act}, s);
  if (Z || o.N % 8 || ld % 8 || so % 8 || sbias % 4 || (reinterpret_cast<uintptr_t>(bias) & 15)) return hipErrorInvalidValue;
  return run(o, EpiBiasActDrop{bias, sbias, Aout, ld, so, act, site.record, site.record_stride, site.args, site.site}, s);
}
hipError_t gemm_dgrad_act(const GemmOperands& o, const bf16_t* Zprev, bf16_t* dZ, int64_t ld, int64_t so, int act,
                          hipStream_t s, const DropRecord& drop) {
  if (drop.mask && (o.N % 8 || ld % 8 || so % 8)) return hipErrorInvalidValue;
  return run(o, EpiDgradAct{Zprev, dZ, ld, so, act, drop.mask, drop.mask_stride, drop.H, drop.n_hyper, drop.col, 1.f}, s);
}

hipError_t gemm_wgrad_optimizer(const GemmOperands& o, const OptArgs& a, int64_t off, int64_t ldc, hipStream_t s) {
  const OptHyper hy{a.H, a.t, a.n_hyper, a.col_lr, a.col_beta1, a.col_wd, a.c0, a.c1, a.c2, a.c3, a.t_mul, a.t_add};
  if (a.optimizer == OPT_SGD_MOMENTUM) return run(o, EpiOptimizer<OPT_SGD_MOMENTUM>{a.W32, a.S0, a.S1, a.W16, a.stride, off, ldc, hy, {}}, s);
  if (a.optimizer == OPT_ADAM) return run(o, EpiOptimizer<OPT_ADAM>{a.W32, a.S0, a.S1, a.W16, a.stride, off, ldc, hy, {}}, s);
  return run(o, EpiOptimizer<OPT_RMSPROP>{a.W32, a.S0, a.S1, a.W16, a.stride, off, ldc, hy, {}}, s);
}

hipError_t gemm_rbf_sum(const GemmOperands& o, const float* na, int64_t sna, const float* nb, int64_t snb, float inv2d,
                        float* partial, int* tiles, hipStream_t s) {
  // tile count as launch_gemm_bf16 will choose it (the caller sizes `partial` with gemm_rbf_tiles, an upper bound)
  const TileShape t = tile_shape(choose_tile(o.M, o.N, o.K, o.batch));
  *tiles = ((o.M + t.bm - 1) / t.bm) * ((o.N + t.bn - 1) / t.bn);
  return run(o, EpiRbfSum{na, sna, nb, snb, inv2d, partial, 0.f}, s);
}
int gemm_rbf_tiles(int M, int N, int) {
  return ((M + 127) / 128) * ((N + 63) / 64);  // the smallest tile gives the most partial sums
}

}  // namespace pbt
