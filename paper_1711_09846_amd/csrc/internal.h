// Host-callable launchers of the population-step kernels.  Every launcher only enqueues on
// `stream` and returns the launch status; none allocates or synchronises.
#pragma once
#include "../../include/pbt.h"
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pbt {

typedef uint16_t bf16_t;

// ---- gemm.hip: population-batched bf16 MFMA GEMM with fused epilogues ------------------------
struct GemmOperands {
  const bf16_t* A; int64_t lda, sa; bool a_m_contig;
  const bf16_t* B; int64_t ldb, sb; bool b_k_contig;
  int M, N, K, batch;
  int inner = 1;                 // two-level batch index: element b reads A at (b / inner) * sa + (b % inner) * sa_in
  int64_t sa_in = 0, sb_in = 0;
  float* colsum = nullptr;       // optional by-product: colsum[b * colsum_stride + n] = sum_k B[k][n]
  int64_t colsum_stride = 0;
  int colsum_k = -1;             // the column sums run over k < colsum_k only (-1: over all of K)
};
hipError_t gemm_store_f32(const GemmOperands& o, float* C, int64_t ldc, int64_t sc, hipStream_t s);
hipError_t gemm_store_bf16(const GemmOperands& o, bf16_t* C, int64_t ldc, int64_t sc, hipStream_t s);
// as gemm_store_bf16 with C of batch element b at (b / o.inner) * sc + (b % o.inner) * sc_in
hipError_t gemm_store_bf16_heads(const GemmOperands& o, bf16_t* C, int64_t ldc, int64_t sc, int64_t sc_in, hipStream_t s);
// C (float) = acc + bias
hipError_t gemm_bias_f32(const GemmOperands& o, const float* bias, int64_t sbias, float* C, int64_t ldc, int64_t sc, hipStream_t s);
// z = acc + bias; Z (may be null) <- z, Aout <- act(z); both [batch][M][ld] bf16 with batch stride so
struct DropArgs {  // where a kernel finds the member's dropout rate and the Philox counter base
  const float* H; int n_hyper; int col;  // column of H holding the rate, -1 = no dropout
  int active;                            // 0 = eval: keep everything
  uint32_t c0; uint64_t seed;            // step index, Philox key
};
// a dropout site applied by the kernel that produces the site's input: Philox site number, where the keep bits go
// (one bit per element of the member's array, record_stride bytes per member; null = no dropout here)
struct DropSite { DropArgs args = {}; int site = 0; uint8_t* record = nullptr; int64_t record_stride = 0; };
// (with a site: N, ld and so multiples of 8; Aout receives act(z), rounded, times the keep factors, rounded)
hipError_t gemm_bias_act(const GemmOperands& o, const float* bias, int64_t sbias, bf16_t* Z, bf16_t* Aout, int64_t ld,
                         int64_t so, int act, hipStream_t s, const DropSite& site = DropSite());
// dZ <- acc * act'(Zprev); with a dropout record (drop.mask != null; needs N and ld multiples of 8) the result is
// rounded and then multiplied by the recorded keep factors of the member (rate in column drop.col of drop.H)
struct DropRecord { const uint8_t* mask = nullptr; int64_t mask_stride = 0; const float* H = nullptr; int n_hyper = 0, col = -1; };
hipError_t gemm_dgrad_act(const GemmOperands& o, const bf16_t* Zprev, bf16_t* dZ, int64_t ld, int64_t so, int act,
                          hipStream_t s, const DropRecord& drop = DropRecord());

// Per-member sum over the whole M x N Gram matrix of exp(-(na[m] + nb[n] - 2 a_m.b_n) * inv2d), as
// per-tile partial sums partial[batch][*tiles]; gemm_rbf_tiles(M, N, batch) is an upper bound of *tiles for sizing `partial`.
int gemm_rbf_tiles(int M, int N, int batch);
hipError_t gemm_rbf_sum(const GemmOperands& o, const float* na, int64_t sna, const float* nb, int64_t snb, float inv2d,
                        float* partial, int* tiles, hipStream_t s);

// ---- kernels.hip ----------------------------------------------------------------------------
hipError_t fill_u32(uint32_t* p, uint32_t v, int64_t n, hipStream_t s);
hipError_t iota_i32(int32_t* p, int n, hipStream_t s);
hipError_t f32_to_bf16(const float* src, bf16_t* dst, int64_t n, hipStream_t s);

// Mini-batch fetch: row r of member i at step `step` is data row floor(x * n_train / 2^32),
// x = word 0 of Philox(step, i, DOMAIN_BATCH, r).  Writes X[P][B][d] (bf16 or float) and Y[P][B];
// also t[i] += 1 (the update count used by this step's optimiser pass).
hipError_t gather_batch(const float* train_x, const int32_t* train_y, int n_train, int d, int P, int B, uint32_t step,
                        uint64_t seed, bf16_t* X16, float* X32, int32_t* Y, int32_t* t, hipStream_t s);

// head.hip -- output layer (C <= 32 classes) + softmax cross-entropy on the matrix cores.
// logits = A W + b with A [P][rows][K] (bf16, batch stride sa; sa = 0 shares A), W bf16 [K][C] at
// W16 + member*sw, b float at bias + member*sbias.  Writes rowloss[member*srowloss + r] and, when
// dlogits != null, dlogits[P][rows][32] (bf16, zero padded) = (softmax - onehot) * gscale.
// labels are [rows] shared (sy = 0) or per member (sy = rows).
// n_pos < 0: softmax cross-entropy against `labels`.  n_pos >= 0 (needs C = 1): logistic loss, rows
// r < n_pos have target 1, the others target 0 (labels unused).  n_pos = -2: no loss; rowloss then
// receives the head outputs as float [P][rows][32] (bias added, zero padded).
hipError_t head_fwd_loss(const bf16_t* A, int64_t sa, const bf16_t* W16, int64_t sw, const float* bias, int64_t sbias,
                         const int32_t* labels, int64_t sy, int P, int rows, int K, int C, float gscale, int n_pos,
                         bf16_t* dlogits, float* rowloss, int64_t srowloss, hipStream_t s);
// dZprev[P][rows][K] = (dlogits W^T) * act'(Zprev)
hipError_t head_dgrad(const bf16_t* dlogits, const bf16_t* W16, int64_t sw, const bf16_t* Zprev, bf16_t* dZprev, int P,
                      int rows, int K, int C, int act, hipStream_t s);
// out[i * out_stride] = scale * sum_r rowval[i][r]   (one wavefront per member, fixed order)
hipError_t row_reduce(const float* rowval, int64_t srow, int P, int rows, float scale, float* out, int out_stride,
                      hipStream_t s);

// Initial population: uniform +-1/sqrt(fan_in) weights (positions outside any layer are zero) and
// hyperparameters from the priors; all in double, rounded once to float.
struct InitArgs {
  float* W32; bf16_t* W16; float* H;
  int64_t stride; int P, n_seg, n_hyper;
  // parameter arrays of one member: fan > 0: uniform in +-1/sqrt(fan); fan == 0: the constant
  int64_t seg_off[PBT_MAX_SEGMENTS], seg_len[PBT_MAX_SEGMENTS]; int seg_fan[PBT_MAX_SEGMENTS]; float seg_const[PBT_MAX_SEGMENTS];
  int prior_kind[8]; double prior_a[8], prior_b[8];  // uniform: a + u (b - a); log: exp(a + u (b - a)), a = ln lo
  uint64_t seed;
};
hipError_t init_population(const InitArgs& a, hipStream_t s);

struct OptArgs {
  float* W32; float* S0; float* S1; bf16_t* W16; const float* G;
  int64_t begin, count;  // range of the member's flat vector to update (multiples of 4)
  const float* H; const int32_t* t;
  int64_t stride; int P; int n_hyper;
  int optimizer;
  int col_lr, col_beta1, col_wd;  // column of H with that role, or -1
  float c0, c1, c2, c3;           // opt_const
  // further ranges of the flat vector handled by the same launch (the biases between fused matrices)
  int n_extra = 0;
  int64_t xbegin[3] = {0, 0, 0}, xcount[3] = {0, 0, 0};
  // Adam's bias correction counts t[i] * t_mul + t_add updates (a network updated several times per step)
  int t_mul = 1, t_add = 0;
};
constexpr int OPT_MAX_RANGES = 4;
hipError_t optimizer_step(const OptArgs& a, hipStream_t s);
// Weight-gradient GEMM (o) whose epilogue applies the optimiser to the matrix at offset `off` (row
// pitch ldc) of every member's flat vector instead of storing the gradient; a.G, a.begin, a.count unused.
hipError_t gemm_wgrad_optimizer(const GemmOperands& o, const OptArgs& a, int64_t off, int64_t ldc, hipStream_t s);

// out[P][rows][d] (bf16) = standard normal latents: element e uses Philox counter
// (c0, member, DOMAIN_LATENT + substream, e / 4); words (0,1) and (2,3) are one Box-Muller pair each
// (cosine branch for even e, sine for odd), evaluated in double.
hipError_t latent_normal(bf16_t* out, int P, int rows, int d, uint32_t c0, int substream, uint64_t seed, hipStream_t s);
// out[batch][rows] = sum_k X[batch][rows][d]^2 (float)
hipError_t row_sqnorm(const bf16_t* X, int batch, int rows, int d, float* out, hipStream_t s);
// gathers rows of a float data set into bf16 X[P][ld_rows][d] rows 0..B-1 (Philox domain 1, counter element
// counter0 + r for row r); t[i] += 1 when bump_t
hipError_t gather_rows(const float* train_x, int n_train, int d, int P, int B, int64_t member_stride, uint32_t step,
                       uint64_t seed, bf16_t* X16, int32_t* t, hipStream_t s, uint32_t counter0 = 0, bool bump_t = true);
// score[i] = -( sxx[i] + syy[0] - 2 sxy[i] ) * inv_n2 where each s is the sum of `tiles` partials
hipError_t mmd_combine(const float* pxx, int txx, const float* pyy, int tyy, const float* pxy, int txy, int P, float inv_n2,
                       float* score, hipStream_t s);

// ---- transformer_kernels.hip ------------------------------------------------------------------
hipError_t embed_fwd(const int32_t* pool, int n_pool, int S, int B, int d, int V, int P, const bf16_t* W16, int64_t stride,
                     int64_t tok_off, int64_t pos_off, uint32_t c0, uint64_t seed, int draw, bf16_t* h, int32_t* tokens,
                     int32_t* targets, int32_t* t, hipStream_t s);
hipError_t embed_bwd(const bf16_t* dh, const int32_t* tokens, int B, int S, int d, int V, int P, float* G, int64_t stride,
                     int64_t tok_off, int64_t pos_off, int32_t* start, int32_t* cursor, int32_t* order, hipStream_t s);
hipError_t layernorm_fwd(const bf16_t* x, int P, int rows, int d, const float* W32, int64_t stride, int64_t g_off, int64_t b_off,
                         bf16_t* y, float* mean, float* rstd, hipStream_t s);
hipError_t layernorm_bwd(const bf16_t* dy, const bf16_t* x, const float* mean, const float* rstd, int P, int rows, int d,
                         const float* W32, int64_t stride, int64_t g_off, const bf16_t* res, bf16_t* out, hipStream_t s);
constexpr int LN_MAX_SLABS = 64;  // row slabs whose partial sums layernorm_param_grad combines
hipError_t layernorm_param_grad(const bf16_t* dy, const bf16_t* x, const float* mean, const float* rstd, int P, int rows, int d,
                                float* G, int64_t stride, int64_t g_off, int64_t b_off, float* part, hipStream_t s);
constexpr int LN_FUSED_SLABS = 64;  // row slabs of the fused LayerNorm backward
// LayerNorm backward (as layernorm_bwd) and the gain / bias gradients (as layernorm_param_grad) in one pass; d <= 2048
// out2 (optional): out multiplied by the recorded keep factors of a dropout site (drop as in gemm_dgrad_act), i.e.
// the gradient that enters the branch behind that site
hipError_t layernorm_bwd_with_param_grad(const bf16_t* dy, const bf16_t* x, const float* mean, const float* rstd, int P, int rows,
                                         int d, const float* W32, int64_t stride, int64_t g_off, int64_t b_off, const bf16_t* res,
                                         bf16_t* out, float* G, float* part, hipStream_t s, bf16_t* out2 = nullptr,
                                         const DropRecord& drop = DropRecord());
hipError_t softmax_fwd(const bf16_t* sc, int P, int64_t rows, int S, float scale, const DropArgs& d, int site, bf16_t* pq,
                       bf16_t* pd, hipStream_t s);
hipError_t softmax_bwd(const bf16_t* pq, bf16_t* dpd, int P, int64_t rows, int S, float scale, const DropArgs& d, int site,
                       hipStream_t s);
// h = res + x * keep and y = LayerNorm(h) in one pass (d <= 2048, rows * d a multiple of 16); record as dropout_apply's mask_out
hipError_t residual_dropout_layernorm(const bf16_t* x, const bf16_t* res, int P, int rows, int d, const DropArgs& dr, int site, bf16_t* h,
                                      uint16_t* record, const float* W32, int64_t stride, int64_t g_off, int64_t b_off, bf16_t* y, float* mean,
                                      float* rstd, hipStream_t s);
// adds up the n_parts partial weight gradients part[P * n_parts][count] (and their column sums colpart[P * n_parts][N])
// of a contraction that was cut into pieces, in piece order, into G at w_off (b_off)
hipError_t wgrad_combine(const float* part, const float* colpart, int n_parts, int P, int64_t count, int N, float* G, int64_t stride,
                         int64_t w_off, int64_t b_off, hipStream_t s);
// Attention of one (member, sequence, head) per workgroup without score or probability arrays in memory, for
// 64-wide heads and sequences of 32, 64, 96 or 128 positions (attention_fused_applies).  qkv: [P][Bc*S][3d]
// (queries, keys, values side by side, heads side by side inside each); o, dO: [P][Bc*S][d]; dqkv like qkv.
// The forward pass leaves the keep bits of its dropout site in `record` (attention_record_bytes; null = not
// wanted); the backward pass (two kernels: dQ, then dK and dV) needs them and attention_stats_bytes of scratch.
constexpr int ATTN_FUSED_HEAD = 64, ATTN_FUSED_MAX_SEQ = 128;
bool attention_fused_applies(int d_model, int heads, int seq);
size_t attention_record_bytes(int P, int Bc, int heads);
size_t attention_stats_bytes(int P, int Bc, int heads);
hipError_t attention_fwd(const bf16_t* qkv, int P, int Bc, int S, int d, int H, float scale, const DropArgs& dr, int site, bf16_t* o,
                         uint32_t* record, hipStream_t s);
hipError_t attention_bwd(const bf16_t* qkv, const bf16_t* dO, int P, int Bc, int S, int d, int H, float scale, const DropArgs& dr,
                         const uint32_t* record, float* stats, bf16_t* dqkv, hipStream_t s);
// out = x * keep (+ res); mask_out (optional) receives the keep bits, mask_in (optional) supplies them (the
// backward pass of a site reads what its forward pass recorded); dropout_mask_bytes sizes such a record
hipError_t dropout_apply(const bf16_t* x, const bf16_t* res, int P, int64_t per_member, const DropArgs& d, int site, bf16_t* out,
                         hipStream_t s, const uint16_t* mask_in = nullptr, uint16_t* mask_out = nullptr);
size_t dropout_mask_bytes(int P, int64_t per_member);
hipError_t xent_rows(const float* logits, const int32_t* targets, int P, int rows, int V, const float* H, int n_hyper, int col_ls,
                     int use_ls, float gscale, bf16_t* dlogits, float* rowloss, hipStream_t s);
hipError_t perplexity_score(const float* rowloss, int P, int rows, float* score, hipStream_t s);
hipError_t tf_scatter_rows(const float* src, int P, int rows, float* dst, int64_t dst_stride, int64_t offset, hipStream_t s);

struct ExploitArgs {
  float* score; const float* score_override; float* H; int32_t* t; int32_t* order; int32_t* donor; int32_t* parent;
  int32_t* recip; int32_t* n_recip;  // recipients (member indices) and their number
  int P, n_trunc, n_hyper;
  float f_lo, f_hi;
  float h_max[8];
  uint32_t round; uint64_t seed;
  int tournament, resample, keep_weights, keep_hypers;  // tournament: opponent drawn from the whole population
  int ttest; double ttest_alpha; const float* hist;     // t-test selection on the score histories [P][12]
  uint32_t resample_thr; int resample_always;     // resample iff word < thr, or always
  int prior_kind[8]; double prior_a[8], prior_b[8];  // as in InitArgs
};
hipError_t rank_select_explore(const ExploitArgs& a, hipStream_t s);
struct CopyArrays {
  void* base[6]; int64_t row_bytes[6]; int n;
  void* stage[6];  // optional staging rows [max_rows][row_bytes] per array (donors that are recipients too)
};
// Row recip[y] of every array <- row donor[recip[y]], y < *n_recip (at most max_rows).  staged: every donor
// row is first gathered into arrs.stage and then scattered, so that a member can be donor and recipient.
hipError_t gather_copy(const CopyArrays& arrs, const int32_t* recip, const int32_t* donor, int max_rows, const int32_t* n_recip,
                       bool staged, hipStream_t s);

// fused_small.hip: whole step of a small fp32 MLP classifier, one workgroup per member, the
// member's weights, optimiser state and activations resident in LDS across n_steps steps.
struct FusedSmallArgs {
  float* W32; float* S0; float* S1; float* G; const float* H; int32_t* t; float* loss; float* score;
  const float* x; const int32_t* y;          // training set (step) or held-out set (eval)
  int64_t stride; int P, B, n_rows, n_layers; int dims[16]; int w_off[16], b_off[16];
  int act, optimizer, n_hyper, col_lr, col_beta1, col_wd; float c0, c1, c2, c3;
  uint32_t step0; int n_steps; uint64_t seed;
  // LDS carve-up in floats, filled by fused_small_plan()
  int lds_w, lds_s0, lds_s1, lds_a[16], lds_z[16], lds_dz[2], lds_rowloss, lds_y, lds_total;
};
// Fills the lds_* fields; returns the dynamic LDS bytes needed (for_eval: no state, no gradients).
size_t fused_small_plan(FusedSmallArgs& a, bool for_eval);
constexpr size_t FUSED_SMALL_MAX_LDS = 160 * 1024;
hipError_t fused_small_step(const FusedSmallArgs& a, hipStream_t s);
hipError_t fused_small_eval(const FusedSmallArgs& a, hipStream_t s);

}  // namespace pbt
