// The language-model workload (Section 4.2.1 of the PBT paper: Transformer networks trained with
// Adam, learning rate and dropout rates adapted per member, scored by a metric that is not the
// training loss).  Host side: parameter layout, scratch carve-up and the kernel sequences of one
// population step and of the perplexity score.  Every dense contraction, the attention products
// included, goes through the population-batched MFMA GEMM; for attention the batch index is
// (member, sequence, head) with a two-level stride.
#include <cmath>
#include <cstring>

#include "dense_host.h"

namespace pbt {

namespace {

struct Dim { int V, d, H, dh, f, S, L; };
// LayerNorm, dropout and residual steps ride on neighbouring kernels when a row fits the fused kernels' registers
// and the keep-bit records are whole bytes per row
bool tf_fused_elementwise(const pbt_config& c) { return c.tf_d_model <= 2048 && c.tf_d_model % 16 == 0 && c.tf_d_ff % 16 == 0; }
Dim dim_of(const pbt_config& c) { return Dim{c.tf_vocab, c.tf_d_model, c.tf_heads, c.tf_d_model / c.tf_heads, c.tf_d_ff, c.tf_seq, c.n_layers}; }

struct Ctx {
  pbt_handle* h; hipStream_t s; Dim D; int P, Bc, n;  // Bc sequences per member in this pass, n = Bc * S rows
  int64_t S_; const float* W32; const bf16_t* W16; float* G;
  bool fused_bwd;   // elementwise steps ride on neighbouring kernels (tf_fused_elementwise): residual + dropout + LayerNorm forward in one kernel, hidden-layer dropout in its GEMM, LayerNorm backward + parameter gradients + the next dropout site in one kernel
  template <class T> T* sc(size_t off) const { return h->sc<T>(off); }
};

// out[P][n][N] = act(in[P][n][K] W[K][N] + b)
pbt_status dense(const Ctx& x, const bf16_t* in, int K, int N, int64_t w, int64_t b, bf16_t* Z, bf16_t* out, int act,
                 const DropSite& site = DropSite()) {
  GemmOperands o{in, K, (int64_t)x.n * K, false, x.W16 + w, N, x.S_, false, x.n, N, K, x.P};
  PBT_LAUNCH(x.h, PBT_K_GEMM_FWD, x.s, gemm_bias_act(o, x.W32 + b, x.S_, Z, out, N, (int64_t)x.n * N, act, x.s, site));
  return PBT_OK;
}
// A small weight matrix over many rows (the attention output projection: 512 x 512 from 4096 rows) gives 256 x 256 tiles
// to a quarter of the compute units, and smaller tiles spend the long contraction on loop overhead (12 % of the MFMA peak):
// its contraction is cut into WGRAD_PARTS pieces, each a tile of its own, and the pieces are added up in order afterwards.
constexpr int WGRAD_PARTS = 4;
bool wgrad_in_parts(int P, int rows, int K, int N) {
  return (int64_t)((K + 255) / 256) * ((N + 255) / 256) * P <= 64 && K >= 256 && N >= 256 && N % 4 == 0 && ((int64_t)K * N) % 4 == 0 &&
         rows % (WGRAD_PARTS * 64) == 0 && rows / WGRAD_PARTS >= 1024;
}
// G[w] = in^T dout, G[b] = column sums of dout
pbt_status wgrad(const Ctx& x, const bf16_t* in, int K, const bf16_t* dout, int N, int64_t w, int64_t b) {
  if ((int64_t)K * N <= x.h->plan.tf.wpart_elems && N <= x.h->plan.tf.wcol_elems && wgrad_in_parts(x.P, x.n, K, N)) {
    float* part = x.sc<float>(x.h->plan.tf.o_wpart);
    float* colpart = x.sc<float>(x.h->plan.tf.o_wcolpart);
    const int rows = x.n / WGRAD_PARTS;
    GemmOperands o{in, K, (int64_t)x.n * K, true, dout, N, (int64_t)x.n * N, false, K, N, rows, x.P * WGRAD_PARTS};
    o.inner = WGRAD_PARTS; o.sa_in = (int64_t)rows * K; o.sb_in = (int64_t)rows * N;
    o.colsum = colpart; o.colsum_stride = N;
    PBT_LAUNCH(x.h, PBT_K_GEMM_WGRAD, x.s, gemm_store_f32(o, part, N, (int64_t)K * N, x.s));
    PBT_HIP(x.h, wgrad_combine(part, colpart, WGRAD_PARTS, x.P, (int64_t)K * N, N, x.G, x.S_, w, b, x.s));
    return PBT_OK;
  }
  // The column sums are a by-product of the GEMM (its first tile row adds up the dout slabs it stages anyway).
  // That tile row finishes last and the launch takes 17 % longer (146 -> 171 us), which is still cheaper than a
  // pass of its own over dout (41 us per layer): 16.78 -> 16.43 ms per population step.
  GemmOperands o{in, K, (int64_t)x.n * K, true, dout, N, (int64_t)x.n * N, false, K, N, x.n, x.P};
  o.colsum = x.G + b; o.colsum_stride = x.S_;
  PBT_LAUNCH(x.h, PBT_K_GEMM_WGRAD, x.s, gemm_store_f32(o, x.G + w, N, x.S_, x.s));
  return PBT_OK;
}
// din[P][n][K] = dout[P][n][N] W^T   (optionally times act'(zprev))
pbt_status dgrad(const Ctx& x, const bf16_t* dout, int N, int K, int64_t w, const bf16_t* zprev, int act, bf16_t* din,
                 const DropRecord& drop = DropRecord()) {
  GemmOperands o{dout, N, (int64_t)x.n * N, false, x.W16 + w, N, x.S_, true, x.n, K, N, x.P};
  if (zprev)
    PBT_LAUNCH(x.h, PBT_K_GEMM_DGRAD, x.s, gemm_dgrad_act(o, zprev, din, K, (int64_t)x.n * K, act, x.s, drop));
  else
    PBT_LAUNCH(x.h, PBT_K_GEMM_DGRAD, x.s, gemm_store_bf16(o, din, K, (int64_t)x.n * K, x.s));
  return PBT_OK;
}

// out = LayerNorm backward of dy (+ res); G[g], G[b] = gradients of gain and bias
// out2 / drop (optional, fused path only): out times the recorded keep factors of a dropout site
pbt_status ln_backward(const Ctx& x, const bf16_t* dy, const bf16_t* in, const float* mean, const float* rstd, int64_t g, int64_t b,
                       const bf16_t* res, bf16_t* out, bf16_t* out2 = nullptr, const DropRecord& drop = DropRecord()) {
  float* part = x.sc<float>(x.h->plan.tf.o_lnpart);
  if (x.fused_bwd) {
    PBT_HIP(x.h, layernorm_bwd_with_param_grad(dy, in, mean, rstd, x.P, x.n, x.D.d, x.W32, x.S_, g, b, res, out, x.G, part, x.s, out2, drop));
    return PBT_OK;
  }
  PBT_HIP(x.h, layernorm_param_grad(dy, in, mean, rstd, x.P, x.n, x.D.d, x.G, x.S_, g, b, part, x.s));
  PBT_HIP(x.h, layernorm_bwd(dy, in, mean, rstd, x.P, x.n, x.D.d, x.W32, x.S_, g, res, out, x.s));
  return PBT_OK;
}

// One attention product over all (member, sequence, head) triples.  Operands live inside
// [P*Bc][S][pitch] arrays at column `col` + head * dh, or inside the [P*Bc][H][S][S] score arrays.
struct Opnd { const bf16_t* p; int64_t pitch, outer, inner; };
Opnd in_rows(const bf16_t* base, int col, int pitch, const Dim& D) { return Opnd{base + col, pitch, (int64_t)D.S * pitch, D.dh}; }
Opnd in_scores(const bf16_t* base, const Dim& D) { return Opnd{base, D.S, (int64_t)D.H * D.S * D.S, (int64_t)D.S * D.S}; }
pbt_status attn_gemm(const Ctx& x, Opnd a, bool a_m_contig, Opnd b, bool b_k_contig, Opnd c, int M, int N, int K) {
  GemmOperands o{a.p, a.pitch, a.outer, a_m_contig, b.p, b.pitch, b.outer, b_k_contig, M, N, K, x.P * x.Bc * x.D.H, x.D.H, a.inner, b.inner};
  PBT_LAUNCH(x.h, PBT_K_HEAD, x.s, gemm_store_bf16_heads(o, const_cast<bf16_t*>(c.p), c.pitch, c.outer, c.inner, x.s));
  return PBT_OK;
}

#define TF_TRY(call) do { pbt_status st_ = (call); if (st_ != PBT_OK) return st_; } while (0)

// Forward through embeddings, blocks and the final LayerNorm + head; leaves float logits.
pbt_status forward(const Ctx& x, const int32_t* pool, int n_pool, uint32_t c0, int draw, int train) {
  pbt_handle* h = x.h;
  const pbt_config& c = h->cfg;
  const TfPlan& t = h->plan.tf;
  const Dim& D = x.D;
  const DropArgs dr{h->st<float>(h->plan.o_hyper), c.n_hyper, t.col_drop, train, c0, c.seed};
  const int64_t per_d = (int64_t)x.n * D.d, per_f = (int64_t)x.n * D.f;
  PBT_LAUNCH(h, PBT_K_FETCH, x.s, embed_fwd(pool, n_pool, D.S, x.Bc, D.d, D.V, x.P, x.W16, x.S_, t.tok, t.pos, c0, c.seed, draw,
                                            x.sc<bf16_t>(t.o_h[0]), x.sc<int32_t>(t.o_tokens), x.sc<int32_t>(t.o_targets),
                                            h->st<int32_t>(h->plan.o_t), x.s));
  bf16_t* tmp_d = x.sc<bf16_t>(t.o_tmp_d[0]);
  bf16_t* score = x.sc<bf16_t>(t.o_score);
  for (int l = 0; l < D.L; ++l) {
    const TfBlockOff& b = t.blk[l];
    bf16_t* hin = x.sc<bf16_t>(t.o_h[l]);
    bf16_t* hmid = x.sc<bf16_t>(t.o_hmid[l]);
    bf16_t* hout = x.sc<bf16_t>(t.o_h[l + 1]);
    bf16_t* u = x.sc<bf16_t>(t.o_u[l]);
    bf16_t* qkv = x.sc<bf16_t>(t.o_qkv[l]);
    bf16_t* pq = x.sc<bf16_t>(t.o_pq[l]);
    bf16_t* pd = x.sc<bf16_t>(t.o_pd[l]);
    bf16_t* o = x.sc<bf16_t>(t.o_o[l]);
    // (on the fused path the LayerNorm at the head of a block rides on the kernel that closes the block before it)
    if (!x.fused_bwd || l == 0)
      PBT_HIP(h, layernorm_fwd(hin, x.P, x.n, D.d, x.W32, x.S_, b.ln1g, b.ln1b, u, x.sc<float>(t.o_mean1[l]), x.sc<float>(t.o_rstd1[l]), x.s));
    TF_TRY(dense(x, u, D.d, 3 * D.d, b.wqkv, b.bqkv, nullptr, qkv, PBT_ACT_NONE));
    if (t.fused_attn) {
      PBT_LAUNCH(h, PBT_K_HEAD, x.s, attention_fwd(qkv, x.P, x.Bc, D.S, D.d, D.H, 1.f / sqrtf((float)D.dh), dr, 4 * l + 0, o,
                                                   train ? x.sc<uint32_t>(t.o_keep[l]) : nullptr, x.s));
    } else {
      TF_TRY(attn_gemm(x, in_rows(qkv, 0, 3 * D.d, D), false, in_rows(qkv, D.d, 3 * D.d, D), true, in_scores(score, D), D.S, D.S, D.dh));
      PBT_HIP(h, softmax_fwd(score, x.P, (int64_t)x.Bc * D.H * D.S, D.S, 1.f / sqrtf((float)D.dh), dr, 4 * l + 0, pq, pd, x.s));
      TF_TRY(attn_gemm(x, in_scores(pd, D), false, in_rows(qkv, 2 * D.d, 3 * D.d, D), false, in_rows(o, 0, D.d, D), D.S, D.dh, D.S));
    }
    TF_TRY(dense(x, o, D.d, D.d, b.wo, b.bo, nullptr, tmp_d, PBT_ACT_NONE));
    bf16_t* u2 = x.sc<bf16_t>(t.o_u2[l]);
    bf16_t* fd = x.sc<bf16_t>(t.o_fd[l]);
    if (x.fused_bwd) {
      // residual + dropout + the next LayerNorm in one kernel; the feed-forward hidden layer's dropout in the epilogue of
      // its GEMM (only the dropped-out activation is kept: it is positive exactly where the pre-activation is positive and
      // the element was kept, and the backward pass multiplies by the keep factor anyway)
      PBT_HIP(h, residual_dropout_layernorm(tmp_d, hin, x.P, x.n, D.d, dr, 4 * l + 1, hmid, x.sc<uint16_t>(t.o_mask[l][0]), x.W32, x.S_, b.ln2g,
                                            b.ln2b, u2, x.sc<float>(t.o_mean2[l]), x.sc<float>(t.o_rstd2[l]), x.s));
      DropSite site;
      if (train) site = DropSite{dr, 4 * l + 2, x.sc<uint8_t>(t.o_mask[l][1]), (int64_t)dropout_mask_bytes(1, per_f)};
      TF_TRY(dense(x, u2, D.d, D.f, b.w1, b.b1, nullptr, fd, PBT_ACT_RELU, site));
      TF_TRY(dense(x, fd, D.f, D.d, b.w2, b.b2, nullptr, tmp_d, PBT_ACT_NONE));
      const bool last = l + 1 == D.L;
      const int64_t ng = last ? t.lnfg : t.blk[l + 1].ln1g, nb = last ? t.lnfb : t.blk[l + 1].ln1b;
      PBT_HIP(h, residual_dropout_layernorm(tmp_d, hmid, x.P, x.n, D.d, dr, 4 * l + 3, hout, x.sc<uint16_t>(t.o_mask[l][2]), x.W32, x.S_, ng, nb,
                                            last ? x.sc<bf16_t>(t.o_uf) : x.sc<bf16_t>(t.o_u[l + 1]),
                                            x.sc<float>(last ? t.o_meanf : t.o_mean1[l + 1]), x.sc<float>(last ? t.o_rstdf : t.o_rstd1[l + 1]), x.s));
      continue;
    }
    PBT_HIP(h, dropout_apply(tmp_d, hin, x.P, per_d, dr, 4 * l + 1, hmid, x.s, nullptr, x.sc<uint16_t>(t.o_mask[l][0])));
    PBT_HIP(h, layernorm_fwd(hmid, x.P, x.n, D.d, x.W32, x.S_, b.ln2g, b.ln2b, u2, x.sc<float>(t.o_mean2[l]), x.sc<float>(t.o_rstd2[l]), x.s));
    // only relu(z) is kept: it is positive exactly where z is, which is all the backward pass needs
    TF_TRY(dense(x, u2, D.d, D.f, b.w1, b.b1, nullptr, x.sc<bf16_t>(t.o_z1[l]), PBT_ACT_RELU));
    PBT_HIP(h, dropout_apply(x.sc<bf16_t>(t.o_z1[l]), nullptr, x.P, per_f, dr, 4 * l + 2, fd, x.s, nullptr, x.sc<uint16_t>(t.o_mask[l][1])));
    TF_TRY(dense(x, fd, D.f, D.d, b.w2, b.b2, nullptr, tmp_d, PBT_ACT_NONE));
    PBT_HIP(h, dropout_apply(tmp_d, hmid, x.P, per_d, dr, 4 * l + 3, hout, x.s, nullptr, x.sc<uint16_t>(t.o_mask[l][2])));
  }
  bf16_t* uf = x.sc<bf16_t>(t.o_uf);
  if (!x.fused_bwd)
    PBT_HIP(h, layernorm_fwd(x.sc<bf16_t>(t.o_h[D.L]), x.P, x.n, D.d, x.W32, x.S_, t.lnfg, t.lnfb, uf, x.sc<float>(t.o_meanf), x.sc<float>(t.o_rstdf), x.s));
  GemmOperands o{uf, D.d, (int64_t)x.n * D.d, false, x.W16 + t.whead, D.V, x.S_, false, x.n, D.V, D.d, x.P};
  PBT_LAUNCH(h, PBT_K_GEMM_FWD, x.s, gemm_bias_f32(o, x.W32 + t.bhead, x.S_, x.sc<float>(t.o_logits), D.V, (int64_t)x.n * D.V, x.s));
  return PBT_OK;
}

Ctx make_ctx(pbt_handle* h, int Bc, hipStream_t s) {
  const Plan& p = h->plan;
  Ctx x{h, s, dim_of(h->cfg), h->cfg.P, Bc, Bc * h->cfg.tf_seq, p.lay.stride, h->st<float>(p.o_w32), h->st<bf16_t>(p.o_w16), h->sc<float>(p.o_grad), false};
  x.fused_bwd = tf_fused_elementwise(h->cfg);
  return x;
}

}  // namespace

pbt_status tf_layout(const pbt_config* c, Plan* pl) {
  const int L = c->n_layers;
  if (c->tf_vocab < 2 || c->tf_d_model < 8 || c->tf_heads < 1 || c->tf_d_ff < 8 || c->tf_seq < 1)
    return fail(nullptr, PBT_EINVAL, "transformer sizes must be positive");
  if (c->tf_d_model % c->tf_heads || (c->tf_d_model / c->tf_heads) % 8 || c->tf_d_model % 8 || c->tf_d_ff % 8 || c->tf_vocab % 8 || c->tf_seq % 8)
    return fail(nullptr, PBT_EUNSUPPORTED, "d_model, head width, d_ff, vocabulary and sequence length must be multiples of 8");
  if (c->tf_seq > 4096) return fail(nullptr, PBT_EUNSUPPORTED, "sequence length above 4096");
  if ((int64_t)c->batch * c->tf_seq > 16000) return fail(nullptr, PBT_EUNSUPPORTED, "more than 16000 positions per member and step");
  if (2 + 12 * L + 4 > PBT_MAX_SEGMENTS || L >= PBT_MAX_DIMS) return fail(nullptr, PBT_EUNSUPPORTED, "too many blocks");
  pbt_layout& lay = pl->lay;
  TfPlan& t = pl->tf;
  std::memset(&lay, 0, sizeof lay);
  const int64_t d = c->tf_d_model, f = c->tf_d_ff, V = c->tf_vocab, S = c->tf_seq;
  int64_t off = 0, n_params = 0;
  auto seg = [&](int64_t len) {
    const int64_t o = off;
    lay.seg_off[lay.n_seg] = o;
    lay.seg_len[lay.n_seg++] = len;
    off = round_up(off + len, SEG_ALIGN);
    n_params += len;
    return o;
  };
  t.tok = seg(V * d);
  t.pos = seg(S * d);
  for (int l = 0; l < L; ++l) {
    TfBlockOff& b = t.blk[l];
    b.ln1g = seg(d); b.ln1b = seg(d); b.wqkv = seg(d * 3 * d); b.bqkv = seg(3 * d); b.wo = seg(d * d); b.bo = seg(d);
    b.ln2g = seg(d); b.ln2b = seg(d); b.w1 = seg(d * f); b.b1 = seg(f); b.w2 = seg(f * d); b.b2 = seg(d);
  }
  t.lnfg = seg(d); t.lnfb = seg(d); t.whead = seg(d * V); t.bhead = seg(V);
  lay.stride = round_up(off, STRIDE_ALIGN);
  lay.n_params = n_params;
  return PBT_OK;
}

pbt_status tf_check_and_plan(const pbt_config* c, Plan* pl, Carver* w) {
  TfPlan& t = pl->tf;
  const Dim D{c->tf_vocab, c->tf_d_model, c->tf_heads, c->tf_d_model / c->tf_heads, c->tf_d_ff, c->tf_seq, c->n_layers};
  const size_t P = c->P, n = (size_t)c->batch * D.S;
  t.fused_attn = attention_fused_applies(D.d, D.H, D.S);
  const size_t nd = P * n * D.d * 2, nf = P * n * D.f * 2, ns = P * (size_t)c->batch * D.H * D.S * D.S * 2;
  t.o_tokens = w->take(P * n * 4);
  t.o_targets = w->take(P * n * 4);
  for (int l = 0; l <= D.L; ++l) t.o_h[l] = w->take(nd);
  for (int l = 0; l < D.L; ++l) {
    t.o_hmid[l] = w->take(nd);
    t.o_mean1[l] = w->take(P * n * 4); t.o_rstd1[l] = w->take(P * n * 4);
    t.o_mean2[l] = w->take(P * n * 4); t.o_rstd2[l] = w->take(P * n * 4);
    t.o_u[l] = w->take(nd); t.o_qkv[l] = w->take(3 * nd); t.o_o[l] = w->take(nd);
    if (t.fused_attn) {
      t.o_keep[l] = w->take(attention_record_bytes((int)P, c->batch, D.H));
      t.o_pq[l] = t.o_pd[l] = 0;
    } else {
      t.o_pq[l] = w->take(ns); t.o_pd[l] = w->take(ns);
      t.o_keep[l] = 0;
    }
    t.o_u2[l] = w->take(nd); t.o_z1[l] = tf_fused_elementwise(*c) ? 0 : w->take(nf); t.o_fd[l] = w->take(nf);
    t.o_mask[l][0] = w->take(dropout_mask_bytes((int)P, (int64_t)n * D.d));
    t.o_mask[l][1] = w->take(dropout_mask_bytes((int)P, (int64_t)n * D.f));
    t.o_mask[l][2] = w->take(dropout_mask_bytes((int)P, (int64_t)n * D.d));
  }
  t.o_meanf = w->take(P * n * 4); t.o_rstdf = w->take(P * n * 4);
  t.o_score = t.fused_attn ? 0 : w->take(ns);
  t.o_attn_stats = t.fused_attn ? w->take(attention_stats_bytes((int)P, c->batch, D.H)) : 0;
  t.o_wpart = t.o_wcolpart = 0;
  t.wpart_elems = t.wcol_elems = 0;
  {
    const int shapes[5][2] = {{D.d, 3 * D.d}, {D.d, D.d}, {D.d, D.f}, {D.f, D.d}, {D.d, D.V}};   // (rows in, columns out) of every weight matrix
    for (const auto& sh : shapes)
      if (wgrad_in_parts((int)P, (int)n, sh[0], sh[1])) {
        t.wpart_elems = std::max<int64_t>(t.wpart_elems, (int64_t)sh[0] * sh[1]);
        t.wcol_elems = std::max<int64_t>(t.wcol_elems, sh[1]);
      }
    if (t.wpart_elems) {
      t.o_wpart = w->take(P * WGRAD_PARTS * (size_t)t.wpart_elems * 4);
      t.o_wcolpart = w->take(P * WGRAD_PARTS * (size_t)t.wcol_elems * 4);
    }
  }
  for (int k = 0; k < 3; ++k) t.o_tmp_d[k] = w->take(nd);
  for (int k = 0; k < 2; ++k) t.o_tmp_f[k] = w->take(nf);
  t.o_dqkv = w->take(3 * nd);
  t.o_uf = w->take(nd);
  t.o_logits = w->take(P * n * D.V * 4);
  t.o_dlogits = w->take(P * n * D.V * 2);
  t.o_rowloss = w->take(P * n * 4);
  t.o_evalrow = w->take(P * (size_t)c->n_eval * D.S * 4);
  t.o_tokstart = w->take(P * ((size_t)D.V + 1) * 4);
  t.o_tokcursor = w->take(P * (size_t)D.V * 4);
  t.o_tokorder = w->take(P * n * 4);
  t.o_lnpart = w->take(P * (size_t)(LN_FUSED_SLABS > LN_MAX_SLABS ? LN_FUSED_SLABS : LN_MAX_SLABS) * 2 * D.d * 4);
  return PBT_OK;
}

pbt_status tf_step(pbt_handle* h, const int32_t* pool, uint32_t step, hipStream_t s) {
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  const TfPlan& t = p.tf;
  const Ctx x = make_ctx(h, c.batch, s);
  const Dim& D = x.D;
  const DropArgs dr{h->st<float>(p.o_hyper), c.n_hyper, t.col_drop, 1, step, c.seed};
  const int64_t per_d = (int64_t)x.n * D.d, per_f = (int64_t)x.n * D.f;
  const float att_scale = 1.f / sqrtf((float)D.dh);
  TF_TRY(forward(x, pool, c.n_train, step, 1, 1));
  float* rowloss = x.sc<float>(t.o_rowloss);
  bf16_t* dl = x.sc<bf16_t>(t.o_dlogits);
  PBT_HIP(h, xent_rows(x.sc<float>(t.o_logits), x.sc<int32_t>(t.o_targets), x.P, x.n, D.V, h->st<float>(p.o_hyper), c.n_hyper, t.col_ls, 1,
                       1.f / (float)x.n, dl, rowloss, s));
  PBT_LAUNCH(h, PBT_K_HEAD, s, row_reduce(rowloss, x.n, x.P, x.n, 1.f / (float)x.n, h->st<float>(p.o_loss), 1, s));

  bf16_t* dh = x.sc<bf16_t>(t.o_tmp_d[0]);   // gradient of the residual stream (ping)
  bf16_t* dh2 = x.sc<bf16_t>(t.o_tmp_d[1]);  // (pong)
  bf16_t* dd = x.sc<bf16_t>(t.o_tmp_d[2]);   // width-d scratch
  bf16_t* du = x.sc<bf16_t>(t.o_uf);         // width-d scratch, free once the head's weight gradient is taken
  bf16_t* df0 = x.sc<bf16_t>(t.o_tmp_f[0]);
  bf16_t* df1 = x.sc<bf16_t>(t.o_tmp_f[1]);
  bf16_t* dqkv = x.sc<bf16_t>(t.o_dqkv);
  bf16_t* dscore = x.sc<bf16_t>(t.o_score);

  // The gradient of a dropout site's input is the gradient of its output times the keep factors the forward pass
  // recorded.  On the fused path that multiply rides on the kernel that produces the gradient (the LayerNorm
  // backward for the two residual-branch sites, the input-gradient GEMM's epilogue for the feed-forward hidden
  // site); otherwise it is a pass of its own.
  const float* Hh = h->st<float>(p.o_hyper);
  auto record = [&](int l, int k, int64_t per_member) {
    return DropRecord{x.sc<uint8_t>(t.o_mask[l][k]), (int64_t)(dropout_mask_bytes(1, per_member)), Hh, c.n_hyper, t.col_drop};
  };
  const bool fb = x.fused_bwd;
  // head and final LayerNorm
  TF_TRY(wgrad(x, x.sc<bf16_t>(t.o_uf), D.d, dl, D.V, t.whead, t.bhead));
  TF_TRY(dgrad(x, dl, D.V, D.d, t.whead, nullptr, 0, du));   // (du: the final LayerNorm's output buffer, free once the head's weight gradient is taken)
  TF_TRY(ln_backward(x, du, x.sc<bf16_t>(t.o_h[D.L]), x.sc<float>(t.o_meanf), x.sc<float>(t.o_rstdf), t.lnfg, t.lnfb, nullptr, dh,
                     fb ? dd : nullptr, fb ? record(D.L - 1, 2, per_d) : DropRecord()));
  for (int l = D.L - 1; l >= 0; --l) {
    const TfBlockOff& b = t.blk[l];
    bf16_t* qkv = x.sc<bf16_t>(t.o_qkv[l]);
    // feed-forward branch
    if (!fb) PBT_HIP(h, dropout_apply(dh, nullptr, x.P, per_d, dr, 4 * l + 3, dd, s, x.sc<uint16_t>(t.o_mask[l][2])));
    TF_TRY(wgrad(x, x.sc<bf16_t>(t.o_fd[l]), D.f, dd, D.d, b.w2, b.b2));
    if (fb) {
      TF_TRY(dgrad(x, dd, D.d, D.f, b.w2, x.sc<bf16_t>(t.o_fd[l]), PBT_ACT_RELU, df1, record(l, 1, per_f)));   // (the forward pass kept no separate relu(z))
    } else {
      TF_TRY(dgrad(x, dd, D.d, D.f, b.w2, x.sc<bf16_t>(t.o_z1[l]), PBT_ACT_RELU, df0));
      PBT_HIP(h, dropout_apply(df0, nullptr, x.P, per_f, dr, 4 * l + 2, df1, s, x.sc<uint16_t>(t.o_mask[l][1])));
    }
    TF_TRY(wgrad(x, x.sc<bf16_t>(t.o_u2[l]), D.d, df1, D.f, b.w1, b.b1));
    TF_TRY(dgrad(x, df1, D.f, D.d, b.w1, nullptr, 0, du));
    TF_TRY(ln_backward(x, du, x.sc<bf16_t>(t.o_hmid[l]), x.sc<float>(t.o_mean2[l]), x.sc<float>(t.o_rstd2[l]), b.ln2g, b.ln2b, dh, dh2,
                       fb ? dd : nullptr, fb ? record(l, 0, per_d) : DropRecord()));
    // attention branch
    if (!fb) PBT_HIP(h, dropout_apply(dh2, nullptr, x.P, per_d, dr, 4 * l + 1, dd, s, x.sc<uint16_t>(t.o_mask[l][0])));
    TF_TRY(wgrad(x, x.sc<bf16_t>(t.o_o[l]), D.d, dd, D.d, b.wo, b.bo));
    TF_TRY(dgrad(x, dd, D.d, D.d, b.wo, nullptr, 0, du));  // du = gradient of the merged head outputs
    if (t.fused_attn) {
      PBT_LAUNCH(h, PBT_K_HEAD, s, attention_bwd(qkv, du, x.P, x.Bc, D.S, D.d, D.H, att_scale, dr, x.sc<uint32_t>(t.o_keep[l]),
                                                 x.sc<float>(t.o_attn_stats), dqkv, s));
    } else {
      const bf16_t* pd = x.sc<bf16_t>(t.o_pd[l]);
      TF_TRY(attn_gemm(x, in_scores(pd, D), true, in_rows(du, 0, D.d, D), false, in_rows(dqkv, 2 * D.d, 3 * D.d, D), D.S, D.dh, D.S));           // dV = Pd^T dO
      TF_TRY(attn_gemm(x, in_rows(du, 0, D.d, D), false, in_rows(qkv, 2 * D.d, 3 * D.d, D), true, in_scores(dscore, D), D.S, D.S, D.dh));          // dPd = dO V^T
      PBT_HIP(h, softmax_bwd(x.sc<bf16_t>(t.o_pq[l]), dscore, x.P, (int64_t)x.Bc * D.H * D.S, D.S, att_scale, dr, 4 * l + 0, s));
      TF_TRY(attn_gemm(x, in_scores(dscore, D), false, in_rows(qkv, D.d, 3 * D.d, D), false, in_rows(dqkv, 0, 3 * D.d, D), D.S, D.dh, D.S));       // dQ = dS K
      TF_TRY(attn_gemm(x, in_scores(dscore, D), true, in_rows(qkv, 0, 3 * D.d, D), false, in_rows(dqkv, D.d, 3 * D.d, D), D.S, D.dh, D.S));        // dK = dS^T Q
    }
    TF_TRY(wgrad(x, x.sc<bf16_t>(t.o_u[l]), D.d, dqkv, 3 * D.d, b.wqkv, b.bqkv));
    TF_TRY(dgrad(x, dqkv, 3 * D.d, D.d, b.wqkv, nullptr, 0, du));
    const bool next = fb && l > 0;   // the block below starts with the backward of its feed-forward output site
    TF_TRY(ln_backward(x, du, x.sc<bf16_t>(t.o_h[l]), x.sc<float>(t.o_mean1[l]), x.sc<float>(t.o_rstd1[l]), b.ln1g, b.ln1b, dh2, dh,
                       next ? dd : nullptr, next ? record(l - 1, 2, per_d) : DropRecord()));
  }
  PBT_HIP(h, embed_bwd(dh, x.sc<int32_t>(t.o_tokens), x.Bc, D.S, D.d, D.V, x.P, x.G, x.S_, t.tok, t.pos, x.sc<int32_t>(t.o_tokstart),
                       x.sc<int32_t>(t.o_tokcursor), x.sc<int32_t>(t.o_tokorder), s));
  OptArgs oa{h->st<float>(p.o_w32), h->st<float>(p.o_opt0), h->st<float>(p.o_opt1), h->st<bf16_t>(p.o_w16), x.G, 0, x.S_,
             h->st<float>(p.o_hyper), h->st<int32_t>(p.o_t), x.S_, x.P, c.n_hyper, PBT_OPT_ADAM, p.col_lr, -1, -1,
             c.opt_const[0], c.opt_const[1], c.opt_const[2], c.opt_const[3]};
  PBT_LAUNCH(h, PBT_K_OPTIMIZER, s, optimizer_step(oa, s));
  return PBT_OK;
}

pbt_status tf_eval(pbt_handle* h, const int32_t* eval_tokens, hipStream_t s) {
  const pbt_config& c = h->cfg;
  const TfPlan& t = h->plan.tf;
  const int S = c.tf_seq;
  float* evalrow = h->sc<float>(t.o_evalrow);
  // chunks of `batch` sequences; per-row losses of chunk k go to a [n_chunks][P][rows] staging area
  // whose per-member rows are summed by the perplexity kernel in a fixed order
  if (c.n_eval % c.batch) return fail(h, PBT_EUNSUPPORTED, "n_eval must be a multiple of batch");
  const int chunks = c.n_eval / c.batch;
  for (int k = 0; k < chunks; ++k) {
    const Ctx x = make_ctx(h, c.batch, s);
    TF_TRY(forward(x, eval_tokens + (int64_t)k * c.batch * (S + 1), c.batch, 0u, 0, 0));
    PBT_HIP(h, xent_rows(x.sc<float>(t.o_logits), x.sc<int32_t>(t.o_targets), x.P, x.n, c.tf_vocab, h->st<float>(h->plan.o_hyper), c.n_hyper, -1, 0,
                         0.f, nullptr, x.sc<float>(t.o_rowloss), s));
    PBT_HIP(h, tf_scatter_rows(x.sc<float>(t.o_rowloss), x.P, x.n, evalrow, (int64_t)c.n_eval * S, (int64_t)k * x.n, s));
  }
  PBT_HIP(h, perplexity_score(evalrow, c.P, c.n_eval * S, h->st<float>(h->plan.o_score), s));
  return PBT_OK;
}

}  // namespace pbt
