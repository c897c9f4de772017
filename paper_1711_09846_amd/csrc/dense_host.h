// Host-side helpers shared by the workload files: forward and backward passes of a stack of dense
// layers as sequences of population-batched GEMM launches.
#pragma once
#include "handle.h"

namespace pbt {

struct Net {  // a view of one of the two MLPs inside the member's flat parameter vector
  int L;
  const int32_t* dims;
  int first;  // index of its first layer in the layout
  int hidden_act, out_act;
};


// Dense layers 0 .. n_dense-1 of `net` on `rows` rows per member: in[l+1] = act(in[l] W_l + b_l).
// A[l] (inputs), Z[l] (pre-activations, may be null when no backward pass follows) are bf16
// [P][rows][width]; the output of the last dense layer goes to `last_out` with batch stride
// `last_stride` (so that it can land inside another network's input buffer).
inline pbt_status forward(pbt_handle* h, const Net& net, int n_dense, int rows, bf16_t* const* A, bf16_t* const* Z, bf16_t* last_out,
                   int64_t last_stride, hipStream_t s) {
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  const int64_t S = p.lay.stride;
  const float* W32 = h->st<float>(p.o_w32);
  const bf16_t* W16 = h->st<bf16_t>(p.o_w16);
  for (int l = 0; l < n_dense; ++l) {
    const int K = net.dims[l], N = net.dims[l + 1];
    const bool last = l == n_dense - 1;
    const int act = (l == net.L - 1) ? net.out_act : net.hidden_act;
    GemmOperands o{A[l], K, (int64_t)rows * K, false, W16 + p.lay.w_off[net.first + l], N, S, false, rows, N, K, c.P};
    bf16_t* out = last && last_out ? last_out : A[l + 1];
    const int64_t so = last && last_out ? last_stride : (int64_t)rows * N;
    PBT_LAUNCH(h, PBT_K_GEMM_FWD, s, gemm_bias_act(o, W32 + p.lay.b_off[net.first + l], S, Z ? Z[l] : nullptr, out, N, so, act, s));
  }
  return PBT_OK;
}

// Backward through dense layers n_dense-1 .. 0 given dZ[n_dense-1]: dZ[l-1] = (dZ[l] W_l^T) * act'(Z[l-1])
// and, when want_wgrad, the weight / bias gradients.  With `fused` null the weight gradient goes to G;
// otherwise the optimiser described by *fused is applied in the weight-gradient GEMM's epilogue (the
// bias gradient still goes to G).  The input gradient of a layer is always taken BEFORE its weight
// gradient, because the fused epilogue rewrites the bf16 weights that the input gradient reads.
// For l = 0 the input gradient is produced only when in_z != null: dIn = (dZ[0] W_0^T) * act'(in_z)
// with activation in_act.
inline pbt_status backward(pbt_handle* h, const Net& net, int n_dense, int rows, bf16_t* const* A, bf16_t* const* Z, bf16_t* const* dZ,
                           bool want_wgrad, const OptArgs* fused, const bf16_t* in_z, bf16_t* in_dz, int in_act, hipStream_t s) {
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  const int64_t S = p.lay.stride;
  const bf16_t* W16 = h->st<bf16_t>(p.o_w16);
  float* G = h->sc<float>(p.o_grad);
  for (int l = n_dense - 1; l >= 0; --l) {
    const int K = net.dims[l], N = net.dims[l + 1];
    const bf16_t* zprev = l > 0 ? Z[l - 1] : in_z;
    bf16_t* dzprev = l > 0 ? dZ[l - 1] : in_dz;
    if (zprev) {
      GemmOperands dg{dZ[l], N, (int64_t)rows * N, false, W16 + p.lay.w_off[net.first + l], N, S, true, rows, K, N, c.P};
      PBT_LAUNCH(h, PBT_K_GEMM_DGRAD, s, gemm_dgrad_act(dg, zprev, dzprev, K, (int64_t)rows * K, l > 0 ? net.hidden_act : in_act, s));
    }
    if (want_wgrad) {
      // (the bias gradient, column sums of dZ_l, is a by-product of the same launch)
      GemmOperands wg{A[l], K, (int64_t)rows * K, true, dZ[l], N, (int64_t)rows * N, false, K, N, rows, c.P};
      wg.colsum = G + p.lay.b_off[net.first + l]; wg.colsum_stride = S;
      if (fused)
        PBT_LAUNCH(h, PBT_K_GEMM_WGRAD, s, gemm_wgrad_optimizer(wg, *fused, p.lay.w_off[net.first + l], N, s));
      else
        PBT_LAUNCH(h, PBT_K_GEMM_WGRAD, s, gemm_store_f32(wg, G + p.lay.w_off[net.first + l], N, S, s));
    }
  }
  return PBT_OK;
}

// The streaming optimiser on what the fused weight-gradient epilogues did not cover: of layers
// first .. first+n-1 (layout indices) the first n_fused had their matrices updated in the GEMM; this
// updates their biases and everything of the remaining layers, up to range_end, merging
// neighbouring ranges into one launch.
inline pbt_status optimizer_rest(pbt_handle* h, OptArgs oa, int first, int n, int n_fused, int64_t range_end, hipStream_t s) {
  const Plan& p = h->plan;
  // collect the ranges, then hand them to the kernel OPT_MAX_RANGES at a time
  int64_t rb[PBT_MAX_DIMS + 1], rc[PBT_MAX_DIMS + 1];
  int n_ranges = 0;
  int64_t begin = -1, end = -1;
  for (int l = first; l < first + n; ++l) {
    const int64_t next = l + 1 < first + n ? p.lay.w_off[l + 1] : range_end;
    const int64_t b = l < first + n_fused ? p.lay.b_off[l] : p.lay.w_off[l];
    if (begin >= 0 && b == end) {
      end = next;
    } else {
      if (begin >= 0) { rb[n_ranges] = begin; rc[n_ranges] = end - begin; ++n_ranges; }
      begin = b;
      end = next;
    }
  }
  if (begin >= 0) { rb[n_ranges] = begin; rc[n_ranges] = end - begin; ++n_ranges; }
  for (int r0 = 0; r0 < n_ranges; r0 += OPT_MAX_RANGES) {
    oa.begin = rb[r0];
    oa.count = rc[r0];
    oa.n_extra = n_ranges - r0 - 1 < OPT_MAX_RANGES - 1 ? n_ranges - r0 - 1 : OPT_MAX_RANGES - 1;
    for (int x = 0; x < oa.n_extra; ++x) { oa.xbegin[x] = rb[r0 + 1 + x]; oa.xcount[x] = rc[r0 + 1 + x]; }
    PBT_LAUNCH(h, PBT_K_OPTIMIZER, s, optimizer_step(oa, s));
  }
  return PBT_OK;
}

}  // namespace pbt
