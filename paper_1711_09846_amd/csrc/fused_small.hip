// Fully fused fp32 population step for networks small enough to live in LDS: one workgroup per
// member gathers its mini-batch, runs forward, softmax cross-entropy, backward and the optimiser
// update, for n_steps consecutive steps, touching HBM only for the data rows.  Members are
// independent between exploit points (Algorithm 1 of the PBT paper), so no grid-wide
// synchronisation is needed and one launch covers a whole ready interval.
//
// Row pitches in LDS are (width + 1) floats so that both "lanes along the batch" and "lanes
// along the features" access patterns are free of bank conflicts.
#include "common.h"
#include "internal.h"
#include "philox.h"

namespace pbt {

size_t fused_small_plan(FusedSmallArgs& a, bool for_eval) {
  int off = 0;
  a.lds_w = off; off += (int)a.stride;
  a.lds_s0 = a.lds_s1 = 0;
  if (!for_eval) {
    a.lds_s0 = off; off += (int)a.stride;
    if (a.optimizer == 1) { a.lds_s1 = off; off += (int)a.stride; }
  }
  int maxd = 0;
  for (int l = 0; l < a.n_layers; ++l) {
    a.lds_a[l] = off; off += a.B * (a.dims[l] + 1);
    a.lds_z[l] = off; off += a.B * (a.dims[l + 1] + 1);
    if (a.dims[l + 1] > maxd) maxd = a.dims[l + 1];
    if (a.dims[l] > maxd) maxd = a.dims[l];
  }
  a.lds_dz[0] = a.lds_dz[1] = 0;
  if (!for_eval) {
    a.lds_dz[0] = off; off += a.B * (maxd + 1);
    a.lds_dz[1] = off; off += a.B * (maxd + 1);
  }
  a.lds_rowloss = off; off += a.B;
  a.lds_y = off; off += a.B;
  a.lds_total = off;
  return (size_t)off * sizeof(float);
}

constexpr int FS_THREADS = 256;

// Forward through all layers for the B rows whose inputs sit in lds_a[0]; leaves logits in
// lds_z[L-1] and per-row losses in lds_rowloss.
__device__ __forceinline__ void fs_forward(const FusedSmallArgs& a, float* lds, int nrows) {
  const int tid = threadIdx.x;
  const float* W = lds + a.lds_w;
  for (int l = 0; l < a.n_layers; ++l) {
    const int K = a.dims[l], N = a.dims[l + 1];
    const float* in = lds + a.lds_a[l];
    float* z = lds + a.lds_z[l];
    const float* Wl = W + a.w_off[l];
    const float* bl = W + a.b_off[l];
    for (int idx = tid; idx < nrows * N; idx += FS_THREADS) {
      const int b = idx / N, n = idx - b * N;
      float acc = 0.f;
      for (int k = 0; k < K; ++k) acc = fmaf(in[b * (K + 1) + k], Wl[k * N + n], acc);
      acc += bl[n];
      z[b * (N + 1) + n] = acc;
      if (l < a.n_layers - 1) lds[a.lds_a[l + 1] + b * (N + 1) + n] = act_fwd(acc, a.act);
    }
    __syncthreads();
  }
}

// Softmax cross-entropy per row; when dz != null also (softmax - onehot) * gscale into dz (pitch C+1).
__device__ __forceinline__ void fs_loss(const FusedSmallArgs& a, float* lds, int nrows, float* dz, float gscale) {
  const int C = a.dims[a.n_layers];
  const float* logits = lds + a.lds_z[a.n_layers - 1];
  const int* y = reinterpret_cast<const int*>(lds + a.lds_y);
  for (int b = threadIdx.x; b < nrows; b += FS_THREADS) {
    const float* lg = logits + b * (C + 1);
    // log-sum-exp with the largest term split off: lse = mx + log1p(sum of the others), which
    // keeps full relative accuracy when one class dominates (small losses)
    float mx = lg[0];
    int cm = 0;
    for (int c = 1; c < C; ++c)
      if (lg[c] > mx) { mx = lg[c]; cm = c; }
    float rest = 0.f;
    for (int c = 0; c < C; ++c)
      if (c != cm) rest += expf(lg[c] - mx);
    const float l1p = log1pf(rest);
    const int yb = y[b];
    lds[a.lds_rowloss + b] = l1p + (mx - lg[yb]);
    if (dz) {
      const float inv = 1.f / (1.f + rest);
      // softmax_y - 1 = -(sum of the other classes' terms) / S: no cancellation when softmax_y -> 1
      float others = (yb == cm) ? 0.f : 1.f;
      for (int c = 0; c < C; ++c)
        if (c != yb && c != cm) others += expf(lg[c] - mx);
      for (int c = 0; c < C; ++c)
        dz[b * (C + 1) + c] = (c == yb ? -others * inv : expf(lg[c] - mx) * inv) * gscale;
    }
  }
  __syncthreads();
}

__device__ __forceinline__ float fs_sum_rowloss(const float* lds_rowloss, int nrows) {
  // first wavefront: lane adds rows lane, lane+64, ... then butterfly; valid in wave 0 only
  float acc = 0.f;
  for (int r = threadIdx.x & 63; r < nrows; r += 64) acc += lds_rowloss[r];
  return wave_sum(acc);
}

__global__ __launch_bounds__(FS_THREADS) void fused_small_step_kernel(FusedSmallArgs a) {
  extern __shared__ float lds[];
  const int i = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int64_t base = (int64_t)i * a.stride;
  const int n = (int)a.stride;
  float* W = lds + a.lds_w;
  float* S0 = lds + a.lds_s0;
  float* S1 = lds + a.lds_s1;
  for (int j = tid; j < n; j += FS_THREADS) {
    W[j] = a.W32[base + j];
    S0[j] = a.S0[base + j];
    if (a.optimizer == 1) S1[j] = a.S1[base + j];
  }
  const float* h = a.H + (int64_t)i * a.n_hyper;
  const float lr = h[a.col_lr];
  const float b1 = (a.optimizer == 1 && a.col_beta1 >= 0) ? h[a.col_beta1] : a.c0;
  const float wd = (a.optimizer == 1 && a.col_wd >= 0) ? h[a.col_wd] : a.c3;
  int t = a.t[i];
  const uint32_t k0 = (uint32_t)a.seed, k1 = (uint32_t)(a.seed >> 32);
  const int L = a.n_layers, B = a.B, d0 = a.dims[0];
  int* ylds = reinterpret_cast<int*>(lds + a.lds_y);
  float last_loss = 0.f;
  __syncthreads();

  for (int s = 0; s < a.n_steps; ++s) {
    const uint32_t step = a.step0 + (uint32_t)s;
    ++t;
    // mini-batch rows (Philox domain 1), one wavefront per row
    for (int r = wave; r < B; r += FS_THREADS / 64) {
      const uint32_t x = philox4x32_10(step, (uint32_t)i, DOMAIN_BATCH, (uint32_t)r, k0, k1).x;
      const int64_t src = (int64_t)philox_bounded(x, (uint32_t)a.n_rows);
      for (int c = lane; c < d0; c += 64) lds[a.lds_a[0] + r * (d0 + 1) + c] = a.x[src * d0 + c];
      if (lane == 0) ylds[r] = a.y[src];
    }
    __syncthreads();
    fs_forward(a, lds, B);
    float* dz = lds + a.lds_dz[0];
    float* dprev = lds + a.lds_dz[1];
    fs_loss(a, lds, B, dz, 1.f / (float)B);
    if (wave == 0) last_loss = fs_sum_rowloss(lds + a.lds_rowloss, B) / (float)B;

    float inv_bc1 = 1.f, inv_bc2 = 1.f;
    if (a.optimizer == 1) {
      inv_bc1 = 1.f / (1.f - powf(b1, (float)t));
      inv_bc2 = 1.f / (1.f - powf(a.c1, (float)t));
    }
    for (int l = L - 1; l >= 0; --l) {
      const int K = a.dims[l], N = a.dims[l + 1];
      const float* in = lds + a.lds_a[l];
      float* Wl = W + a.w_off[l];
      // input gradient first: it needs W_l from before the update
      if (l > 0) {
        const float* zp = lds + a.lds_z[l - 1];
        for (int idx = tid; idx < B * K; idx += FS_THREADS) {
          const int k = idx / B, b = idx - k * B;  // lanes along the batch
          float acc = 0.f;
          for (int nn = 0; nn < N; ++nn) acc = fmaf(dz[b * (N + 1) + nn], Wl[k * N + nn], acc);
          dprev[b * (K + 1) + k] = acc * act_bwd(zp[b * (K + 1) + k], a.act);
        }
      }
      __syncthreads();
      // weight and bias gradient, optimiser update in place (idx < K*N: weights; then N biases)
      for (int idx = tid; idx < K * N + N; idx += FS_THREADS) {
        float g = 0.f;
        int p;
        if (idx < K * N) {
          const int k = idx / N, nn = idx - k * N;
          for (int b = 0; b < B; ++b) g = fmaf(in[b * (K + 1) + k], dz[b * (N + 1) + nn], g);
          p = a.w_off[l] + idx;
        } else {
          const int nn = idx - K * N;
          for (int b = 0; b < B; ++b) g += dz[b * (N + 1) + nn];
          p = a.b_off[l] + nn;
        }
        if (s == a.n_steps - 1) a.G[base + p] = g;
        float w = W[p];
        if (a.optimizer == 0) {
          const float v = a.c0 * S0[p] + g;
          S0[p] = v;
          w = w - lr * v;
        } else if (a.optimizer == 1) {
          const float m = b1 * S0[p] + (1.f - b1) * g;
          const float v = a.c1 * S1[p] + (1.f - a.c1) * g * g;
          S0[p] = m;
          S1[p] = v;
          w = w - lr * ((m * inv_bc1) / (sqrtf(v * inv_bc2) + a.c2) + wd * w);
        } else {
          const float v = a.c0 * S0[p] + (1.f - a.c0) * g * g;
          S0[p] = v;
          w = w - lr * g / sqrtf(v + a.c1);
        }
        W[p] = w;
      }
      __syncthreads();
      float* tmp = dz; dz = dprev; dprev = tmp;
    }
  }
  for (int j = tid; j < n; j += FS_THREADS) {
    a.W32[base + j] = W[j];
    a.S0[base + j] = S0[j];
    if (a.optimizer == 1) a.S1[base + j] = S1[j];
  }
  if (tid == 0) {
    a.t[i] = t;
    a.loss[i] = last_loss;
  }
}

hipError_t fused_small_step(const FusedSmallArgs& a, hipStream_t s) {
  const size_t bytes = (size_t)a.lds_total * sizeof(float);
  if (bytes > FUSED_SMALL_MAX_LDS) return hipErrorInvalidValue;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fused_small_step_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fused_small_step_kernel, dim3(a.P), dim3(FS_THREADS), bytes, s, a);
  return hipGetLastError();
}

// eval: score[i] = -(mean cross-entropy over the held-out rows), chunks of B rows through LDS.
__global__ __launch_bounds__(FS_THREADS) void fused_small_eval_kernel(FusedSmallArgs a) {
  extern __shared__ float lds[];
  const int i = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int64_t base = (int64_t)i * a.stride;
  float* W = lds + a.lds_w;
  for (int j = tid; j < (int)a.stride; j += FS_THREADS) W[j] = a.W32[base + j];
  int* ylds = reinterpret_cast<int*>(lds + a.lds_y);
  const int d0 = a.dims[0];
  float total = 0.f;  // meaningful in wave 0
  __syncthreads();
  for (int r0 = 0; r0 < a.n_rows; r0 += a.B) {
    const int nrows = a.n_rows - r0 < a.B ? a.n_rows - r0 : a.B;
    for (int r = wave; r < nrows; r += FS_THREADS / 64) {
      const int64_t src = r0 + r;
      for (int c = lane; c < d0; c += 64) lds[a.lds_a[0] + r * (d0 + 1) + c] = a.x[src * d0 + c];
      if (lane == 0) ylds[r] = a.y[src];
    }
    __syncthreads();
    fs_forward(a, lds, nrows);
    fs_loss(a, lds, nrows, nullptr, 0.f);
    if (wave == 0) total += fs_sum_rowloss(lds + a.lds_rowloss, nrows);
    __syncthreads();
  }
  if (tid == 0) a.score[i] = -total / (float)a.n_rows;
}

hipError_t fused_small_eval(const FusedSmallArgs& a, hipStream_t s) {
  const size_t bytes = (size_t)a.lds_total * sizeof(float);
  if (bytes > FUSED_SMALL_MAX_LDS) return hipErrorInvalidValue;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fused_small_eval_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fused_small_eval_kernel, dim3(a.P), dim3(FS_THREADS), bytes, s, a);
  return hipGetLastError();
}

}  // namespace pbt
