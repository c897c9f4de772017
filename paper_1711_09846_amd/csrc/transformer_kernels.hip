// Row-wise and element-wise kernels of the transformer workload: embedding gather and its gradient,
// LayerNorm forward / backward, causal softmax with dropout forward / backward, dropout and
// residual updates with counter-based (Philox) masks, and the label-smoothed cross-entropy over a
// large vocabulary.  All activations are bf16 in memory; arithmetic is fp32.
//
// Dropout: element e of site s (member i, step c0) keeps its value iff word e % 4 of the Philox
// counter (c0, i, DOMAIN_DROPOUT + s, e / 4) is >= floor(p * 2^32) (capped at 2^32 - 1); kept values
// are scaled by the float nearest to 1 / (1 - p).  p is the member's own rate, read from H on the
// device.  Where a bf16 value times that factor (plus a bf16 residual) is rounded to bf16 again, the
// arithmetic is done in double and rounded once: with round rates such as 0.25 or 0.3 a seventh or
// so of such products are dyadic and a good share of the sums lie within 1e-8 (relative) of the
// midpoint of two bf16 values, closer than fp32 can resolve.
#include "common.h"
#include "internal.h"
#include "philox.h"
#include "dropout.h"

namespace pbt {

// tokens outside the vocabulary are mapped to its ends so that no table read leaves its array
__device__ __forceinline__ int32_t clamp_token(int32_t tok, int V) { return tok < 0 ? 0 : tok >= V ? V - 1 : tok; }

// ---- embeddings ------------------------------------------------------------------------------
// h[i][b][s][:] = tok[token] + pos[s]; tokens are drawn here: sequence b of member i is pool row
// floor(x * n_pool / 2^32), x from Philox domain 1; also copies the targets and bumps t.
__global__ __launch_bounds__(64) void embed_fwd_kernel(const int32_t* __restrict__ pool, int n_pool, int S, int B, int d, int V,
                                                       const bf16_t* __restrict__ W16, int64_t stride, int64_t tok_off,
                                                       int64_t pos_off, uint32_t c0, uint32_t k0, uint32_t k1, int draw,
                                                       bf16_t* __restrict__ h, int32_t* __restrict__ tokens,
                                                       int32_t* __restrict__ targets, int32_t* __restrict__ t) {
  const int s = blockIdx.x, b = blockIdx.y, i = blockIdx.z;
  int64_t row = b;
  if (draw) row = philox_bounded(philox4x32_10(c0, (uint32_t)i, DOMAIN_BATCH, (uint32_t)b, k0, k1).x, (uint32_t)n_pool);
  const int32_t tok = clamp_token(pool[row * (S + 1) + s], V);
  const int64_t r = ((int64_t)i * B + b) * S + s;
  const bf16_t* __restrict__ te = W16 + (int64_t)i * stride + tok_off + (int64_t)tok * d;
  const bf16_t* __restrict__ pe = W16 + (int64_t)i * stride + pos_off + (int64_t)s * d;
  for (int c = threadIdx.x; c < d; c += 64) h[r * d + c] = f2bf(bf2f(te[c]) + bf2f(pe[c]));
  if (threadIdx.x == 0) {
    tokens[r] = tok;
    targets[r] = clamp_token(pool[row * (S + 1) + s + 1], V);
    if (draw && s == 0 && b == 0) t[i] += 1;
  }
}
hipError_t embed_fwd(const int32_t* pool, int n_pool, int S, int B, int d, int V, int P, const bf16_t* W16, int64_t stride,
                     int64_t tok_off, int64_t pos_off, uint32_t c0, uint64_t seed, int draw, bf16_t* h, int32_t* tokens,
                     int32_t* targets, int32_t* t, hipStream_t s) {
  hipLaunchKernelGGL(embed_fwd_kernel, dim3(S, B, P), dim3(64), 0, s, pool, n_pool, S, B, d, V, W16, stride, tok_off, pos_off, c0,
                     (uint32_t)seed, (uint32_t)(seed >> 32), draw, h, tokens, targets, t);
  return hipGetLastError();
}

// Gradient of the embedding tables, in a fixed summation order (no floating-point atomics):
//   1. count the positions of every token (integer atomics), 2. the counts become list starts and every position
//   is filed under its token, positions ascending,
//   3. one workgroup per (token, member) adds up the rows of its list; tokens that do not occur get
//   zeros.  The position table's gradient sums the B rows that share a position.
__global__ __launch_bounds__(256) void tok_count_kernel(const int32_t* __restrict__ tokens, int n, int V, int32_t* __restrict__ start) {
  const int i = blockIdx.y;
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r < n) atomicAdd(&start[(int64_t)i * (V + 1) + tokens[(int64_t)i * n + r]], 1);
}

// counts -> list starts (exclusive prefix sum over the vocabulary), one workgroup per member
__global__ __launch_bounds__(256) void tok_start_kernel(int V, int n, int32_t* __restrict__ start) {
  __shared__ int32_t part[256];
  const int i = blockIdx.x, tid = threadIdx.x;
  int32_t* __restrict__ st = start + (int64_t)i * (V + 1);
  const int span = (V + 255) / 256;   // a span of consecutive tokens per thread
  const int v0 = tid * span, v1 = min(V, v0 + span);
  int32_t sum = 0;
  for (int v = v0; v < v1; ++v) sum += st[v];
  part[tid] = sum;
  __syncthreads();
  if (tid == 0) {
    int32_t run = 0;
    for (int k = 0; k < 256; ++k) { const int32_t c = part[k]; part[k] = run; run += c; }
  }
  __syncthreads();
  int32_t run = part[tid];
  for (int v = v0; v < v1; ++v) { const int32_t c = st[v]; st[v] = run; run += c; }
  if (tid == 255) st[V] = n;
}

// Files every position under its token, positions ascending: position r goes to start[token] + (number of earlier
// positions of the member with the same token).  A workgroup takes 256 positions and counts by looking at all earlier
// tokens of the member, staged in LDS (n^2 / 2 integer compares per member, spread over the whole device: with one
// workgroup per member walking the positions in order this step took 150 us on 16 of 256 compute units).
__global__ __launch_bounds__(256) void tok_place_kernel(const int32_t* __restrict__ tokens, int n, int V, const int32_t* __restrict__ start,
                                                        int32_t* __restrict__ order) {
  extern __shared__ __attribute__((aligned(16))) int32_t s_tok[];   // tokens of positions 0 .. base + 255
  const int i = blockIdx.y, base = blockIdx.x * 256, tid = threadIdx.x;
  const int32_t* __restrict__ tk = tokens + (int64_t)i * n;
  const int upto = min(n, base + 256);
  // (16-byte loads, several in flight: n is a multiple of 4 and so is upto)
#pragma unroll 4
  for (int r = tid * 4; r < upto; r += 1024) *reinterpret_cast<int4*>(s_tok + r) = *reinterpret_cast<const int4*>(tk + r);
  for (int r = upto + tid; r < base + 256; r += 256) s_tok[r] = -1;   // (a ragged last workgroup reads its whole 256)
  __syncthreads();
  const int r = base + tid;
  if (r >= n) return;
  const int32_t tok = s_tok[r];
  int rank = 0;
  // (whole groups of four below the workgroup's first position: the same 16-byte LDS read for every lane)
#pragma unroll 8
  for (int j = 0; j < base; j += 4) {   // (base is a multiple of 256; unrolled so that several reads are in flight)
    const int4 q = *reinterpret_cast<const int4*>(s_tok + j);
    rank += (q.x == tok ? 1 : 0) + (q.y == tok ? 1 : 0) + (q.z == tok ? 1 : 0) + (q.w == tok ? 1 : 0);
  }
#pragma unroll 8
  for (int j = 0; j < 256; ++j) rank += (base + j < r && s_tok[base + j] == tok) ? 1 : 0;
  order[(int64_t)i * n + start[(int64_t)i * (V + 1) + tok] + rank] = r;
}

__global__ __launch_bounds__(128) void tok_sum_kernel(const bf16_t* __restrict__ dh, const int32_t* __restrict__ start,
                                                      const int32_t* __restrict__ order, int n, int d, int V, float* __restrict__ G,
                                                      int64_t stride, int64_t tok_off) {
  const int v = blockIdx.x, i = blockIdx.y;
  const int32_t b = start[(int64_t)i * (V + 1) + v], e = start[(int64_t)i * (V + 1) + v + 1];
  const int32_t* __restrict__ ord = order + (int64_t)i * n;
  const bf16_t* __restrict__ g = dh + (int64_t)i * n * d;
  for (int c0 = threadIdx.x * 4; c0 < d; c0 += 512) {
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    for (int k = b; k < e; ++k) {
      const uint2 x = *reinterpret_cast<const uint2*>(g + (int64_t)ord[k] * d + c0);
      a0 += __uint_as_float(x.x << 16); a1 += __uint_as_float(x.x & 0xffff0000u);
      a2 += __uint_as_float(x.y << 16); a3 += __uint_as_float(x.y & 0xffff0000u);
    }
    *reinterpret_cast<float4*>(G + (int64_t)i * stride + tok_off + (int64_t)v * d + c0) = make_float4(a0, a1, a2, a3);
  }
}

__global__ __launch_bounds__(128) void pos_sum_kernel(const bf16_t* __restrict__ dh, int B, int S, int d, float* __restrict__ G,
                                                      int64_t stride, int64_t pos_off) {
  const int sp = blockIdx.x, i = blockIdx.y;
  const bf16_t* __restrict__ g = dh + (int64_t)i * B * S * d;
  for (int c0 = threadIdx.x * 4; c0 < d; c0 += 512) {
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    for (int b = 0; b < B; ++b) {
      const uint2 x = *reinterpret_cast<const uint2*>(g + ((int64_t)b * S + sp) * d + c0);
      a0 += __uint_as_float(x.x << 16); a1 += __uint_as_float(x.x & 0xffff0000u);
      a2 += __uint_as_float(x.y << 16); a3 += __uint_as_float(x.y & 0xffff0000u);
    }
    *reinterpret_cast<float4*>(G + (int64_t)i * stride + pos_off + (int64_t)sp * d + c0) = make_float4(a0, a1, a2, a3);
  }
}

// start: int32 [P][V + 1], cursor: int32 [P][V], order: int32 [P][B * S] (scratch)
hipError_t embed_bwd(const bf16_t* dh, const int32_t* tokens, int B, int S, int d, int V, int P, float* G, int64_t stride,
                     int64_t tok_off, int64_t pos_off, int32_t* start, int32_t* cursor, int32_t* order, hipStream_t s) {
  const int n = B * S;
  if (d % 4) return hipErrorInvalidValue;
  hipError_t e = fill_u32(reinterpret_cast<uint32_t*>(start), 0u, (int64_t)P * (V + 1), s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(tok_count_kernel, dim3((n + 255) / 256, P), dim3(256), 0, s, tokens, n, V, start);
  (void)cursor;
  if ((size_t)(n + 255) * sizeof(int32_t) > 64 * 1024 || n % 4) return hipErrorInvalidValue;   // (a member's tokens are staged in LDS)
  hipLaunchKernelGGL(tok_start_kernel, dim3(P), dim3(256), 0, s, V, n, start);
  hipLaunchKernelGGL(tok_place_kernel, dim3((n + 255) / 256, P), dim3(256), (size_t)((n + 255) / 256 * 256) * sizeof(int32_t), s, tokens, n, V, start, order);
  hipLaunchKernelGGL(tok_sum_kernel, dim3(V, P), dim3(128), 0, s, dh, start, order, n, d, V, G, stride, tok_off);
  hipLaunchKernelGGL(pos_sum_kernel, dim3(S, P), dim3(128), 0, s, dh, B, S, d, G, stride, pos_off);
  return hipGetLastError();
}

// ---- LayerNorm -------------------------------------------------------------------------------
// One wavefront per row, eight consecutive elements (one 16-byte access) per lane and pass; a row
// is at most a few KB, so the second and third pass over it are served by the caches.
// y = (x - mean) * rstd * g + b, eps = 1e-5; mean and rstd are kept.
constexpr float LN_EPS = 1e-5f;
__device__ __forceinline__ void load8(const bf16_t* p, float* v) {
  const uint4 u = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) { v[2 * q] = __uint_as_float(w[q] << 16); v[2 * q + 1] = __uint_as_float(w[q] & 0xffff0000u); }
}
__device__ __forceinline__ void load8(const float* p, float* v) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void store8(bf16_t* p, const float* v) {
  *reinterpret_cast<uint4*>(p) = make_uint4(f2bf_pair(v[0], v[1]), f2bf_pair(v[2], v[3]), f2bf_pair(v[4], v[5]), f2bf_pair(v[6], v[7]));
}

__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const bf16_t* __restrict__ x, int rows_per_member, int d,
                                                            const float* __restrict__ W32, int64_t stride, int64_t g_off,
                                                            int64_t b_off, bf16_t* __restrict__ y, float* __restrict__ mean,
                                                            float* __restrict__ rstd) {
  const int i = blockIdx.y;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (r >= rows_per_member) return;
  const int64_t row = (int64_t)i * rows_per_member + r;
  const bf16_t* __restrict__ xr = x + row * d;
  float s = 0.f;
  for (int c = lane * 8; c < d; c += 512) {
    float v[8];
    load8(xr + c, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) s += v[e];
  }
  const float mu = wave_sum(s) / (float)d;
  float var = 0.f;
  for (int c = lane * 8; c < d; c += 512) {
    float v[8];
    load8(xr + c, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) { const float t = v[e] - mu; var = fmaf(t, t, var); }
  }
  const float rs = rsqrtf(wave_sum(var) / (float)d + LN_EPS);
  const float* __restrict__ g = W32 + (int64_t)i * stride + g_off;
  const float* __restrict__ b = W32 + (int64_t)i * stride + b_off;
  for (int c = lane * 8; c < d; c += 512) {
    float v[8], gv[8], bv[8];
    load8(xr + c, v);
    load8(g + c, gv);
    load8(b + c, bv);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (v[e] - mu) * rs * gv[e] + bv[e];
    store8(y + row * d + c, v);
  }
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
}
hipError_t layernorm_fwd(const bf16_t* x, int P, int rows, int d, const float* W32, int64_t stride, int64_t g_off, int64_t b_off,
                         bf16_t* y, float* mean, float* rstd, hipStream_t s) {
  if (d % 8 || g_off % 4 || b_off % 4 || stride % 4) return hipErrorInvalidValue;
  hipLaunchKernelGGL(layernorm_fwd_kernel, dim3((rows + 3) / 4, P), dim3(256), 0, s, x, rows, d, W32, stride, g_off, b_off, y, mean, rstd);
  return hipGetLastError();
}

// dx = rstd (dy g - mean(dy g) - xhat mean(dy g xhat)); out = dx (+ res when res != null), bf16.
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ x,
                                                            const float* __restrict__ mean, const float* __restrict__ rstd,
                                                            int rows_per_member, int d, const float* __restrict__ W32,
                                                            int64_t stride, int64_t g_off, const bf16_t* __restrict__ res,
                                                            bf16_t* __restrict__ out) {
  const int i = blockIdx.y;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (r >= rows_per_member) return;
  const int64_t row = (int64_t)i * rows_per_member + r;
  const float mu = mean[row], rs = rstd[row];
  const float* __restrict__ g = W32 + (int64_t)i * stride + g_off;
  float a = 0.f, b = 0.f;
  for (int c = lane * 8; c < d; c += 512) {
    float dv[8], xv[8], gv[8];
    load8(dy + row * d + c, dv);
    load8(x + row * d + c, xv);
    load8(g + c, gv);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float dyg = dv[e] * gv[e];
      a += dyg;
      b = fmaf(dyg, (xv[e] - mu) * rs, b);
    }
  }
  a = wave_sum(a) / (float)d;
  b = wave_sum(b) / (float)d;
  for (int c = lane * 8; c < d; c += 512) {
    float dv[8], xv[8], gv[8], o[8];
    load8(dy + row * d + c, dv);
    load8(x + row * d + c, xv);
    load8(g + c, gv);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float xh = (xv[e] - mu) * rs;
      o[e] = rs * (dv[e] * gv[e] - a - xh * b);
    }
    if (res) {
      float rv[8];
      load8(res + row * d + c, rv);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] += rv[e];
    }
    store8(out + row * d + c, o);
  }
}
hipError_t layernorm_bwd(const bf16_t* dy, const bf16_t* x, const float* mean, const float* rstd, int P, int rows, int d,
                         const float* W32, int64_t stride, int64_t g_off, const bf16_t* res, bf16_t* out, hipStream_t s) {
  if (d % 8 || g_off % 4 || stride % 4) return hipErrorInvalidValue;
  hipLaunchKernelGGL(layernorm_bwd_kernel, dim3((rows + 3) / 4, P), dim3(256), 0, s, dy, x, mean, rstd, rows, d, W32, stride, g_off, res, out);
  return hipGetLastError();
}

// dg[c] = sum_r dy[r][c] xhat[r][c], db[c] = sum_r dy[r][c].  Two passes with a fixed summation order:
// a workgroup covers 64 columns of one slab of rows (4 row groups of 64 threads, combined through
// LDS) and writes a partial sum; a second kernel adds the slabs' partial sums in slab order.
__global__ __launch_bounds__(256) void layernorm_param_grad_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ x,
                                                                   const float* __restrict__ mean, const float* __restrict__ rstd,
                                                                   int rows_per_member, int d, int rows_per_slab,
                                                                   float* __restrict__ part) {
  __shared__ float pg[4][64], pb[4][64];
  const int i = blockIdx.z, slab = blockIdx.y, n_slabs = gridDim.y;
  const int cl = threadIdx.x & 63, rg = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  const int r_end = min(rows_per_member, (slab + 1) * rows_per_slab);
  float ag = 0.f, ab = 0.f;
  if (c < d) {
    for (int r = slab * rows_per_slab + rg; r < r_end; r += 4) {
      const int64_t row = (int64_t)i * rows_per_member + r;
      const float v = bf2f(dy[row * d + c]);
      ab += v;
      ag = fmaf(v, (bf2f(x[row * d + c]) - mean[row]) * rstd[row], ag);
    }
  }
  pg[rg][cl] = ag;
  pb[rg][cl] = ab;
  __syncthreads();
  if (rg == 0 && c < d) {
    float* __restrict__ out = part + ((int64_t)i * n_slabs + slab) * 2 * d;
    out[c] = ((pg[0][cl] + pg[1][cl]) + pg[2][cl]) + pg[3][cl];
    out[d + c] = ((pb[0][cl] + pb[1][cl]) + pb[2][cl]) + pb[3][cl];
  }
}
// adds the slabs' partial sums in a fixed order: a workgroup covers 64 of the 2 d columns (gains, then biases), its
// four thread groups each add a quarter of the slabs in slab order, and the four results are added in group order
__global__ __launch_bounds__(256) void layernorm_param_combine_kernel(const float* __restrict__ part, int n_slabs, int d,
                                                                      float* __restrict__ G, int64_t stride, int64_t g_off, int64_t b_off) {
  __shared__ float red[4][64];
  const int i = blockIdx.y;
  const int cl = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;  // 0..2d-1
  const int per = (n_slabs + 3) / 4;
  float acc = 0.f;
  if (c < 2 * d)
    for (int k = grp * per; k < min(n_slabs, (grp + 1) * per); ++k) acc += part[((int64_t)i * n_slabs + k) * 2 * d + c];
  red[grp][cl] = acc;
  __syncthreads();
  if (grp == 0 && c < 2 * d)
    G[(int64_t)i * stride + (c < d ? g_off + c : b_off + c - d)] = ((red[0][cl] + red[1][cl]) + red[2][cl]) + red[3][cl];
}
// part: float [P][LN_MAX_SLABS][2][d] (scratch)
hipError_t layernorm_param_grad(const bf16_t* dy, const bf16_t* x, const float* mean, const float* rstd, int P, int rows, int d,
                                float* G, int64_t stride, int64_t g_off, int64_t b_off, float* part, hipStream_t s) {
  int n_slabs = (rows + 127) / 128;
  if (n_slabs > LN_MAX_SLABS) n_slabs = LN_MAX_SLABS;
  const int rows_per_slab = (rows + n_slabs - 1) / n_slabs;
  hipLaunchKernelGGL(layernorm_param_grad_kernel, dim3((d + 63) / 64, n_slabs, P), dim3(256), 0, s, dy, x, mean, rstd, rows, d,
                     rows_per_slab, part);
  hipLaunchKernelGGL(layernorm_param_combine_kernel, dim3((2 * d + 63) / 64, P), dim3(256), 0, s, part, n_slabs, d, G, stride, g_off, b_off);
  return hipGetLastError();
}

// LayerNorm backward and the gradients of its gain and bias in one pass over dy and x: a workgroup takes a slab
// of rows (wavefront w the rows w, w + 4, ... of the slab), a lane owns the same 8 J columns in every row, so the
// gain is read once, a row is read once (it stays in registers between the two reductions and the output) and
// the per-column sums dg += dy xhat, db += dy accumulate in registers; the four wavefronts are combined through
// LDS in wavefront order and the slab's partial sums go to `part`, which layernorm_param_combine_kernel adds in
// slab order.  J = ceil(d / 512).
template <int J>
__global__ __launch_bounds__(256) void layernorm_bwd_fused_kernel(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ x,
                                                                  const float* __restrict__ mean, const float* __restrict__ rstd,
                                                                  int rows_per_member, int d, int rows_per_slab,
                                                                  const float* __restrict__ W32, int64_t stride, int64_t g_off,
                                                                  const bf16_t* __restrict__ res, bf16_t* __restrict__ out,
                                                                  float* __restrict__ part, bf16_t* __restrict__ out2, DropRecord drop) {
  extern __shared__ float red[];  // [4][2][d]
  const int i = blockIdx.y, slab = blockIdx.x, n_slabs = gridDim.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* __restrict__ g = W32 + (int64_t)i * stride + g_off;
  float drop_scale = 1.f;
  if (out2) {
    const float p = drop.col >= 0 ? drop.H[(int64_t)i * drop.n_hyper + drop.col] : 0.f;
    drop_scale = p > 0.f ? (float)(1.0 / (1.0 - (double)p)) : 1.f;
  }
  float gv[J][8], ag[J][8], ab[J][8];
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int c = lane * 8 + 512 * j;
#pragma unroll
    for (int e = 0; e < 8; ++e) { gv[j][e] = 0.f; ag[j][e] = 0.f; ab[j][e] = 0.f; }
    if (c < d) load8(g + c, gv[j]);
  }
  const int r_end = min(rows_per_member, (slab + 1) * rows_per_slab);
  for (int r = slab * rows_per_slab + wave; r < r_end; r += 4) {
    const int64_t row = (int64_t)i * rows_per_member + r;
    const float mu = mean[row], rs = rstd[row];
    float dv[J][8], xv[J][8];
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const int c = lane * 8 + 512 * j;
      if (c < d) {
        load8(dy + row * d + c, dv[j]);
        load8(x + row * d + c, xv[j]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float dyg = dv[j][e] * gv[j][e];
          a += dyg;
          b = fmaf(dyg, (xv[j][e] - mu) * rs, b);
        }
      }
    }
    a = wave_sum(a) / (float)d;
    b = wave_sum(b) / (float)d;
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const int c = lane * 8 + 512 * j;
      if (c < d) {
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = (xv[j][e] - mu) * rs;
          o[e] = rs * (dv[j][e] * gv[j][e] - a - xh * b);
          ab[j][e] += dv[j][e];
          ag[j][e] = fmaf(dv[j][e], xh, ag[j][e]);
        }
        if (res) {
          float rv[8];
          load8(res + row * d + c, rv);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] += rv[e];
        }
        store8(out + row * d + c, o);
        if (out2) {
          // the stored (bf16) value times the recorded keep factor, rounded once more
          const uint32_t bits = drop.mask[(int64_t)i * drop.mask_stride + (((int64_t)r * d + c) >> 3)];
          bf16_t w[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) w[e] = (bits >> e) & 1u ? d2bf((double)bf2f(f2bf(o[e])) * (double)drop_scale) : (bf16_t)(f2bf(o[e]) & 0x8000u);  // x * 0 keeps the sign
          *reinterpret_cast<uint4*>(out2 + row * d + c) = make_uint4(w[0] | ((uint32_t)w[1] << 16), w[2] | ((uint32_t)w[3] << 16),
                                                                      w[4] | ((uint32_t)w[5] << 16), w[6] | ((uint32_t)w[7] << 16));
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int c = lane * 8 + 512 * j;
    if (c < d) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        red[(wave * 2 + 0) * d + c + e] = ag[j][e];
        red[(wave * 2 + 1) * d + c + e] = ab[j][e];
      }
    }
  }
  __syncthreads();
  float* __restrict__ po = part + ((int64_t)i * n_slabs + slab) * 2 * d;
  for (int c = threadIdx.x; c < 2 * d; c += 256) {
    const int which = c / d, col = c - which * d;
    po[c] = ((red[(0 * 2 + which) * d + col] + red[(1 * 2 + which) * d + col]) + red[(2 * 2 + which) * d + col]) + red[(3 * 2 + which) * d + col];
  }
}
// out = LayerNorm backward of dy (+ res), G[g_off], G[b_off] = gradients of gain and bias; part: float
// [P][LN_FUSED_SLABS][2][d] (scratch).  d <= 2048.
hipError_t layernorm_bwd_with_param_grad(const bf16_t* dy, const bf16_t* x, const float* mean, const float* rstd, int P, int rows,
                                         int d, const float* W32, int64_t stride, int64_t g_off, int64_t b_off, const bf16_t* res,
                                         bf16_t* out, float* G, float* part, hipStream_t s, bf16_t* out2, const DropRecord& drop) {
  if (d % 8 || g_off % 4 || b_off % 4 || stride % 4 || d > 2048) return hipErrorInvalidValue;
  if (out2 && !drop.mask) return hipErrorInvalidValue;
  int n_slabs = (rows + 15) / 16;
  if (n_slabs > LN_FUSED_SLABS) n_slabs = LN_FUSED_SLABS;
  const int rows_per_slab = (rows + n_slabs - 1) / n_slabs;
  const size_t lds = (size_t)8 * d * sizeof(float);
  const dim3 grid(n_slabs, P);
  if (d <= 512)
    hipLaunchKernelGGL(layernorm_bwd_fused_kernel<1>, grid, dim3(256), lds, s, dy, x, mean, rstd, rows, d, rows_per_slab, W32, stride, g_off, res, out, part, out2, drop);
  else if (d <= 1024)
    hipLaunchKernelGGL(layernorm_bwd_fused_kernel<2>, grid, dim3(256), lds, s, dy, x, mean, rstd, rows, d, rows_per_slab, W32, stride, g_off, res, out, part, out2, drop);
  else
    hipLaunchKernelGGL(layernorm_bwd_fused_kernel<4>, grid, dim3(256), lds, s, dy, x, mean, rstd, rows, d, rows_per_slab, W32, stride, g_off, res, out, part, out2, drop);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(layernorm_param_combine_kernel, dim3((2 * d + 63) / 64, P), dim3(256), 0, s, part, n_slabs, d, G, stride, g_off, b_off);
  return hipGetLastError();
}

// ---- causal softmax with dropout -------------------------------------------------------------
// Rows of the [P][B][H][S][S] score array; LPR lanes share a row (64 / LPR rows per wavefront) and each
// lane owns runs of four consecutive keys, i.e. one Philox counter and 8-byte accesses.
// p = softmax over positions <= t of score * scale; writes p (kept for the backward pass) and
// p * keep (the operand of P V).
template <int LPR> __device__ __forceinline__ float group_max(float v) {
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
template <int LPR> __device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ void unpack4(uint2 x, float* v) {
  v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xffff0000u);
  v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xffff0000u);
}
__device__ __forceinline__ uint2 pack4(const float* v) {
  return make_uint2(f2bf_pair(v[0], v[1]), f2bf_pair(v[2], v[3]));
}

template <int LPR>
__global__ __launch_bounds__(256) void softmax_fwd_kernel(const bf16_t* __restrict__ sc, int64_t rows_per_member, int S, float scale,
                                                          DropArgs d, int site, bf16_t* __restrict__ pq, bf16_t* __restrict__ pd) {
  constexpr int RPW = 64 / LPR;
  const int i = blockIdx.y;
  const int lane = threadIdx.x & 63, l = lane % LPR;
  const int64_t r = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + lane / LPR;
  if (r >= rows_per_member) return;
  const int t = (int)(r % S);  // query position: attends to keys 0..t
  const int64_t base = ((int64_t)i * rows_per_member + r) * S;
  const DropRate dr = drop_rate(d.H, d.n_hyper, d.col, i, d.active);
  float mx = -INFINITY;
  for (int c = l * 4; c <= t; c += LPR * 4) {
    float v[4];
    unpack4(*reinterpret_cast<const uint2*>(sc + base + c), v);
#pragma unroll
    for (int k = 0; k < 4; ++k) if (c + k <= t) mx = fmaxf(mx, v[k] * scale);
  }
  mx = group_max<LPR>(mx);
  float se = 0.f;
  for (int c = l * 4; c <= t; c += LPR * 4) {
    float v[4];
    unpack4(*reinterpret_cast<const uint2*>(sc + base + c), v);
#pragma unroll
    for (int k = 0; k < 4; ++k) if (c + k <= t) se += expf(v[k] * scale - mx);
  }
  const float inv = 1.f / group_sum<LPR>(se);
  for (int c = l * 4; c < S; c += LPR * 4) {
    float p[4] = {0.f, 0.f, 0.f, 0.f}, f[4];
    if (c <= t) {
      float v[4];
      unpack4(*reinterpret_cast<const uint2*>(sc + base + c), v);
#pragma unroll
      for (int k = 0; k < 4; ++k) if (c + k <= t) p[k] = expf(v[k] * scale - mx) * inv;
    }
    *reinterpret_cast<uint2*>(pq + base + c) = pack4(p);
    // (beyond the diagonal p is zero whatever the keep factors are: no Philox call for those groups)
    if (c <= t) {
      drop_factors4(d, dr, i, site, (uint32_t)(((uint64_t)r * S + c) >> 2), f);
#pragma unroll
      for (int k = 0; k < 4; ++k) p[k] *= f[k];
    }
    *reinterpret_cast<uint2*>(pd + base + c) = pack4(p);
  }
}

// ds = p (dp - sum_c dp p) * scale with dp = dpd * keep; in place over dpd.  NG = groups of four keys per lane
// (S <= 4 NG LPR): the lane's part of the row (p and dp) stays in registers between the dot product and the
// result, so every keep factor is drawn once.
template <int LPR, int NG>
__global__ __launch_bounds__(256) void softmax_bwd_kernel(const bf16_t* __restrict__ pq, bf16_t* __restrict__ dpd, int64_t rows_per_member,
                                                          int S, float scale, DropArgs d, int site) {
  constexpr int RPW = 64 / LPR;
  const int i = blockIdx.y;
  const int lane = threadIdx.x & 63, l = lane % LPR;
  const int64_t r = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + lane / LPR;
  if (r >= rows_per_member) return;
  const int t = (int)(r % S);
  const int64_t base = ((int64_t)i * rows_per_member + r) * S;
  const DropRate dr = drop_rate(d.H, d.n_hyper, d.col, i, d.active);
  // p is zero beyond the diagonal, so the dot product and the non-zero results stop there
  float p[NG][4], dp[NG][4];
  float dot = 0.f;
#pragma unroll
  for (int j = 0; j < NG; ++j) {
    const int c = (l + j * LPR) * 4;
    if (c <= t) {
      float g[4], f[4];
      unpack4(*reinterpret_cast<const uint2*>(pq + base + c), p[j]);
      unpack4(*reinterpret_cast<const uint2*>(dpd + base + c), g);
      drop_factors4(d, dr, i, site, (uint32_t)(((uint64_t)r * S + c) >> 2), f);
#pragma unroll
      for (int k = 0; k < 4; ++k) { dp[j][k] = g[k] * f[k]; dot = fmaf(dp[j][k], p[j][k], dot); }
    }
  }
  dot = group_sum<LPR>(dot);
#pragma unroll
  for (int j = 0; j < NG; ++j) {
    const int c = (l + j * LPR) * 4;
    if (c < S) {
      float o[4] = {0.f, 0.f, 0.f, 0.f};
      if (c <= t) {
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = p[j][k] * (dp[j][k] - dot) * scale;
      }
      *reinterpret_cast<uint2*>(dpd + base + c) = pack4(o);
    }
  }
}

template <int LPR>
static void launch_softmax(bool fwd, const bf16_t* a, bf16_t* b, bf16_t* c, int P, int64_t rows, int S, float scale, const DropArgs& d, int site, hipStream_t s) {
  const int64_t rows_per_block = 4 * (64 / LPR);
  const dim3 grid((unsigned)((rows + rows_per_block - 1) / rows_per_block), P);
  if (fwd) hipLaunchKernelGGL(softmax_fwd_kernel<LPR>, grid, dim3(256), 0, s, a, rows, S, scale, d, site, b, c);
  else if (S <= 4 * LPR) hipLaunchKernelGGL((softmax_bwd_kernel<LPR, 1>), grid, dim3(256), 0, s, a, b, rows, S, scale, d, site);
  else if (S <= 16 * LPR) hipLaunchKernelGGL((softmax_bwd_kernel<LPR, 4>), grid, dim3(256), 0, s, a, b, rows, S, scale, d, site);
  else hipLaunchKernelGGL((softmax_bwd_kernel<LPR, 16>), grid, dim3(256), 0, s, a, b, rows, S, scale, d, site);
}
static hipError_t softmax_dispatch(bool fwd, const bf16_t* a, bf16_t* b, bf16_t* c, int P, int64_t rows, int S, float scale, const DropArgs& d, int site, hipStream_t s) {
  if (S % 4 || S > 4096) return hipErrorInvalidValue;   // (the backward kernel keeps a row in registers: at most 16 groups of four keys per lane)
  if (S <= 64) launch_softmax<16>(fwd, a, b, c, P, rows, S, scale, d, site, s);
  else if (S <= 128) launch_softmax<32>(fwd, a, b, c, P, rows, S, scale, d, site, s);
  else launch_softmax<64>(fwd, a, b, c, P, rows, S, scale, d, site, s);
  return hipGetLastError();
}
hipError_t softmax_fwd(const bf16_t* sc, int P, int64_t rows, int S, float scale, const DropArgs& d, int site, bf16_t* pq,
                       bf16_t* pd, hipStream_t s) {
  return softmax_dispatch(true, sc, pq, pd, P, rows, S, scale, d, site, s);
}
hipError_t softmax_bwd(const bf16_t* pq, bf16_t* dpd, int P, int64_t rows, int S, float scale, const DropArgs& d, int site,
                       hipStream_t s) {
  return softmax_dispatch(false, pq, dpd, nullptr, P, rows, S, scale, d, site, s);
}

// ---- dropout / residual ----------------------------------------------------------------------
// out = x * keep (+ res when res != null).  A thread takes DROP_GROUPS consecutive groups of four
// elements (one Philox call each): 32-byte runs per thread and a quarter of the wavefronts that one
// group per thread would launch (at one group the launch rate of wavefronts, not memory, set the time).
constexpr int DROP_GROUPS = 4;
__device__ __forceinline__ void dropout_group(uint2 xv, bool has_res, uint2 rv, const float* f, uint2* out) {
  // bf16 x float products are exact in double
  double v[4] = {(double)__uint_as_float(xv.x << 16) * (double)f[0], (double)__uint_as_float(xv.x & 0xffff0000u) * (double)f[1],
                 (double)__uint_as_float(xv.y << 16) * (double)f[2], (double)__uint_as_float(xv.y & 0xffff0000u) * (double)f[3]};
  if (has_res) {
    v[0] = (double)__uint_as_float(rv.x << 16) + v[0]; v[1] = (double)__uint_as_float(rv.x & 0xffff0000u) + v[1];
    v[2] = (double)__uint_as_float(rv.y << 16) + v[2]; v[3] = (double)__uint_as_float(rv.y & 0xffff0000u) + v[3];
  }
  out->x = d2bf(v[0]) | ((uint32_t)d2bf(v[1]) << 16);
  out->y = d2bf(v[2]) | ((uint32_t)d2bf(v[3]) << 16);
}
__device__ __forceinline__ void bits_to_factors(uint32_t bits, float scale, float* f) {
#pragma unroll
  for (int k = 0; k < 4; ++k) f[k] = (bits >> k) & 1u ? scale : 0.f;
}
// mask_out (may be null): the forward pass records the keep bits, one 16-bit word per thread (four groups);
// mask_in (may be null): the backward pass of the same site and step reads them instead of repeating the
// Philox calls, whose 32-bit multiplies, not memory, bound this kernel.
__global__ __launch_bounds__(256) void dropout_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ res,
                                                      int64_t per_member, DropArgs d, int site, bf16_t* __restrict__ out,
                                                      const uint16_t* __restrict__ mask_in, uint16_t* __restrict__ mask_out) {
  const int i = blockIdx.y;
  const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t first = tid * DROP_GROUPS;   // first group of this thread
  const int64_t groups = per_member / 4;
  if (first >= groups) return;
  const DropRate dr = drop_rate(d.H, d.n_hyper, d.col, i, d.active);
  const int64_t o = (int64_t)i * per_member + first * 4;
  const int64_t words = (groups + DROP_GROUPS - 1) / DROP_GROUPS;   // mask words per member
  uint32_t word = mask_in ? mask_in[(int64_t)i * words + tid] : 0u, made = 0u;
  auto group_bits = [&](int g) {
    const uint32_t bits = mask_in ? (word >> (4 * g)) & 15u : drop_bits4(d, dr, i, site, (uint32_t)(first + g));
    made |= bits << (4 * g);
    return bits;
  };
  if (first + DROP_GROUPS <= groups && ((reinterpret_cast<uintptr_t>(x + o) | reinterpret_cast<uintptr_t>(out + o) |
                                         (res ? reinterpret_cast<uintptr_t>(res + o) : 0)) & 15) == 0) {
    uint4 xv[DROP_GROUPS / 2], rv[DROP_GROUPS / 2], ov[DROP_GROUPS / 2];
#pragma unroll
    for (int h = 0; h < DROP_GROUPS / 2; ++h) {
      xv[h] = *reinterpret_cast<const uint4*>(x + o + 8 * h);
      rv[h] = res ? *reinterpret_cast<const uint4*>(res + o + 8 * h) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int h = 0; h < DROP_GROUPS / 2; ++h) {
      float f[4];
      uint2 lo, hi;
      bits_to_factors(group_bits(2 * h), dr.scale, f);
      dropout_group(make_uint2(xv[h].x, xv[h].y), res != nullptr, make_uint2(rv[h].x, rv[h].y), f, &lo);
      bits_to_factors(group_bits(2 * h + 1), dr.scale, f);
      dropout_group(make_uint2(xv[h].z, xv[h].w), res != nullptr, make_uint2(rv[h].z, rv[h].w), f, &hi);
      ov[h] = make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
#pragma unroll
    for (int h = 0; h < DROP_GROUPS / 2; ++h) *reinterpret_cast<uint4*>(out + o + 8 * h) = ov[h];
  } else {
    for (int g = 0; g < DROP_GROUPS && first + g < groups; ++g) {
      float f[4];
      uint2 pk;
      bits_to_factors(group_bits(g), dr.scale, f);
      const uint2 rv = res ? *reinterpret_cast<const uint2*>(res + o + 4 * g) : make_uint2(0, 0);
      dropout_group(*reinterpret_cast<const uint2*>(x + o + 4 * g), res != nullptr, rv, f, &pk);
      *reinterpret_cast<uint2*>(out + o + 4 * g) = pk;
    }
  }
  if (mask_out) mask_out[(int64_t)i * words + tid] = (uint16_t)made;
}
size_t dropout_mask_bytes(int P, int64_t per_member) {
  const int64_t groups = per_member / 4;
  return (size_t)P * (size_t)((groups + DROP_GROUPS - 1) / DROP_GROUPS) * sizeof(uint16_t);
}
hipError_t dropout_apply(const bf16_t* x, const bf16_t* res, int P, int64_t per_member, const DropArgs& d, int site, bf16_t* out,
                         hipStream_t s, const uint16_t* mask_in, uint16_t* mask_out) {
  if (per_member % 4) return hipErrorInvalidValue;
  const int64_t threads = (per_member / 4 + DROP_GROUPS - 1) / DROP_GROUPS;
  hipLaunchKernelGGL(dropout_kernel, dim3((unsigned)((threads + 255) / 256), P), dim3(256), 0, s, x, res, per_member, d, site, out,
                     mask_in, mask_out);
  return hipGetLastError();
}

// h = res + x * keep (one rounding, as dropout_kernel) followed by the LayerNorm of h, in one pass: a wavefront
// per row, a lane owns the same 8 J columns (J = ceil(d / 512)); h is written for the residual stream and the
// backward pass, the keep bits go to the site's record (bit e % 8 of byte e / 8 of the member's array), and the
// normalised row is formed from the rounded h while it is still in registers, so h is not read back.
template <int J>
__global__ __launch_bounds__(256) void residual_dropout_layernorm_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ res,
                                                                         int rows_per_member, int d, DropArgs dr, int site,
                                                                         bf16_t* __restrict__ h, uint8_t* __restrict__ record, int64_t record_stride,
                                                                         const float* __restrict__ W32, int64_t stride, int64_t g_off, int64_t b_off,
                                                                         bf16_t* __restrict__ y, float* __restrict__ mean, float* __restrict__ rstd) {
  const int i = blockIdx.y;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (r >= rows_per_member) return;
  const int64_t row = (int64_t)i * rows_per_member + r;
  const DropRate rate = drop_rate(dr.H, dr.n_hyper, dr.col, i, dr.active);
  float v[J][8];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int c = lane * 8 + 512 * j;
    if (c < d) {
      const int64_t e = (int64_t)r * d + c;   // element index inside the member's array
      const uint4 xv = *reinterpret_cast<const uint4*>(x + row * d + c), rv = *reinterpret_cast<const uint4*>(res + row * d + c);
      const uint32_t b0 = drop_bits4(dr, rate, i, site, (uint32_t)(e >> 2)), b1 = drop_bits4(dr, rate, i, site, (uint32_t)(e >> 2) + 1u);
      float f[4];
      uint2 lo, hi;
      bits_to_factors(b0, rate.scale, f);
      dropout_group(make_uint2(xv.x, xv.y), true, make_uint2(rv.x, rv.y), f, &lo);
      bits_to_factors(b1, rate.scale, f);
      dropout_group(make_uint2(xv.z, xv.w), true, make_uint2(rv.z, rv.w), f, &hi);
      const uint4 hv = make_uint4(lo.x, lo.y, hi.x, hi.y);
      *reinterpret_cast<uint4*>(h + row * d + c) = hv;
      if (record) record[(int64_t)i * record_stride + (e >> 3)] = (uint8_t)(b0 | (b1 << 4));
      const uint32_t w[4] = {hv.x, hv.y, hv.z, hv.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) { v[j][2 * q] = __uint_as_float(w[q] << 16); v[j][2 * q + 1] = __uint_as_float(w[q] & 0xffff0000u); }
#pragma unroll
      for (int k = 0; k < 8; ++k) s += v[j][k];
    }
  }
  const float mu = wave_sum(s) / (float)d;
  float var = 0.f;
#pragma unroll
  for (int j = 0; j < J; ++j)
    if (lane * 8 + 512 * j < d) {
#pragma unroll
      for (int k = 0; k < 8; ++k) { const float t = v[j][k] - mu; var = fmaf(t, t, var); }
    }
  const float rs = rsqrtf(wave_sum(var) / (float)d + LN_EPS);
  const float* __restrict__ g = W32 + (int64_t)i * stride + g_off;
  const float* __restrict__ b = W32 + (int64_t)i * stride + b_off;
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int c = lane * 8 + 512 * j;
    if (c < d) {
      float gv[8], bv[8], o[8];
      load8(g + c, gv);
      load8(b + c, bv);
#pragma unroll
      for (int k = 0; k < 8; ++k) o[k] = (v[j][k] - mu) * rs * gv[k] + bv[k];
      store8(y + row * d + c, o);
    }
  }
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
}
hipError_t residual_dropout_layernorm(const bf16_t* x, const bf16_t* res, int P, int rows, int d, const DropArgs& dr, int site, bf16_t* h,
                                      uint16_t* record, const float* W32, int64_t stride, int64_t g_off, int64_t b_off, bf16_t* y, float* mean,
                                      float* rstd, hipStream_t s) {
  // (the record is the bit array dropout_kernel writes, which has no padding between members when their size is a multiple of 16)
  if (d % 8 || ((int64_t)rows * d) % 16 || g_off % 4 || b_off % 4 || stride % 4 || d > 2048) return hipErrorInvalidValue;
  const dim3 grid((rows + 3) / 4, P);
  uint8_t* rec = reinterpret_cast<uint8_t*>(record);
  const int64_t rstride = (int64_t)rows * d / 8;
#define PBT_RDL(J) hipLaunchKernelGGL(residual_dropout_layernorm_kernel<J>, grid, dim3(256), 0, s, x, res, rows, d, dr, site, h, rec, rstride, W32, stride, g_off, b_off, y, mean, rstd)
  if (d <= 512) PBT_RDL(1);
  else if (d <= 1024) PBT_RDL(2);
  else PBT_RDL(4);
#undef PBT_RDL
  return hipGetLastError();
}

// ---- weight gradients formed in several parts of the contraction -------------------------------------------
// G[i][w_off + e] = sum over parts q (in order) of part[(i * n_parts + q)][e], e < count (a multiple of 4), and
// likewise the bias gradient from the parts' column sums: the second half of a weight-gradient product whose
// contraction was cut into n_parts pieces so that a small matrix still gives every compute unit a tile.
__global__ __launch_bounds__(256) void wgrad_combine_kernel(const float* __restrict__ part, const float* __restrict__ colpart, int n_parts,
                                                            int64_t count, int N, float* __restrict__ G, int64_t stride, int64_t w_off, int64_t b_off) {
  const int i = blockIdx.y;
  const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (e < count) {
    float4 a = *reinterpret_cast<const float4*>(part + (int64_t)i * n_parts * count + e);
    for (int q = 1; q < n_parts; ++q) {
      const float4 b = *reinterpret_cast<const float4*>(part + ((int64_t)i * n_parts + q) * count + e);
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    *reinterpret_cast<float4*>(G + (int64_t)i * stride + w_off + e) = a;
  }
  if (e < N) {   // (N is a multiple of 4 too)
    float4 a = *reinterpret_cast<const float4*>(colpart + (int64_t)i * n_parts * N + e);
    for (int q = 1; q < n_parts; ++q) {
      const float4 b = *reinterpret_cast<const float4*>(colpart + ((int64_t)i * n_parts + q) * N + e);
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    *reinterpret_cast<float4*>(G + (int64_t)i * stride + b_off + e) = a;
  }
}
hipError_t wgrad_combine(const float* part, const float* colpart, int n_parts, int P, int64_t count, int N, float* G, int64_t stride,
                         int64_t w_off, int64_t b_off, hipStream_t s) {
  if (count % 4 || N % 4 || w_off % 4 || b_off % 4 || stride % 4 || n_parts < 1 || N > count) return hipErrorInvalidValue;
  hipLaunchKernelGGL(wgrad_combine_kernel, dim3((unsigned)((count / 4 + 255) / 256), P), dim3(256), 0, s, part, colpart, n_parts, count, N, G, stride, w_off, b_off);
  return hipGetLastError();
}

// ---- label-smoothed cross-entropy over the vocabulary -----------------------------------------
// One workgroup per row of float logits[rows][V].  loss = lse - (1-e) l_y - (e/V) sum l;
// dlogits = (softmax - ((1-e) onehot + e/V)) * gscale as bf16 (when dlogits != null).
__global__ __launch_bounds__(256) void xent_kernel(const float* __restrict__ logits, const int32_t* __restrict__ targets, int rows_per_member,
                                                   int V, const float* __restrict__ H, int n_hyper, int col_ls, int use_ls, float gscale,
                                                   bf16_t* __restrict__ dlogits, float* __restrict__ rowloss) {
  __shared__ float red[4];
  const int i = blockIdx.y;
  const int64_t row = (int64_t)i * rows_per_member + blockIdx.x;
  const float* __restrict__ l = logits + row * V;
  const float eps = (use_ls && col_ls >= 0) ? H[(int64_t)i * n_hyper + col_ls] : 0.f;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float mx = -INFINITY;
  for (int c = threadIdx.x; c < V; c += 256) mx = fmaxf(mx, l[c]);
  mx = wave_max(mx);
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float se = 0.f, sl = 0.f;
  for (int c = threadIdx.x; c < V; c += 256) { se += expf(l[c] - mx); sl += l[c]; }
  se = wave_sum(se);
  if (lane == 0) red[wave] = se;
  __syncthreads();
  se = ((red[0] + red[1]) + red[2]) + red[3];
  __syncthreads();
  sl = wave_sum(sl);
  if (lane == 0) red[wave] = sl;
  __syncthreads();
  sl = ((red[0] + red[1]) + red[2]) + red[3];
  const float lse = mx + logf(se);
  const int y = targets[row];
  if (threadIdx.x == 0) rowloss[row] = lse - (1.f - eps) * l[y] - eps * (sl / (float)V);
  if (dlogits) {
    const float inv = 1.f / se, u = eps / (float)V;
    bf16_t* __restrict__ dl = dlogits + row * V;
    for (int c = threadIdx.x; c < V; c += 256)
      dl[c] = f2bf((expf(l[c] - mx) * inv - u - (c == y ? 1.f - eps : 0.f)) * gscale);
  }
}
// The same with the whole row held in registers (V <= 2048 G, V a multiple of 8): every thread owns G
// runs of 8 consecutive logits, so the row is read once with 16-byte loads and the gradient leaves in
// 16-byte stores.
template <int G>
__global__ __launch_bounds__(256) void xent_rowreg_kernel(const float* __restrict__ logits, const int32_t* __restrict__ targets, int rows_per_member,
                                                          int V, const float* __restrict__ H, int n_hyper, int col_ls, int use_ls, float gscale,
                                                          bf16_t* __restrict__ dlogits, float* __restrict__ rowloss) {
  __shared__ float red[4];
  const int i = blockIdx.y;
  const int64_t row = (int64_t)i * rows_per_member + blockIdx.x;
  const float* __restrict__ l = logits + row * V;
  const float eps = (use_ls && col_ls >= 0) ? H[(int64_t)i * n_hyper + col_ls] : 0.f;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float v[G][8];
  float mx = -INFINITY, sl = 0.f;
#pragma unroll
  for (int j = 0; j < G; ++j) {
    const int c0 = (j * 256 + threadIdx.x) * 8;
    if (c0 < V) {
      const float4 a = *reinterpret_cast<const float4*>(l + c0), b = *reinterpret_cast<const float4*>(l + c0 + 4);
      v[j][0] = a.x; v[j][1] = a.y; v[j][2] = a.z; v[j][3] = a.w; v[j][4] = b.x; v[j][5] = b.y; v[j][6] = b.z; v[j][7] = b.w;
#pragma unroll
      for (int k = 0; k < 8; ++k) { mx = fmaxf(mx, v[j][k]); sl += v[j][k]; }
    }
  }
  mx = wave_max(mx);
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float se = 0.f;
#pragma unroll
  for (int j = 0; j < G; ++j) {
    if ((j * 256 + threadIdx.x) * 8 < V) {
#pragma unroll
      for (int k = 0; k < 8; ++k) { v[j][k] = expf(v[j][k] - mx); se += v[j][k]; }
    }
  }
  se = wave_sum(se);
  if (lane == 0) red[wave] = se;
  __syncthreads();
  se = ((red[0] + red[1]) + red[2]) + red[3];
  __syncthreads();
  sl = wave_sum(sl);
  if (lane == 0) red[wave] = sl;
  __syncthreads();
  sl = ((red[0] + red[1]) + red[2]) + red[3];
  const int y = targets[row];
  if (threadIdx.x == 0) rowloss[row] = mx + logf(se) - (1.f - eps) * l[y] - eps * (sl / (float)V);
  if (dlogits) {
    const float inv = 1.f / se, u = eps / (float)V;
    bf16_t* __restrict__ dl = dlogits + row * V;
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int c0 = (j * 256 + threadIdx.x) * 8;
      if (c0 < V) {
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 8; k += 2) {
          const float g0 = (v[j][k] * inv - u - (c0 + k == y ? 1.f - eps : 0.f)) * gscale;
          const float g1 = (v[j][k + 1] * inv - u - (c0 + k + 1 == y ? 1.f - eps : 0.f)) * gscale;
          w[k / 2] = f2bf_pair(g0, g1);
        }
        *reinterpret_cast<uint4*>(dl + c0) = make_uint4(w[0], w[1], w[2], w[3]);
      }
    }
  }
}

hipError_t xent_rows(const float* logits, const int32_t* targets, int P, int rows, int V, const float* H, int n_hyper, int col_ls,
                     int use_ls, float gscale, bf16_t* dlogits, float* rowloss, hipStream_t s) {
  const dim3 grid(rows, P), block(256);
  if (V % 8 == 0 && V <= 2048)
    hipLaunchKernelGGL(xent_rowreg_kernel<1>, grid, block, 0, s, logits, targets, rows, V, H, n_hyper, col_ls, use_ls, gscale, dlogits, rowloss);
  else if (V % 8 == 0 && V <= 4096)
    hipLaunchKernelGGL(xent_rowreg_kernel<2>, grid, block, 0, s, logits, targets, rows, V, H, n_hyper, col_ls, use_ls, gscale, dlogits, rowloss);
  else if (V % 8 == 0 && V <= 8192)
    hipLaunchKernelGGL(xent_rowreg_kernel<4>, grid, block, 0, s, logits, targets, rows, V, H, n_hyper, col_ls, use_ls, gscale, dlogits, rowloss);
  else
    hipLaunchKernelGGL(xent_kernel, grid, block, 0, s, logits, targets, rows, V, H, n_hyper, col_ls, use_ls, gscale, dlogits, rowloss);
  return hipGetLastError();
}

// dst[i][offset + r] = src[i][r]: collects the per-row losses of one eval chunk
__global__ void scatter_rows_kernel(const float* __restrict__ src, int rows, float* __restrict__ dst, int64_t dst_stride, int64_t offset) {
  const int i = blockIdx.y;
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < rows) dst[(int64_t)i * dst_stride + offset + r] = src[(int64_t)i * rows + r];
}
hipError_t tf_scatter_rows(const float* src, int P, int rows, float* dst, int64_t dst_stride, int64_t offset, hipStream_t s) {
  hipLaunchKernelGGL(scatter_rows_kernel, dim3((rows + 255) / 256, P), dim3(256), 0, s, src, rows, dst, dst_stride, offset);
  return hipGetLastError();
}

// score[i] = -exp(mean of rowloss[i][:])   (perplexity, negated), one wavefront per member
__global__ __launch_bounds__(64) void perplexity_kernel(const float* __restrict__ rowloss, int rows, float* __restrict__ score) {
  const int i = blockIdx.x;
  float acc = 0.f;
  for (int r = threadIdx.x; r < rows; r += 64) acc += rowloss[(int64_t)i * rows + r];
  acc = wave_sum(acc);
  if (threadIdx.x == 0) score[i] = -expf(acc / (float)rows);
}
hipError_t perplexity_score(const float* rowloss, int P, int rows, float* score, hipStream_t s) {
  hipLaunchKernelGGL(perplexity_kernel, dim3(P), dim3(64), 0, s, rowloss, rows, score);
  return hipGetLastError();
}

}  // namespace pbt
