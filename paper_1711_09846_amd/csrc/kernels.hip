// Memory-bound and small kernels of the population step: mini-batch fetch, output layer with
// softmax cross-entropy, bias gradients, per-member reductions, the fused per-member optimiser
// and the on-device exploit/explore pass (rank, truncation selection, gather-copy, perturb).
#include "common.h"
#include "internal.h"
#include "optim_math.h"
#include "philox.h"

namespace pbt {

// ---- fills and conversions -------------------------------------------------------------------

__global__ void fill_u32_kernel(uint32_t* p, uint32_t v, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}
hipError_t fill_u32(uint32_t* p, uint32_t v, int64_t n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const int blocks = (int)((n + 1023) / 1024 > 8192 ? 8192 : (n + 1023) / 1024);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks), dim3(256), 0, s, p, v, n);
  return hipGetLastError();
}

__global__ void iota_i32_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = i;
}
hipError_t iota_i32(int32_t* p, int n, hipStream_t s) {
  hipLaunchKernelGGL(iota_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p, n);
  return hipGetLastError();
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = f2bf(src[i]);
}
hipError_t f32_to_bf16(const float* src, bf16_t* dst, int64_t n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const int blocks = (int)((n + 1023) / 1024 > 16384 ? 16384 : (n + 1023) / 1024);
  hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(blocks), dim3(256), 0, s, src, dst, n);
  return hipGetLastError();
}

// ---- initial population ----------------------------------------------------------------------
// grid (chunks, parameter arrays, P): one thread per element of one parameter array.  The value at
// position p of the member's flat vector depends on p alone (word p % 4 of Philox counter
// (0, member, DOMAIN_INIT_W, p / 4)), not on how the grid is cut.
__global__ __launch_bounds__(256) void init_population_kernel(InitArgs a) {
  const int i = blockIdx.z, seg = blockIdx.y;
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const uint32_t k0 = (uint32_t)a.seed, k1 = (uint32_t)(a.seed >> 32);
  if (e < a.seg_len[seg]) {
    const int64_t p = a.seg_off[seg] + e;
    float v = a.seg_const[seg];
    if (a.seg_fan[seg] > 0) {
      const u32x4 w = philox4x32_10(0u, (uint32_t)i, DOMAIN_INIT_W, (uint32_t)(p >> 2), k0, k1);
      const uint32_t x = (p & 3) == 0 ? w.x : (p & 3) == 1 ? w.y : (p & 3) == 2 ? w.z : w.w;
      v = (float)((2.0 * philox_unit(x) - 1.0) / sqrt((double)a.seg_fan[seg]));
    }
    a.W32[(int64_t)i * a.stride + p] = v;
    if (a.W16) a.W16[(int64_t)i * a.stride + p] = f2bf(v);
  }
  if (blockIdx.x == 0 && seg == 0 && threadIdx.x < a.n_hyper) {
    const int k = threadIdx.x;
    const double u = philox_unit(philox4x32_10(0u, (uint32_t)i, DOMAIN_INIT_H, (uint32_t)k, k0, k1).x);
    const double lin = a.prior_a[k] + u * (a.prior_b[k] - a.prior_a[k]);
    a.H[i * a.n_hyper + k] = (float)(a.prior_kind[k] == 1 ? exp(lin) : lin);
  }
}
hipError_t init_population(const InitArgs& a, hipStream_t s) {
  int64_t longest = 1;
  for (int k = 0; k < a.n_seg; ++k) longest = a.seg_len[k] > longest ? a.seg_len[k] : longest;
  hipLaunchKernelGGL(init_population_kernel, dim3((unsigned)((longest + 255) / 256), a.n_seg, a.P), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ---- mini-batch fetch ------------------------------------------------------------------------
// grid (B, P); one workgroup copies one data row.

__global__ __launch_bounds__(64) void gather_batch_kernel(const float* __restrict__ train_x,
                                                          const int32_t* __restrict__ train_y, int n_train, int d, int B,
                                                          uint32_t step, uint32_t k0, uint32_t k1,
                                                          bf16_t* __restrict__ X16, float* __restrict__ X32,
                                                          int32_t* __restrict__ Y, int32_t* __restrict__ t) {
  const int r = blockIdx.x, i = blockIdx.y;
  const uint32_t x = philox4x32_10(step, (uint32_t)i, DOMAIN_BATCH, (uint32_t)r, k0, k1).x;
  const int64_t src = (int64_t)philox_bounded(x, (uint32_t)n_train);
  const int64_t dst = ((int64_t)i * B + r) * d;
  const float* __restrict__ row = train_x + src * d;
  if (X16) {
    for (int c = threadIdx.x; c < d; c += 64) X16[dst + c] = f2bf(row[c]);
  } else {
    for (int c = threadIdx.x; c < d; c += 64) X32[dst + c] = row[c];
  }
  if (threadIdx.x == 0) {
    Y[(int64_t)i * B + r] = train_y[src];
    if (r == 0) t[i] += 1;
  }
}
hipError_t gather_batch(const float* train_x, const int32_t* train_y, int n_train, int d, int P, int B, uint32_t step,
                        uint64_t seed, bf16_t* X16, float* X32, int32_t* Y, int32_t* t, hipStream_t s) {
  hipLaunchKernelGGL(gather_batch_kernel, dim3(B, P), dim3(64), 0, s, train_x, train_y, n_train, d, B, step,
                     (uint32_t)seed, (uint32_t)(seed >> 32), X16, X32, Y, t);
  return hipGetLastError();
}

// Per-member reduction of per-row values with wavefront shuffles: lane l adds rows l, l+64, ...
// in order, then a butterfly over the 64 lanes.
__global__ __launch_bounds__(64) void row_reduce_kernel(const float* __restrict__ rowval, int64_t srow, int rows,
                                                        float scale, float* __restrict__ out, int out_stride) {
  const int i = blockIdx.x;
  const float* __restrict__ p = rowval + (int64_t)i * srow;
  float acc = 0.f;
  for (int r = threadIdx.x; r < rows; r += 64) acc += p[r];
  acc = wave_sum(acc);
  if (threadIdx.x == 0) out[(int64_t)i * out_stride] = acc * scale;
}
hipError_t row_reduce(const float* rowval, int64_t srow, int P, int rows, float scale, float* out, int out_stride,
                      hipStream_t s) {
  hipLaunchKernelGGL(row_reduce_kernel, dim3(P), dim3(64), 0, s, rowval, srow, rows, scale, out, out_stride);
  return hipGetLastError();
}

// ---- fused per-member optimiser --------------------------------------------------------------
// Streams a range of every member's parameters once: reads theta, gradient and state, writes theta,
// state and the bf16 shadow (update rules in optim_math.h).  One float4 per thread per array (two or four per
// thread, all loads issued first, were slower on every workload: 397 -> 416 -> 431 us on the wide MLP's separate
// pass, 1820 -> 1876 / 1855 us on the transformer).
constexpr int OPT_VEC_PER_THREAD = 1;

template <int OPT>
__global__ __launch_bounds__(256) void optimizer_kernel(OptArgs a) {
  const int i = blockIdx.y;
  const OptHyper hy{a.H, a.t, a.n_hyper, a.col_lr, a.col_beta1, a.col_wd, a.c0, a.c1, a.c2, a.c3, a.t_mul, a.t_add};
  const OptScalars sc = opt_scalars<OPT>(hy, i);
#pragma unroll
  for (int u = 0; u < OPT_VEC_PER_THREAD; ++u) {
    // vector index over the concatenation of the ranges
    int64_t v = ((int64_t)blockIdx.x * OPT_VEC_PER_THREAD + u) * 256 + threadIdx.x;
    int64_t begin = a.begin, nvec = a.count / 4;
    for (int x = 0; x < a.n_extra && v >= nvec; ++x) {
      v -= nvec;
      begin = a.xbegin[x];
      nvec = a.xcount[x] / 4;
    }
    if (v >= nvec) break;
    const int64_t o = (int64_t)i * a.stride + begin + v * 4;
    float4 w = stream_load(a.W32 + o);
    const float4 g = stream_load(a.G + o);
    float4 s0 = stream_load(a.S0 + o);
    float4 s1 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (OPT == OPT_ADAM) s1 = stream_load(a.S1 + o);
    float* wp = reinterpret_cast<float*>(&w);
    const float* gp = reinterpret_cast<const float*>(&g);
    float* s0p = reinterpret_cast<float*>(&s0);
    float* s1p = reinterpret_cast<float*>(&s1);
#pragma unroll
    for (int e = 0; e < 4; ++e) opt_update<OPT>(wp[e], gp[e], s0p[e], s1p[e], sc, hy);
    stream_store(w, a.W32 + o);
    stream_store(s0, a.S0 + o);
    if (OPT == OPT_ADAM) stream_store(s1, a.S1 + o);
    if (a.W16) {
      uint2 pk;
      pk.x = f2bf_pair(wp[0], wp[1]);
      pk.y = f2bf_pair(wp[2], wp[3]);
      *reinterpret_cast<uint2*>(a.W16 + o) = pk;
    }
  }
}
hipError_t optimizer_step(const OptArgs& a, hipStream_t s) {
  if (a.begin % 4 || a.count % 4 || a.count <= 0 || a.begin + a.count > a.stride) return hipErrorInvalidValue;
  if (a.n_extra < 0 || a.n_extra > OPT_MAX_RANGES - 1) return hipErrorInvalidValue;
  int64_t nvec = a.count / 4;
  for (int x = 0; x < a.n_extra; ++x) {
    if (a.xbegin[x] % 4 || a.xcount[x] % 4 || a.xcount[x] <= 0 || a.xbegin[x] + a.xcount[x] > a.stride) return hipErrorInvalidValue;
    nvec += a.xcount[x] / 4;
  }
  const int per_block = 256 * OPT_VEC_PER_THREAD;
  dim3 grid((unsigned)((nvec + per_block - 1) / per_block), a.P);
  if (a.optimizer == 0)
    hipLaunchKernelGGL(optimizer_kernel<0>, grid, dim3(256), 0, s, a);
  else if (a.optimizer == 1)
    hipLaunchKernelGGL(optimizer_kernel<1>, grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(optimizer_kernel<2>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

// ---- GAN workload: latents, real-row gather, squared norms, MMD combination -------------------

__global__ __launch_bounds__(256) void latent_normal_kernel(bf16_t* __restrict__ out, int64_t per_member, uint32_t c0,
                                                            uint32_t domain, uint32_t k0, uint32_t k1) {
  const int i = blockIdx.y;
  const int64_t blk = (int64_t)blockIdx.x * 256 + threadIdx.x;  // block of 4 elements
  if (blk * 4 >= per_member) return;
  const u32x4 w = philox4x32_10(c0, (uint32_t)i, domain, (uint32_t)blk, k0, k1);
  const double r1 = sqrt(-2.0 * log(philox_unit(w.x))), a1 = 6.283185307179586476925 * philox_unit(w.y);
  const double r2 = sqrt(-2.0 * log(philox_unit(w.z))), a2 = 6.283185307179586476925 * philox_unit(w.w);
  const double v[4] = {r1 * cos(a1), r1 * sin(a1), r2 * cos(a2), r2 * sin(a2)};
  bf16_t* __restrict__ o = out + (int64_t)i * per_member + blk * 4;
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (blk * 4 + e < per_member) o[e] = f2bf((float)v[e]);
}
hipError_t latent_normal(bf16_t* out, int P, int rows, int d, uint32_t c0, int substream, uint64_t seed, hipStream_t s) {
  const int64_t per_member = (int64_t)rows * d;
  const int64_t blocks4 = (per_member + 3) / 4;
  hipLaunchKernelGGL(latent_normal_kernel, dim3((unsigned)((blocks4 + 255) / 256), P), dim3(256), 0, s, out, per_member, c0,
                     (uint32_t)(DOMAIN_LATENT + substream), (uint32_t)seed, (uint32_t)(seed >> 32));
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void gather_rows_kernel(const float* __restrict__ train_x, int n_train, int d,
                                                          int64_t member_stride, uint32_t step, uint32_t k0, uint32_t k1,
                                                          bf16_t* __restrict__ X16, int32_t* __restrict__ t, uint32_t counter0) {
  const int r = blockIdx.x, i = blockIdx.y;
  const uint32_t x = philox4x32_10(step, (uint32_t)i, DOMAIN_BATCH, counter0 + (uint32_t)r, k0, k1).x;
  const float* __restrict__ row = train_x + (int64_t)philox_bounded(x, (uint32_t)n_train) * d;
  bf16_t* __restrict__ o = X16 + (int64_t)i * member_stride + (int64_t)r * d;
  if ((d & 3) == 0) {  // rows are 16-byte aligned: four floats in, four bf16 out per access
    for (int c = threadIdx.x * 4; c < d; c += 1024) {
      const float4 v = *reinterpret_cast<const float4*>(row + c);
      uint2 pk;
      pk.x = f2bf_pair(v.x, v.y);
      pk.y = f2bf_pair(v.z, v.w);
      *reinterpret_cast<uint2*>(o + c) = pk;
    }
  } else {
    for (int c = threadIdx.x; c < d; c += 256) o[c] = f2bf(row[c]);
  }
  if (t != nullptr && threadIdx.x == 0 && r == 0) t[i] += 1;
}
hipError_t gather_rows(const float* train_x, int n_train, int d, int P, int B, int64_t member_stride, uint32_t step,
                       uint64_t seed, bf16_t* X16, int32_t* t, hipStream_t s, uint32_t counter0, bool bump_t) {
  if ((d & 3) == 0 && (member_stride & 3)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gather_rows_kernel, dim3(B, P), dim3(256), 0, s, train_x, n_train, d, member_stride, step,
                     (uint32_t)seed, (uint32_t)(seed >> 32), X16, bump_t ? t : nullptr, counter0);
  return hipGetLastError();
}

// one wavefront per row: lanes stride over the row, butterfly sum
__global__ __launch_bounds__(256) void row_sqnorm_kernel(const bf16_t* __restrict__ X, int64_t n_rows, int d,
                                                         float* __restrict__ out) {
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= n_rows) return;
  const bf16_t* __restrict__ p = X + r * d;
  float acc = 0.f;
  for (int c = threadIdx.x & 63; c < d; c += 64) {
    const float v = bf2f(p[c]);
    acc = fmaf(v, v, acc);
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) out[r] = acc;
}
hipError_t row_sqnorm(const bf16_t* X, int batch, int rows, int d, float* out, hipStream_t s) {
  const int64_t n_rows = (int64_t)batch * rows;
  hipLaunchKernelGGL(row_sqnorm_kernel, dim3((unsigned)((n_rows + 3) / 4)), dim3(256), 0, s, X, n_rows, d, out);
  return hipGetLastError();
}

// one wavefront per member; tiles added in a fixed order (lane-strided, then butterfly)
__global__ __launch_bounds__(64) void mmd_combine_kernel(const float* __restrict__ pxx, int txx,
                                                         const float* __restrict__ pyy, int tyy,
                                                         const float* __restrict__ pxy, int txy, float inv_n2,
                                                         float* __restrict__ score) {
  const int i = blockIdx.x;
  float sxx = 0.f, syy = 0.f, sxy = 0.f;
  for (int k = threadIdx.x; k < txx; k += 64) sxx += pxx[(int64_t)i * txx + k];
  for (int k = threadIdx.x; k < tyy; k += 64) syy += pyy[k];
  for (int k = threadIdx.x; k < txy; k += 64) sxy += pxy[(int64_t)i * txy + k];
  sxx = wave_sum(sxx);
  syy = wave_sum(syy);
  sxy = wave_sum(sxy);
  if (threadIdx.x == 0) score[i] = -((sxx * inv_n2 + syy * inv_n2) - 2.f * (sxy * inv_n2));
}
hipError_t mmd_combine(const float* pxx, int txx, const float* pyy, int tyy, const float* pxy, int txy, int P, float inv_n2,
                       float* score, hipStream_t s) {
  hipLaunchKernelGGL(mmd_combine_kernel, dim3(P), dim3(64), 0, s, pxx, txx, pyy, tyy, pxy, txy, inv_n2, score);
  return hipGetLastError();
}

// ---- exploit / explore -----------------------------------------------------------------------
// One workgroup ranks the population by counting: member i's position is the number of members
// that rank above it under the total order (score descending; equal scores: lower index first;
// -inf below every finite score; NaN below -inf).  The bottom n_trunc members then pick a donor
// from the top n_trunc with one Philox word each and perturb the donor's hyperparameters.

__device__ __forceinline__ bool ranks_above(float sj, int j, float si, int i) {
  const bool nj = sj != sj, ni = si != si;
  if (nj != ni) return ni;
  if (!nj && sj != si) return sj > si;
  return j < i;
}

// ---- Welch's t-test (Section 4.1.1, Exploit (a)) in double -----------------------------------
// Continued fraction of the incomplete beta function, evaluated with the modified Lentz scheme.
__device__ double beta_cf(double a, double b, double x) {
  const double tiny = 1e-300;
  double c = 1.0, d = 1.0 - (a + b) * x / (a + 1.0);
  if (fabs(d) < tiny) d = tiny;
  d = 1.0 / d;
  double h = d;
  for (int m = 1; m <= 400; ++m) {
    const double m2 = 2.0 * m;
    double num = m * (b - m) * x / ((a + m2 - 1.0) * (a + m2));
    d = 1.0 + num * d; if (fabs(d) < tiny) d = tiny;
    c = 1.0 + num / c; if (fabs(c) < tiny) c = tiny;
    d = 1.0 / d;
    h *= d * c;
    num = -(a + m) * (a + b + m) * x / ((a + m2) * (a + m2 + 1.0));
    d = 1.0 + num * d; if (fabs(d) < tiny) d = tiny;
    c = 1.0 + num / c; if (fabs(c) < tiny) c = tiny;
    d = 1.0 / d;
    const double del = d * c;
    h *= del;
    if (fabs(del - 1.0) < 1e-16) break;
  }
  return h;
}
// regularised incomplete beta function I_x(a, b)
__device__ double beta_inc(double a, double b, double x) {
  if (x <= 0.0) return 0.0;
  if (x >= 1.0) return 1.0;
  const double front = exp(lgamma(a + b) - lgamma(a) - lgamma(b) + a * log(x) + b * log1p(-x));
  if (x < (a + 1.0) / (a + b + 2.0)) return front * beta_cf(a, b, x) / a;
  return 1.0 - front * beta_cf(b, a, 1.0 - x) / b;
}
// P(T_nu > t), t >= 0
__device__ double student_sf(double t, double nu) { return 0.5 * beta_inc(0.5 * nu, 0.5, nu / (nu + t * t)); }

// mean and variance-of-the-mean (s^2 / n, s^2 unbiased) of a member's recorded scores, oldest first
__device__ int hist_stats(const float* __restrict__ hrow, double* mean, double* vmean) {
  const int n = __float_as_int(hrow[10]);
  const int m = n < 10 ? n : 10;
  if (m < 2) return m;
  double acc = 0.0;
  for (int k = 0; k < m; ++k) acc += (double)hrow[(n - m + k) % 10];
  const double mu = acc / (double)m;
  double ss = 0.0;
  for (int k = 0; k < m; ++k) { const double dv = (double)hrow[(n - m + k) % 10] - mu; ss += dv * dv; }
  *mean = mu;
  *vmean = ss / (double)(m - 1) / (double)m;
  return m;
}

__global__ __launch_bounds__(1024) void rank_select_explore_kernel(ExploitArgs a) {
  __shared__ float sc[1024];
  __shared__ int ord[1024];
  __shared__ int place[1024];
  __shared__ int is_rec[1024];
  const int i = threadIdx.x;
  const bool live = i < a.P;
  const float* __restrict__ src = a.score_override ? a.score_override : a.score;
  if (live) sc[i] = src[i];
  __syncthreads();
  int pos = 0;
  if (live) {
    const float si = sc[i];
    for (int j = 0; j < a.P; ++j) pos += (j != i && ranks_above(sc[j], j, si, i)) ? 1 : 0;
    ord[pos] = i;
    place[i] = pos;
  }
  __syncthreads();
  // exploit: who copies from whom (decided on the scores before the pass)
  const uint32_t k0 = (uint32_t)a.seed, k1 = (uint32_t)(a.seed >> 32);
  const int first_bottom = a.P - a.n_trunc;
  int d = -1;
  if (live) {
    const uint32_t x = philox4x32_10(a.round, (uint32_t)i, DOMAIN_DONOR, 0u, k0, k1).x;
    if (a.tournament) {
      if (a.P > 1) {
        int j = (int)philox_bounded(x, (uint32_t)(a.P - 1));
        j += j >= i ? 1 : 0;
        if (!a.ttest) {
          if (place[j] < pos) d = j;
        } else {
          double mi, vi, mj, vj;
          const int ni = hist_stats(a.hist + (int64_t)i * 12, &mi, &vi), nj = hist_stats(a.hist + (int64_t)j * 12, &mj, &vj);
          if (ni >= 2 && nj >= 2 && mj > mi) {
            if (vi + vj == 0.0) {
              d = j;
            } else {
              const double t = (mj - mi) / sqrt(vi + vj);
              const double nu = (vi + vj) * (vi + vj) / (vi * vi / (double)(ni - 1) + vj * vj / (double)(nj - 1));
              if (student_sf(t, nu) < a.ttest_alpha) d = j;
            }
          }
        }
      }
    } else if (a.n_trunc > 0 && pos >= first_bottom) {
      d = ord[philox_bounded(x, (uint32_t)a.n_trunc)];
    }
    is_rec[i] = d >= 0;
  }
  // the donor's values as they are before anybody writes (a donor can be a recipient in a tournament)
  int t_d = 0;
  float h_d[8];
  if (d >= 0) {
    t_d = a.t[d];
    for (int k = 0; k < a.n_hyper; ++k) h_d[k] = a.H[d * a.n_hyper + k];
  }
  __syncthreads();
  if (!live) return;
  a.order[i] = ord[i];
  if (i == 0) {
    int n = 0;
    for (int j = 0; j < a.P; ++j) n += is_rec[j];
    a.n_recip[0] = n;
  }
  a.donor[i] = d;
  if (d < 0) {
    if (a.score_override) a.score[i] = sc[i];
    return;
  }
  int slot = pos - first_bottom;  // truncation: bottom set in rank order
  if (a.tournament) {
    slot = 0;
    for (int j = 0; j < i; ++j) slot += is_rec[j];
  }
  a.recip[slot] = i;
  a.parent[i] = d;
  if (!a.keep_weights) {
    a.t[i] = t_d;
    a.score[i] = sc[d];
  } else if (a.score_override) {
    a.score[i] = sc[i];
  }
  if (a.keep_hypers) return;
  for (int k = 0; k < a.n_hyper; ++k) {
    const u32x4 w = philox4x32_10(a.round, (uint32_t)i, DOMAIN_EXPLORE, (uint32_t)k, k0, k1);
    float v = h_d[k];
    if (a.resample) {
      if (a.resample_always || w.y < a.resample_thr) {
        const double lin = a.prior_a[k] + philox_unit(w.z) * (a.prior_b[k] - a.prior_a[k]);
        v = (float)(a.prior_kind[k] == 1 ? exp(lin) : lin);
      }
    } else {
      // one IEEE float multiply (no contraction possible: nothing is added)
      v = __fmul_rn(v, (w.x & 1u) ? a.f_hi : a.f_lo);
    }
    a.H[i * a.n_hyper + k] = v > a.h_max[k] ? a.h_max[k] : v;
  }
}
hipError_t rank_select_explore(const ExploitArgs& a, hipStream_t s) {
  if (a.P > 1024) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rank_select_explore_kernel, dim3(1), dim3(1024), 0, s, a);
  return hipGetLastError();
}

// Gather-copy: recipient recip[y] receives a byte copy of row donor[recip[y]] of every array.
// grid (chunks, rows, arrays); 16-byte vectors, four in flight per thread.  pass 0: row to row;
// pass 1: donor row -> staging row y; pass 2: staging row y -> recipient row.
constexpr int COPY_UNROLL = 4;
__global__ __launch_bounds__(256) void gather_copy_kernel(CopyArrays arrs, const int32_t* __restrict__ recip,
                                                          const int32_t* __restrict__ donor, const int32_t* __restrict__ n_recip,
                                                          int pass) {
  if ((int)blockIdx.y >= n_recip[0]) return;
  const int r = recip[blockIdx.y];
  const int d = donor[r];
  const int64_t rb = arrs.row_bytes[blockIdx.z];
  char* const base = static_cast<char*>(arrs.base[blockIdx.z]);
  char* const stage = static_cast<char*>(arrs.stage[blockIdx.z]) + (int64_t)blockIdx.y * rb;
  const uint4* __restrict__ src = reinterpret_cast<const uint4*>(pass == 2 ? stage : base + (int64_t)d * rb);
  uint4* __restrict__ dst = reinterpret_cast<uint4*>(pass == 1 ? stage : base + (int64_t)r * rb);
  const int64_t nvec = rb / 16;
  const int64_t span = (int64_t)gridDim.x * 256;
  for (int64_t v0 = (int64_t)blockIdx.x * 256 + threadIdx.x; v0 < nvec; v0 += span * COPY_UNROLL) {
    uint4 tmp[COPY_UNROLL];
#pragma unroll
    for (int u = 0; u < COPY_UNROLL; ++u) {
      const int64_t v = v0 + u * span;
      if (v < nvec) tmp[u] = src[v];
    }
#pragma unroll
    for (int u = 0; u < COPY_UNROLL; ++u) {
      const int64_t v = v0 + u * span;
      if (v < nvec) dst[v] = tmp[u];
    }
  }
}
hipError_t gather_copy(const CopyArrays& arrs, const int32_t* recip, const int32_t* donor, int max_rows, const int32_t* n_recip,
                       bool staged, hipStream_t s) {
  if (max_rows <= 0 || arrs.n <= 0) return hipSuccess;
  int64_t maxvec = 0;
  for (int k = 0; k < arrs.n; ++k) maxvec = arrs.row_bytes[k] / 16 > maxvec ? arrs.row_bytes[k] / 16 : maxvec;
  int64_t chunks = (maxvec + 256 * COPY_UNROLL - 1) / (256 * COPY_UNROLL);
  if (chunks > 2048) chunks = 2048;
  if (chunks < 1) chunks = 1;
  const dim3 grid((unsigned)chunks, max_rows, arrs.n);
  if (!staged) {
    hipLaunchKernelGGL(gather_copy_kernel, grid, dim3(256), 0, s, arrs, recip, donor, n_recip, 0);
  } else {
    hipLaunchKernelGGL(gather_copy_kernel, grid, dim3(256), 0, s, arrs, recip, donor, n_recip, 1);
    hipLaunchKernelGGL(gather_copy_kernel, grid, dim3(256), 0, s, arrs, recip, donor, n_recip, 2);
  }
  return hipGetLastError();
}

}  // namespace pbt
