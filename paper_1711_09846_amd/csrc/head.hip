// Output layer of the classifier networks on the matrix cores: a "skinny" contraction whose
// output width C (classes) is at most 32.
//
//   forward   logits[rows][C] = A[rows][K] W[K][C] + b, fused with softmax cross-entropy and its
//             gradient with respect to the logits (rounded to bf16, row pitch 32, zero padded);
//   backward  dZprev[rows][K] = (dlogits[rows][32] W^T) * act'(Zprev).
//
// The A operand of v_mfma_f32_32x32x16_bf16 (row = lane % 32, eight consecutive k per lane) is exactly
// a 16-byte global load of a K-contiguous row, so the large operand never passes through LDS; only
// the small weight matrix is staged there (transposed to K-contiguous, which is what the B operand
// needs).  Forward: a workgroup owns 32 rows and its four wavefronts share the contraction (wavefront
// w takes the k-blocks of 16 with index = w mod 4, so that together they read whole 128-byte lines
// of a row); the partial sums are added in wavefront order.  Backward: a wavefront owns 32 rows and
// passes its 32x64 block through LDS so that memory sees 16-byte accesses of whole 128-byte rows.
#include "common.h"
#include "internal.h"

namespace pbt {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

constexpr int HEAD_NP = 32;         // padded class count = MFMA tile width
constexpr int HEAD_ROWS = 128;      // rows per workgroup of the backward kernel (4 wavefronts x 32)
constexpr int HEAD_FWD_ROWS = 32;   // rows per workgroup of the forward kernel

__device__ __forceinline__ bf16x8_t load_frag(const bf16_t* p, bool valid) {
  uint4 v = make_uint4(0, 0, 0, 0);
  if (valid) v = *reinterpret_cast<const uint4*>(p);
  return *reinterpret_cast<bf16x8_t*>(&v);
}

// grid (ceil(rows / 32), P); dynamic LDS = 32 * (K + 8) bf16 + 4 * 32 * 33 floats
__global__ __launch_bounds__(256) void head_fwd_loss_kernel(const bf16_t* __restrict__ A, int64_t sa,
                                                            const bf16_t* __restrict__ W16, int64_t sw,
                                                            const float* __restrict__ bias, int64_t sbias,
                                                            const int32_t* __restrict__ labels, int64_t sy, int rows,
                                                            int K, int C, float gscale, int n_pos,
                                                            bf16_t* __restrict__ dlogits,
                                                            float* __restrict__ rowloss, int64_t srowloss) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int pitch = K + 8;
  bf16_t* Wt = reinterpret_cast<bf16_t*>(smem);                                  // [32][K + 8], rows >= C unused
  float* Lg = reinterpret_cast<float*>(smem + (size_t)HEAD_NP * pitch * 2);      // [4 wavefronts][32][33]
  const int i = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r_lane = blockIdx.x * HEAD_FWD_ROWS + (lane & 31);
  const int kq = (lane >> 5) * 8;
  const bf16_t* __restrict__ arow = A + (int64_t)i * sa + (int64_t)r_lane * K + kq;
  const bool row_ok = r_lane < rows;
  // the first rows' fragments are requested before the weights are staged
  constexpr int AHEAD = 8;
  bf16x8_t af[AHEAD];
#pragma unroll
  for (int j = 0; j < AHEAD; ++j) {
    const int k0 = (wave + 4 * j) * 16;
    af[j] = load_frag(arow + k0, row_ok && k0 + kq + 8 <= K);
  }
  // stage W[K][C] transposed; rows >= C of the 32-wide class tile are never read (their lanes use zeros)
  const bf16_t* __restrict__ W = W16 + (int64_t)i * sw;
  if ((reinterpret_cast<uintptr_t>(W) & 15) == 0) {
    for (int v = threadIdx.x; v < K * C / 8; v += 256) {   // K is a multiple of 8
      const uint4 x = *reinterpret_cast<const uint4*>(W + (int64_t)v * 8);
      const uint32_t w[4] = {x.x, x.y, x.z, x.w};
      int k = v * 8 / C, c = v * 8 - k * C;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        Wt[c * pitch + k] = (bf16_t)(q & 1 ? w[q >> 1] >> 16 : w[q >> 1] & 0xffffu);
        if (++c == C) { c = 0; ++k; }
      }
    }
  } else {
    for (int e = threadIdx.x; e < K * C; e += 256) {
      const int k = e / C, c = e - k * C;
      Wt[c * pitch + k] = W[e];
    }
  }
  __syncthreads();

  const bf16_t* brow = Wt + (lane & 31) * pitch + kq;
  f32x16_t acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  for (int kb = wave * 16; kb < K; kb += 64 * AHEAD) {
    bf16x8_t cur[AHEAD];
#pragma unroll
    for (int j = 0; j < AHEAD; ++j) cur[j] = af[j];
#pragma unroll
    for (int j = 0; j < AHEAD; ++j) {
      const int k0 = kb + 64 * (AHEAD + j);
      af[j] = load_frag(arow + k0, row_ok && k0 + kq + 8 <= K);
    }
#pragma unroll
    for (int j = 0; j < AHEAD; ++j) {
      const int k0 = kb + 64 * j;
      if (k0 < K) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur[j], load_frag(brow + k0, (lane & 31) < C && k0 + kq + 8 <= K), acc, 0, 0, 0);
    }
  }
#pragma unroll
  for (int e = 0; e < 16; ++e)
    Lg[(wave * 32 + 8 * (e / 4) + 4 * (lane >> 5) + (e % 4)) * 33 + (lane & 31)] = acc[e];
  __syncthreads();
  // partial sums of the four wavefronts, added in wavefront order
  for (int e = threadIdx.x; e < 32 * 32; e += 256) {
    const int o = (e >> 5) * 33 + (e & 31);
    Lg[o] = ((Lg[o] + Lg[32 * 33 + o]) + Lg[2 * 32 * 33 + o]) + Lg[3 * 32 * 33 + o];
  }
  __syncthreads();

  if (threadIdx.x < HEAD_FWD_ROWS) {
    const int r = blockIdx.x * HEAD_FWD_ROWS + threadIdx.x;
    if (r < rows) {
      const float* __restrict__ b = bias + (int64_t)i * sbias;
      float* lg = Lg + threadIdx.x * 33;
      if (n_pos == -2) {
        // no loss here: hand the head outputs (bias added, zero padded to 32) to the caller's loss kernel
        float* __restrict__ o = rowloss + ((int64_t)i * rows + r) * HEAD_NP;
        for (int c = 0; c < HEAD_NP; ++c) o[c] = c < C ? lg[c] + b[c] : 0.f;
      } else if (n_pos >= 0) {
        // logistic loss on one logit: target 1 for rows < n_pos, else 0.
        // loss = softplus(-l) or softplus(l) = max(x, 0) + log1p(exp(-|x|)); dl = sigmoid(l) - target
        const float l = lg[0] + b[0];
        const float target = r < n_pos ? 1.f : 0.f;
        const float x = r < n_pos ? -l : l;
        const float en = expf(-fabsf(l));
        rowloss[(int64_t)i * srowloss + r] = fmaxf(x, 0.f) + log1pf(en);
        if (dlogits) {
          const float sig = l >= 0.f ? 1.f / (1.f + en) : en / (1.f + en);
          bf16_t* __restrict__ d = dlogits + ((int64_t)i * rows + r) * HEAD_NP;
          d[0] = f2bf((sig - target) * gscale);
          for (int c = 1; c < HEAD_NP; ++c) d[c] = 0;
        }
      } else {
        float mx = -INFINITY;
        int cm = 0;
        for (int c = 0; c < C; ++c) {
          lg[c] += b[c];
          if (lg[c] > mx) { mx = lg[c]; cm = c; }
        }
        // log-sum-exp with the largest term split off: lse = mx + log1p(sum of the others)
        const int y = labels[(int64_t)i * sy + r];
        float rest = 0.f, others = (y == cm) ? 0.f : 1.f;
        for (int c = 0; c < C; ++c) {
          if (c == cm) continue;
          const float ex = expf(lg[c] - mx);
          rest += ex;
          if (c != y) others += ex;
        }
        rowloss[(int64_t)i * srowloss + r] = log1pf(rest) + (mx - lg[y]);
        if (dlogits) {
          // softmax_y - 1 = -(sum of the other classes' terms) / S: no cancellation as softmax_y -> 1
          const float inv = 1.f / (1.f + rest);
          bf16_t* __restrict__ d = dlogits + ((int64_t)i * rows + r) * HEAD_NP;
          for (int c = 0; c < HEAD_NP; ++c) {
            float v = 0.f;
            if (c < C) v = (c == y ? -others * inv : expf(lg[c] - mx) * inv) * gscale;
            d[c] = f2bf(v);
          }
        }
      }
    }
  }
}

hipError_t head_fwd_loss(const bf16_t* A, int64_t sa, const bf16_t* W16, int64_t sw, const float* bias, int64_t sbias,
                         const int32_t* labels, int64_t sy, int P, int rows, int K, int C, float gscale, int n_pos,
                         bf16_t* dlogits, float* rowloss, int64_t srowloss, hipStream_t s) {
  if (C > HEAD_NP || C < 1 || K % 8 || (n_pos >= 0 && C != 1)) return hipErrorInvalidValue;
  const size_t lds = (size_t)HEAD_NP * (K + 8) * 2 + (size_t)4 * 32 * 33 * 4;
  if (lds > 160 * 1024) return hipErrorInvalidValue;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(head_fwd_loss_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  dim3 grid((rows + HEAD_FWD_ROWS - 1) / HEAD_FWD_ROWS, P);
  hipLaunchKernelGGL(head_fwd_loss_kernel, grid, dim3(256), lds, s, A, sa, W16, sw, bias, sbias, labels, sy, rows, K, C,
                     gscale, n_pos, dlogits, rowloss, srowloss);
  return hipGetLastError();
}

// grid (ceil(K / 64), ceil(rows / 128), P).  The contraction runs over the 32 padded classes, i.e.
// two MFMAs per 32x32 output block (one when C <= 16).
constexpr int DG_COLS = 64;
constexpr int DG_PITCH = DG_COLS + 4;   // floats: 16-byte writes of a wavefront spread over all banks
__global__ __launch_bounds__(256) void head_dgrad_kernel(const bf16_t* __restrict__ dlogits,
                                                         const bf16_t* __restrict__ W16, int64_t sw,
                                                         const bf16_t* __restrict__ Zprev, bf16_t* __restrict__ dZprev,
                                                         int rows, int K, int C, int act) {
  __shared__ __attribute__((aligned(16))) bf16_t Ws[DG_COLS * 40];   // [64 columns k][32 classes + 8]
  __shared__ __attribute__((aligned(16))) float Cs[4 * 32 * DG_PITCH];  // one 32 x 64 strip per wavefront
  const int i = blockIdx.z;
  const int k_base = blockIdx.x * DG_COLS;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bf16_t* __restrict__ W = W16 + (int64_t)i * sw;
  for (int e = threadIdx.x; e < DG_COLS * HEAD_NP; e += 256) {
    const int kk = e / HEAD_NP, c = e % HEAD_NP;
    const int k = k_base + kk;
    Ws[kk * 40 + c] = (k < K && c < C) ? W[(int64_t)k * C + c] : (bf16_t)0;
  }
  __syncthreads();
  const int r_lane = blockIdx.y * HEAD_ROWS + wave * 32 + (lane & 31);
  const int cq = (lane >> 5) * 8;
  const bf16_t* __restrict__ drow = dlogits + ((int64_t)i * rows + r_lane) * HEAD_NP + cq;
  const bool row_ok = r_lane < rows;
  const bf16x8_t a0 = load_frag(drow, row_ok);
  const bf16x8_t a1 = load_frag(drow + 16, row_ok && C > 16);
  // The W fragment goes first, so the accumulator holds the transposed block: lane -> row, register
  // e -> column 8*(e/4) + 4*(lane/32) + e%4.  Each wavefront writes its 32 x 64 block to its own LDS
  // strip (16-byte writes) and reads it back as runs of 8 columns: a run is one 16-byte access of
  // Zprev and dZprev, eight lanes cover a 128-byte row segment.
  float* Cw = Cs + wave * 32 * DG_PITCH;
#pragma unroll
  for (int j = 0; j < DG_COLS / 32; ++j) {
    f32x16_t acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    const bf16_t* brow = Ws + (j * 32 + (lane & 31)) * 40 + cq;
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_frag(brow, true), a0, acc, 0, 0, 0);
    if (C > 16) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_frag(brow + 16, true), a1, acc, 0, 0, 0);
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *reinterpret_cast<float4*>(Cw + (lane & 31) * DG_PITCH + j * 32 + 8 * q + 4 * (lane >> 5)) =
          make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  const bool vec = (K % 8) == 0;
#pragma unroll
  for (int pass = 0; pass < 32 * (DG_COLS / 8) / 64; ++pass) {
    const int run = pass * 64 + lane;
    const int row = run / (DG_COLS / 8), col = (run % (DG_COLS / 8)) * 8;
    const int r = blockIdx.y * HEAD_ROWS + wave * 32 + row, k = k_base + col;
    if (r >= rows || k >= K) continue;
    const float4 lo = *reinterpret_cast<const float4*>(Cw + row * DG_PITCH + col);
    const float4 hi = *reinterpret_cast<const float4*>(Cw + row * DG_PITCH + col + 4);
    const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    const int64_t o = ((int64_t)i * rows + r) * K + k;
    if (vec && k + 8 <= K) {
      const uint4 z = *reinterpret_cast<const uint4*>(Zprev + o);
      const uint32_t zw[4] = {z.x, z.y, z.z, z.w};
      float zf[8], d[8];
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        zf[2 * h] = __uint_as_float(zw[h] << 16);
        zf[2 * h + 1] = __uint_as_float(zw[h] & 0xffff0000u);
      }
      act_bwd_scale8(v, zf, d, act);
      *reinterpret_cast<uint4*>(dZprev + o) =
          make_uint4(f2bf_pair(d[0], d[1]), f2bf_pair(d[2], d[3]), f2bf_pair(d[4], d[5]), f2bf_pair(d[6], d[7]));
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (k + e < K) dZprev[o + e] = f2bf(v[e] * act_bwd(bf2f(Zprev[o + e]), act));
    }
  }
}

hipError_t head_dgrad(const bf16_t* dlogits, const bf16_t* W16, int64_t sw, const bf16_t* Zprev, bf16_t* dZprev, int P,
                      int rows, int K, int C, int act, hipStream_t s) {
  if (C > HEAD_NP || C < 1) return hipErrorInvalidValue;
  dim3 grid((K + DG_COLS - 1) / DG_COLS, (rows + HEAD_ROWS - 1) / HEAD_ROWS, P);
  hipLaunchKernelGGL(head_dgrad_kernel, grid, dim3(256), 0, s, dlogits, W16, sw, Zprev, dZprev, rows, K, C, act);
  return hipGetLastError();
}

}  // namespace pbt
