// Causal self-attention of one (member, sequence, head) per workgroup, forward and backward, for sequences of
// at most 128 positions and 64-wide heads: the S x S score, probability and gradient matrices live in MFMA
// accumulators and never reach memory.  This is the attention of the transformer whose `step` the population
// runs (Section 3, Eq. 2 of the PBT paper; Section 4.2 for the workload).
//
// What is computed, with q() = rounding to bf16 (the same points as the unfused kernels):
//   forward   s = q(Q K^T), p = softmax over keys <= query of s / sqrt(dh), pd = q(p * keep), o = q(pd V)
//   backward  dpd = q(dO V^T), dp = dpd * keep, pq = q(p), ds = q(pq (dp - sum_keys dp pq) / sqrt(dh)),
//             dQ = q(ds K), dK = q(ds^T Q), dV = q(pd^T dO)
// keep = 0 or the member's 1 / (1 - rate), drawn by the forward pass (one Philox block per four consecutive
// keys of a query) and left behind as one bit per (query, key) for the backward pass, which recomputes s and p.
//
// Layout.  v_mfma_f32_32x32x16_bf16(X, Y, acc): lane l supplies row l % 32 of X and of Y, eight consecutive
// contraction indices each (chosen by l / 32); afterwards acc[e] of lane l is the product for X row
// 8 (e / 4) + 4 (l / 32) + e % 4 and Y row l % 32.  Wavefront w owns the 32 queries 32 w .. 32 w + 31 as Y rows
// and walks the key blocks 0 .. w as X rows, so a lane holds, for its query, runs of four consecutive keys:
// the row reductions of the softmax are sums over registers plus one exchange with lane l ^ 32, a run of four
// keys is one Philox block, and the probabilities are already in the right registers to be the Y operand of
// the next product (its contraction index, the key, runs over registers; the other operand is read from a
// transposed copy in LDS with the same permutation of keys).  Products that contract over queries (dK, dV)
// are formed by a second kernel with the roles exchanged (keys on lanes, queries on registers), which repeats
// the two small score products instead of transposing four S x S matrices through LDS; the row statistics it
// needs (maximum, 1 / sum, sum_keys dp pq: three floats per query) are left in memory by the first.  Two
// kernels rather than two passes of one: wavefront w has w + 1 blocks of work in the first and S / 32 - w in
// the second, and a barrier between them would keep every wavefront waiting for the slowest twice.
#include "common.h"
#include "dropout.h"
#include "internal.h"

namespace pbt {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 frag_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float acc_t;

constexpr int DH = ATTN_FUSED_HEAD, SMAX = ATTN_FUSED_MAX_SEQ;
constexpr int TP = SMAX + 4;   // LDS pitch (elements) of a transposed [DH][S] operand: rows 2 banks apart

__device__ __forceinline__ float round_bf16(float x) { return bf2f(f2bf(x)); }
__device__ __forceinline__ float bf_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf_hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }

// ---- operands in LDS ------------------------------------------------------------------------------------
// Every operand (Q, K, V or dO of one head: S rows of DH values, 128 bytes each, `pitch` apart in memory) is
// fetched once with eight neighbouring lanes on a row, 16 bytes each -- read straight from memory in the MFMA
// operand pattern, a wavefront's load touches 32 rows and the L1 takes 64 separate accesses for it, which is
// what bounded these kernels -- and then written to LDS either as rows (the X / Y operand of a product that
// contracts over DH) or transposed (the X operand of a product that contracts over positions).
struct Staged { uint4 v[SMAX * 8 / 256]; };
__device__ __forceinline__ void fetch_rows(const bf16_t* __restrict__ src, int64_t pitch, int S, Staged& r) {
#pragma unroll
  for (int j = 0; j < SMAX * 8 / 256; ++j) {
    const int it = threadIdx.x + 256 * j;
    const int row = min(it >> 3, S - 1);   // (past the operand: the last row again, never used)
    r.v[j] = *reinterpret_cast<const uint4*>(src + (int64_t)row * pitch + (it & 7) * 8);
  }
}
// rows of DH values, unpadded; the 16-byte chunks of a row are permuted by the row's index so that the 32 rows
// an operand read touches spread over all banks
__device__ __forceinline__ int row_offset(int row, int chunk) { return row * DH + (((chunk ^ (row >> 1)) & 7) << 3); }
__device__ __forceinline__ void put_rows(const Staged& r, int S, bf16_t* lds) {
#pragma unroll
  for (int j = 0; j < SMAX * 8 / 256; ++j) {
    const int it = threadIdx.x + 256 * j;
    if (it < S * 8) *reinterpret_cast<uint4*>(lds + row_offset(it >> 3, it & 7)) = r.v[j];
  }
}
// lds[c * TP + row] = operand[row][c].  Lanes 8 apart hold neighbouring rows: they exchange half of their chunk
// so that each writes four 4-byte pairs (row, row + 1) instead of eight 2-byte values.
__device__ __forceinline__ void put_transposed(const Staged& r, int S, bf16_t* lds) {
#pragma unroll
  for (int j = 0; j < SMAX * 8 / 256; ++j) {
    const int it = threadIdx.x + 256 * j;
    if (it >= S * 8) break;   // (uniform over the workgroup: S * 8 is a multiple of 256)
    const int row = it >> 3, cc = it & 7, odd = row & 1;
    const uint4 v = r.v[j];
    const uint32_t g0 = __shfl_xor(odd ? v.x : v.z, 8), g1 = __shfl_xor(odd ? v.y : v.w, 8);
    // the even row's and the odd row's four values of columns 8 cc + i0 .. + 3
    const uint32_t e0 = odd ? g0 : v.x, e1 = odd ? g1 : v.y, o0 = odd ? v.z : g0, o1 = odd ? v.w : g1;
    uint32_t* out = reinterpret_cast<uint32_t*>(lds) + (8 * cc + 4 * odd) * (TP / 2) + (row >> 1);
    out[0] = (e0 & 0xffffu) | (o0 << 16);
    out[TP / 2] = (e0 >> 16) | (o0 & 0xffff0000u);
    out[2 * (TP / 2)] = (e1 & 0xffffu) | (o1 << 16);
    out[3 * (TP / 2)] = (e1 >> 16) | (o1 & 0xffff0000u);
  }
}

__device__ __forceinline__ acc_t zero_acc() {
  acc_t a;
#pragma unroll
  for (int e = 0; e < 16; ++e) a[e] = 0.f;
  return a;
}
// X rows (row xrow of xl) . Y rows (row yrow of yl) over the DH values, both stored as rows
__device__ __forceinline__ acc_t product_dh(const bf16_t* xl, int xrow, const bf16_t* yl, int yrow, int hf) {
  acc_t a = zero_acc();
#pragma unroll
  for (int c = 0; c < DH / 16; ++c)
    a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const frag_t*>(xl + row_offset(xrow, 2 * c + hf)),
                                                *reinterpret_cast<const frag_t*>(yl + row_offset(yrow, 2 * c + hf)), a, 0, 0, 0);
  return a;
}
// X operand for a product whose contraction index runs over the registers of an accumulator block: rows of a
// transposed copy, contraction indices 32 blk + 16 half + {4 hf .. 4 hf + 3} and the same + 8
__device__ __forceinline__ frag_t transposed_frag(const bf16_t* lds, int row, int blk, int half, int hf) {
  const bf16_t* p = lds + row * TP + 32 * blk + 16 * half + 4 * hf;
  const uint2 lo = *reinterpret_cast<const uint2*>(p), hi = *reinterpret_cast<const uint2*>(p + 8);
  const uint4 v = make_uint4(lo.x, lo.y, hi.x, hi.y);
  return __builtin_bit_cast(frag_t, v);
}
// Y operand from accumulator-layout values already rounded and packed in pairs (registers 8 half .. 8 half + 7)
__device__ __forceinline__ frag_t packed_frag(const uint32_t* pairs, int half) {
  const uint4 u = make_uint4(pairs[4 * half], pairs[4 * half + 1], pairs[4 * half + 2], pairs[4 * half + 3]);
  return __builtin_bit_cast(frag_t, u);
}
// A wavefront's 32 x DH result (two accumulator blocks: lane = row, registers = runs of four columns), rounded,
// to memory rows `pitch` apart.  Written straight from the accumulators every store would touch 32 rows with 8
// bytes each; instead the block goes through the wavefront's own 32 rows of an LDS operand region it no longer
// needs (rows first .. first + 31 of `region`, which no other wavefront reads) and leaves as whole 128-byte rows.
// LDS operations of one wavefront execute in order, so no barrier is involved.
__device__ __forceinline__ void store_rows(const acc_t* acc, bf16_t* region, int first, int lane, bf16_t* __restrict__ dst, int64_t pitch) {
  const int lr = lane & 31, hf = lane >> 5;
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      *reinterpret_cast<uint2*>(region + row_offset(first + lr, 4 * nb + g) + 4 * hf) =
          make_uint2(f2bf_pair(acc[nb][4 * g], acc[nb][4 * g + 1]), f2bf_pair(acc[nb][4 * g + 2], acc[nb][4 * g + 3]));
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = (lane >> 3) + 8 * j, cc = lane & 7;
    *reinterpret_cast<uint4*>(dst + (int64_t)row * pitch + 8 * cc) = *reinterpret_cast<const uint4*>(region + row_offset(first + row, cc));
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

struct AttnDims { int d, H, S, Bc; float scale; };

// Record of the keep bits: one 32-bit word per (member, sequence, head, query, key block); bit k = key
// 32 kb + k of that query kept.  Words of key blocks past the query's own are never written or read.
__device__ __forceinline__ int64_t record_index(const AttnDims& a, int member, int b, int h, int t, int kb) {
  return ((((int64_t)member * a.Bc + b) * a.H + h) * SMAX + t) * 4 + kb;
}
// row statistics: [member][sequence][head][3][SMAX] floats
__device__ __forceinline__ int64_t stat_index(const AttnDims& a, int member, int b, int h) {
  return (((int64_t)member * a.Bc + b) * a.H + h) * 3 * SMAX;
}
// x where bit k of word is set, else 0
__device__ __forceinline__ float keep_or_zero(uint32_t word, int k, float x) {
  return __uint_as_float(__float_as_uint(x) & (uint32_t)((int32_t)(word << (31 - k)) >> 31));
}

// exp(v - max) for the scores of wavefront w's queries (lane's query t = 32 w + lane % 32) against key blocks
// 0 .. w, in the accumulator layout (register e of block kb: key 32 kb + 8 (e / 4) + 4 hf + e % 4; 0 for keys
// past the query), the row maximum and 1 / row sum.  Kr, Qr: K and Q as rows in LDS.
__device__ __forceinline__ void softmax_rows(const bf16_t* Kr, const bf16_t* Qr, int w, int lr, int hf, float scale, float (*p)[16], float& mx, float& inv) {
  mx = -INFINITY;
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    if (kb > w) break;
    const acc_t s = product_dh(Kr, 32 * kb + lr, Qr, 32 * w + lr, hf);
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      p[kb][e] = round_bf16(s[e]) * scale;
      if (kb == w && 8 * (e / 4) + 4 * hf + e % 4 > lr) p[kb][e] = -INFINITY;
      mx = fmaxf(mx, p[kb][e]);
    }
  }
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  float se = 0.f;
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    if (kb > w) break;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      p[kb][e] = __expf(p[kb][e] - mx);   // (-inf gives 0)
      se += p[kb][e];
    }
  }
  se += __shfl_xor(se, 32);
  inv = 1.f / se;
}

}  // namespace

__global__ __launch_bounds__(256) void attention_fwd_kernel(const bf16_t* __restrict__ qkv, AttnDims a, DropArgs dr, int site,
                                                            bf16_t* __restrict__ o, uint32_t* __restrict__ record) {
  __shared__ __attribute__((aligned(16))) bf16_t Kr[SMAX * DH];
  __shared__ __attribute__((aligned(16))) bf16_t Qr[SMAX * DH];
  __shared__ __attribute__((aligned(16))) bf16_t Vt[DH * TP];
  const int member = blockIdx.y, b = blockIdx.x / a.H, h = blockIdx.x % a.H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, lr = lane & 31, hf = lane >> 5;
  const int NB = a.S / 32;
  const int64_t row0 = ((int64_t)member * a.Bc + b) * a.S;          // first row of this sequence
  const int64_t pitch = 3 * (int64_t)a.d;
  const bf16_t* Q = qkv + row0 * pitch + h * DH;
  {
    Staged q, k, v;
    fetch_rows(Q, pitch, a.S, q);
    fetch_rows(Q + a.d, pitch, a.S, k);
    fetch_rows(Q + 2 * a.d, pitch, a.S, v);
    put_rows(q, a.S, Qr);
    put_rows(k, a.S, Kr);
    put_transposed(v, a.S, Vt);
  }
  __syncthreads();
  if (w >= NB) return;
  const DropRate rate = drop_rate(dr.H, dr.n_hyper, dr.col, member, dr.active);
  const int t = 32 * w + lr;                                           // this lane's query
  const uint64_t prow = ((uint64_t)(b * a.H + h) * a.S + t) * a.S;     // element index of (query, key 0) in the site

  float p[4][16];
  float mx, inv;
  softmax_rows(Kr, Qr, w, lr, hf, a.scale, p, mx, inv);

  acc_t oacc[2] = {zero_acc(), zero_acc()};
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    if (kb > w) break;
    uint32_t pd[8];
    uint32_t word = 0u;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int c = 32 * kb + 8 * g + 4 * hf;   // first key of the run
      const uint32_t bits = c <= t ? drop_bits4(dr, rate, member, site, (uint32_t)((prow + c) >> 2)) : 0u;
      word |= bits << (8 * g);
#pragma unroll
      for (int j = 0; j < 4; j += 2)
        pd[2 * g + j / 2] = f2bf_pair(p[kb][4 * g + j] * inv * keep_or_zero(bits, j, rate.scale), p[kb][4 * g + j + 1] * inv * keep_or_zero(bits, j + 1, rate.scale));
    }
    if (record) {
      const uint32_t full = (word << (4 * hf)) | (__shfl_xor(word, 32) << (4 * (1 - hf)));
      if (hf == 0) record[record_index(a, member, b, h, t, kb)] = full;
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const frag_t pf = packed_frag(pd, half);
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
        oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(transposed_frag(Vt, 32 * nb + lr, kb, half, hf), pf, oacc[nb], 0, 0, 0);
    }
  }
  store_rows(oacc, Qr, 32 * w, lane, o + (row0 + 32 * w) * a.d + h * DH, a.d);   // (only this wavefront reads its queries' rows of Qr)
}

// Backward, first kernel: queries on lanes.  Row statistics, ds, dQ.  K and Q occupy two LDS regions for the
// scores, V and dO (fetched at the start, held in registers meanwhile) the same two for dpd.  What has to stay
// live across the key blocks is kept as packed bf16, which is what pq and dpd are anyway.
__global__ __launch_bounds__(256, 3) void attention_bwd_dq_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dO, AttnDims a, DropArgs dr,
                                                                  const uint32_t* __restrict__ record, bf16_t* __restrict__ dqkv, float* __restrict__ stats) {
  __shared__ __attribute__((aligned(16))) bf16_t Xr[SMAX * DH];   // K, then V
  __shared__ __attribute__((aligned(16))) bf16_t Yr[SMAX * DH];   // Q, then dO
  __shared__ __attribute__((aligned(16))) bf16_t Kt[DH * TP];
  const int member = blockIdx.y, b = blockIdx.x / a.H, h = blockIdx.x % a.H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, lr = lane & 31, hf = lane >> 5;
  const int NB = a.S / 32;
  const int64_t row0 = ((int64_t)member * a.Bc + b) * a.S;
  const int64_t pitch = 3 * (int64_t)a.d;
  const bf16_t* Q = qkv + row0 * pitch + h * DH;
  const bf16_t* dOh = dO + row0 * a.d + h * DH;
  const int t = 32 * w + lr;
  Staged v, g;
  {
    Staged q, k;
    fetch_rows(Q, pitch, a.S, q);
    fetch_rows(Q + a.d, pitch, a.S, k);
    fetch_rows(Q + 2 * a.d, pitch, a.S, v);
    fetch_rows(dOh, a.d, a.S, g);
    put_rows(q, a.S, Yr);
    put_rows(k, a.S, Xr);
    put_transposed(k, a.S, Kt);
  }
  const DropRate rate = drop_rate(dr.H, dr.n_hyper, dr.col, member, dr.active);
  uint32_t words[4] = {0u, 0u, 0u, 0u};
  if (w < NB) {
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
      if (kb <= w) words[kb] = record[record_index(a, member, b, h, t, kb)] >> (4 * hf);   // bit 8 g + j: this lane's key 8 g + 4 hf + j
  }
  __syncthreads();
  float mx = 0.f, inv = 0.f;
  uint32_t pq[4][8];
  if (w < NB) {
    float p[4][16];
    softmax_rows(Xr, Yr, w, lr, hf, a.scale, p, mx, inv);
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      if (kb > w) break;
#pragma unroll
      for (int e = 0; e < 16; e += 2) pq[kb][e / 2] = f2bf_pair(p[kb][e] * inv, p[kb][e + 1] * inv);
    }
  }
  __syncthreads();   // every wavefront is done with K and Q
  put_rows(v, a.S, Xr);
  put_rows(g, a.S, Yr);
  __syncthreads();
  if (w >= NB) return;
  // (pq is zero for keys past the query, so dp needs no mask of its own: those terms vanish from the sum and from ds)
  uint32_t dpd[4][8];
  float dot = 0.f;
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    if (kb > w) break;
    const acc_t gacc = product_dh(Xr, 32 * kb + lr, Yr, t, hf);
#pragma unroll
    for (int e = 0; e < 16; e += 2) {
      dpd[kb][e / 2] = f2bf_pair(gacc[e], gacc[e + 1]);
      const float d0 = keep_or_zero(words[kb], 8 * (e / 4) + e % 4, rate.scale) * bf_lo(dpd[kb][e / 2]);
      const float d1 = keep_or_zero(words[kb], 8 * (e / 4) + e % 4 + 1, rate.scale) * bf_hi(dpd[kb][e / 2]);
      dot = fmaf(d0, bf_lo(pq[kb][e / 2]), dot);
      dot = fmaf(d1, bf_hi(pq[kb][e / 2]), dot);
    }
  }
  dot += __shfl_xor(dot, 32);
  if (hf == 0) {
    float* st = stats + stat_index(a, member, b, h);
    st[t] = mx; st[SMAX + t] = inv; st[2 * SMAX + t] = dot;
  }
  acc_t dq[2] = {zero_acc(), zero_acc()};
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    if (kb > w) break;
    uint32_t ds[8];
#pragma unroll
    for (int e = 0; e < 16; e += 2) {
      const float d0 = keep_or_zero(words[kb], 8 * (e / 4) + e % 4, rate.scale) * bf_lo(dpd[kb][e / 2]);
      const float d1 = keep_or_zero(words[kb], 8 * (e / 4) + e % 4 + 1, rate.scale) * bf_hi(dpd[kb][e / 2]);
      ds[e / 2] = f2bf_pair(bf_lo(pq[kb][e / 2]) * (d0 - dot) * a.scale, bf_hi(pq[kb][e / 2]) * (d1 - dot) * a.scale);
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const frag_t sf = packed_frag(ds, half);
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
        dq[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(transposed_frag(Kt, 32 * nb + lr, kb, half, hf), sf, dq[nb], 0, 0, 0);
    }
  }
  store_rows(dq, Yr, 32 * w, lane, dqkv + (row0 + 32 * w) * pitch + h * DH, pitch);   // (only this wavefront reads its queries' rows of Yr)
}

// Backward, second kernel: keys on lanes (wavefront w owns keys 32 w .. 32 w + 31), queries on registers.
// dK, dV.  Q and K occupy two LDS regions for the transposed scores, dO and V the same two for dpd^T.
__global__ __launch_bounds__(256, 2) void attention_bwd_dkv_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dO, AttnDims a, DropArgs dr,
                                                                   const uint32_t* __restrict__ record, const float* __restrict__ stats,
                                                                   bf16_t* __restrict__ dqkv) {
  __shared__ __attribute__((aligned(16))) bf16_t Xr[SMAX * DH];   // Q, then dO
  __shared__ __attribute__((aligned(16))) bf16_t Yr[SMAX * DH];   // K, then V
  __shared__ __attribute__((aligned(16))) bf16_t Qt[DH * TP];
  __shared__ __attribute__((aligned(16))) bf16_t dOt[DH * TP];
  __shared__ __attribute__((aligned(16))) float st[3 * SMAX];     // row maximum, 1 / row sum, sum_keys dp pq of every query
  __shared__ __attribute__((aligned(16))) uint32_t rec[SMAX * 4]; // keep bits: [query][key block]
  const int member = blockIdx.y, b = blockIdx.x / a.H, h = blockIdx.x % a.H;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, lr = lane & 31, hf = lane >> 5;
  const int NB = a.S / 32;
  const int64_t row0 = ((int64_t)member * a.Bc + b) * a.S;
  const int64_t pitch = 3 * (int64_t)a.d;
  const bf16_t* Q = qkv + row0 * pitch + h * DH;
  const bf16_t* dOh = dO + row0 * a.d + h * DH;
  Staged v, g;
  {
    Staged q, k;
    fetch_rows(Q, pitch, a.S, q);
    fetch_rows(Q + a.d, pitch, a.S, k);
    fetch_rows(Q + 2 * a.d, pitch, a.S, v);
    fetch_rows(dOh, a.d, a.S, g);
    // (3 * SMAX floats and SMAX * 4 words: 16 bytes per thread for the first 96 and the first 128 threads)
    if (threadIdx.x < 3 * SMAX / 4)
      reinterpret_cast<float4*>(st)[threadIdx.x] = reinterpret_cast<const float4*>(stats + stat_index(a, member, b, h))[threadIdx.x];
    if (threadIdx.x < SMAX)
      reinterpret_cast<uint4*>(rec)[threadIdx.x] = reinterpret_cast<const uint4*>(record + record_index(a, member, b, h, 0, 0))[threadIdx.x];
    put_rows(q, a.S, Xr);
    put_rows(k, a.S, Yr);
    put_transposed(q, a.S, Qt);
    put_transposed(g, a.S, dOt);
  }
  const DropRate rate = drop_rate(dr.H, dr.n_hyper, dr.col, member, dr.active);
  __syncthreads();
  const int key = 32 * w + lr;
  uint32_t sv[4][8];   // q(s) of the query blocks w .. NB - 1, packed
  if (w < NB) {
#pragma unroll
    for (int qb = 0; qb < 4; ++qb) {
      if (qb < w) continue;
      if (qb >= NB) break;
      const acc_t s = product_dh(Xr, 32 * qb + lr, Yr, key, hf);
#pragma unroll
      for (int e = 0; e < 16; e += 2) sv[qb][e / 2] = f2bf_pair(s[e], s[e + 1]);
    }
  }
  __syncthreads();   // every wavefront is done with Q and K
  put_rows(g, a.S, Xr);
  put_rows(v, a.S, Yr);
  __syncthreads();
  if (w >= NB) return;
  acc_t dk[2] = {zero_acc(), zero_acc()}, dv[2] = {zero_acc(), zero_acc()};
#pragma unroll
  for (int qb = 0; qb < 4; ++qb) {
    if (qb < w) continue;
    if (qb >= NB) break;
    const acc_t gacc = product_dh(Xr, 32 * qb + lr, Yr, key, hf);
    uint32_t pd[8], ds[8];
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const int tq = 32 * qb + 8 * gq + 4 * hf;   // four consecutive queries
      const float4 rmax = *reinterpret_cast<const float4*>(st + tq), rinv = *reinterpret_cast<const float4*>(st + SMAX + tq),
                   rdot = *reinterpret_cast<const float4*>(st + 2 * SMAX + tq);
      const float mxs[4] = {rmax.x, rmax.y, rmax.z, rmax.w}, invs[4] = {rinv.x, rinv.y, rinv.z, rinv.w}, dots[4] = {rdot.x, rdot.y, rdot.z, rdot.w};
      float pdv[4], dsv[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int e = 4 * gq + j;
        const float sc = (e & 1 ? bf_hi(sv[qb][e / 2]) : bf_lo(sv[qb][e / 2])) * a.scale;
        float pr = __expf(sc - mxs[j]) * invs[j];
        if (qb == w && lr > 8 * gq + 4 * hf + j) pr = 0.f;   // key past the query
        const float f = keep_or_zero(rec[(tq + j) * 4 + w] >> lr, 0, rate.scale);
        pdv[j] = pr * f;
        dsv[j] = round_bf16(pr) * (round_bf16(gacc[e]) * f - dots[j]) * a.scale;
      }
      pd[2 * gq] = f2bf_pair(pdv[0], pdv[1]); pd[2 * gq + 1] = f2bf_pair(pdv[2], pdv[3]);
      ds[2 * gq] = f2bf_pair(dsv[0], dsv[1]); ds[2 * gq + 1] = f2bf_pair(dsv[2], dsv[3]);
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const frag_t pf = packed_frag(pd, half), sf = packed_frag(ds, half);
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        dv[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(transposed_frag(dOt, 32 * nb + lr, qb, half, hf), pf, dv[nb], 0, 0, 0);
        dk[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(transposed_frag(Qt, 32 * nb + lr, qb, half, hf), sf, dk[nb], 0, 0, 0);
      }
    }
  }
  bf16_t* krows = dqkv + (row0 + 32 * w) * pitch + a.d + h * DH;
  store_rows(dk, Yr, 32 * w, lane, krows, pitch);   // (only this wavefront reads its keys' rows of Yr)
  store_rows(dv, Yr, 32 * w, lane, krows + a.d, pitch);
}

bool attention_fused_applies(int d_model, int heads, int seq) {
  return heads > 0 && d_model / heads == DH && d_model % heads == 0 && seq % 32 == 0 && seq >= 32 && seq <= SMAX;
}
size_t attention_record_bytes(int P, int Bc, int heads) { return (size_t)P * Bc * heads * SMAX * 4 * 4; }
size_t attention_stats_bytes(int P, int Bc, int heads) { return (size_t)P * Bc * heads * 3 * SMAX * 4; }

hipError_t attention_fwd(const bf16_t* qkv, int P, int Bc, int S, int d, int H, float scale, const DropArgs& dr, int site, bf16_t* o,
                         uint32_t* record, hipStream_t s) {
  if (!attention_fused_applies(d, H, S) || d % 8) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attention_fwd_kernel, dim3(Bc * H, P), dim3(256), 0, s, qkv, AttnDims{d, H, S, Bc, scale}, dr, site, o, record);
  return hipGetLastError();
}
hipError_t attention_bwd(const bf16_t* qkv, const bf16_t* dO, int P, int Bc, int S, int d, int H, float scale, const DropArgs& dr,
                         const uint32_t* record, float* stats, bf16_t* dqkv, hipStream_t s) {
  if (!attention_fused_applies(d, H, S) || d % 8 || !record || !stats) return hipErrorInvalidValue;
  const AttnDims a{d, H, S, Bc, scale};
  hipLaunchKernelGGL(attention_bwd_dq_kernel, dim3(Bc * H, P), dim3(256), 0, s, qkv, dO, a, dr, record, dqkv, stats);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attention_bwd_dkv_kernel, dim3(Bc * H, P), dim3(256), 0, s, qkv, dO, a, dr, record, stats, dqkv);
  return hipGetLastError();
}

}  // namespace pbt
