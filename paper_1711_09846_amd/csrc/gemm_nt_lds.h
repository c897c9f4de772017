// Variant of the population-batched GEMM for two K-contiguous operands (C = A B^T with A [M][K] and
// B [N][K]: the input-gradient layout, attention scores) whose tiles lie wholly inside the operands.
//
// The slabs go from memory straight into LDS (global_load_lds_dwordx4: lane l of a wavefront deposits
// its 16 bytes at LDS base + 16 l), not through registers.  What a compute unit can have in flight is
// then bounded by LDS, not by the registers left over beside the accumulators: four stages of 32 KB
// (256 + 256 rows x 32 k) keep three slabs on their way while one is multiplied, where the register
// path holds one 64 KB slab.  With a load latency near 2 us and 128 flop per byte for a 256x256
// tile, bytes in flight are what bounds the long contractions.
//
// LDS rows are unpadded (64 bytes = four 16-byte slots); conflicts are avoided by permuting the slots
// on the way in: slot s of LDS row r holds k-slot s ^ ((r >> 2) & 3), which each lane arranges by
// choosing which 16 bytes of its row it fetches.  A fragment read (16 consecutive rows, one k-slot
// per LDS cycle) then touches 16 different 16-byte bank groups.
#pragma once
#include "gemm_bf16.h"

namespace pbt {

constexpr int NTL_BM = 256, NTL_BN = 256, NTL_BK = 32, NTL_STAGES = 4, NTL_THREADS = 512;
constexpr int NTL_STAGE_ELEMS = (NTL_BM + NTL_BN) * NTL_BK;          // bf16 elements per stage
constexpr int NTL_LDS_BYTES = NTL_STAGES * NTL_STAGE_ELEMS * 2;      // 128 KB

template <class Epilogue>
__global__ __launch_bounds__(NTL_THREADS) void gemm_nt_lds_kernel(GemmArgs g, Epilogue epi) {
  constexpr int BM = NTL_BM, BN = NTL_BN, BK = NTL_BK, WM = 2, WN = 4;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];

  const int total = g.tiles_m * g.tiles_n * g.batch;
  int id = xcd_remap(blockIdx.x, total);
  const int per_member = g.tiles_m * g.tiles_n;
  const int member = id / per_member;
  id -= member * per_member;
  const int group = id / (GROUP_M * g.tiles_n);
  const int first_m = group * GROUP_M;
  const int rows_in_group = g.tiles_m - first_m < GROUP_M ? g.tiles_m - first_m : GROUP_M;
  id -= group * GROUP_M * g.tiles_n;
  const int tm = first_m + id % rows_in_group;
  const int tn = id / rows_in_group;
  const int m0 = tm * BM, n0 = tn * BN;

  const bf16_t* __restrict__ A = g.A + (int64_t)(member / g.inner) * g.sa + (int64_t)(member % g.inner) * g.sa_in;
  const bf16_t* __restrict__ B = g.B + (int64_t)(member / g.inner) * g.sb + (int64_t)(member % g.inner) * g.sb_in;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // loads: a wavefront instruction fills 16 LDS rows; wavefront w owns row chunks w, w + 8 (A) and
  // w + 16, w + 24 (B) of every slab.  Lane l -> row l / 4 of the chunk, LDS slot l % 4, which is to
  // hold k-slot (l % 4) ^ f with f = ((row >> 2) & 3) = (l >> 4) & 3 (chunks start at multiples of 16).
  const int ld_row = lane >> 2, ld_kslot = (lane & 3) ^ ((lane >> 4) & 3);
  const bf16_t* src[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r = (wave + 8 * j) * 16 + ld_row;  // row of the 512-row slab
    src[j] = r < BM ? A + (int64_t)(m0 + r) * g.lda + ld_kslot * 8 : B + (int64_t)(n0 + r - BM) * g.ldb + ld_kslot * 8;
  }
  auto issue_slab = [&](int slab) {
    bf16_t* stage = smem + (slab % NTL_STAGES) * NTL_STAGE_ELEMS;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(src[j] + (int64_t)slab * BK),
                                       (void __attribute__((address_space(3)))*)(stage + (wave + 8 * j) * 16 * BK), 16, 0, 0);
  };

  // Fragment reads: lane -> row frag_row of a 32-row block, k-slot kk / 8 + lane / 32.  The compiler
  // does not know which LDS stage a direct load fills, so before any LDS read (and at every
  // __syncthreads) it would wait for ALL loads in flight, which is the one thing this kernel must not
  // do.  The K loop therefore issues its LDS reads, counter waits and barriers as assembly: loads
  // return in issue order, so "at most the two younger slabs outstanding" (vmcnt) is exactly "my part
  // of this slab has landed", and the barrier then makes everybody's part visible.
  typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
  const int frag_row = lane & 31, frag_f = (frag_row >> 2) & 3, frag_half = lane >> 5;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) bf16_t*)smem;
  // byte addresses inside a stage for the two 16-wide steps of a slab (the slot permutation is an XOR,
  // so the two steps need an address each); A blocks are 2048 bytes apart, B starts 16384 bytes in
  const uint32_t a_row = (uint32_t)(wm * (BM / WM) + frag_row) * (BK * 2), b_row = (uint32_t)(BM + wn * (BN / WN) + frag_row) * (BK * 2);
  const uint32_t step_off[2] = {(uint32_t)(((0 + frag_half) ^ frag_f) * 16), (uint32_t)(((2 + frag_half) ^ frag_f) * 16)};

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int n_slabs = g.K / BK;
  // Software pipeline.  All four stages are filled up front.  Inside the loop the LDS reads of the next
  // MFMA group are always issued before the MFMAs of the current one, so they run in the matrix
  // pipe's shadow, and the slab barrier sits between the two groups of a slab:
  //   read step-1 operands of slab s | MFMAs step 0 | barrier for slab s+1, refill the stage of slab s,
  //   read step-0 operands of slab s+1 | MFMAs step 1.
  auto wait_and_barrier = [&](int younger_slabs) {  // my loads of the slab have landed; then everybody's
    if (younger_slabs >= 3) asm volatile("s_waitcnt vmcnt(12)\n\ts_barrier" ::: "memory");
    else if (younger_slabs == 2) asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");
    else if (younger_slabs == 1) asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
  };
  static_assert(TM == 4 && TN == 2, "the read sequence below is written for 128x64 wavefront tiles");
  u32x4_t fa[2][TM], fb[2][TN];
  auto read_step = [&](int slab, int st) {
    const uint32_t stage = lds0 + (uint32_t)(slab % NTL_STAGES) * (NTL_STAGE_ELEMS * 2);
    const uint32_t pa = stage + a_row + step_off[st], pb = stage + b_row + step_off[st];
    asm volatile("ds_read_b128 %0, %6\n\tds_read_b128 %1, %6 offset:2048\n\tds_read_b128 %2, %6 offset:4096\n\t"
                 "ds_read_b128 %3, %6 offset:6144\n\tds_read_b128 %4, %7\n\tds_read_b128 %5, %7 offset:2048"
                 : "=&v"(fa[st][0]), "=&v"(fa[st][1]), "=&v"(fa[st][2]), "=&v"(fa[st][3]), "=&v"(fb[st][0]), "=&v"(fb[st][1])
                 : "v"(pa), "v"(pb));
  };
  auto mfma_step = [&](int st) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fb[st][j]), __builtin_bit_cast(bf16x8_t, fa[st][i]), acc[i][j], 0, 0, 0);
  };
#pragma unroll
  for (int s = 0; s < NTL_STAGES; ++s)
    if (s < n_slabs) issue_slab(s);
  wait_and_barrier(n_slabs - 1 < NTL_STAGES - 1 ? n_slabs - 1 : NTL_STAGES - 1);
  read_step(0, 0);
  for (int s = 0; s < n_slabs; ++s) {
    read_step(s, 1);
    // LDS reads return in order: six still out = the step-0 operands are here
    asm volatile("s_waitcnt lgkmcnt(6)" : "+v"(fa[0][0]), "+v"(fa[0][1]), "+v"(fa[0][2]), "+v"(fa[0][3]), "+v"(fb[0][0]), "+v"(fb[0][1]));
    mfma_step(0);
    // all my reads of slab s are complete before I pass the barrier that frees its stage
    // (tied to the last accumulator of the group so that the wait stays behind those MFMAs)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(fa[1][0]), "+v"(fa[1][1]), "+v"(fa[1][2]), "+v"(fa[1][3]), "+v"(fb[1][0]), "+v"(fb[1][1]), "+v"(acc[TM - 1][TN - 1]));
    if (s + 1 < n_slabs) {
      const int last_issued = s + NTL_STAGES - 1 < n_slabs - 1 ? s + NTL_STAGES - 1 : n_slabs - 1;
      wait_and_barrier(last_issued - (s + 1));
      if (s + NTL_STAGES < n_slabs) issue_slab(s + NTL_STAGES);  // into the stage slab s occupied
      read_step(s + 1, 0);
    }
    mfma_step(1);
  }
  asm volatile("s_barrier" ::: "memory");  // every wavefront is done with the last slab

  // epilogue as in gemm_bf16_kernel: transposed accumulator blocks through wave-private LDS strips
  constexpr int WCOLS = BN / WN, CPITCH = WCOLS + 4, RUNS = WCOLS / 8;
  static_assert(WM * WN * 32 * CPITCH * 4 <= NTL_LDS_BYTES, "C strips must fit the LDS");
  float* const Cw = reinterpret_cast<float*>(smem) + wave * 32 * CPITCH;
  epi.begin(member);
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(Cw + (lane & 31) * CPITCH + j * 32 + 8 * q + 4 * (lane >> 5)) =
            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    typename Epilogue::RunData rund[32 * RUNS / 64];
    if constexpr (Epilogue::HAS_RUNDATA) {
#pragma unroll
      for (int q = 0; q < 32 * RUNS / 64; ++q) {
        const int run = q * 64 + lane;
        rund[q] = epi.load_run(m0 + wm * (BM / WM) + i * 32 + run / RUNS, n0 + wn * WCOLS + (run % RUNS) * 8, 8);
      }
    }
#pragma unroll
    for (int q = 0; q < 32 * RUNS / 64; ++q) {
      const int run = q * 64 + lane;
      const int row = run / RUNS, col = (run % RUNS) * 8;
      const int m = m0 + wm * (BM / WM) + i * 32 + row, n = n0 + wn * WCOLS + col;
      const float4 lo = *reinterpret_cast<const float4*>(Cw + row * CPITCH + col);
      const float4 hi = *reinterpret_cast<const float4*>(Cw + row * CPITCH + col + 4);
      const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      if constexpr (Epilogue::HAS_RUNDATA) epi.apply8(member, m, n, v, 8, rund[q]);
      else epi.apply8(member, m, n, v, 8);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  if constexpr (Epilogue::HAS_FINISH) epi.finish(member, tm * g.tiles_n + tn, g.tiles_m * g.tiles_n);
}

// True when the operands of launch_gemm_bf16 fit this kernel: both K-contiguous, whole 256x256 tiles,
// whole slabs, 16-byte aligned rows, and enough tiles and slabs for the pipeline to pay.
inline bool nt_lds_applies(const GemmArgs& g, bool a_m_contig, bool b_k_contig) {
  if (a_m_contig || !b_k_contig) return false;
  // (K = 512 was tried inside the transformer step: the feed-forward input gradient went from 171 to 189 us per launch)
  if (g.M % NTL_BM || g.N % NTL_BN || g.K % NTL_BK || g.K < 1024) return false;
  if (g.lda % 8 || g.ldb % 8 || g.sa % 8 || g.sb % 8 || g.sa_in % 8 || g.sb_in % 8) return false;
  if ((reinterpret_cast<uintptr_t>(g.A) | reinterpret_cast<uintptr_t>(g.B)) & 15) return false;
  return (int64_t)(g.M / NTL_BM) * (g.N / NTL_BN) * g.batch >= 256;
}

template <class Epilogue>
hipError_t launch_gemm_nt_lds(const GemmArgs& g0, const Epilogue& epi, hipStream_t stream) {
  GemmArgs g = g0;
  g.tiles_m = g.M / NTL_BM;
  g.tiles_n = g.N / NTL_BN;
  auto kernel = gemm_nt_lds_kernel<Epilogue>;
  static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, NTL_LDS_BYTES);
  if (attr != hipSuccess) return attr;
  const int64_t total = (int64_t)g.tiles_m * g.tiles_n * g.batch;
  if (total > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kernel, dim3((unsigned)total), dim3(NTL_THREADS), NTL_LDS_BYTES, stream, g, epi);
  return hipGetLastError();
}

}  // namespace pbt
