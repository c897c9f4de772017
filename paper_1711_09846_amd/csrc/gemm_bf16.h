// Population-batched GEMM on the gfx950 matrix cores: bf16 operands, fp32
// accumulate, one output tile per workgroup, member index = batch dimension.
//
// This is the dense contraction of `step` (Section 3, Eq. 2 of the PBT paper):
// forward Y = X W, input gradient dX = dY W^T and weight gradient dW = X^T dY
// for every member of the population in one launch.
//
// Tiling (wave64): a workgroup of WM x WN wavefronts owns a BM x BN tile of C;
// each wavefront owns a (BM/WM) x (BN/WN) sub-tile made of 32x32 accumulator
// blocks fed by v_mfma_f32_32x32x16_bf16.  The K loop moves BK wide slabs of A
// and B from HBM into registers (16-byte loads), then into LDS in a
// "K-contiguous" layout, so that every MFMA operand is one 16-byte LDS read.
// Operands whose memory layout is contiguous along M or N instead of K (W in
// the forward pass, X and dY in the weight gradient) are transposed in
// registers on their way into LDS.  The loads of slab k+1 (k+2 with two LDS
// buffers) are in flight while slab k is multiplied.
//
// The epilogue is a functor applied to runs of 8 consecutive columns; it fuses
// bias + activation (forward) or the activation derivative (input gradient).
#pragma once
#include <type_traits>

#include "common.h"
#include "dropout.h"
#include "optim_math.h"

namespace pbt {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

struct GemmArgs {
  const bf16_t* A;
  int64_t lda, sa;
  const bf16_t* B;
  int64_t ldb, sb;
  int M, N, K, batch;
  int tiles_m, tiles_n;
  // two-level batch index (attention: outer = sequence, inner = head): the operand of batch element b
  // starts at (b / inner) * s? + (b % inner) * s?_in
  int inner;
  int64_t sa_in, sb_in;
  // optional by-product: colsum[b * colsum_stride + n] = sum_k B[k][n] (float), written by the first tile
  // row of every batch element from the B slabs it stages anyway (the bias gradient of a weight-gradient
  // contraction, whose B operand is dZ); null = not wanted
  float* colsum = nullptr;
  int64_t colsum_stride = 0;
  int colsum_k = 0;   // the column sums run over k < colsum_k (the launcher sets K when the caller gives no limit)
};

// LDS row pitch in elements for a slab width BK: +8 keeps 16-byte alignment and skews the banks
constexpr int gemm_pitch(int bk) { return bk + 8; }
// Within an LDS row the 16-byte slots (8 k values each) are permuted by the row's group of sixteen:
// slot' = slot ^ ((row / 16) & mask).  The transposing writers (lanes 8 rows apart, same slot) would
// otherwise all hit two bank groups, because 8 row pitches are a multiple of half the bank period; the
// XOR spreads them over all banks.  Readers take 16 consecutive rows of one slot per LDS cycle, and
// the odd slot pitch already spreads those, so the permutation has to be constant over such a group:
// keyed by row / 8 it costs every fragment read 4 to 8 extra cycles (measured), keyed by row / 16 none.
template <int BK>
__device__ __forceinline__ int lds_offset(int row, int k) {
  constexpr int MASK = (BK / 8 < 8 ? BK / 8 : 8) - 1;
  return row * gemm_pitch(BK) + ((((k >> 3) ^ ((row >> 4) & MASK)) << 3) | (k & 7));
}

// ---- global -> register staging -------------------------------------------------------------
// Operand tile of ROWS x BK (ROWS along M or N).  KCONTIG: memory is [row][k].
// Otherwise memory is [k][row] and a thread fetches a KB x 8 block (KB k-rows of
// 8 consecutive rows each) that it transposes before the LDS write.

template <int ROWS, int GEMM_BK, bool KCONTIG, int THREADS>
struct TileLoader {
  static constexpr int GEMM_PITCH = gemm_pitch(GEMM_BK);
  static constexpr int CHUNKS = ROWS * GEMM_BK / 8;            // 16-byte pieces per tile
  static constexpr int PER_THREAD = CHUNKS / THREADS;     // pieces per thread
  static constexpr int KB = PER_THREAD;                        // k-rows per thread in the transposed case
  static_assert(CHUNKS % THREADS == 0, "tile must divide evenly over the workgroup");
  uint4 r[PER_THREAD];

  // base points at this member's operand; row0 / k0 select the tile; nrows / K bound it.
  __device__ __forceinline__ void load(const bf16_t* __restrict__ base, int64_t ld, int row0, int k0, int nrows, int K) {
    const int t = threadIdx.x;
    if constexpr (KCONTIG) {
#pragma unroll
      for (int j = 0; j < PER_THREAD; ++j) {
        const int c = t + THREADS * j;
        const int row = row0 + c / (GEMM_BK / 8);
        const int k = k0 + (c % (GEMM_BK / 8)) * 8;
        r[j] = fetch8(base, (int64_t)row * ld + k, row < nrows, K - k);
      }
    } else {
      const int rb = t % (ROWS / 8);
      const int kb = t / (ROWS / 8);
      const int row = row0 + rb * 8;
#pragma unroll
      for (int j = 0; j < KB; ++j) {
        const int k = k0 + kb * KB + j;
        r[j] = fetch8(base, (int64_t)k * ld + row, k < K, nrows - row);
      }
    }
  }

  // The same tile when its K range lies wholly inside the operand: straight 16-byte loads, no guards.
  // Rows past the operand's last row (a ragged last tile in M or N) read the last row (K-contiguous
  // operand) or the last whole group of eight rows (the other layout; the launcher checks that the row
  // count is a multiple of 8 then): always in bounds, and the epilogue drops those rows' results.
  __device__ __forceinline__ void load_interior(const bf16_t* __restrict__ base, int64_t ld, int row0, int k0, int nrows) {
    const int t = threadIdx.x;
    if constexpr (KCONTIG) {
#pragma unroll
      for (int j = 0; j < PER_THREAD; ++j) {
        const int c = t + THREADS * j;
        const int row = min(row0 + c / (GEMM_BK / 8), nrows - 1);
        r[j] = *reinterpret_cast<const uint4*>(base + (int64_t)row * ld + k0 + (c % (GEMM_BK / 8)) * 8);
      }
    } else {
      const int rb = t % (ROWS / 8);
      const int kb = t / (ROWS / 8);
      const int row = min(row0 + rb * 8, nrows - 8);
#pragma unroll
      for (int j = 0; j < KB; ++j)
        r[j] = *reinterpret_cast<const uint4*>(base + (int64_t)(k0 + kb * KB + j) * ld + row);
    }
  }

  // 8 consecutive elements starting at base[off]; `valid` false or `left` <= 0 gives zeros,
  // 0 < left < 8 loads only the first `left` elements.
  static __device__ __forceinline__ uint4 fetch8(const bf16_t* __restrict__ base, int64_t off, bool valid, int left) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (valid && left >= 8) {
      v = *reinterpret_cast<const uint4*>(base + off);
    } else if (valid && left > 0) {
      bf16_t e[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) e[i] = i < left ? base[off + i] : (bf16_t)0;
      v.x = e[0] | ((uint32_t)e[1] << 16);
      v.y = e[2] | ((uint32_t)e[3] << 16);
      v.z = e[4] | ((uint32_t)e[5] << 16);
      v.w = e[6] | ((uint32_t)e[7] << 16);
    }
    return v;
  }

  __device__ __forceinline__ void store(bf16_t* __restrict__ lds) const {
    const int t = threadIdx.x;
    if constexpr (KCONTIG) {
#pragma unroll
      for (int j = 0; j < PER_THREAD; ++j) {
        const int c = t + THREADS * j;
        const int row = c / (GEMM_BK / 8);
        const int k = (c % (GEMM_BK / 8)) * 8;
        *reinterpret_cast<uint4*>(lds + lds_offset<GEMM_BK>(row, k)) = r[j];
      }
    } else {
      const int rb = t % (ROWS / 8);
      const int kb = t / (ROWS / 8);
      // r[j] holds rows rb*8 .. rb*8+7 at k = kb*KB + j.  Emit, per row, KB consecutive k values.
      const uint32_t* w = reinterpret_cast<const uint32_t*>(r);  // w[j*4 + q]: rows 2q (low half), 2q+1 (high half)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint32_t lo[KB / 2 > 0 ? KB / 2 : 1], hi[KB / 2 > 0 ? KB / 2 : 1];
#pragma unroll
        for (int j = 0; j < KB; j += 2) {
          const uint32_t a = w[j * 4 + q], b = w[(j + 1) * 4 + q];
          lo[j / 2] = (a & 0xffffu) | (b << 16);          // row 2q:   k = j, j+1
          hi[j / 2] = (a >> 16) | (b & 0xffff0000u);      // row 2q+1: k = j, j+1
        }
        bf16_t* p0 = lds + lds_offset<GEMM_BK>(rb * 8 + 2 * q, kb * KB);      // both rows are in the same group of sixteen
        bf16_t* p1 = p0 + GEMM_PITCH;
        if constexpr (KB == 2) {
          *reinterpret_cast<uint32_t*>(p0) = lo[0];
          *reinterpret_cast<uint32_t*>(p1) = hi[0];
        } else if constexpr (KB == 4) {
          *reinterpret_cast<uint2*>(p0) = make_uint2(lo[0], lo[1]);
          *reinterpret_cast<uint2*>(p1) = make_uint2(hi[0], hi[1]);
        } else {
          static_assert(KB == 8, "unsupported tile shape");
          *reinterpret_cast<uint4*>(p0) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
          *reinterpret_cast<uint4*>(p1) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        }
      }
    }
  }
};

// Workgroups are handed to the 8 XCDs round-robin by linear id.  Remap the id
// so that each XCD works on a contiguous run of tiles (neighbouring tiles
// share an A or B slab, which then stays in that XCD's L2).
__device__ __forceinline__ int xcd_remap(int id, int total) {
  constexpr int XCDS = 8;
  const int per = total / XCDS;
  if (id >= per * XCDS) return id;  // ragged tail keeps its place
  return (id % XCDS) * per + id / XCDS;
}

// Tile order inside one batch element: tiles are numbered down groups of GROUP_M tile rows, so that the
// workgroups resident on an XCD at one time (consecutive numbers) form a block of tiles that shares
// few A and B slabs and keeps them in that XCD's L2.
constexpr int GROUP_M = 8;

template <int BM, int BN, int GEMM_BK, int WM, int WN, bool A_MCONTIG, bool B_KCONTIG, bool DOUBLE_BUF, class Epilogue>
__global__ __launch_bounds__(WM * WN * 64) void gemm_bf16_kernel(GemmArgs g, Epilogue epi) {
  constexpr int THREADS = WM * WN * 64;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int GEMM_PITCH = gemm_pitch(GEMM_BK);
  constexpr int SLAB = (BM + BN) * GEMM_PITCH;  // elements of one A + B slab pair
  // LDS (sized by the launcher): one or two slab pairs during the K loop, then (reused) a 32-row strip of C
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

  TileLoader<BM, GEMM_BK, !A_MCONTIG, THREADS> la;
  TileLoader<BN, GEMM_BK, B_KCONTIG, THREADS> lb;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int frag_row = lane & 31, frag_k = (lane >> 5) * 8;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // A functor that reads what it updates (the optimiser) takes runs of 4 columns, consecutive lanes side
  // by side (whole 256-byte row segments per access, which streaming loads need: nothing keeps the other
  // half of a line).  The runs of the first 32-row strip are requested right after the K loop, each later
  // strip's while the one before it is applied.
  constexpr int WCOLS = BN / WN, RUNS4 = WCOLS / 4, NQ4 = 32 * RUNS4 / 64;
  epi.begin(member);

  // (half of the first strip goes out ahead of the K loop so that memory is never left idle while the
  // workgroups of a compute unit are all busy with their operands; all of it would cost an occupancy step)
  typename Epilogue::Fetched pre[NQ4];
  constexpr int EARLY_RUNS = NQ4 / 2;
  auto fetch_first_strip = [&](int q0, int q1) {
    if constexpr (Epilogue::PREFETCH) {
#pragma unroll
      for (int q = 0; q < NQ4; ++q) {
        if (q < q0 || q >= q1) continue;
        const int run = q * 64 + lane;
        const int m = m0 + wm * (BM / WM) + run / RUNS4, n = n0 + wn * WCOLS + (run % RUNS4) * 4;
        if (m < g.M && n < g.N) pre[q] = epi.fetch(m, n, g.N - n < 4 ? g.N - n : 4);
      }
    }
  };
  fetch_first_strip(0, EARLY_RUNS);

  // (only the weight-gradient functors carry this code: elsewhere its registers would cost an occupancy step)
  const bool want_colsum = Epilogue::COLSUM && g.colsum != nullptr && tm == 0;
  float csum = 0.f;

  // One K loop per kind of launch: straight 16-byte loads when K is a multiple of the slab depth (ragged
  // last tiles in M or N read clamped rows), the guarded loads otherwise; keeping the two apart keeps the
  // guards' branches out of the common loop.
  auto k_loop = [&](auto interior_tag) {
    constexpr bool INTERIOR = decltype(interior_tag)::value;
    auto fetch_slab = [&](int k) {
      if constexpr (INTERIOR) {
        la.load_interior(A, g.lda, m0, k, g.M);
        lb.load_interior(B, g.ldb, n0, k, g.N);
      } else {
        la.load(A, g.lda, m0, k, g.M, g.K);
        lb.load(B, g.ldb, n0, k, g.N, g.K);
      }
    };
    // the MFMAs of one slab
    auto multiply_slab = [&](const bf16_t* As, const bf16_t* Bs) {
#pragma unroll
      for (int kk = 0; kk < GEMM_BK; kk += 16) {
        bf16x8_t af[TM], bfr[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
          af[i] = *reinterpret_cast<const bf16x8_t*>(As + lds_offset<GEMM_BK>(wm * (BM / WM) + i * 32 + frag_row, kk + frag_k));
#pragma unroll
        for (int j = 0; j < TN; ++j)
          bfr[j] = *reinterpret_cast<const bf16x8_t*>(Bs + lds_offset<GEMM_BK>(wn * (BN / WN) + j * 32 + frag_row, kk + frag_k));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
      }
    };
    // column sums of the B slab in LDS (rows of Bs are columns n; the slot permutation only reorders k)
    auto colsum_slab = [&](const bf16_t* Bs, int k0) {
      if constexpr (Epilogue::COLSUM) if (want_colsum && (int)threadIdx.x < BN && k0 < g.colsum_k) {
        const bool whole = k0 + GEMM_BK <= g.colsum_k;   // (uniform: only the slab that straddles the limit masks)
#pragma unroll
        for (int ks = 0; ks < GEMM_BK; ks += 8) {
          const uint4 v = *reinterpret_cast<const uint4*>(Bs + lds_offset<GEMM_BK>((int)threadIdx.x, ks));
          const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const float lo = __uint_as_float(w[q] << 16), hi = __uint_as_float(w[q] & 0xffff0000u);
            csum += whole || k0 + ks + 2 * q < g.colsum_k ? lo : 0.f;
            csum += whole || k0 + ks + 2 * q + 1 < g.colsum_k ? hi : 0.f;
          }
        }
      }
    };
    if constexpr (DOUBLE_BUF) {
      // slab s+1 goes from registers into the other LDS buffer and slab s+2 leaves for the registers
      // before slab s is multiplied: one barrier per slab, and a load has a whole slab's MFMAs to land
      fetch_slab(0);
      la.store(smem);
      lb.store(smem + BM * GEMM_PITCH);
      if (GEMM_BK < g.K) fetch_slab(GEMM_BK);
      __syncthreads();
      int buf = 0;
      for (int k0 = 0; k0 < g.K; k0 += GEMM_BK, buf ^= 1) {
        if (k0 + GEMM_BK < g.K) {
          la.store(smem + (buf ^ 1) * SLAB);
          lb.store(smem + (buf ^ 1) * SLAB + BM * GEMM_PITCH);
          if (k0 + 2 * GEMM_BK < g.K) fetch_slab(k0 + 2 * GEMM_BK);
        }
        multiply_slab(smem + buf * SLAB, smem + buf * SLAB + BM * GEMM_PITCH);
        colsum_slab(smem + buf * SLAB + BM * GEMM_PITCH, k0);
        __syncthreads();
      }
    } else {
      fetch_slab(0);
      for (int k0 = 0; k0 < g.K; k0 += GEMM_BK) {
        __syncthreads();  // previous slab fully consumed
        la.store(smem);
        lb.store(smem + BM * GEMM_PITCH);
        __syncthreads();
        if (k0 + GEMM_BK < g.K) fetch_slab(k0 + GEMM_BK);
        multiply_slab(smem, smem + BM * GEMM_PITCH);
        colsum_slab(smem + BM * GEMM_PITCH, k0);
      }
    }
  };
  // (uniform over the launch: a ragged K needs the zero fill of the guarded loads; ragged M or N only
  // needs in-bounds addresses, unless the operand is stored eight rows per 16 bytes and does not end on one)
  const bool a_rows_ok = A_MCONTIG ? (g.M % 8 == 0 && g.M >= 8) : true;
  const bool b_rows_ok = B_KCONTIG ? true : (g.N % 8 == 0 && g.N >= 8);
  if (g.K % GEMM_BK == 0 && a_rows_ok && b_rows_ok) k_loop(std::true_type{});
  else k_loop(std::false_type{});

  if constexpr (Epilogue::COLSUM) if (want_colsum && (int)threadIdx.x < BN && n0 + (int)threadIdx.x < g.N)
    g.colsum[(int64_t)member * g.colsum_stride + n0 + threadIdx.x] = csum;

  // Epilogue.  The MFMAs above take the B fragment as their first operand, so an accumulator block
  // holds the transposed product: lane -> row m (lane % 32) of C, register e -> column
  // 8*(e/4) + 4*(lane/32) + e%4, i.e. a lane holds runs of four consecutive columns.  To reach memory
  // with 16-byte accesses of whole 128-byte rows, every wavefront passes its accumulators, one row of
  // 32x32 blocks at a time, through a private LDS region (16-byte writes, no conflicts at a pitch of
  // 4 mod 64 floats) and reads them back as runs of 8 consecutive columns for the functor.  LDS
  // operations of one wavefront execute in order, so no workgroup barrier is needed between strips.
  constexpr int CPITCH = WCOLS + 4, RUNS = WCOLS / 8;
  static_assert(WM * WN * 32 * CPITCH * 4 <= SLAB * 2, "C strips must fit the slab LDS");
  float* const Cw = reinterpret_cast<float*>(smem) + wave * 32 * CPITCH;
  fetch_first_strip(EARLY_RUNS, NQ4);
  // A lane handles the same eight columns in every run, so what a functor needs per column (the bias) is
  // read once, here: read inside the runs, after the stores of the run before, each run paid a memory
  // latency of its own (more than half of a K = 512 tile's lifetime).  (Ahead of the K loop the eight
  // registers would cost the 128x128 kernel its third workgroup per compute unit.)
  static_assert(64 % RUNS == 0, "a lane's runs must share their columns");
  float colv[8];
  if constexpr (Epilogue::HAS_COLS) epi.load_cols(n0 + wn * WCOLS + (lane % RUNS) * 8, g.N, colv);
  __syncthreads();  // every wavefront is done with the slabs
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    // a functor that reads what it updates asks for all of a strip's runs first, so that their
    // latencies overlap each other and the staging below
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(Cw + (lane & 31) * CPITCH + j * 32 + 8 * q + 4 * (lane >> 5)) =
            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if constexpr (Epilogue::PREFETCH) {
#pragma unroll
      for (int q = 0; q < NQ4; ++q) {
        const int run = q * 64 + lane;
        const int row = run / RUNS4, col = (run % RUNS4) * 4;
        const int m = m0 + wm * (BM / WM) + i * 32 + row, n = n0 + wn * WCOLS + col;
        const float4 x = *reinterpret_cast<const float4*>(Cw + row * CPITCH + col);
        if (m < g.M && n < g.N) {
          const float v[4] = {x.x, x.y, x.z, x.w};
          epi.apply4_fetched(pre[q], m, n, v, g.N - n < 4 ? g.N - n : 4);
        }
        // the registers of this run are free again: the same run of the next strip goes into them
        if (i + 1 < TM && m + 32 < g.M && n < g.N) pre[q] = epi.fetch(m + 32, n, g.N - n < 4 ? g.N - n : 4);
      }
    } else {
      typename Epilogue::RunData rund[32 * RUNS / 64];
      if constexpr (Epilogue::HAS_RUNDATA) {
#pragma unroll
        for (int q = 0; q < 32 * RUNS / 64; ++q) {
          const int run = q * 64 + lane;
          const int m = m0 + wm * (BM / WM) + i * 32 + run / RUNS, n = n0 + wn * WCOLS + (run % RUNS) * 8;
          rund[q] = typename Epilogue::RunData{};
          if (m < g.M && n < g.N) rund[q] = epi.load_run(m, n, g.N - n < 8 ? g.N - n : 8);
        }
      }
#pragma unroll
      for (int q = 0; q < 32 * RUNS / 64; ++q) {
        const int run = q * 64 + lane;
        const int row = run / RUNS, col = (run % RUNS) * 8;
        const int m = m0 + wm * (BM / WM) + i * 32 + row, n = n0 + wn * WCOLS + col;
        const float4 lo = *reinterpret_cast<const float4*>(Cw + row * CPITCH + col);
        const float4 hi = *reinterpret_cast<const float4*>(Cw + row * CPITCH + col + 4);
        if (m < g.M && n < g.N) {
          const float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
          if constexpr (Epilogue::HAS_COLS) epi.apply8(member, m, n, v, g.N - n < 8 ? g.N - n : 8, colv);
          else if constexpr (Epilogue::HAS_RUNDATA) epi.apply8(member, m, n, v, g.N - n < 8 ? g.N - n : 8, rund[q]);
          else epi.apply8(member, m, n, v, g.N - n < 8 ? g.N - n : 8);
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
  if constexpr (Epilogue::HAS_FINISH) epi.finish(member, tm * g.tiles_n + tn, g.tiles_m * g.tiles_n);
}

// ---- epilogues ------------------------------------------------------------------------------

// Every epilogue receives runs of up to 8 consecutive columns of one row: v[0..count-1] are the
// accumulator values of C[m][n .. n+count-1].  Full, 16-byte aligned runs use vector accesses.

__device__ __forceinline__ uint4 pack_bf16x8(const float* v) {
  return make_uint4(f2bf_pair(v[0], v[1]), f2bf_pair(v[2], v[3]), f2bf_pair(v[4], v[5]), f2bf_pair(v[6], v[7]));
}
__device__ __forceinline__ void unpack_bf16x8(uint4 p, float* v) {
  const uint32_t w[4] = {p.x, p.y, p.z, p.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    v[2 * q] = __uint_as_float(w[q] << 16);
    v[2 * q + 1] = __uint_as_float(w[q] & 0xffff0000u);
  }
}
__device__ __forceinline__ bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

__device__ __forceinline__ void store_bf16_run(bf16_t* dst, const float* v, int count) {
  if (count == 8 && aligned16(dst)) {
    *reinterpret_cast<uint4*>(dst) = pack_bf16x8(v);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (e < count) dst[e] = f2bf(v[e]);
  }
}

// Every functor's begin(member) moves its pointers to the member's arrays once, so that apply8 is
// left with m * pitch + n.
struct EpiStoreF32 {
  static constexpr bool HAS_FINISH = false;
  static constexpr bool PREFETCH = false;
  static constexpr bool COLSUM = true;   // weight gradients: the bias gradient can ride along
  static constexpr bool HAS_COLS = false;
  static constexpr bool HAS_RUNDATA = false;
  struct Fetched {};
  struct RunData {};
  float* C;
  int64_t ldc, sc;
  __device__ __forceinline__ void begin(int member) { C += (int64_t)member * sc; }
  __device__ __forceinline__ void apply8(int, int m, int n, const float* v, int count) const {
    float* dst = C + (int64_t)m * ldc + n;
    if (count == 8 && aligned16(dst)) {
      *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
      *reinterpret_cast<float4*>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
    } else {
      for (int e = 0; e < count; ++e) dst[e] = v[e];
    }
  }
};

struct EpiStoreBF16 {
  static constexpr bool HAS_FINISH = false;
  static constexpr bool PREFETCH = false;
  static constexpr bool COLSUM = false;
  static constexpr bool HAS_COLS = false;
  static constexpr bool HAS_RUNDATA = false;
  struct Fetched {};
  struct RunData {};
  bf16_t* C;
  int64_t ldc, sc;
  int inner = 1;       // two-level batch index as in GemmArgs
  int64_t sc_in = 0;
  __device__ __forceinline__ void begin(int member) { C += (int64_t)(member / inner) * sc + (int64_t)(member % inner) * sc_in; }
  __device__ __forceinline__ void apply8(int, int m, int n, const float* v, int count) const {
    store_bf16_run(C + (int64_t)m * ldc + n, v, count);
  }
};

// Output layer over a large vocabulary: logits = acc + b[n], kept in float.  (Streaming stores for the logits made
// this launch 4 % faster and the two that follow it slower by more: plain stores.)
struct EpiBiasF32 {
  static constexpr bool HAS_FINISH = false;
  static constexpr bool PREFETCH = false;
  static constexpr bool COLSUM = false;
  static constexpr bool HAS_COLS = true;
  static constexpr bool HAS_RUNDATA = false;
  struct Fetched {};
  struct RunData {};
  const float* bias;
  int64_t sbias;
  float* C;
  int64_t ldc, sc;
  __device__ __forceinline__ void begin(int member) { bias += (int64_t)member * sbias; C += (int64_t)member * sc; }
  // the eight biases of the lane's columns (the same for every run the lane handles), zero past N
  __device__ __forceinline__ void load_cols(int n, int N, float* b) const {
    if (n + 8 <= N && aligned16(bias + n)) {
      const float4 lo = *reinterpret_cast<const float4*>(bias + n), hi = *reinterpret_cast<const float4*>(bias + n + 4);
      b[0] = lo.x; b[1] = lo.y; b[2] = lo.z; b[3] = lo.w; b[4] = hi.x; b[5] = hi.y; b[6] = hi.z; b[7] = hi.w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) b[e] = n + e < N ? bias[n + e] : 0.f;
    }
  }
  __device__ __forceinline__ void apply8(int, int m, int n, const float* v, int count, const float* b) const {
    float* dst = C + (int64_t)m * ldc + n;
    if (count == 8 && aligned16(dst)) {
      *reinterpret_cast<float4*>(dst) = make_float4(v[0] + b[0], v[1] + b[1], v[2] + b[2], v[3] + b[3]);
      *reinterpret_cast<float4*>(dst + 4) = make_float4(v[4] + b[4], v[5] + b[5], v[6] + b[6], v[7] + b[7]);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (e < count) dst[e] = v[e] + b[e];
    }
  }
};

// Forward layer: z = acc + b[n]; stores z (for the backward pass, may be null) and act(z), both bf16.
struct EpiBiasAct {
  static constexpr bool HAS_FINISH = false;
  static constexpr bool PREFETCH = false;
  static constexpr bool COLSUM = false;
  static constexpr bool HAS_COLS = true;
  static constexpr bool HAS_RUNDATA = false;
  struct Fetched {};
  struct RunData {};
  const float* bias;  // + member * sbias + n
  int64_t sbias;
  bf16_t* Z;
  bf16_t* Aout;
  int64_t ld, so;
  int act;
  __device__ __forceinline__ void begin(int member) {
    bias += (int64_t)member * sbias;
    if (Z) Z += (int64_t)member * so;
    Aout += (int64_t)member * so;
  }
  // the eight biases of the lane's columns (the same for every run the lane handles), zero past N
  __device__ __forceinline__ void load_cols(int n, int N, float* b) const {
    if (n + 8 <= N && aligned16(bias + n)) {
      const float4 lo = *reinterpret_cast<const float4*>(bias + n), hi = *reinterpret_cast<const float4*>(bias + n + 4);
      b[0] = lo.x; b[1] = lo.y; b[2] = lo.z; b[3] = lo.w; b[4] = hi.x; b[5] = hi.y; b[6] = hi.z; b[7] = hi.w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) b[e] = n + e < N ? bias[n + e] : 0.f;
    }
  }
  __device__ __forceinline__ void apply8(int, int m, int n, const float* v, int count, const float* b) const {
    float z[8], a[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = e < count ? v[e] + b[e] : 0.f;
    act_fwd8(z, a, act);
    const int64_t o = (int64_t)m * ld + n;
    if (Z) store_bf16_run(Z + o, z, count);
    store_bf16_run(Aout + o, a, count);
  }
};

// Forward layer followed by a dropout site: the stored activation is act(acc + b[n]), rounded, times the keep factor
// of its element (Philox block (m ld + n) / 4 of the site, as the stand-alone dropout kernel draws it), rounded
// again; the keep bits go to the site's record (bit e % 8 of byte e / 8 of the member's [rows][ld] array).  N and ld
// are multiples of 8.  (A functor of its own: inside EpiBiasAct the extra state cost the 256x256 kernel its
// registers, 156 -> 860 us per launch.)
struct EpiBiasActDrop {
  static constexpr bool HAS_FINISH = false;
  static constexpr bool PREFETCH = false;
  static constexpr bool COLSUM = false;
  static constexpr bool HAS_COLS = true;
  static constexpr bool HAS_RUNDATA = false;
  struct Fetched {};
  struct RunData {};
  const float* bias;
  int64_t sbias;
  bf16_t* Aout;
  int64_t ld, so;
  int act;
  uint8_t* rec;
  int64_t rec_stride;   // bytes of record per member
  DropArgs drop;
  int site;
  int member_ = 0;
  DropRate rate = {0u, 1.f};
  __device__ __forceinline__ void begin(int member) {
    bias += (int64_t)member * sbias;
    Aout += (int64_t)member * so;
    rec += (int64_t)member * rec_stride;
    rate = drop_rate(drop.H, drop.n_hyper, drop.col, member, drop.active);
    member_ = member;
  }
  __device__ __forceinline__ void load_cols(int n, int N, float* b) const {
    const float4 lo = *reinterpret_cast<const float4*>(bias + n), hi = *reinterpret_cast<const float4*>(bias + n + 4);
    b[0] = lo.x; b[1] = lo.y; b[2] = lo.z; b[3] = lo.w; b[4] = hi.x; b[5] = hi.y; b[6] = hi.z; b[7] = hi.w;
  }
  __device__ __forceinline__ void apply8(int, int m, int n, const float* v, int, const float* b) const {
    float z[8], a[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = v[e] + b[e];
    act_fwd8(z, a, act);
    const int64_t o = (int64_t)m * ld + n;
    const uint32_t b0 = drop_bits4(drop, rate, member_, site, (uint32_t)(o >> 2)), b1 = drop_bits4(drop, rate, member_, site, (uint32_t)(o >> 2) + 1u);
    const uint32_t bits = b0 | (b1 << 4);
    bf16_t out[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = (bits >> e) & 1u ? bf16_times_float(f2bf(a[e]), rate.scale) : (bf16_t)(f2bf(a[e]) & 0x8000u);
    *reinterpret_cast<uint4*>(Aout + o) = make_uint4(out[0] | ((uint32_t)out[1] << 16), out[2] | ((uint32_t)out[3] << 16),
                                                     out[4] | ((uint32_t)out[5] << 16), out[6] | ((uint32_t)out[7] << 16));
    rec[o >> 3] = (uint8_t)bits;
  }
};

// Input gradient: dz_prev = acc * act'(z_prev), bf16.  With a dropout record (mask != null) the result is then
// multiplied by the keep factor of the site that followed the activation in the forward pass: the value is
// rounded to bf16, multiplied by 0 or by the member's scale (the float nearest 1 / (1 - p), p from column col
// of H) in double, and rounded once more.  The record holds one bit per element of the member's [rows][ld]
// array (bit e % 8 of byte e / 8), as the forward pass of that site left it.
struct EpiDgradAct {
  static constexpr bool HAS_FINISH = false;
  static constexpr bool PREFETCH = false;
  static constexpr bool COLSUM = false;
  static constexpr bool HAS_COLS = false;
  static constexpr bool HAS_RUNDATA = true;
  struct Fetched {};
  struct RunData { uint4 z = {0u, 0u, 0u, 0u}; uint32_t bits = 0u; };
  const bf16_t* Zprev;
  bf16_t* dZ;
  int64_t ld, so;
  int act;
  const uint8_t* mask = nullptr;
  int64_t mask_stride = 0;       // bytes of record per member
  const float* H = nullptr;
  int n_hyper = 0, col = -1;
  float scale = 1.f;
  __device__ __forceinline__ void begin(int member) {
    Zprev += (int64_t)member * so; dZ += (int64_t)member * so;
    if (mask) {
      mask += (int64_t)member * mask_stride;
      const float p = col >= 0 ? H[(int64_t)member * n_hyper + col] : 0.f;
      scale = p > 0.f ? (float)(1.0 / (1.0 - (double)p)) : 1.f;
    }
  }
  // the run of z the result is scaled by (and the run's eight record bits): requested for all runs of a strip
  // before the first is applied (read inside apply8, after the store of the run before, every run paid a memory
  // latency of its own)
  __device__ __forceinline__ RunData load_run(int m, int n, int count) const {
    const int64_t o = (int64_t)m * ld + n;
    RunData r;
    r.bits = mask ? mask[o >> 3] : 0u;   // (the launcher only attaches a record to arrays whose rows are whole runs of eight)
    if (count == 8 && aligned16(Zprev + o)) { r.z = *reinterpret_cast<const uint4*>(Zprev + o); return r; }
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (e < count) w[e >> 1] |= (uint32_t)Zprev[o + e] << (16 * (e & 1));
    r.z = make_uint4(w[0], w[1], w[2], w[3]);
    return r;
  }
  __device__ __forceinline__ void apply8(int, int m, int n, const float* v, int count, const RunData& run) const {
    const int64_t o = (int64_t)m * ld + n;
    float z[8], d[8];
    unpack_bf16x8(run.z, z);
    act_bwd_scale8(v, z, d, act);
    if (mask) {
      bf16_t out[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] = (run.bits >> e) & 1u ? bf16_times_float(f2bf(d[e]), scale) : (bf16_t)(f2bf(d[e]) & 0x8000u);  // x * 0 keeps the sign
      *reinterpret_cast<uint4*>(dZ + o) = make_uint4(out[0] | ((uint32_t)out[1] << 16), out[2] | ((uint32_t)out[3] << 16),
                                                     out[4] | ((uint32_t)out[5] << 16), out[6] | ((uint32_t)out[7] << 16));
      return;
    }
    store_bf16_run(dZ + o, d, count);
  }
};

// Weight gradient with the optimiser applied in place: v = dW[m][n .. n+3] never goes to memory;
// the run of theta, its optimiser state and the bf16 shadow is read, updated and written back
// (16-byte streaming accesses).  Saves writing and re-reading the gradient (8 of 34 bytes per
// parameter and step).  The layer's input-gradient GEMM must already have read the bf16 shadow.
template <int OPT>
struct EpiOptimizer {
  static constexpr bool HAS_FINISH = false;
  static constexpr bool PREFETCH = true;
  static constexpr bool COLSUM = true;
  static constexpr bool HAS_COLS = false;
  static constexpr bool HAS_RUNDATA = false;
  struct Fetched { float w[4], s0[4], s1[4]; };  // one run of theta and its state, read ahead of use
  struct RunData {};
  float* W32; float* S0; float* S1; bf16_t* W16;
  int64_t stride, off, ldc;   // member stride, offset of the matrix in the member's vector, row pitch
  OptHyper hy;
  OptScalars sc;
  __device__ __forceinline__ void begin(int member) { sc = opt_scalars<OPT>(hy, member); off += (int64_t)member * stride; }
  __device__ __forceinline__ Fetched fetch(int m, int n, int count) const {
    Fetched f;
    const int64_t o = off + (int64_t)m * ldc + n;
    if (count == 4 && (o & 3) == 0) {
      const float4 a = stream_load(W32 + o), b = stream_load(S0 + o);
      f.w[0] = a.x; f.w[1] = a.y; f.w[2] = a.z; f.w[3] = a.w;
      f.s0[0] = b.x; f.s0[1] = b.y; f.s0[2] = b.z; f.s0[3] = b.w;
      if (OPT == OPT_ADAM) {
        const float4 c = stream_load(S1 + o);
        f.s1[0] = c.x; f.s1[1] = c.y; f.s1[2] = c.z; f.s1[3] = c.w;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        f.w[e] = e < count ? W32[o + e] : 0.f;
        f.s0[e] = e < count ? S0[o + e] : 0.f;
        f.s1[e] = (OPT == OPT_ADAM && e < count) ? S1[o + e] : 0.f;
      }
    }
    return f;
  }
  __device__ __forceinline__ void apply4_fetched(Fetched& f, int m, int n, const float* v, int count) const {
    const int64_t o = off + (int64_t)m * ldc + n;
#pragma unroll
    for (int e = 0; e < 4; ++e) opt_update<OPT>(f.w[e], e < count ? v[e] : 0.f, f.s0[e], f.s1[e], sc, hy);
    if (count == 4 && (o & 3) == 0) {
      stream_store(make_float4(f.w[0], f.w[1], f.w[2], f.w[3]), W32 + o);
      stream_store(make_float4(f.s0[0], f.s0[1], f.s0[2], f.s0[3]), S0 + o);
      if (OPT == OPT_ADAM) stream_store(make_float4(f.s1[0], f.s1[1], f.s1[2], f.s1[3]), S1 + o);
      if (W16) *reinterpret_cast<uint2*>(W16 + o) = make_uint2(f2bf_pair(f.w[0], f.w[1]), f2bf_pair(f.w[2], f.w[3]));
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (e < count) {
          W32[o + e] = f.w[e];
          S0[o + e] = f.s0[e];
          if (OPT == OPT_ADAM) S1[o + e] = f.s1[e];
          if (W16) W16[o + e] = f2bf(f.w[e]);
        }
    }
  }
};

// Tile shapes.  128x128 tiles (four wavefronts, three workgroups per compute unit) unless that leaves
// the 256 compute units with fewer than four workgroups each to hide latency with; then 128x64.
// Long contractions of large matrices take 256x256 tiles (eight wavefronts of 128x64, LDS slabs
// double-buffered, one workgroup per compute unit): the L2 -> LDS traffic per flop halves, which
// lifts the steady-state rate from about 880 to 1100 TFLOP/s (measured, 4096 x 2048 x K, batch 16);
// a tile's fixed cost (first loads, epilogue) is no longer hidden by other workgroups on the compute
// unit, so short contractions stay with 128x128.
enum GemmTile { TILE_128x64 = 0, TILE_128x128, TILE_256x256 };
struct TileShape { int bm, bn; };
inline TileShape tile_shape(GemmTile t) {
  switch (t) {
    case TILE_128x64: return {128, 64};
    case TILE_256x256: return {256, 256};
    default: return {128, 128};
  }
}
inline int64_t tile_count(int M, int N, int batch, int bm, int bn) { return (int64_t)((M + bm - 1) / bm) * ((N + bn - 1) / bn) * batch; }
inline GemmTile choose_tile(int M, int N, int K, int batch) {
  constexpr int CUS = 256;
  // (three quarters of the compute units busy with 256x256 tiles still beat all of them on smaller ones)
  // K = 512 stays with 128x128: timed alone, 256x256 tiles are 5-20 % faster there (4096 rows x 16 members,
  // N = 512 ... 8192), but inside the transformer step, with the fused epilogues and whatever the previous kernel
  // left in the caches, the same launches came out 9 % slower (forward class 206 -> 225 us, step +0.6 ms; for the
  // feed-forward layers alone +0.8 ms, for the vocabulary head alone +0.15 ms).
  if (K >= 1024 && M > 128 && N > 128 && tile_count(M, N, batch, 256, 256) >= CUS * 3 / 4) return TILE_256x256;
  // (double-buffered 128x128 and 128x64 variants were tried for the long, narrow weight gradients (K >= 2048 with at
  // most two tiles per compute unit) and for all 128x128 launches: no change for the former, 3 % slower for the latter)
  if ((tile_count(M, N, batch, 128, 128) < 4 * CUS && N > 64) || (N <= 64 && N > 32)) return TILE_128x64;
  return TILE_128x128;
}

template <int BM, int BN, int BK, int WM, int WN, bool DOUBLE_BUF, bool A_M, bool B_K, class Epilogue>
hipError_t launch_gemm_kernel(const GemmArgs& g, const Epilogue& epi, hipStream_t stream) {
  constexpr int SLAB_BYTES = (BM + BN) * gemm_pitch(BK) * 2;
  constexpr int LDS_BYTES = SLAB_BYTES * (DOUBLE_BUF ? 2 : 1);
  auto kernel = gemm_bf16_kernel<BM, BN, BK, WM, WN, A_M, B_K, DOUBLE_BUF, Epilogue>;
  if constexpr (LDS_BYTES > 64 * 1024) {
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (attr != hipSuccess) return attr;
  }
  const int64_t total = (int64_t)g.tiles_m * g.tiles_n * g.batch;
  hipLaunchKernelGGL(kernel, dim3((unsigned)total), dim3(WM * WN * 64), LDS_BYTES, stream, g, epi);
  return hipGetLastError();
}

template <int BM, int BN, int BK, int WM, int WN, bool DOUBLE_BUF, class Epilogue>
hipError_t launch_gemm_tile(const GemmArgs& g0, bool a_m_contig, bool b_k_contig, const Epilogue& epi, hipStream_t stream) {
  GemmArgs g = g0;
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = (g.N + BN - 1) / BN;
  const int64_t total = (int64_t)g.tiles_m * g.tiles_n * g.batch;
  if (total <= 0 || total > 0x7fffffff) return hipErrorInvalidValue;
  if (!a_m_contig && !b_k_contig) return launch_gemm_kernel<BM, BN, BK, WM, WN, DOUBLE_BUF, false, false>(g, epi, stream);
  if (!a_m_contig && b_k_contig) return launch_gemm_kernel<BM, BN, BK, WM, WN, DOUBLE_BUF, false, true>(g, epi, stream);
  if (a_m_contig && !b_k_contig) return launch_gemm_kernel<BM, BN, BK, WM, WN, DOUBLE_BUF, true, false>(g, epi, stream);
  return launch_gemm_kernel<BM, BN, BK, WM, WN, DOUBLE_BUF, true, true>(g, epi, stream);
}

// Sum over the tile of exp(-(|a_m|^2 + |b_n|^2 - 2 a_m.b_n) / (2 d)): the RBF kernel of the MMD
// score evaluated on the Gram tile while it is still in the accumulators.  Every thread adds its
// elements in a fixed order, the wavefront and then the wavefronts are combined in a fixed
// order, and the tile's sum goes to partial[member][tile]; a later pass adds the tiles.
struct EpiRbfSum {
  static constexpr bool HAS_FINISH = true;
  static constexpr bool PREFETCH = false;
  static constexpr bool COLSUM = false;
  static constexpr bool HAS_COLS = false;
  static constexpr bool HAS_RUNDATA = false;
  struct Fetched {};
  struct RunData {};
  __device__ __forceinline__ void begin(int member) { na += (int64_t)member * sna; nb += (int64_t)member * snb; }
  const float* na;  // squared norms of the A rows, + member * sna
  int64_t sna;
  const float* nb;
  int64_t snb;
  float inv2d;
  float* partial;
  float sum;
  __device__ __forceinline__ void apply8(int member, int m, int n, const float* v, int count) {
    const float nam = na[m];
    const float* nbn = nb + n;
    for (int e = 0; e < count; ++e) sum += expf(-(nam + nbn[e] - 2.f * v[e]) * inv2d);
  }
  __device__ __forceinline__ void finish(int member, int tile, int tiles) {
    __shared__ float wsum[8];
    const float w = wave_sum(sum);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = w;
    __syncthreads();
    if (threadIdx.x == 0) {
      float t = wsum[0];
      for (unsigned k = 1; k < blockDim.x / 64; ++k) t += wsum[k];
      partial[(int64_t)member * tiles + tile] = t;
    }
  }
};

// Host-side launcher.  Caller guarantees 16-byte alignment of pitches / strides / bases.
template <class Epilogue>
hipError_t launch_gemm_bf16(const bf16_t* A, int64_t lda, int64_t sa, bool a_m_contig, const bf16_t* B, int64_t ldb,
                            int64_t sb, bool b_k_contig, int M, int N, int K, int batch, const Epilogue& epi,
                            hipStream_t stream, int inner = 1, int64_t sa_in = 0, int64_t sb_in = 0, float* colsum = nullptr,
                            int64_t colsum_stride = 0, int colsum_k = -1) {
  GemmArgs g;
  g.A = A; g.lda = lda; g.sa = sa;
  g.B = B; g.ldb = ldb; g.sb = sb;
  g.M = M; g.N = N; g.K = K; g.batch = batch;
  g.tiles_m = g.tiles_n = 0;
  g.inner = inner < 1 ? 1 : inner; g.sa_in = sa_in; g.sb_in = sb_in;
  g.colsum = colsum; g.colsum_stride = colsum_stride; g.colsum_k = colsum_k < 0 ? K : colsum_k;
  switch (choose_tile(M, N, K, batch)) {
    case TILE_256x256: return launch_gemm_tile<256, 256, 64, 2, 4, true, Epilogue>(g, a_m_contig, b_k_contig, epi, stream);
    case TILE_128x64: return launch_gemm_tile<128, 64, 64, 2, 2, false, Epilogue>(g, a_m_contig, b_k_contig, epi, stream);
    default: return launch_gemm_tile<128, 128, 64, 2, 2, false, Epilogue>(g, a_m_contig, b_k_contig, epi, stream);
  }
}

}  // namespace pbt
