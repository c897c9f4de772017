// Dropout decisions shared by the transformer's kernels: element e of site s of member i at step c0 is kept
// iff word e % 4 of the Philox block (c0, i, DOMAIN_DROPOUT + s, e / 4) is >= floor(p * 2^32), p the member's
// own rate (a hyperparameter, Section 4.2 of the PBT paper lists dropout among the adapted ones); kept values
// are multiplied by the float nearest 1 / (1 - p).
#pragma once
#include "common.h"
#include "internal.h"
#include "philox.h"

namespace pbt {

struct DropRate { uint32_t thr; float scale; };

__device__ __forceinline__ DropRate drop_rate(const float* H, int n_hyper, int col, int member, int active) {
  DropRate r{0u, 1.f};
  if (active && col >= 0) {
    const float p = H[(int64_t)member * n_hyper + col];
    if (p > 0.f) {
      const double t = floor((double)p * 4294967296.0);
      r.thr = t >= 4294967295.0 ? 4294967295u : (uint32_t)t;
      r.scale = (float)(1.0 / (1.0 - (double)p));
    }
  }
  return r;
}

// keep factors (0 or scale) of the four elements 4*blk .. 4*blk+3 of a site
__device__ __forceinline__ void drop_factors4(const DropArgs& d, const DropRate& r, int member, int site, uint32_t blk, float* f) {
  if (r.thr == 0u) { f[0] = f[1] = f[2] = f[3] = r.scale; return; }
  const u32x4 w = philox4x32_10(d.c0, (uint32_t)member, (uint32_t)(DOMAIN_DROPOUT + site), blk, (uint32_t)d.seed, (uint32_t)(d.seed >> 32));
  f[0] = w.x >= r.thr ? r.scale : 0.f;
  f[1] = w.y >= r.thr ? r.scale : 0.f;
  f[2] = w.z >= r.thr ? r.scale : 0.f;
  f[3] = w.w >= r.thr ? r.scale : 0.f;
}

// keep bits (bit k = element 4*blk + k kept) of one group, from the Philox words or, when the pass that made
// them left them behind, from its record
__device__ __forceinline__ uint32_t drop_bits4(const DropArgs& d, const DropRate& r, int member, int site, uint32_t blk) {
  if (r.thr == 0u) return 15u;
  const u32x4 w = philox4x32_10(d.c0, (uint32_t)member, (uint32_t)(DOMAIN_DROPOUT + site), blk, (uint32_t)d.seed, (uint32_t)(d.seed >> 32));
  return (w.x >= r.thr ? 1u : 0u) | (w.y >= r.thr ? 2u : 0u) | (w.z >= r.thr ? 4u : 0u) | (w.w >= r.thr ? 8u : 0u);
}

}  // namespace pbt
