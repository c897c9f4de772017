// The per-member optimiser update as device functions, shared by the streaming optimiser kernel
// and by the weight-gradient GEMM epilogue that applies the update while the gradient tile is
// still on chip.
//   SGD-momentum  v <- mu v + g;  theta <- theta - lr v
//   Adam          m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2
//                 theta <- theta - lr ( (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps) + wd theta )
//   RMSProp       s <- rho s + (1-rho) g^2;  theta <- theta - lr g / sqrt(s + eps)
// lr / beta1 / weight decay come from the member's row of H on the device, so an explore pass
// changes the very next update without host involvement.
#pragma once
#include "common.h"

namespace pbt {

enum { OPT_SGD_MOMENTUM = 0, OPT_ADAM = 1, OPT_RMSPROP = 2 };

struct OptHyper {  // where the member's hyperparameters and constants come from
  const float* H; const int32_t* t; int n_hyper;
  int col_lr, col_beta1, col_wd;  // column of H with that role, or -1
  float c0, c1, c2, c3;           // SGD {mu}; Adam {beta1, beta2, eps, wd}; RMSProp {rho, eps}
  int t_mul = 1, t_add = 0;       // updates counted by the bias correction: t[member] * t_mul + t_add
};

struct OptScalars { float lr, b1, wd, inv_bc1, inv_bc2; };

template <int OPT>
__device__ __forceinline__ OptScalars opt_scalars(const OptHyper& a, int member) {
  const float* __restrict__ h = a.H + (int64_t)member * a.n_hyper;
  OptScalars s;
  s.lr = h[a.col_lr];
  s.b1 = a.c0; s.wd = a.c3; s.inv_bc1 = 1.f; s.inv_bc2 = 1.f;
  if (OPT == OPT_ADAM) {
    if (a.col_beta1 >= 0) s.b1 = h[a.col_beta1];
    if (a.col_wd >= 0) s.wd = h[a.col_wd];
    const float tt = (float)(a.t[member] * a.t_mul + a.t_add);
    s.inv_bc1 = 1.f / (1.f - powf(s.b1, tt));
    s.inv_bc2 = 1.f / (1.f - powf(a.c1, tt));
  }
  return s;
}

template <int OPT>
__device__ __forceinline__ void opt_update(float& w, float g, float& s0, float& s1, const OptScalars& s, const OptHyper& a) {
  if (OPT == OPT_SGD_MOMENTUM) {
    s0 = a.c0 * s0 + g;
    w = w - s.lr * s0;
  } else if (OPT == OPT_ADAM) {
    s0 = s.b1 * s0 + (1.f - s.b1) * g;
    s1 = a.c1 * s1 + (1.f - a.c1) * g * g;
    const float mh = s0 * s.inv_bc1;
    const float vh = s1 * s.inv_bc2;
    w = w - s.lr * (mh / (sqrtf(vh) + a.c2) + s.wd * w);
  } else {
    s0 = a.c0 * s0 + (1.f - a.c0) * g * g;
    w = w - s.lr * g / sqrtf(s0 + a.c1);
  }
}

// theta, gradient and optimiser state are touched once per step: stream them past the caches
// (nontemporal), so that the bf16 shadow, which the next step's GEMMs read, is what stays resident.
typedef float vf4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 stream_load(const float* p) {
  const vf4_t v = __builtin_nontemporal_load(reinterpret_cast<const vf4_t*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void stream_store(float4 x, float* p) {
  const vf4_t v = {x.x, x.y, x.z, x.w};
  __builtin_nontemporal_store(v, reinterpret_cast<vf4_t*>(p));
}

}  // namespace pbt
