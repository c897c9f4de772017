// The actor-critic workload (Section 4.1.1 of the PBT paper: A3C-style agents trained with RMSProp,
// learning rate and entropy cost adapted per member, evaluated by the last 10 episodic returns).
// Device kernels for the trajectory bookkeeping and the loss, and the host-side kernel sequence.
#include <cstring>

#include "common.h"
#include "dense_host.h"
#include "philox.h"

namespace pbt {

constexpr int HIST_SLOTS = 10, HIST_PITCH = 12;  // ring of returns, slot 10 = count (int bits), slot 11 unused

// Per member: copies actions and rewards of the B drawn trajectories (the same Philox draws as the
// observation gather) and pushes the unroll's return (mean over trajectories of the summed
// rewards, accumulated in double in a fixed order) into the member's history ring.
__global__ __launch_bounds__(64) void a2c_fetch_aux_kernel(const int32_t* __restrict__ pool_act,
                                                           const float* __restrict__ pool_rew, int n_traj, int B, int T,
                                                           uint32_t step, uint32_t k0, uint32_t k1,
                                                           int32_t* __restrict__ act, float* __restrict__ rew,
                                                           float* __restrict__ hist) {
  const int i = blockIdx.x;
  __shared__ double tsum[64];
  double mean = 0.0;
  for (int r0 = 0; r0 < B; r0 += 64) {
    const int r = r0 + threadIdx.x;
    double sacc = 0.0;
    if (r < B) {
      const uint32_t x = philox4x32_10(step, (uint32_t)i, DOMAIN_BATCH, (uint32_t)r, k0, k1).x;
      const int64_t src = (int64_t)philox_bounded(x, (uint32_t)n_traj) * T;
      const int64_t dst = ((int64_t)i * B + r) * T;
      for (int t = 0; t < T; ++t) {
        act[dst + t] = pool_act[src + t];
        const float rv = pool_rew[src + t];
        rew[dst + t] = rv;
        sacc += (double)rv;
      }
    }
    tsum[threadIdx.x] = sacc;
    __syncthreads();
    if (threadIdx.x == 0)
      for (int k = 0; k < 64 && r0 + k < B; ++k) mean += tsum[k];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    float* hrow = hist + (int64_t)i * HIST_PITCH;
    const int n = __float_as_int(hrow[HIST_SLOTS]);
    hrow[n % HIST_SLOTS] = (float)(mean / (double)B);
    hrow[HIST_SLOTS] = __int_as_float(n + 1);
  }
}

// Loss and its gradient with respect to the head outputs, one workgroup per member.
// Phase 1: the rewards of the member's trajectories are brought into LDS by all threads, then one
//   thread per trajectory walks it backwards in place for the bootstrapped returns
//   R_T = V(s_T), R_t = r_t + gamma R_{t+1}.
// Phase 2 (one thread per transition) evaluates, with A_t = R_t - V_t and R_t constants,
//   loss_t = -A_t log pi(a_t) + value_cost (R_t - V_t)^2 - entropy_cost H_t
//   dlogit_c = ( -A_t (1[c = a_t] - pi_c) + entropy_cost pi_c (log pi_c + H_t) ) / n
//   dV_t = 2 value_cost (V_t - R_t) / n,   n = B T;  the bootstrap rows get zeros.
// out: head outputs float [P][B][T+1][32] (n_act logits, then the value).  The exponentials of a row
// are evaluated once and kept in registers.  The per-thread losses are combined in a fixed order
// (lane butterfly, then the wavefronts in order).
__global__ __launch_bounds__(1024) void a2c_loss_kernel(const float* __restrict__ out, const int32_t* __restrict__ act,
                                                        const float* __restrict__ rew, const float* __restrict__ H,
                                                        int n_hyper, int col_ent, int B, int T, int n_act, float gamma,
                                                        float value_cost, bf16_t* __restrict__ dout, float* __restrict__ loss) {
  extern __shared__ float Rl[];  // [B][T]
  __shared__ float wsum[16];
  const int i = blockIdx.x;
  const int threads = blockDim.x;
  const float ent_cost = H[i * n_hyper + col_ent];
  const float inv_n = 1.f / (float)(B * T);
  for (int e = threadIdx.x; e < B * T; e += threads) Rl[e] = rew[(int64_t)i * B * T + e];
  __syncthreads();
  for (int r = threadIdx.x; r < B; r += threads) {
    float R = out[(((int64_t)i * B + r) * (T + 1) + T) * 32 + n_act];
    for (int t = T - 1; t >= 0; --t) {
      R = Rl[r * T + t] + gamma * R;
      Rl[r * T + t] = R;
    }
  }
  __syncthreads();
  float lacc = 0.f;
  for (int idx = threadIdx.x; idx < B * (T + 1); idx += threads) {
    const int r = idx / (T + 1), t = idx - r * (T + 1);
    const float4* __restrict__ lg4 = reinterpret_cast<const float4*>(out + ((int64_t)i * B * (T + 1) + idx) * 32);
    uint4* __restrict__ d4 = reinterpret_cast<uint4*>(dout + ((int64_t)i * B * (T + 1) + idx) * 32);
    if (t == T) {
#pragma unroll
      for (int q = 0; q < 4; ++q) d4[q] = make_uint4(0, 0, 0, 0);
      continue;
    }
    float lg[32];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const float4 x = lg4[q];
      lg[4 * q] = x.x; lg[4 * q + 1] = x.y; lg[4 * q + 2] = x.z; lg[4 * q + 3] = x.w;
    }
    const int a = act[((int64_t)i * B + r) * T + t];
    const float R = Rl[r * T + t];
    float v = 0.f, la = 0.f, mx = -INFINITY;
#pragma unroll
    for (int c = 0; c < 32; ++c) {
      if (c < n_act) mx = fmaxf(mx, lg[c]);
      if (c == n_act) v = lg[c];
      if (c == a) la = lg[c];
    }
    const float adv = R - v;
    float ex[32], se = 0.f;
#pragma unroll
    for (int c = 0; c < 32; ++c) {
      ex[c] = c < n_act ? expf(lg[c] - mx) : 0.f;
      se += ex[c];
    }
    const float lse = mx + logf(se), inv_se = 1.f / se;
    float ent = 0.f;
#pragma unroll
    for (int c = 0; c < 32; ++c)
      if (c < n_act) ent -= ex[c] * inv_se * (lg[c] - lse);
    lacc += -adv * (la - lse) + value_cost * adv * adv - ent_cost * ent;
    float dv[32];
#pragma unroll
    for (int c = 0; c < 32; ++c) {
      const float pi = ex[c] * inv_se, lp = lg[c] - lse;
      dv[c] = c < n_act ? (-adv * ((c == a ? 1.f : 0.f) - pi) + ent_cost * pi * (lp + ent)) * inv_n
              : c == n_act ? 2.f * value_cost * (v - R) * inv_n : 0.f;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
      d4[q] = make_uint4(f2bf_pair(dv[8 * q], dv[8 * q + 1]), f2bf_pair(dv[8 * q + 2], dv[8 * q + 3]),
                         f2bf_pair(dv[8 * q + 4], dv[8 * q + 5]), f2bf_pair(dv[8 * q + 6], dv[8 * q + 7]));
  }
  lacc = wave_sum(lacc);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = lacc;
  __syncthreads();
  if (threadIdx.x == 0) {
    float total = 0.f;
    for (int w = 0; w < threads / 64; ++w) total += wsum[w];
    loss[i] = total * inv_n;
  }
}

// score = mean of the last min(count, 10) returns (double accumulation), -inf when there are none
__global__ void a2c_score_kernel(const float* __restrict__ hist, int P, float* __restrict__ score) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= P) return;
  const float* hrow = hist + (int64_t)i * HIST_PITCH;
  const int n = __float_as_int(hrow[HIST_SLOTS]);
  const int m = n < HIST_SLOTS ? n : HIST_SLOTS;
  if (m == 0) { score[i] = -INFINITY; return; }
  // oldest first, as a list that keeps the most recent entries would hold them
  double acc = 0.0;
  for (int k = 0; k < m; ++k) acc += (double)hrow[(n - m + k) % HIST_SLOTS];
  score[i] = (float)(acc / (double)m);
}

pbt_status a2c_check_and_plan(const pbt_config* c, Plan* pl, Carver* w) {
  A2CPlan& a = pl->a2c;
  const int L = c->n_layers;
  if (L < 2) return fail(nullptr, PBT_EUNSUPPORTED, "the actor-critic network needs at least one torso layer before its head");
  if (c->unroll < 1) return fail(nullptr, PBT_EINVAL, "unroll must be positive");
  // the step passes one optimiser-state array and no beta1 / decay columns to the update kernels
  if (c->optimizer != PBT_OPT_RMSPROP && c->optimizer != PBT_OPT_SGD_MOMENTUM)
    return fail(nullptr, PBT_EUNSUPPORTED, "the actor-critic workload is built for RMSProp and SGD with momentum");
  if ((int64_t)c->batch * c->unroll * 4 > 48 * 1024) return fail(nullptr, PBT_EUNSUPPORTED, "batch x unroll above 12288 transitions per member");
  if (c->dims[L] < 2 || c->dims[L] > 32) return fail(nullptr, PBT_EUNSUPPORTED, "head width (actions + value) must be 2..32");
  for (int l = 0; l < L; ++l)
    if (c->dims[l] % 8) return fail(nullptr, PBT_EUNSUPPORTED, "torso widths must be multiples of 8");
  if (!(c->gamma >= 0.f && c->gamma <= 1.f)) return fail(nullptr, PBT_EINVAL, "gamma outside [0, 1]");
  const int64_t P = c->P, R = (int64_t)c->batch * (c->unroll + 1);
  a.rows = (int)R;
  for (int l = 0; l < L; ++l) {
    a.o_a[l] = w->take((size_t)P * R * c->dims[l] * 2);
    if (l < L - 1) {
      a.o_z[l] = w->take((size_t)P * R * c->dims[l + 1] * 2);
      a.o_dz[l] = w->take((size_t)P * R * c->dims[l + 1] * 2);
    }
  }
  a.o_out = w->take((size_t)P * R * 32 * 4);
  a.o_dout = w->take((size_t)P * R * 32 * 2);
  a.o_act = w->take((size_t)P * c->batch * c->unroll * 4);
  a.o_rew = w->take((size_t)P * c->batch * c->unroll * 4);
  a.o_lat = a.o_gout = 0;
  if (c->on_policy) {
    if (c->latent_dim < 1 || c->latent_dim > 64) return fail(nullptr, PBT_EINVAL, "latent_dim outside 1..64");
    // (LDS of the generator's kernels: the latents of a member's trajectories, plus an action each in the transition
    // kernel or a 64-component slab of the observation matrix, 65 doubles per latent component, in the observation kernel)
    if ((int64_t)c->batch * (c->latent_dim * 8 + 4) + (int64_t)c->latent_dim * 65 * 8 > 64 * 1024)
      return fail(nullptr, PBT_EUNSUPPORTED, "batch x latent_dim too large for the trajectory generator's LDS");
    if ((int64_t)R * c->dims[0] >= (1LL << 31)) return fail(nullptr, PBT_EUNSUPPORTED, "more than 2^31 observation elements per member");
    a.o_lat = w->take((size_t)P * c->batch * c->latent_dim * 8);
    for (int l = 1; l < L; ++l) a.o_ga[l] = w->take((size_t)P * c->batch * c->dims[l] * 2);
    a.o_gout = w->take((size_t)P * c->batch * 32 * 4);
  }
  return PBT_OK;
}

// Forward, loss, backward and update on the unroll that sits in the step's input buffers (observations in
// the first activation buffer, actions and rewards in theirs).
static pbt_status a2c_update(pbt_handle* h, hipStream_t s) {
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  const A2CPlan& a = p.a2c;
  const int P = c.P, B = c.batch, T = c.unroll, L = c.n_layers, R = a.rows;
  const int Kh = c.dims[L - 1], C = c.dims[L];
  const int64_t S = p.lay.stride;
  const Net net{L, c.dims, 0, c.act, PBT_ACT_NONE};
  bf16_t* A[PBT_MAX_DIMS]; bf16_t* Z[PBT_MAX_DIMS]; bf16_t* dZ[PBT_MAX_DIMS];
  for (int l = 0; l < L; ++l) { A[l] = h->sc<bf16_t>(a.o_a[l]); Z[l] = l < L - 1 ? h->sc<bf16_t>(a.o_z[l]) : nullptr; dZ[l] = l < L - 1 ? h->sc<bf16_t>(a.o_dz[l]) : nullptr; }
  const float* W32 = h->st<float>(p.o_w32);
  const bf16_t* W16 = h->st<bf16_t>(p.o_w16);
  float* G = h->sc<float>(p.o_grad);
  float* out = h->sc<float>(a.o_out);
  bf16_t* dout = h->sc<bf16_t>(a.o_dout);
  int32_t* act = h->sc<int32_t>(a.o_act);
  float* rew = h->sc<float>(a.o_rew);
  pbt_status st;
  if ((st = forward(h, net, L - 1, R, A, Z, nullptr, 0, s)) != PBT_OK) return st;
  PBT_LAUNCH(h, PBT_K_HEAD, s, head_fwd_loss(A[L - 1], (int64_t)R * Kh, W16 + p.lay.w_off[L - 1], S, W32 + p.lay.b_off[L - 1], S, nullptr,
                                             0, P, R, Kh, C, 0.f, -2, nullptr, out, 0, s));
  hipLaunchKernelGGL(a2c_loss_kernel, dim3(P), dim3(B * (T + 1) > 512 ? 1024 : B * (T + 1) > 256 ? 512 : 256), (size_t)B * T * sizeof(float), s, out, act, rew, h->st<float>(p.o_hyper), c.n_hyper, a.col_ent, B, T,
                     C - 1, c.gamma, c.value_cost, dout, h->st<float>(p.o_loss));
  PBT_HIP(h, hipGetLastError());
  {
    // (the bias gradient, column sums of dout, is a by-product of the same launch)
    GemmOperands wg{A[L - 1], Kh, (int64_t)R * Kh, true, dout, 32, (int64_t)R * 32, false, Kh, C, R, P};
    wg.colsum = G + p.lay.b_off[L - 1]; wg.colsum_stride = S;
    PBT_LAUNCH(h, PBT_K_HEAD, s, gemm_store_f32(wg, G + p.lay.w_off[L - 1], C, S, s));
  }
  PBT_LAUNCH(h, PBT_K_HEAD, s, head_dgrad(dout, W16 + p.lay.w_off[L - 1], S, Z[L - 2], dZ[L - 2], P, R, Kh, C, c.act, s));
  OptArgs oa{h->st<float>(p.o_w32), h->st<float>(p.o_opt0), nullptr, h->st<bf16_t>(p.o_w16), G, 0, S, h->st<float>(p.o_hyper),
             h->st<int32_t>(p.o_t), S, P, c.n_hyper, c.optimizer, p.col_lr, -1, -1, c.opt_const[0], c.opt_const[1], c.opt_const[2],
             c.opt_const[3]};
  const bool fused = c.fuse_optimizer != 0;
  if ((st = backward(h, net, L - 1, R, A, Z, dZ, true, fused ? &oa : nullptr, nullptr, nullptr, 0, s)) != PBT_OK) return st;
  if (fused) return optimizer_rest(h, oa, 0, L, L - 1, S, s);
  PBT_LAUNCH(h, PBT_K_OPTIMIZER, s, optimizer_step(oa, s));
  return PBT_OK;
}

pbt_status a2c_step(pbt_handle* h, const float* obs, const int32_t* actions, const float* rewards, uint32_t step, hipStream_t s) {
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  const A2CPlan& a = p.a2c;
  const int P = c.P, B = c.batch, T = c.unroll, R = a.rows;
  // a trajectory is one "row" of (T+1) * d observations; B of them are drawn per member
  PBT_LAUNCH(h, PBT_K_FETCH, s, gather_rows(obs, c.n_train, (T + 1) * c.dims[0], P, B, (int64_t)R * c.dims[0], step, c.seed,
                                            h->sc<bf16_t>(a.o_a[0]), h->st<int32_t>(p.o_t), s));
  hipLaunchKernelGGL(a2c_fetch_aux_kernel, dim3(P), dim3(64), 0, s, actions, rewards, c.n_train, B, T, step, (uint32_t)c.seed,
                     (uint32_t)(c.seed >> 32), h->sc<int32_t>(a.o_act), h->sc<float>(a.o_rew), h->st<float>(p.o_hist));
  PBT_HIP(h, hipGetLastError());
  return a2c_update(h, s);
}

// ---- on-policy unrolls (Section 4.1.1: agents act with their current policy) -------------------------

constexpr uint32_t DOMAIN_ENV = 32;

// Four standard normals from one Philox counter: Box-Muller on the word pairs (0,1) and (2,3), in double.
__device__ __forceinline__ void env_normal4(uint32_t step, uint32_t member, uint32_t domain, uint32_t counter, uint32_t k0,
                                            uint32_t k1, double* v) {
  const u32x4 w = philox4x32_10(step, member, domain, counter, k0, k1);
  // (cos and sin of 2 pi u through sincospi(2 u): no reduction of a large argument modulo pi)
  const double r1 = sqrt(-2.0 * log(philox_unit(w.x))), r2 = sqrt(-2.0 * log(philox_unit(w.z)));
  double s1, c1, s2, c2;
  sincospi(2.0 * philox_unit(w.y), &s1, &c1);
  sincospi(2.0 * philox_unit(w.w), &s2, &c2);
  v[0] = r1 * c1; v[1] = r1 * s1; v[2] = r2 * c2; v[3] = r2 * s2;
}
// The same four normals to float accuracy (relative error about 2e-7), for values that are stored as bf16 anyway
// (the observation noise: 512 of them per trajectory and time step, where the double-precision log, sqrt and
// sincospi above were the whole cost of the generator).  The uniforms and the argument reductions stay in double:
// -log(u) through log1p(u - 1) above one half (u - 1 is exact in double, so no digits are lost next to 1), and the
// angle 2 pi u reduced to pi f with |f| <= 1/4 before it is rounded to float, then rotated back by quadrant.
__device__ __forceinline__ void env_normal_pair_f32(uint32_t wr, uint32_t wa, float* cosv, float* sinv) {
  const double u = philox_unit(wr);
  const float nl = u > 0.5 ? -log1pf((float)(u - 1.0)) : -logf((float)u);
  const float r = sqrtf(2.f * nl);
  const double x = 2.0 * philox_unit(wa);          // angle / pi, in (0, 2)
  const double q = rint(2.0 * x);                  // nearest multiple of 1/2
  const float f = (float)(x - 0.5 * q);
  const float s0 = sinpif(f), c0 = cospif(f);
  const int k = (int)q & 3;
  const float s = k == 0 ? s0 : k == 1 ? c0 : k == 2 ? -s0 : -c0;
  const float c = k == 0 ? c0 : k == 1 ? -s0 : k == 2 ? -c0 : s0;
  *cosv = r * c; *sinv = r * s;
}
__device__ __forceinline__ void env_normal4_f32(uint32_t step, uint32_t member, uint32_t domain, uint32_t counter, uint32_t k0,
                                                uint32_t k1, float* v) {
  const u32x4 w = philox4x32_10(step, member, domain, counter, k0, k1);
  env_normal_pair_f32(w.x, w.y, &v[0], &v[1]);
  env_normal_pair_f32(w.z, w.w, &v[2], &v[3]);
}
__device__ __forceinline__ double env_normal(uint32_t step, uint32_t member, uint32_t domain, uint32_t e, uint32_t k0, uint32_t k1) {
  double v[4];
  env_normal4(step, member, domain, e >> 2, k0, k1, v);
  return v[e & 3];
}

struct EnvArgs {
  A2CEnv env;
  int nz, n_act, d, B, T, rows;        // rows = B (T + 1) observation rows per member
  uint32_t step, k0, k1;
  double* z;                           // [P][B][nz]
  const float* head_out;               // [P][B][32]: head outputs of the policy at time t - 1
  int32_t* act; float* rew;            // [P][B][T]
  bf16_t* obs;                         // [P][rows][d]
  int32_t* t_count;
};

// One time step of the latent system for all trajectories of one member (one workgroup per member).
// t > 0: one thread per trajectory draws a_{t-1} from the policy's head outputs and books r_{t-1}; then one
// thread per (trajectory, four latent components) moves the latent to z_t (four normals = one Philox counter).
// t = 0: z_0 is drawn.
__global__ __launch_bounds__(256) void a2c_env_transition_kernel(EnvArgs a, int t) {
  extern __shared__ double zs[];                 // [B][nz] latent before the transition
  int* action = reinterpret_cast<int*>(zs + (size_t)a.B * a.nz);   // [B]
  const int i = blockIdx.x;
  const int nz = a.nz, B = a.B, T = a.T, tt = t - 1;
  double* zm = a.z + (int64_t)i * B * nz;
  if (t > 0) {
    for (int e = threadIdx.x; e < B * nz; e += blockDim.x) zs[e] = zm[e];
    __syncthreads();
    for (int r = threadIdx.x; r < B; r += blockDim.x) {
      const float* lg = a.head_out + ((int64_t)i * B + r) * 32;
      double mx = -INFINITY;
      for (int c = 0; c < a.n_act; ++c) mx = fmax(mx, (double)lg[c]);
      double ex[32], se = 0.0;
      for (int c = 0; c < a.n_act; ++c) { ex[c] = exp((double)lg[c] - mx); se += ex[c]; }
      const double u = philox_unit(philox4x32_10(a.step, i, DOMAIN_ENV + 2, (uint32_t)(r * T + tt), a.k0, a.k1).x);
      double cdf = 0.0;
      int act = 0;
      for (int c = 0; c < a.n_act; ++c) { cdf += ex[c] / se; act += cdf <= u ? 1 : 0; }
      act = act < a.n_act - 1 ? act : a.n_act - 1;
      double rw = 0.0;
      for (int k = 0; k < nz; ++k) rw += a.env.w[k] * zs[r * nz + k];
      rw += a.env.noise[1] * env_normal(a.step, i, DOMAIN_ENV + 3, (uint32_t)(r * T + tt), a.k0, a.k1);
      a.act[((int64_t)i * B + r) * T + tt] = act;
      a.rew[((int64_t)i * B + r) * T + tt] = (float)rw;
      action[r] = act;
    }
    __syncthreads();
  }
  // element e = (trajectory, component) of the normal stream of this time step: z_0 (t = 0) or zeta_{t-1}
  const uint32_t domain = t == 0 ? DOMAIN_ENV + 0 : DOMAIN_ENV + 4;
  const int quads = (nz + 3) / 4;
  for (int item = threadIdx.x; item < B * quads; item += blockDim.x) {
    const int r = item / quads, k0 = (item - r * quads) * 4;
    const uint32_t e0 = (uint32_t)((t == 0 ? r : r * T + tt) * nz + k0);
    double v[4];
    if ((e0 & 3u) == 0) {
      env_normal4(a.step, i, domain, e0 >> 2, a.k0, a.k1, v);
    } else {
      for (int q = 0; q < 4; ++q) v[q] = env_normal(a.step, i, domain, e0 + q, a.k0, a.k1);
    }
    for (int q = 0; q < 4 && k0 + q < nz; ++q) {
      const int k = k0 + q;
      double zn = v[q];
      if (t > 0) {
        double acc = 0.0;
        for (int j = 0; j < nz; ++j) acc += a.env.A[k * nz + j] * zs[r * nz + j];
        zn = acc + a.env.B[k * a.n_act + action[r]] + a.env.noise[2] * v[q];
      }
      zm[r * nz + k] = zn;
    }
  }
  if (t == 0 && threadIdx.x == 0) a.t_count[i] += 1;
}

// The observations o_t of all trajectories of one member (blockIdx.y) for a slab of 64 observation components
// (blockIdx.x), written where the step (and the policy's next forward pass) reads them.  The slab's rows of C go
// through LDS, transposed, so that neighbouring lanes read neighbouring addresses there (read from memory in the
// order the sum wants them, a wavefront's load touched 64 separate lines and the L1's access rate set the time);
// a thread handles runs of four components, i.e. one Philox counter.
constexpr int OBS_SLAB = 64;   // (the plan's LDS check assumes 64)
__global__ __launch_bounds__(256) void a2c_env_observe_kernel(EnvArgs a, int t) {
  extern __shared__ double obs_lds[];
  const int nz = a.nz, B = a.B, i = blockIdx.y, j_first = blockIdx.x * OBS_SLAB;
  double* Ct = obs_lds;                         // [nz][OBS_SLAB + 1]
  double* zs = obs_lds + nz * (OBS_SLAB + 1);   // [B][nz]
  for (int e = threadIdx.x; e < OBS_SLAB * nz; e += blockDim.x) {
    const int j = e / nz, k = e - j * nz;
    Ct[k * (OBS_SLAB + 1) + j] = j_first + j < a.d ? a.env.C[(int64_t)(j_first + j) * nz + k] : 0.0;
  }
  for (int e = threadIdx.x; e < B * nz; e += blockDim.x) zs[e] = a.z[(int64_t)i * B * nz + e];
  __syncthreads();
  constexpr int RUNS = OBS_SLAB / 4;
  for (int item = threadIdx.x; item < B * RUNS; item += blockDim.x) {
    const int r = item / RUNS, g = item - r * RUNS, j0 = j_first + 4 * g;
    if (j0 >= a.d) continue;
    const int64_t row = (int64_t)r * (a.T + 1) + t;
    float v[4];
    env_normal4_f32(a.step, i, DOMAIN_ENV + 1, (uint32_t)((row * a.d + j0) >> 2), a.k0, a.k1, v);
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int k = 0; k < nz; ++k) {
      const double zk = zs[r * nz + k];
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] += Ct[k * (OBS_SLAB + 1) + 4 * g + e] * zk;
    }
    float o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (float)(acc[e] + a.env.noise[0] * (double)v[e]);
    *reinterpret_cast<uint2*>(a.obs + ((int64_t)i * a.rows + row) * a.d + j0) = make_uint2(f2bf_pair(o[0], o[1]), f2bf_pair(o[2], o[3]));
  }
}

// ---- the whole unroll of one member in one kernel -------------------------------------------------------------
// One workgroup per member runs the T + 1 rounds of (transition and action draw, observation, policy) back to
// back: latents, the round's observations and the hidden activations stay in LDS, the member's bf16 weights are
// streamed through LDS a 64-deep slab at a time (fetched with eight neighbouring lanes on 128 contiguous bytes,
// transposed on the way in through a lane exchange, the next slab's loads in flight while this one is multiplied),
// and every layer is a 32 x N x K product on the matrix cores with the trajectories as one 32-row block.  The same
// arithmetic as the kernels above and the batched GEMMs (bf16 operands, float accumulation, bias and activation in
// float, activations rounded to bf16 between layers, float head outputs); sums run in a different order.
// Shapes: at most 32 trajectories, observation width a multiple of 64, hidden widths 64, 128 or 256, at most 32
// head outputs.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 ro_frag_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float ro_acc_t;
constexpr int RO_WP = 64 + 4;     // LDS pitch (elements) of a transposed weight slab [N][64]
constexpr int RO_MAX_HIDDEN = 3;
constexpr int RO_THREADS = 512;   // 8 wavefronts: with one workgroup per compute unit, two per SIMD to overlap each other's latencies

struct RolloutArgs {
  EnvArgs e;
  const bf16_t* W16; const float* W32; int64_t stride;
  int n_hidden, act, hmax;
  int dims[RO_MAX_HIDDEN + 2];
  int64_t w_off[RO_MAX_HIDDEN + 1], b_off[RO_MAX_HIDDEN + 1];
};

// Wt[n][k] (pitch RO_WP) = W[k0 + k][n] for k < 64, n < N: rows of N contiguous values in memory.  A thread
// holds N / 32 pieces of 16 bytes; piece `it` is row (it % 512) / 8, columns 64 (it / 512) + 8 (it % 8) ...
struct RoStaged { uint4 v[4]; };
template <int N>
__device__ __forceinline__ void ro_fetch(const bf16_t* __restrict__ W, int k0, RoStaged& r) {
#pragma unroll
  for (int j = 0; j < N / 64; ++j) {
    const int it = threadIdx.x + RO_THREADS * j;
    r.v[j] = *reinterpret_cast<const uint4*>(W + (int64_t)(k0 + ((it & 511) >> 3)) * N + 64 * (it >> 9) + 8 * (it & 7));
  }
}
template <int N>
__device__ __forceinline__ void ro_put(const RoStaged& r, bf16_t* Wt) {
#pragma unroll
  for (int j = 0; j < N / 64; ++j) {
    const int it = threadIdx.x + RO_THREADS * j;
    const int row = (it & 511) >> 3, n0 = 64 * (it >> 9) + 8 * (it & 7), odd = row & 1;
    const uint4 v = r.v[j];
    // lanes 8 apart hold rows k and k ^ 1: they exchange halves so that each writes four (k, k + 1) pairs
    const uint32_t g0 = __shfl_xor(odd ? v.x : v.z, 8), g1 = __shfl_xor(odd ? v.y : v.w, 8);
    const uint32_t e0 = odd ? g0 : v.x, e1 = odd ? g1 : v.y, o0 = odd ? v.z : g0, o1 = odd ? v.w : g1;
    uint32_t* out = reinterpret_cast<uint32_t*>(Wt) + (n0 + 4 * odd) * (RO_WP / 2) + (row >> 1);
    out[0] = (e0 & 0xffffu) | (o0 << 16);
    out[RO_WP / 2] = (e0 >> 16) | (o0 & 0xffff0000u);
    out[2 * (RO_WP / 2)] = (e1 & 0xffffu) | (o1 << 16);
    out[3 * (RO_WP / 2)] = (e1 >> 16) | (o1 & 0xffff0000u);
  }
}
__device__ __forceinline__ ro_frag_t ro_wfrag(const bf16_t* Wt, int n, int c, int hf) {
  const bf16_t* p = Wt + n * RO_WP + 16 * c + 8 * hf;   // 8-byte aligned
  const uint2 lo = *reinterpret_cast<const uint2*>(p), hi = *reinterpret_cast<const uint2*>(p + 4);
  const uint4 v = make_uint4(lo.x, lo.y, hi.x, hi.y);
  return __builtin_bit_cast(ro_frag_t, v);
}

// out[r][n] = act(sum_k in[r][k] W[k][n] + b[n]) for the 32 rows in LDS; N in {64, 128, 256}, K a multiple of 64
template <int N>
__device__ __forceinline__ void ro_dense(const bf16_t* in, int pin, int K, const bf16_t* __restrict__ W, const float* __restrict__ bias,
                                         int act, bf16_t* out, int pout, bf16_t* Wt) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, lr = lane & 31, hf = lane >> 5;
  const bool mine = w < N / 32;   // wavefront w owns columns 32 w .. 32 w + 31
  ro_acc_t acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  // Three register sets: the slabs k0 + 64 and k0 + 128 are on their way while slab k0 is written to LDS and
  // multiplied (one workgroup per compute unit: nothing else hides the memory latency).  Every slab step issues
  // the same loads, past the end of W's rows too (the last slab again, never multiplied), so that the number of
  // loads in flight at each wait is known when the kernel is compiled; with conditional loads every wait was for
  // all of them, i.e. a full memory latency per slab.
  const int last = K - 64;
  RoStaged st[3];
  ro_fetch<N>(W, 0, st[0]);
  ro_fetch<N>(W, min(64, last), st[1]);
  ro_fetch<N>(W, min(128, last), st[2]);
  auto slab = [&](RoStaged& r, int k0) {
    ro_put<N>(r, Wt);
    __syncthreads();
    ro_fetch<N>(W, min(k0 + 192, last), r);
    if (mine && k0 < K) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const ro_frag_t af = *reinterpret_cast<const ro_frag_t*>(in + lr * pin + k0 + 16 * c + 8 * hf);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ro_wfrag(Wt, 32 * w + lr, c, hf), af, acc, 0, 0, 0);
      }
    }
    __syncthreads();
  };
  for (int k0 = 0; k0 < K; k0 += 192) {
    slab(st[0], k0);
    slab(st[1], k0 + 64);
    slab(st[2], k0 + 128);
  }
  // accumulator register e of lane (lr, hf): row lr, column 32 w + 8 (e / 4) + 4 hf + e % 4
  if (mine) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int n0 = 32 * w + 8 * g + 4 * hf;
      const float4 b = *reinterpret_cast<const float4*>(bias + n0);
      const float a0 = act_fwd(acc[4 * g] + b.x, act), a1 = act_fwd(acc[4 * g + 1] + b.y, act);
      const float a2 = act_fwd(acc[4 * g + 2] + b.z, act), a3 = act_fwd(acc[4 * g + 3] + b.w, act);
      *reinterpret_cast<uint2*>(out + lr * pout + n0) = make_uint2(f2bf_pair(a0, a1), f2bf_pair(a2, a3));
    }
  }
  __syncthreads();
}

// hout[r][c] = sum_k in[r][k] W[k][c] + b[c] for c < C <= 32 (float): the whole K x C matrix is staged at once
__device__ __forceinline__ void ro_head(const bf16_t* in, int pin, int K, const bf16_t* __restrict__ W, const float* __restrict__ bias, int C,
                                        float* hout, bf16_t* Wt) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, lr = lane & 31, hf = lane >> 5;
  const int pw = K + 8;
  for (int e = threadIdx.x; e < 32 * K; e += RO_THREADS) {
    const int c = e / K, k = e - c * K;
    Wt[c * pw + k] = c < C ? W[(int64_t)k * C + c] : (bf16_t)0;
  }
  __syncthreads();
  // the eight wavefronts share the contraction (k-blocks of 16 in turn); partial sums are added in wavefront order
  ro_acc_t acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  for (int kb = w; kb < K / 16; kb += RO_THREADS / 64) {
    const ro_frag_t af = *reinterpret_cast<const ro_frag_t*>(in + lr * pin + 16 * kb + 8 * hf);
    const ro_frag_t wf = *reinterpret_cast<const ro_frag_t*>(Wt + lr * pw + 16 * kb + 8 * hf);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, af, acc, 0, 0, 0);
  }
  __syncthreads();   // the staged weights are not needed any more: their space takes the partial sums
  float* part = reinterpret_cast<float*>(Wt);   // [8][32][33]
#pragma unroll
  for (int e = 0; e < 16; ++e) part[(w * 32 + lr) * 33 + 8 * (e / 4) + 4 * hf + e % 4] = acc[e];
  __syncthreads();
  for (int e = threadIdx.x; e < 32 * 32; e += RO_THREADS) {
    const int r = e >> 5, c = e & 31;
    float sum = part[r * 33 + c];
    for (int v = 1; v < RO_THREADS / 64; ++v) sum += part[(32 * v + r) * 33 + c];
    hout[e] = sum + (c < C ? bias[c] : 0.f);
  }
  __syncthreads();
}

// bytes of the kernel's LDS ahead of the 16-byte aligned activation buffers
__host__ __device__ inline size_t ro_front_bytes(int nz, int n_act, int d) {
  const size_t b = (size_t)(2 * 32 * nz + nz * nz + nz * n_act + nz) * 8 + (size_t)(nz * (d + 1) + 32 * nz + 32 * 32 + 32) * 4;
  return (b + 15) & ~(size_t)15;
}
__global__ __launch_bounds__(RO_THREADS) void a2c_rollout_kernel(RolloutArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char ro_lds[];
  const EnvArgs& e = a.e;
  const int i = blockIdx.x, nz = e.nz, B = e.B, T = e.T, d = e.d, n_act = e.n_act;
  // LDS.  doubles: latents (two copies), A, B, w of the latent system; floats: C transposed (kept for the whole
  // unroll), the round's latents, head outputs; actions; then, 16-byte aligned, the observations, two activation
  // buffers and the weight slab (which doubles as scratch of the action draw and of the head)
  double* zs = reinterpret_cast<double*>(ro_lds);                 // [2][32][nz]
  double* As = zs + 2 * 32 * nz;                                  // [nz][nz]
  double* Bs = As + nz * nz;                                      // [nz][n_act]
  double* ws = Bs + nz * n_act;                                   // [nz]
  float* Ct = reinterpret_cast<float*>(ws + nz);                  // [nz][d + 1]
  float* zf = Ct + nz * (d + 1);                                  // [32][nz]
  float* hout = zf + 32 * nz;                                     // [32][32]
  int* action = reinterpret_cast<int*>(hout + 32 * 32);           // [32]
  bf16_t* X0 = reinterpret_cast<bf16_t*>(ro_lds + ro_front_bytes(nz, n_act, d));   // [32][d + 8]
  bf16_t* XA = X0 + 32 * (d + 8);                                 // [32][hmax + 8]
  bf16_t* XB = XA + 32 * (a.hmax + 8);
  bf16_t* Wt = XB + 32 * (a.hmax + 8);                            // [256][RO_WP]
  double* ex = reinterpret_cast<double*>(Wt);                     // [32][32] during the action draw
  const bf16_t* W16 = a.W16 + (int64_t)i * a.stride;
  const float* W32 = a.W32 + (int64_t)i * a.stride;
  if (threadIdx.x == 0) e.t_count[i] += 1;
  for (int x = threadIdx.x; x < nz * nz; x += RO_THREADS) As[x] = e.env.A[x];
  for (int x = threadIdx.x; x < nz * n_act; x += RO_THREADS) Bs[x] = e.env.B[x];
  for (int x = threadIdx.x; x < nz; x += RO_THREADS) ws[x] = e.env.w[x];
  for (int x = threadIdx.x; x < d * nz; x += RO_THREADS) {
    const int j = x / nz, k = x - j * nz;
    Ct[k * (d + 1) + j] = (float)e.env.C[x];
  }
  const double noise_obs = e.env.noise[0], noise_rew = e.env.noise[1], noise_lat = e.env.noise[2];
  // rows past the last trajectory stay zero in every activation buffer
  for (int x = threadIdx.x; x < 32 * (d + 8) / 2; x += RO_THREADS) reinterpret_cast<uint32_t*>(X0)[x] = 0u;
  const int quads = (nz + 3) / 4;
  __syncthreads();
  for (int t = 0; t <= T; ++t) {
    const int tt = t - 1;
    double* zo = zs + (t & 1) * 32 * nz;          // latents before this round's transition
    double* zn_ = zs + ((t + 1) & 1) * 32 * nz;   // and after
    if (t > 0) {
      // a_{t-1} from the head outputs: the exponentials with one thread per (trajectory, action), then the
      // cumulative distribution with one thread per trajectory
      for (int x = threadIdx.x; x < B * 32; x += RO_THREADS) {
        const int r = x >> 5, c = x & 31;
        const float* lg = hout + r * 32;
        float mx = -INFINITY;
        for (int q = 0; q < n_act; ++q) mx = fmaxf(mx, lg[q]);
        ex[x] = c < n_act ? exp((double)lg[c] - (double)mx) : 0.0;
      }
      __syncthreads();
      for (int r = threadIdx.x; r < B; r += RO_THREADS) {
        double se = 0.0;
        for (int c = 0; c < n_act; ++c) se += ex[r * 32 + c];
        const double u = philox_unit(philox4x32_10(e.step, i, DOMAIN_ENV + 2, (uint32_t)(r * T + tt), e.k0, e.k1).x);
        double cdf = 0.0;
        int act = 0;
        for (int c = 0; c < n_act; ++c) { cdf += ex[r * 32 + c] / se; act += cdf <= u ? 1 : 0; }
        act = act < n_act - 1 ? act : n_act - 1;
        double rw = 0.0;
        for (int k = 0; k < nz; ++k) rw += ws[k] * zo[r * nz + k];
        rw += noise_rew * env_normal(e.step, i, DOMAIN_ENV + 3, (uint32_t)(r * T + tt), e.k0, e.k1);
        e.act[((int64_t)i * B + r) * T + tt] = act;
        e.rew[((int64_t)i * B + r) * T + tt] = (float)rw;
        action[r] = act;
      }
      __syncthreads();
    }
    const uint32_t domain = t == 0 ? DOMAIN_ENV + 0 : DOMAIN_ENV + 4;
    for (int item = threadIdx.x; item < B * quads; item += RO_THREADS) {
      const int r = item / quads, k0 = (item - r * quads) * 4;
      const uint32_t e0 = (uint32_t)((t == 0 ? r : r * T + tt) * nz + k0);
      double v[4];
      if ((e0 & 3u) == 0) {
        env_normal4(e.step, i, domain, e0 >> 2, e.k0, e.k1, v);
      } else {
        for (int q = 0; q < 4; ++q) v[q] = env_normal(e.step, i, domain, e0 + q, e.k0, e.k1);
      }
      for (int q = 0; q < 4 && k0 + q < nz; ++q) {
        const int k = k0 + q;
        double zv = v[q];
        if (t > 0) {
          double acc = 0.0;
          for (int j = 0; j < nz; ++j) acc += As[k * nz + j] * zo[r * nz + j];
          zv = acc + Bs[k * n_act + action[r]] + noise_lat * v[q];
        }
        zn_[r * nz + k] = zv;
        zf[r * nz + k] = (float)zv;
      }
    }
    __syncthreads();
    // observations of round t: to memory (the update reads them) and to X0 (the policy's input).  The sum C z runs
    // in float (the result is stored as bf16; the latents themselves stay in double from round to round).
    {
      const int runs = d / 4;
      for (int item = threadIdx.x; item < B * runs; item += RO_THREADS) {
        const int r = item / runs, g = item - r * runs, j0 = 4 * g;
        const int64_t row = (int64_t)r * (T + 1) + t;
        float v[4];
        env_normal4_f32(e.step, i, DOMAIN_ENV + 1, (uint32_t)((row * d + j0) >> 2), e.k0, e.k1, v);
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < nz; ++k) {
          const float zk = zf[r * nz + k];
#pragma unroll
          for (int q = 0; q < 4; ++q) acc[q] = fmaf(Ct[k * (d + 1) + j0 + q], zk, acc[q]);
        }
        float o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) o[q] = fmaf((float)noise_obs, v[q], acc[q]);
        const uint2 packed = make_uint2(f2bf_pair(o[0], o[1]), f2bf_pair(o[2], o[3]));
        *reinterpret_cast<uint2*>(e.obs + ((int64_t)i * e.rows + row) * d + j0) = packed;
        *reinterpret_cast<uint2*>(X0 + r * (d + 8) + j0) = packed;
      }
      __syncthreads();
    }
    if (t == T) break;
    // the policy on the round's observations
    const bf16_t* in = X0;
    int pin = d + 8, K = d;
    for (int l = 0; l < a.n_hidden; ++l) {
      bf16_t* out = l & 1 ? XB : XA;
      const int N = a.dims[l + 1];
      if (N == 256) ro_dense<256>(in, pin, K, W16 + a.w_off[l], W32 + a.b_off[l], a.act, out, a.hmax + 8, Wt);
      else if (N == 128) ro_dense<128>(in, pin, K, W16 + a.w_off[l], W32 + a.b_off[l], a.act, out, a.hmax + 8, Wt);
      else ro_dense<64>(in, pin, K, W16 + a.w_off[l], W32 + a.b_off[l], a.act, out, a.hmax + 8, Wt);
      in = out; pin = a.hmax + 8; K = a.dims[l + 1];
    }
    ro_head(in, pin, K, W16 + a.w_off[a.n_hidden], W32 + a.b_off[a.n_hidden], a.dims[a.n_hidden + 1], hout, Wt);
  }
}

// LDS of the kernel above for a shape, 0 if the shape is not covered
static size_t rollout_lds_bytes(const pbt_config& c) {
  const int L = c.n_layers, d = c.dims[0], C = c.dims[L];
  if (c.batch > 32 || d % 64 || L - 1 < 1 || L - 1 > RO_MAX_HIDDEN || C > 32) return 0;
  int hmax = 0;
  for (int l = 1; l < L; ++l) {
    if (c.dims[l] != 64 && c.dims[l] != 128 && c.dims[l] != 256) return 0;
    hmax = c.dims[l] > hmax ? c.dims[l] : hmax;
  }
  const size_t wt = (size_t)256 * RO_WP * 2;   // also holds the head's [32][K + 8] bf16 and its 8 x 32 x 33 partial sums
  if ((size_t)32 * (hmax + 8) * 2 > wt || (size_t)(RO_THREADS / 64) * 32 * 33 * 4 > wt) return 0;
  if ((size_t)32 * 32 * 8 > wt) return 0;      // (and the exponentials of the action draw)
  const size_t bytes = ro_front_bytes(c.latent_dim, C - 1, d) + (size_t)32 * (d + 8) * 2 + (size_t)2 * 32 * (hmax + 8) * 2 + wt;
  return bytes <= 160 * 1024 ? bytes : 0;
}

// Pushes the unroll's return (mean over trajectories of the summed rewards, in double, trajectories in order)
// into the member's history ring.
__global__ __launch_bounds__(64) void a2c_push_return_kernel(const float* __restrict__ rew, int B, int T, float* __restrict__ hist) {
  const int i = blockIdx.x;
  __shared__ double tsum[64];
  double mean = 0.0;
  for (int r0 = 0; r0 < B; r0 += 64) {
    const int r = r0 + threadIdx.x;
    double sacc = 0.0;
    if (r < B)
      for (int t = 0; t < T; ++t) sacc += (double)rew[((int64_t)i * B + r) * T + t];
    tsum[threadIdx.x] = sacc;
    __syncthreads();
    if (threadIdx.x == 0)
      for (int k = 0; k < 64 && r0 + k < B; ++k) mean += tsum[k];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    float* hrow = hist + (int64_t)i * HIST_PITCH;
    const int n = __float_as_int(hrow[HIST_SLOTS]);
    hrow[n % HIST_SLOTS] = (float)(mean / (double)B);
    hrow[HIST_SLOTS] = __int_as_float(n + 1);
  }
}

pbt_status a2c_step_on_policy(pbt_handle* h, const A2CEnv& env, uint32_t step, hipStream_t s) {
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  const A2CPlan& a = p.a2c;
  const int P = c.P, B = c.batch, T = c.unroll, L = c.n_layers, R = a.rows, d = c.dims[0];
  const int Kh = c.dims[L - 1], C = c.dims[L];
  const int64_t S = p.lay.stride;
  const float* W32 = h->st<float>(p.o_w32);
  const bf16_t* W16 = h->st<bf16_t>(p.o_w16);
  bf16_t* obs = h->sc<bf16_t>(a.o_a[0]);
  float* gout = h->sc<float>(a.o_gout);
  EnvArgs ea{env, c.latent_dim, C - 1, d, B, T, R, step, (uint32_t)c.seed, (uint32_t)(c.seed >> 32), h->sc<double>(a.o_lat), gout,
             h->sc<int32_t>(a.o_act), h->sc<float>(a.o_rew), obs, h->st<int32_t>(p.o_t)};
  if (const size_t lds = rollout_lds_bytes(c)) {
    RolloutArgs ra{};
    ra.e = ea; ra.W16 = W16; ra.W32 = W32; ra.stride = S; ra.n_hidden = L - 1; ra.act = c.act; ra.hmax = 0;
    for (int l = 0; l <= L; ++l) ra.dims[l] = c.dims[l];
    for (int l = 1; l < L; ++l) ra.hmax = c.dims[l] > ra.hmax ? c.dims[l] : ra.hmax;
    for (int l = 0; l < L; ++l) { ra.w_off[l] = p.lay.w_off[l]; ra.b_off[l] = p.lay.b_off[l]; }
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(a2c_rollout_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    PBT_HIP(h, attr);
    hipLaunchKernelGGL(a2c_rollout_kernel, dim3(P), dim3(RO_THREADS), lds, s, ra);
    PBT_HIP(h, hipGetLastError());
    hipLaunchKernelGGL(a2c_push_return_kernel, dim3(P), dim3(64), 0, s, h->sc<float>(a.o_rew), B, T, h->st<float>(p.o_hist));
    PBT_HIP(h, hipGetLastError());
    return a2c_update(h, s);
  }
  for (int t = 0; t <= T; ++t) {
    hipLaunchKernelGGL(a2c_env_transition_kernel, dim3(P), dim3(256), (size_t)B * c.latent_dim * sizeof(double) + (size_t)B * sizeof(int), s, ea, t);
    PBT_HIP(h, hipGetLastError());
    hipLaunchKernelGGL(a2c_env_observe_kernel, dim3((d + OBS_SLAB - 1) / OBS_SLAB, P), dim3(256),
                       ((size_t)c.latent_dim * (OBS_SLAB + 1) + (size_t)B * c.latent_dim) * sizeof(double), s, ea, t);
    PBT_HIP(h, hipGetLastError());
    if (t == T) break;
    // the policy on the B observations of time t: rows t, t + (T+1), ... of the member's observation buffer
    for (int l = 0; l < L - 1; ++l) {
      const int K = c.dims[l], N = c.dims[l + 1];
      const bf16_t* in = l == 0 ? obs + (int64_t)t * d : h->sc<bf16_t>(a.o_ga[l]);
      GemmOperands o{in, l == 0 ? (int64_t)(T + 1) * d : (int64_t)K, l == 0 ? (int64_t)R * d : (int64_t)B * K, false,
                     W16 + p.lay.w_off[l], N, S, false, B, N, K, P};
      PBT_LAUNCH(h, PBT_K_FETCH, s, gemm_bias_act(o, W32 + p.lay.b_off[l], S, nullptr, h->sc<bf16_t>(a.o_ga[l + 1]), N, (int64_t)B * N, c.act, s));
    }
    PBT_LAUNCH(h, PBT_K_FETCH, s, head_fwd_loss(h->sc<bf16_t>(a.o_ga[L - 1]), (int64_t)B * Kh, W16 + p.lay.w_off[L - 1], S, W32 + p.lay.b_off[L - 1], S,
                                                nullptr, 0, P, B, Kh, C, 0.f, -2, nullptr, gout, 0, s));
  }
  hipLaunchKernelGGL(a2c_push_return_kernel, dim3(P), dim3(64), 0, s, h->sc<float>(a.o_rew), B, T, h->st<float>(p.o_hist));
  PBT_HIP(h, hipGetLastError());
  return a2c_update(h, s);
}

pbt_status a2c_eval(pbt_handle* h, hipStream_t s) {
  const int P = h->cfg.P;
  hipLaunchKernelGGL(a2c_score_kernel, dim3((P + 63) / 64), dim3(64), 0, s, h->st<float>(h->plan.o_hist), P, h->st<float>(h->plan.o_score));
  PBT_HIP(h, hipGetLastError());
  return PBT_OK;
}

}  // namespace pbt
