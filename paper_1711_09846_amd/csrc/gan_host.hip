// The GAN workload (Section 4.3.1 of the PBT paper: generator and discriminator trained with Adam,
// each with its own learning rate per member, both copied on exploit, scored by a sample-quality
// metric that is not the training loss).  Host side: checks, scratch carve-up and the kernel
// sequences of one population step (discriminator update, then generator update through the updated
// discriminator) and of the MMD score.
#include <cstring>

#include "common.h"
#include "dense_host.h"
#include "philox.h"

namespace pbt {

namespace {

// ---- kernels of the WGAN-GP step (Section 4.3.1) -------------------------------------------------

constexpr uint32_t DOMAIN_GP_EPS = 14;

// Rows 2B .. 3B-1 of the critic's input buffer: xhat_r = eps_r x_r + (1 - eps_r) G(z)_r from the real rows
// 0 .. B-1 and the generated rows B .. 2B-1 (both bf16 already), eps_r from Philox counter
// (step, member, 14, counter0 + r); the sum is formed in double and rounded once.
__global__ __launch_bounds__(256) void wgan_interpolate_kernel(bf16_t* __restrict__ X, int B, int D, uint32_t step, uint32_t counter0,
                                                               uint32_t k0, uint32_t k1) {
  const int r = blockIdx.x, i = blockIdx.y;
  const double eps = philox_unit(philox4x32_10(step, (uint32_t)i, DOMAIN_GP_EPS, counter0 + (uint32_t)r, k0, k1).x);
  bf16_t* __restrict__ base = X + (int64_t)i * 3 * B * D;
  const bf16_t* __restrict__ xr = base + (int64_t)r * D;
  const bf16_t* __restrict__ xf = base + (int64_t)(B + r) * D;
  bf16_t* __restrict__ xh = base + (int64_t)(2 * B + r) * D;
  for (int c = threadIdx.x; c < D; c += blockDim.x)
    xh[c] = d2bf(eps * (double)bf2f(xr[c]) + (1.0 - eps) * (double)bf2f(xf[c]));
}

// One workgroup per member.  out: the critic's outputs, float [P][rows][32], column 0.
// critic (rows = 3B): loss[2 i] = mean out[B..2B) - mean out[0..B) (the penalty is added later), and the
// gradient of the outputs: -1/B on the real rows, +1/B on the generated rows, 1 on the interpolated rows (which
// starts the input-gradient pass).  generator (rows = B): loss[2 i + 1] = -mean out, gradient -1/B.
__global__ __launch_bounds__(256) void wgan_head_kernel(const float* __restrict__ out, int B, int rows, int generator,
                                                        bf16_t* __restrict__ dlogits, float* __restrict__ loss) {
  const int i = blockIdx.x;
  for (int r = threadIdx.x; r < rows; r += blockDim.x) {
    const float d = generator ? -1.f / (float)B : r < B ? -1.f / (float)B : r < 2 * B ? 1.f / (float)B : 1.f;
    uint4* __restrict__ row = reinterpret_cast<uint4*>(dlogits + ((int64_t)i * rows + r) * 32);
    row[0] = make_uint4((uint32_t)f2bf(d), 0u, 0u, 0u);
    row[1] = row[2] = row[3] = make_uint4(0u, 0u, 0u, 0u);
  }
  if (threadIdx.x == 0) {
    const float* __restrict__ o = out + (int64_t)i * rows * 32;
    double real = 0.0, fake = 0.0;
    if (generator) {
      for (int r = 0; r < B; ++r) fake += (double)o[r * 32];
      loss[2 * i + 1] = (float)(-fake / (double)B);
    } else {
      for (int r = 0; r < B; ++r) real += (double)o[r * 32];
      for (int r = B; r < 2 * B; ++r) fake += (double)o[r * 32];
      loss[2 * i] = (float)(fake / (double)B - real / (double)B);
    }
  }
}

// One workgroup per member.  g: the critic's input gradient on the interpolated rows, float [P][B][D].
// penalty = weight * mean_r (|g_r| - 1)^2 is added to loss[2 i]; c_r = (2 weight / B) (|g_r| - 1) / |g_r| g_r,
// the gradient of the penalty with respect to g_r, goes (bf16) to rows 2B .. 3B-1 of the critic's input
// buffer, where the weight-gradient contraction of the first layer finds it.  Row norms are summed in double,
// lanes in a fixed butterfly order, rows in order.
__global__ __launch_bounds__(256) void wgan_penalty_kernel(const float* __restrict__ g, int B, int D, float weight,
                                                           bf16_t* __restrict__ X, float* __restrict__ loss) {
  extern __shared__ double sq[];  // [B] squared deviations
  const int i = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
  for (int r = wave; r < B; r += waves) {
    const float* __restrict__ gr = g + ((int64_t)i * B + r) * D;
    double acc = 0.0;
    for (int c = lane; c < D; c += 64) acc += (double)gr[c] * (double)gr[c];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    const double norm = sqrt(acc);
    const double scale = (2.0 * (double)weight / (double)B) * ((norm - 1.0) / norm);
    bf16_t* __restrict__ xr = X + ((int64_t)i * 3 * B + 2 * B + r) * D;
    for (int c = lane; c < D; c += 64) xr[c] = d2bf(scale * (double)gr[c]);
    if (lane == 0) sq[r] = (norm - 1.0) * (norm - 1.0);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double total = 0.0;
    for (int r = 0; r < B; ++r) total += sq[r];
    loss[2 * i] = (float)((double)loss[2 * i] + (double)weight * total / (double)B);
  }
}

Net gen_net(const pbt_config& c) { return Net{c.n_layers, c.dims, 0, c.act, c.act_out}; }
Net dis_net(const pbt_config& c) { return Net{c.n_layers2, c.dims2, c.n_layers, c.act2, PBT_ACT_NONE}; }

struct Bufs {
  bf16_t* gA[PBT_MAX_DIMS]; bf16_t* gZ[PBT_MAX_DIMS]; bf16_t* gdZ[PBT_MAX_DIMS];
  bf16_t* dA[PBT_MAX_DIMS]; bf16_t* dZ[PBT_MAX_DIMS]; bf16_t* ddZ[PBT_MAX_DIMS];
};

Bufs bufs_of(pbt_handle* h) {
  const pbt_config& c = h->cfg;
  const GanPlan& g = h->plan.gan;
  Bufs b;
  std::memset(&b, 0, sizeof b);
  b.gA[0] = h->sc<bf16_t>(g.o_zin);
  for (int l = 0; l < c.n_layers; ++l) {
    b.gA[l + 1] = h->sc<bf16_t>(g.o_ga[l]);
    b.gZ[l] = h->sc<bf16_t>(g.o_gz[l]);
    b.gdZ[l] = h->sc<bf16_t>(g.o_gdz[l]);
  }
  b.dA[0] = h->sc<bf16_t>(g.o_dx);
  for (int l = 0; l < c.n_layers2 - 1; ++l) {
    b.dA[l + 1] = h->sc<bf16_t>(g.o_da[l]);
    b.dZ[l] = h->sc<bf16_t>(g.o_dz[l]);
    b.ddZ[l] = h->sc<bf16_t>(g.o_ddz[l]);
  }
  return b;
}

OptArgs adam_args(pbt_handle* h, int64_t begin, int64_t count, int col_lr) {
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  return OptArgs{h->st<float>(p.o_w32), h->st<float>(p.o_opt0), h->st<float>(p.o_opt1), h->st<bf16_t>(p.o_w16), h->sc<float>(p.o_grad),
             begin, count, h->st<float>(p.o_hyper), h->st<int32_t>(p.o_t), p.lay.stride, c.P, c.n_hyper, PBT_OPT_ADAM, col_lr, -1, -1,
             c.opt_const[0], c.opt_const[1], c.opt_const[2], c.opt_const[3]};
}

}  // namespace

pbt_status gan_check_and_plan(const pbt_config* c, Plan* pl, Carver* w) {
  GanPlan& g = pl->gan;
  const int Lg = c->n_layers, Ld = c->n_layers2;
  if (Ld < 2) return fail(nullptr, PBT_EUNSUPPORTED, "the discriminator needs at least one hidden layer");
  if (c->dims2[0] != c->dims[Lg]) return fail(nullptr, PBT_EINVAL, "discriminator input width must equal generator output width");
  if (c->dims2[Ld] != 1) return fail(nullptr, PBT_EINVAL, "the discriminator must end in one logit");
  for (int l = 0; l <= Lg; ++l)
    if (c->dims[l] % 8) return fail(nullptr, PBT_EUNSUPPORTED, "generator widths must be multiples of 8");
  for (int l = 0; l < Ld; ++l)
    if (c->dims2[l] < 1 || c->dims2[l] % 8) return fail(nullptr, PBT_EUNSUPPORTED, "discriminator widths must be multiples of 8");
  if (c->act_out < PBT_ACT_NONE || c->act_out > PBT_ACT_TANH || c->act2 < PBT_ACT_NONE || c->act2 > PBT_ACT_TANH)
    return fail(nullptr, PBT_EINVAL, "unknown activation");
  g.n_g = Lg;
  g.n_d = Ld;
  g.eval_rows = c->n_eval;
  const bool wgan = c->gan_objective == 1;
  if (c->gan_objective != 0 && c->gan_objective != 1) return fail(nullptr, PBT_EINVAL, "gan_objective is 0 (logistic) or 1 (WGAN-GP)");
  if (wgan && (c->n_critic < 1 || c->n_critic > 64)) return fail(nullptr, PBT_EINVAL, "n_critic outside 1..64");
  if (wgan && !(c->gp_weight >= 0.f)) return fail(nullptr, PBT_EINVAL, "gp_weight must be >= 0");
  if (wgan && c->fuse_optimizer) return fail(nullptr, PBT_EUNSUPPORTED, "the WGAN-GP step uses the separate optimiser pass");
  if (wgan && 3 + c->n_critic > 10) return fail(nullptr, PBT_EUNSUPPORTED, "at most 7 critic updates per step (latent sub-streams 3 .. 9)");
  // critic buffers hold real + generated rows, and for WGAN-GP the interpolated rows behind them
  const int64_t P = c->P, B = c->batch, R = (wgan ? 3 : 2) * B, E = c->n_eval, D = c->dims2[0];
  g.o_zin = w->take((size_t)P * B * c->dims[0] * 2);
  for (int l = 0; l < Lg; ++l) {
    g.o_ga[l] = w->take((size_t)P * B * c->dims[l + 1] * 2);
    g.o_gz[l] = w->take((size_t)P * B * c->dims[l + 1] * 2);
    g.o_gdz[l] = w->take((size_t)P * B * c->dims[l + 1] * 2);
  }
  g.o_dx = w->take((size_t)P * R * D * 2);
  for (int l = 0; l < Ld - 1; ++l) {
    g.o_da[l] = w->take((size_t)P * R * c->dims2[l + 1] * 2);
    g.o_dz[l] = w->take((size_t)P * R * c->dims2[l + 1] * 2);
    g.o_ddz[l] = w->take((size_t)P * R * c->dims2[l + 1] * 2);
  }
  g.o_dlogits = w->take((size_t)P * R * 32 * 2);
  g.o_rowloss = w->take((size_t)P * R * 4);
  g.o_hout = g.o_gin = 0;
  if (wgan) {
    g.o_hout = w->take((size_t)P * R * 32 * 4);
    g.o_gin = w->take((size_t)P * B * D * 4);
  }
  // eval: latents, two ping-pong hidden buffers, generated rows, held-out rows (bf16), norms, partial sums
  int64_t maxh = 8;
  for (int l = 1; l < Lg; ++l) maxh = c->dims[l] > maxh ? c->dims[l] : maxh;
  g.o_ez = w->take((size_t)P * E * c->dims[0] * 2);
  g.o_ea[0] = w->take((size_t)P * E * maxh * 2);
  g.o_ea[1] = w->take((size_t)P * E * maxh * 2);
  g.o_ex = w->take((size_t)P * E * D * 2);
  g.o_ey = w->take((size_t)E * D * 2);
  g.o_nx = w->take((size_t)P * E * 4);
  g.o_ny = w->take((size_t)E * 4);
  g.o_pxx = w->take((size_t)gemm_rbf_tiles((int)E, (int)E, (int)P) * P * 4);
  g.o_pyy = w->take((size_t)gemm_rbf_tiles((int)E, (int)E, 1) * 4);
  g.o_pxy = w->take((size_t)gemm_rbf_tiles((int)E, (int)E, (int)P) * P * 4);
  return PBT_OK;
}

// Section 4.3.1: n_critic updates of the critic on the WGAN-GP objective, then one update of the generator.
// The critic's buffers hold 3B rows per member: real, generated, interpolated.  The penalty's gradient with
// respect to the weights rides on the ordinary weight-gradient contractions: the input-gradient pass from
// d out = 1 leaves dz_l of the interpolated rows next to the ordinary dz_l, and the rows of the layer inputs
// that belong to the interpolated samples are overwritten by c_l (c_0 = d penalty / d g, c_{l+1} =
// (c_l W_l) * act'(z_l)), so that X_l^T dZ_l over all 3B rows is the Wasserstein gradient plus the penalty's.
static pbt_status gan_step_wgan(pbt_handle* h, const float* train_x, uint32_t step, hipStream_t s) {
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  const GanPlan& g = p.gan;
  const int P = c.P, B = c.batch, R = 3 * B, D = c.dims2[0], K = c.n_critic;
  const int64_t S = p.lay.stride;
  const Net gnet = gen_net(c), dnet = dis_net(c);
  Bufs b = bufs_of(h);
  const float* W32 = h->st<float>(p.o_w32);
  const bf16_t* W16 = h->st<bf16_t>(p.o_w16);
  float* G = h->sc<float>(p.o_grad);
  bf16_t* dlogits = h->sc<bf16_t>(g.o_dlogits);
  float* hout = h->sc<float>(g.o_hout);
  float* gin = h->sc<float>(g.o_gin);
  float* loss = h->st<float>(p.o_loss);
  const int Ld = c.n_layers2, Kh = c.dims2[Ld - 1];
  const int first = c.n_layers, head = c.n_layers + Ld - 1;  // layout indices of the critic's first and output layer
  const uint32_t k0 = (uint32_t)c.seed, k1 = (uint32_t)(c.seed >> 32);
  pbt_status st;
  for (int k = 0; k < K; ++k) {
    PBT_LAUNCH(h, PBT_K_FETCH, s, gather_rows(train_x, c.n_train, D, P, B, (int64_t)R * D, step, c.seed, b.dA[0], h->st<int32_t>(p.o_t), s,
                                              (uint32_t)(k * B), k == 0));
    PBT_LAUNCH(h, PBT_K_FETCH, s, latent_normal(b.gA[0], P, B, c.dims[0], step, 3 + k, c.seed, s));
    if ((st = forward(h, gnet, gnet.L, B, b.gA, nullptr, b.dA[0] + (int64_t)B * D, (int64_t)R * D, s)) != PBT_OK) return st;
    hipLaunchKernelGGL(wgan_interpolate_kernel, dim3(B, P), dim3(256), 0, s, b.dA[0], B, D, step, (uint32_t)(k * B), k0, k1);
    PBT_HIP(h, hipGetLastError());
    if ((st = forward(h, dnet, Ld - 1, R, b.dA, b.dZ, nullptr, 0, s)) != PBT_OK) return st;
    PBT_LAUNCH(h, PBT_K_HEAD, s, head_fwd_loss(b.dA[Ld - 1], (int64_t)R * Kh, W16 + p.lay.w_off[head], S, W32 + p.lay.b_off[head], S,
                                               nullptr, 0, P, R, Kh, 1, 0.f, -2, nullptr, hout, 0, s));
    hipLaunchKernelGGL(wgan_head_kernel, dim3(P), dim3(256), 0, s, hout, B, R, 0, dlogits, loss);
    PBT_HIP(h, hipGetLastError());
    // input gradients of every layer on all 3B rows (no weight gradients yet), down to g = dz_0 W_0^T on the interpolated rows
    PBT_LAUNCH(h, PBT_K_HEAD, s, head_dgrad(dlogits, W16 + p.lay.w_off[head], S, b.dZ[Ld - 2], b.ddZ[Ld - 2], P, R, Kh, 1, dnet.hidden_act, s));
    if ((st = backward(h, dnet, Ld - 1, R, b.dA, b.dZ, b.ddZ, false, nullptr, nullptr, nullptr, 0, s)) != PBT_OK) return st;
    {
      const int N0 = c.dims2[1];
      GemmOperands o{b.ddZ[0] + (int64_t)2 * B * N0, N0, (int64_t)R * N0, false, W16 + p.lay.w_off[first], N0, S, true, B, D, N0, P};
      PBT_LAUNCH(h, PBT_K_GEMM_DGRAD, s, gemm_store_f32(o, gin, D, (int64_t)B * D, s));
    }
    hipLaunchKernelGGL(wgan_penalty_kernel, dim3(P), dim3(256), (size_t)B * sizeof(double), s, gin, B, D, c.gp_weight, b.dA[0], loss);
    PBT_HIP(h, hipGetLastError());
    // c_{l+1} = (c_l W_l) * act'(z_l) on the interpolated rows, written over those rows of the next layer's input
    for (int l = 0; l < Ld - 1; ++l) {
      const int Kl = c.dims2[l], Nl = c.dims2[l + 1];
      GemmOperands o{b.dA[l] + (int64_t)2 * B * Kl, Kl, (int64_t)R * Kl, false, W16 + p.lay.w_off[first + l], Nl, S, false, B, Nl, Kl, P};
      PBT_LAUNCH(h, PBT_K_GEMM_FWD, s, gemm_dgrad_act(o, b.dZ[l] + (int64_t)2 * B * Nl, b.dA[l + 1] + (int64_t)2 * B * Nl, Nl, (int64_t)R * Nl,
                                                      dnet.hidden_act, s));
    }
    // weight gradients over all 3B rows; bias gradients (column sums) over the real and generated rows only
    for (int l = 0; l < Ld - 1; ++l) {
      const int Kl = c.dims2[l], Nl = c.dims2[l + 1];
      GemmOperands wg{b.dA[l], Kl, (int64_t)R * Kl, true, b.ddZ[l], Nl, (int64_t)R * Nl, false, Kl, Nl, R, P};
      wg.colsum = G + p.lay.b_off[first + l]; wg.colsum_stride = S; wg.colsum_k = 2 * B;
      PBT_LAUNCH(h, PBT_K_GEMM_WGRAD, s, gemm_store_f32(wg, G + p.lay.w_off[first + l], Nl, S, s));
    }
    {
      GemmOperands wg{b.dA[Ld - 1], Kh, (int64_t)R * Kh, true, dlogits, 32, (int64_t)R * 32, false, Kh, 1, R, P};
      wg.colsum = G + p.lay.b_off[head]; wg.colsum_stride = S; wg.colsum_k = 2 * B;
      PBT_LAUNCH(h, PBT_K_HEAD, s, gemm_store_f32(wg, G + p.lay.w_off[head], 1, S, s));
    }
    OptArgs oa_d = adam_args(h, g.d_begin, g.d_count, g.col_lr_d);
    oa_d.t_mul = K; oa_d.t_add = k + 1 - K;   // the critic has had K (t - 1) + k + 1 updates
    PBT_LAUNCH(h, PBT_K_OPTIMIZER, s, optimizer_step(oa_d, s));
  }
  // ---- generator update through the updated critic: L_G = -mean D(G(z'))
  PBT_LAUNCH(h, PBT_K_FETCH, s, latent_normal(b.gA[0], P, B, c.dims[0], step, 1, c.seed, s));
  if ((st = forward(h, gnet, gnet.L, B, b.gA, b.gZ, nullptr, 0, s)) != PBT_OK) return st;
  bf16_t* dA[PBT_MAX_DIMS];
  std::memcpy(dA, b.dA, sizeof dA);
  dA[0] = b.gA[gnet.L];
  if ((st = forward(h, dnet, Ld - 1, B, dA, b.dZ, nullptr, 0, s)) != PBT_OK) return st;
  PBT_LAUNCH(h, PBT_K_HEAD, s, head_fwd_loss(dA[Ld - 1], (int64_t)B * Kh, W16 + p.lay.w_off[head], S, W32 + p.lay.b_off[head], S,
                                             nullptr, 0, P, B, Kh, 1, 0.f, -2, nullptr, hout, 0, s));
  hipLaunchKernelGGL(wgan_head_kernel, dim3(P), dim3(256), 0, s, hout, B, B, 1, dlogits, loss);
  PBT_HIP(h, hipGetLastError());
  PBT_LAUNCH(h, PBT_K_HEAD, s, head_dgrad(dlogits, W16 + p.lay.w_off[head], S, b.dZ[Ld - 2], b.ddZ[Ld - 2], P, B, Kh, 1, dnet.hidden_act, s));
  if ((st = backward(h, dnet, Ld - 1, B, dA, b.dZ, b.ddZ, false, nullptr, b.gZ[gnet.L - 1], b.gdZ[gnet.L - 1], gnet.out_act, s)) != PBT_OK) return st;
  if ((st = backward(h, gnet, gnet.L, B, b.gA, b.gZ, b.gdZ, true, nullptr, nullptr, nullptr, 0, s)) != PBT_OK) return st;
  PBT_LAUNCH(h, PBT_K_OPTIMIZER, s, optimizer_step(adam_args(h, 0, g.g_count, g.col_lr_g), s));
  return PBT_OK;
}

pbt_status gan_step(pbt_handle* h, const float* train_x, uint32_t step, hipStream_t s) {
  if (h->cfg.gan_objective == 1) return gan_step_wgan(h, train_x, step, s);
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  const GanPlan& g = p.gan;
  const int P = c.P, B = c.batch, R = 2 * B, D = c.dims2[0];
  const int64_t S = p.lay.stride;
  const Net gnet = gen_net(c), dnet = dis_net(c);
  Bufs b = bufs_of(h);
  const float* W32 = h->st<float>(p.o_w32);
  const bf16_t* W16 = h->st<bf16_t>(p.o_w16);
  float* G = h->sc<float>(p.o_grad);
  bf16_t* dlogits = h->sc<bf16_t>(g.o_dlogits);
  float* rowloss = h->sc<float>(g.o_rowloss);
  float* loss = h->st<float>(p.o_loss);
  const int Ld = c.n_layers2, Kh = c.dims2[Ld - 1];
  const int head = c.n_layers + Ld - 1;  // layout index of the discriminator's output layer
  pbt_status st;

  // ---- discriminator update: B real rows (0..B-1) and B generated rows (B..2B-1), generator fixed
  PBT_LAUNCH(h, PBT_K_FETCH, s, gather_rows(train_x, c.n_train, D, P, B, (int64_t)R * D, step, c.seed, b.dA[0], h->st<int32_t>(p.o_t), s));
  PBT_LAUNCH(h, PBT_K_FETCH, s, latent_normal(b.gA[0], P, B, c.dims[0], step, 0, c.seed, s));
  if ((st = forward(h, gnet, gnet.L, B, b.gA, nullptr, b.dA[0] + (int64_t)B * D, (int64_t)R * D, s)) != PBT_OK) return st;
  if ((st = forward(h, dnet, Ld - 1, R, b.dA, b.dZ, nullptr, 0, s)) != PBT_OK) return st;
  PBT_LAUNCH(h, PBT_K_HEAD, s, head_fwd_loss(b.dA[Ld - 1], (int64_t)R * Kh, W16 + p.lay.w_off[head], S, W32 + p.lay.b_off[head], S,
                                             nullptr, 0, P, R, Kh, 1, 1.f / (float)B, B, dlogits, rowloss, R, s));
  PBT_LAUNCH(h, PBT_K_HEAD, s, row_reduce(rowloss, R, P, R, 1.f / (float)B, loss, 2, s));
  {
    GemmOperands wg{b.dA[Ld - 1], Kh, (int64_t)R * Kh, true, dlogits, 32, (int64_t)R * 32, false, Kh, 1, R, P};
    wg.colsum = G + p.lay.b_off[head]; wg.colsum_stride = S;   // the bias gradient, a by-product of the same launch
    PBT_LAUNCH(h, PBT_K_HEAD, s, gemm_store_f32(wg, G + p.lay.w_off[head], 1, S, s));
  }
  PBT_LAUNCH(h, PBT_K_HEAD, s, head_dgrad(dlogits, W16 + p.lay.w_off[head], S, b.dZ[Ld - 2], b.ddZ[Ld - 2], P, R, Kh, 1, dnet.hidden_act, s));
  const bool fused = c.fuse_optimizer != 0;
  const OptArgs oa_d = adam_args(h, g.d_begin, g.d_count, g.col_lr_d), oa_g = adam_args(h, 0, g.g_count, g.col_lr_g);
  if ((st = backward(h, dnet, Ld - 1, R, b.dA, b.dZ, b.ddZ, true, fused ? &oa_d : nullptr, nullptr, nullptr, 0, s)) != PBT_OK) return st;
  if (fused) {
    if ((st = optimizer_rest(h, oa_d, c.n_layers, Ld, Ld - 1, S, s)) != PBT_OK) return st;
  } else {
    PBT_LAUNCH(h, PBT_K_OPTIMIZER, s, optimizer_step(oa_d, s));
  }

  // ---- generator update: B fresh generated rows through the updated discriminator
  PBT_LAUNCH(h, PBT_K_FETCH, s, latent_normal(b.gA[0], P, B, c.dims[0], step, 1, c.seed, s));
  if ((st = forward(h, gnet, gnet.L, B, b.gA, b.gZ, nullptr, 0, s)) != PBT_OK) return st;
  {
    bf16_t* dA[PBT_MAX_DIMS];
    std::memcpy(dA, b.dA, sizeof dA);
    dA[0] = b.gA[gnet.L];  // the discriminator reads the generator's output directly
    if ((st = forward(h, dnet, Ld - 1, B, dA, b.dZ, nullptr, 0, s)) != PBT_OK) return st;
    PBT_LAUNCH(h, PBT_K_HEAD, s, head_fwd_loss(dA[Ld - 1], (int64_t)B * Kh, W16 + p.lay.w_off[head], S, W32 + p.lay.b_off[head], S,
                                               nullptr, 0, P, B, Kh, 1, 1.f / (float)B, B, dlogits, rowloss, B, s));
    PBT_LAUNCH(h, PBT_K_HEAD, s, row_reduce(rowloss, B, P, B, 1.f / (float)B, loss + 1, 2, s));
    PBT_LAUNCH(h, PBT_K_HEAD, s, head_dgrad(dlogits, W16 + p.lay.w_off[head], S, b.dZ[Ld - 2], b.ddZ[Ld - 2], P, B, Kh, 1, dnet.hidden_act, s));
    // through the discriminator down to its input, no weight gradients; the input gradient is
    // multiplied by the derivative of the generator's output activation on the way
    if ((st = backward(h, dnet, Ld - 1, B, dA, b.dZ, b.ddZ, false, nullptr, b.gZ[gnet.L - 1], b.gdZ[gnet.L - 1], gnet.out_act, s)) != PBT_OK) return st;
  }
  if ((st = backward(h, gnet, gnet.L, B, b.gA, b.gZ, b.gdZ, true, fused ? &oa_g : nullptr, nullptr, nullptr, 0, s)) != PBT_OK) return st;
  if (fused) return optimizer_rest(h, oa_g, 0, gnet.L, gnet.L, g.g_count, s);
  PBT_LAUNCH(h, PBT_K_OPTIMIZER, s, optimizer_step(oa_g, s));
  return PBT_OK;
}

pbt_status gan_eval(pbt_handle* h, const float* eval_x, hipStream_t s) {
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  const GanPlan& g = p.gan;
  const int P = c.P, E = c.n_eval, D = c.dims2[0];
  const Net gnet = gen_net(c);
  bf16_t* X = h->sc<bf16_t>(g.o_ex);
  bf16_t* Y = h->sc<bf16_t>(g.o_ey);
  float* nx = h->sc<float>(g.o_nx);
  float* ny = h->sc<float>(g.o_ny);
  // generated rows: latents (sub-stream 2, step index 0) through the generator
  bf16_t* A[PBT_MAX_DIMS];
  A[0] = h->sc<bf16_t>(g.o_ez);
  for (int l = 0; l < gnet.L; ++l) A[l + 1] = h->sc<bf16_t>(g.o_ea[l & 1]);
  PBT_LAUNCH(h, PBT_K_FETCH, s, latent_normal(A[0], P, E, c.dims[0], 0u, 2, c.seed, s));
  pbt_status st = forward(h, gnet, gnet.L, E, A, nullptr, X, (int64_t)E * D, s);
  if (st != PBT_OK) return st;
  PBT_HIP(h, f32_to_bf16(eval_x, Y, (int64_t)E * D, s));
  PBT_HIP(h, row_sqnorm(X, P, E, D, nx, s));
  PBT_HIP(h, row_sqnorm(Y, 1, E, D, ny, s));
  const float inv2d = 1.f / (2.f * (float)D);
  int txx = 0, tyy = 0, txy = 0;
  GemmOperands xx{X, D, (int64_t)E * D, false, X, D, (int64_t)E * D, true, E, E, D, P};
  PBT_HIP(h, gemm_rbf_sum(xx, nx, E, nx, E, inv2d, h->sc<float>(g.o_pxx), &txx, s));
  GemmOperands yy{Y, D, 0, false, Y, D, 0, true, E, E, D, 1};
  PBT_HIP(h, gemm_rbf_sum(yy, ny, 0, ny, 0, inv2d, h->sc<float>(g.o_pyy), &tyy, s));
  GemmOperands xy{X, D, (int64_t)E * D, false, Y, D, 0, true, E, E, D, P};
  PBT_HIP(h, gemm_rbf_sum(xy, nx, E, ny, 0, inv2d, h->sc<float>(g.o_pxy), &txy, s));
  PBT_HIP(h, mmd_combine(h->sc<float>(g.o_pxx), txx, h->sc<float>(g.o_pyy), tyy, h->sc<float>(g.o_pxy), txy, P,
                         1.f / ((float)E * (float)E), h->st<float>(p.o_score), s));
  return PBT_OK;
}

}  // namespace pbt
