// C ABI of the population step: configuration checks, carving of the caller's device buffers,
// and the kernel sequences behind pbt_step / pbt_eval / pbt_exploit_explore.
#include "dense_host.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

using namespace pbt;

namespace {
thread_local std::string g_last_error = "";

// Working memory of pbt_step_static: one array per GPU inside the library's own image, so that the call
// needs no buffer from an allocator.  In host code the array's name is only a handle for the symbol
// lookup below; kernels are given the looked-up device address, as they are given a caller's buffer.
constexpr size_t STATIC_SCRATCH_BYTES = PBT_STATIC_SCRATCH_BYTES;
__device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
char* g_static_scratch[MAX_DEVICES] = {};   // device address of `scratch` on each GPU, resolved once per GPU

// Device address of the current GPU's copy of the array (looked up on first use on that GPU).
hipError_t static_scratch_ptr(char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  if (!g_static_scratch[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_static_scratch[dev] = static_cast<char*>(p);
  }
  *out = g_static_scratch[dev];
  return hipSuccess;
}
}

namespace pbt {
pbt_status fail(pbt_handle* h, pbt_status code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (h) h->err = buf;
  g_last_error = buf;
  return code;
}
}  // namespace pbt

namespace {

pbt_status check_config(const pbt_config* c, Plan* pl) {
  if (!c) return fail(nullptr, PBT_EINVAL, "config is NULL");
  if (c->workload != PBT_WL_CLASSIFIER && c->workload != PBT_WL_GAN && c->workload != PBT_WL_A2C && c->workload != PBT_WL_TRANSFORMER)
    return fail(nullptr, PBT_EUNSUPPORTED, "workload %d not built", c->workload);
  const bool gan = c->workload == PBT_WL_GAN;
  const bool tf = c->workload == PBT_WL_TRANSFORMER;
  const bool a2c = c->workload == PBT_WL_A2C;
  if (c->P < 1 || c->P > PBT_MAX_P) return fail(nullptr, PBT_EINVAL, "P = %d outside 1..%d", c->P, PBT_MAX_P);
  if (c->batch < 1) return fail(nullptr, PBT_EINVAL, "batch must be positive");
  if (c->n_layers < 1 || c->n_layers >= PBT_MAX_DIMS) return fail(nullptr, PBT_EINVAL, "n_layers = %d outside 1..%d", c->n_layers, PBT_MAX_DIMS - 1);
  for (int l = 0; l <= c->n_layers && !tf; ++l)
    if (c->dims[l] < 1) return fail(nullptr, PBT_EINVAL, "dims[%d] must be positive", l);
  if (c->act < PBT_ACT_NONE || c->act > PBT_ACT_TANH) return fail(nullptr, PBT_EINVAL, "unknown activation %d", c->act);
  if (c->optimizer < PBT_OPT_SGD_MOMENTUM || c->optimizer > PBT_OPT_RMSPROP) return fail(nullptr, PBT_EINVAL, "unknown optimizer %d", c->optimizer);
  if (c->compute_dtype != PBT_DTYPE_FP32 && c->compute_dtype != PBT_DTYPE_BF16) return fail(nullptr, PBT_EINVAL, "unknown compute_dtype %d", c->compute_dtype);
  if (c->n_hyper < 1 || c->n_hyper > PBT_MAX_HYPER) return fail(nullptr, PBT_EINVAL, "n_hyper = %d outside 1..%d", c->n_hyper, PBT_MAX_HYPER);
  if (c->n_trunc < 0 || 2 * (int64_t)c->n_trunc > c->P) return fail(nullptr, PBT_EINVAL, "need 0 <= 2*n_trunc <= P (top and bottom sets must not overlap)");
  if (c->n_train < 1 || c->n_eval < 1) return fail(nullptr, PBT_EINVAL, "n_train and n_eval must be positive");
  if (c->exploit_mode < PBT_EXPLOIT_TRUNCATION || c->exploit_mode > PBT_EXPLOIT_TTEST) return fail(nullptr, PBT_EINVAL, "unknown exploit_mode %d", c->exploit_mode);
  if (c->on_policy != 0 && c->on_policy != 1) return fail(nullptr, PBT_EINVAL, "on_policy is 0 or 1");
  if (c->on_policy && !a2c) return fail(nullptr, PBT_EINVAL, "on_policy needs the actor-critic workload");
  if (c->exploit_mode == PBT_EXPLOIT_TTEST) {
    if (!a2c) return fail(nullptr, PBT_EINVAL, "t-test selection needs the score history of the actor-critic workload");
    if (!(c->ttest_alpha > 0.f && c->ttest_alpha <= 1.f)) return fail(nullptr, PBT_EINVAL, "ttest_alpha must be in (0, 1]");
  }
  if (c->explore_mode != PBT_EXPLORE_PERTURB && c->explore_mode != PBT_EXPLORE_RESAMPLE) return fail(nullptr, PBT_EINVAL, "unknown explore_mode %d", c->explore_mode);
  if (!(c->resample_prob >= 0.f)) return fail(nullptr, PBT_EINVAL, "resample_prob must be >= 0");
  if ((c->keep_weights != 0 && c->keep_weights != 1) || (c->keep_hypers != 0 && c->keep_hypers != 1)) return fail(nullptr, PBT_EINVAL, "keep_weights / keep_hypers are 0 or 1");
  if (c->keep_weights && c->keep_hypers) return fail(nullptr, PBT_EINVAL, "keep_weights and keep_hypers together leave exploit nothing to do");
  if (!gan && !tf && c->dims[c->n_layers] > 32) return fail(nullptr, PBT_EUNSUPPORTED, "more than 32 outputs in the last layer");
  pl->a2c.col_ent = -1;
  pl->tf.col_drop = pl->tf.col_ls = -1;
  pl->col_lr = pl->col_beta1 = pl->col_wd = -1;
  pl->gan.col_lr_g = pl->gan.col_lr_d = -1;
  for (int k = 0; k < c->n_hyper; ++k) {
    if (c->hyper_role[k] == PBT_ROLE_LR) pl->col_lr = k;
    else if (c->hyper_role[k] == PBT_ROLE_BETA1) pl->col_beta1 = k;
    else if (c->hyper_role[k] == PBT_ROLE_WD) pl->col_wd = k;
    else if (c->hyper_role[k] == PBT_ROLE_LR_G) pl->gan.col_lr_g = k;
    else if (c->hyper_role[k] == PBT_ROLE_LR_D) pl->gan.col_lr_d = k;
    else if (c->hyper_role[k] == PBT_ROLE_ENTROPY_COST) pl->a2c.col_ent = k;
    else if (c->hyper_role[k] == PBT_ROLE_DROPOUT) pl->tf.col_drop = k;
    else if (c->hyper_role[k] == PBT_ROLE_LABEL_SMOOTH) pl->tf.col_ls = k;
    else return fail(nullptr, PBT_EINVAL, "unknown hyper_role[%d] = %d", k, c->hyper_role[k]);
    if (std::isnan(c->hyper_max[k])) return fail(nullptr, PBT_EINVAL, "hyper_max[%d] is NaN", k);
  }
  if (gan) {
    if (pl->gan.col_lr_g < 0 || pl->gan.col_lr_d < 0) return fail(nullptr, PBT_EINVAL, "the GAN workload needs a generator and a discriminator learning-rate column");
    return PBT_OK;
  }
  if (pl->gan.col_lr_g >= 0 || pl->gan.col_lr_d >= 0) return fail(nullptr, PBT_EINVAL, "generator / discriminator learning-rate columns need the GAN workload");
  if (pl->col_lr < 0) return fail(nullptr, PBT_EINVAL, "no hyperparameter column has the learning-rate role");
  if (!tf && (pl->tf.col_drop >= 0 || pl->tf.col_ls >= 0)) return fail(nullptr, PBT_EINVAL, "dropout / label-smoothing columns need the transformer workload");
  if (tf) {
    // a rate of 1 would drop everything and divide by zero; explore clamps at hyper_max
    if (pl->tf.col_drop >= 0 && !(c->hyper_max[pl->tf.col_drop] < 1.f)) return fail(nullptr, PBT_EINVAL, "hyper_max of the dropout column must be below 1");
    if (pl->tf.col_ls >= 0 && !(c->hyper_max[pl->tf.col_ls] < 1.f)) return fail(nullptr, PBT_EINVAL, "hyper_max of the label-smoothing column must be below 1");
  }
  if (a2c != (pl->a2c.col_ent >= 0)) return fail(nullptr, PBT_EINVAL, "an entropy-cost column goes with the actor-critic workload, and only with it");
  if (c->optimizer != PBT_OPT_ADAM && (pl->col_beta1 >= 0 || pl->col_wd >= 0))
    return fail(nullptr, PBT_EINVAL, "beta1 / weight-decay columns need the Adam optimizer");
  // explore only clamps at hyper_max: at beta1 >= 1 the bias correction 1 / (1 - beta1^t) is infinite or negative
  if (pl->col_beta1 >= 0 && !(c->hyper_max[pl->col_beta1] < 1.f)) return fail(nullptr, PBT_EINVAL, "hyper_max of the beta1 column must be below 1");
  return PBT_OK;
}

pbt_status make_plan(const pbt_config* c, Plan* pl) {
  pbt_status st = check_config(c, pl);
  if (st != PBT_OK) return st;
  const int L = c->n_layers;
  const int64_t P = c->P, B = c->batch;
  const bool gan = c->workload == PBT_WL_GAN;
  const bool tf = c->workload == PBT_WL_TRANSFORMER;
  // parameter layout (GAN: generator layers, then discriminator layers)
  pbt_layout& lay = pl->lay;
  std::memset(&lay, 0, sizeof lay);
  int64_t off = 0, n_params = 0;
  int n_all = 0;
  int all_dims[2 * PBT_MAX_DIMS][2];
  for (int l = 0; l < L; ++l) { all_dims[n_all][0] = c->dims[l]; all_dims[n_all++][1] = c->dims[l + 1]; }
  if (gan) {
    if (c->n_layers2 < 1 || L + c->n_layers2 >= PBT_MAX_DIMS) return fail(nullptr, PBT_EINVAL, "generator + discriminator layers must number 2..%d", PBT_MAX_DIMS - 1);
    for (int l = 0; l < c->n_layers2; ++l) { all_dims[n_all][0] = c->dims2[l]; all_dims[n_all++][1] = c->dims2[l + 1]; }
  }
  if (tf) n_all = 0;
  for (int l = 0; l < n_all; ++l) {
    lay.w_off[l] = off;
    lay.seg_off[lay.n_seg] = off;
    lay.seg_len[lay.n_seg++] = (int64_t)all_dims[l][0] * all_dims[l][1];
    off = round_up(off + (int64_t)all_dims[l][0] * all_dims[l][1], SEG_ALIGN);
    lay.b_off[l] = off;
    lay.seg_off[lay.n_seg] = off;
    lay.seg_len[lay.n_seg++] = all_dims[l][1];
    off = round_up(off + all_dims[l][1], SEG_ALIGN);
    n_params += (int64_t)all_dims[l][0] * all_dims[l][1] + all_dims[l][1];
    if (gan && l == L - 1) pl->gan.g_count = off;
  }
  lay.stride = round_up(off, STRIDE_ALIGN);
  lay.n_params = n_params;
  if (tf) {
    pbt_status tst = tf_layout(c, pl);
    if (tst != PBT_OK) return tst;
  }
  const bool bf16 = c->compute_dtype == PBT_DTYPE_BF16;
  const bool adam = c->optimizer == PBT_OPT_ADAM;

  Carver s;
  const size_t pw = (size_t)P * lay.stride;
  pl->o_w32 = s.take(pw * 4);
  pl->o_opt0 = s.take(pw * 4);
  pl->o_opt1 = adam ? s.take(pw * 4) : 0;
  pl->o_w16 = bf16 ? s.take(pw * 2) : 0;
  pl->o_hyper = s.take((size_t)P * c->n_hyper * 4);
  pl->o_score = s.take(P * 4);
  pl->n_loss = gan ? 2 : 1;
  pl->o_loss = s.take(P * 4 * pl->n_loss);
  pl->o_t = s.take(P * 4);
  pl->o_order = s.take(P * 4);
  pl->o_donor = s.take(P * 4);
  pl->o_parent = s.take(P * 4);
  pl->o_recip = s.take(P * 4);
  pl->o_nrecip = s.take(4);
  pl->o_hist = c->workload == PBT_WL_A2C ? s.take(P * 12 * 4) : 0;
  pl->state_bytes = s.off;

  Carver w;
  pl->o_grad = w.take(pw * 4);
  for (int k = 0; k < 6; ++k) pl->o_stage[k] = 0;
  if (c->exploit_mode != PBT_EXPLOIT_TRUNCATION && !c->keep_weights) {
    // a member can be donor and recipient: donor rows pass through these staging rows (same order as in pbt_exploit_explore)
    int k = 0;
    pl->o_stage[k++] = w.take(pw * 4);
    pl->o_stage[k++] = w.take(pw * 4);
    if (adam) pl->o_stage[k++] = w.take(pw * 4);
    if (bf16) pl->o_stage[k++] = w.take(pw * 2);
    if (c->workload == PBT_WL_A2C) pl->o_stage[k++] = w.take(P * 12 * 4);
  }
  pl->fused_small = false;
  pl->eval_chunk = 0;
  if (gan) {
    if (!bf16 || !adam) return fail(nullptr, PBT_EUNSUPPORTED, "the GAN workload is built for bf16 compute with Adam");
    pl->gan.d_begin = pl->gan.g_count;
    pl->gan.d_count = lay.stride - pl->gan.g_count;
    pbt_status gst = gan_check_and_plan(c, pl, &w);
    if (gst != PBT_OK) return gst;
  } else if (tf) {
    if (!bf16 || !adam) return fail(nullptr, PBT_EUNSUPPORTED, "the transformer workload is built for bf16 compute with Adam");
    if (c->n_eval % c->batch) return fail(nullptr, PBT_EUNSUPPORTED, "the transformer workload needs n_eval to be a multiple of batch");
    pbt_status tst = tf_check_and_plan(c, pl, &w);
    if (tst != PBT_OK) return tst;
  } else if (c->workload == PBT_WL_A2C) {
    if (!bf16) return fail(nullptr, PBT_EUNSUPPORTED, "the actor-critic workload is built for bf16 compute");
    pbt_status ast = a2c_check_and_plan(c, pl, &w);
    if (ast != PBT_OK) return ast;
  } else if (!bf16) {
    FusedSmallArgs fa;
    std::memset(&fa, 0, sizeof fa);
    fa.stride = lay.stride; fa.B = (int)B; fa.n_layers = L; fa.optimizer = c->optimizer;
    for (int l = 0; l <= L; ++l) fa.dims[l] = c->dims[l];
    if (lay.stride > (1 << 20) || fused_small_plan(fa, false) > FUSED_SMALL_MAX_LDS)
      return fail(nullptr, PBT_EUNSUPPORTED,
                  "fp32 compute is built only for networks whose weights, optimiser state and one mini-batch of "
                  "activations fit the 160 KB LDS of a compute unit; use bf16 compute for larger ones");
    pl->fused_small = true;
  } else {
    for (int l = 0; l < L; ++l) {
      const bool head = l == L - 1;
      if (!head && (c->dims[l] % 8 || c->dims[l + 1] % 8))
        return fail(nullptr, PBT_EUNSUPPORTED, "bf16 hidden layers need widths that are multiples of 8 (layer %d)", l);
    }
    if (L >= 2 && c->dims[L - 1] % 8) return fail(nullptr, PBT_EUNSUPPORTED, "last hidden width must be a multiple of 8");
    pl->o_y = w.take(P * B * 4);
    pl->o_dlogits = w.take((size_t)P * B * 32 * 2);  // bf16, row pitch 32
    pl->o_rowloss = w.take(P * B * 4);
    for (int l = 0; l < L; ++l) {
      pl->o_act[l] = w.take((size_t)P * B * c->dims[l] * 2);       // input of layer l
      if (l < L - 1) {
        pl->o_z[l] = w.take((size_t)P * B * c->dims[l + 1] * 2);   // pre-activation of layer l
        pl->o_dz[l] = w.take((size_t)P * B * c->dims[l + 1] * 2);  // gradient w.r.t. it
      }
    }
    // eval: held-out set in bf16 (shared), two ping-pong activation buffers per chunk, per-row losses
    int64_t maxh = 8;
    for (int l = 1; l < L; ++l) maxh = c->dims[l] > maxh ? c->dims[l] : maxh;
    int chunk = c->eval_chunk;
    if (chunk <= 0) {
      const int64_t budget = (int64_t)256 << 20;  // bytes per ping-pong buffer
      chunk = (int)(budget / (P * maxh * 2));
      if (chunk > c->n_eval) chunk = c->n_eval;
      if (chunk >= 128) chunk = chunk / 128 * 128;
      if (chunk < 1) chunk = 1;
    }
    if (chunk > c->n_eval) chunk = c->n_eval;
    pl->eval_chunk = chunk;
    pl->o_evalx = w.take((size_t)c->n_eval * c->dims[0] * 2);
    pl->o_evala[0] = w.take((size_t)P * chunk * maxh * 2);
    pl->o_evala[1] = w.take((size_t)P * chunk * maxh * 2);
    pl->o_evalrow = w.take((size_t)P * c->n_eval * 4);
  }
  pl->scratch_bytes = w.off;
  return PBT_OK;
}

struct ArrInfo { size_t off; size_t elem; int64_t cols; bool in_scratch; };

pbt_status arr_info(pbt_handle* h, int which, ArrInfo* ai) {
  const Plan& p = h->plan;
  const pbt_config& c = h->cfg;
  const int64_t S = p.lay.stride;
  switch (which) {
    case PBT_ARR_W32: *ai = {p.o_w32, 4, S, false}; return PBT_OK;
    case PBT_ARR_OPT0: *ai = {p.o_opt0, 4, S, false}; return PBT_OK;
    case PBT_ARR_OPT1:
      if (c.optimizer != PBT_OPT_ADAM) return fail(h, PBT_EINVAL, "OPT1 exists only with Adam");
      *ai = {p.o_opt1, 4, S, false}; return PBT_OK;
    case PBT_ARR_W16:
      if (c.compute_dtype != PBT_DTYPE_BF16) return fail(h, PBT_EINVAL, "W16 exists only with bf16 compute");
      *ai = {p.o_w16, 2, S, false}; return PBT_OK;
    case PBT_ARR_GRAD: *ai = {p.o_grad, 4, S, true}; return PBT_OK;
    case PBT_ARR_HYPER: *ai = {p.o_hyper, 4, c.n_hyper, false}; return PBT_OK;
    case PBT_ARR_SCORE: *ai = {p.o_score, 4, 1, false}; return PBT_OK;
    case PBT_ARR_LOSS: *ai = {p.o_loss, 4, p.n_loss, false}; return PBT_OK;
    case PBT_ARR_T: *ai = {p.o_t, 4, 1, false}; return PBT_OK;
    case PBT_ARR_ORDER: *ai = {p.o_order, 4, 1, false}; return PBT_OK;
    case PBT_ARR_DONOR: *ai = {p.o_donor, 4, 1, false}; return PBT_OK;
    case PBT_ARR_PARENT: *ai = {p.o_parent, 4, 1, false}; return PBT_OK;
    case PBT_ARR_HIST:
      if (c.workload != PBT_WL_A2C) return fail(h, PBT_EINVAL, "HIST exists only in the actor-critic workload");
      *ai = {p.o_hist, 4, 12, false}; return PBT_OK;
    case PBT_ARR_TRAJ_OBS: case PBT_ARR_TRAJ_ACT: case PBT_ARR_TRAJ_REW:
      if (c.workload != PBT_WL_A2C) return fail(h, PBT_EINVAL, "the unroll arrays exist only in the actor-critic workload");
      if (which == PBT_ARR_TRAJ_OBS) *ai = {p.a2c.o_a[0], 2, (int64_t)p.a2c.rows * c.dims[0], true};
      else if (which == PBT_ARR_TRAJ_ACT) *ai = {p.a2c.o_act, 4, (int64_t)c.batch * c.unroll, true};
      else *ai = {p.a2c.o_rew, 4, (int64_t)c.batch * c.unroll, true};
      return PBT_OK;
    default: return fail(h, PBT_EINVAL, "unknown array id %d", which);
  }
}

void fill_fused(pbt_handle* h, FusedSmallArgs* fa) {
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  std::memset(fa, 0, sizeof *fa);
  fa->W32 = h->st<float>(p.o_w32);
  fa->S0 = h->st<float>(p.o_opt0);
  fa->S1 = c.optimizer == PBT_OPT_ADAM ? h->st<float>(p.o_opt1) : nullptr;
  fa->G = h->sc<float>(p.o_grad);
  fa->H = h->st<float>(p.o_hyper);
  fa->t = h->st<int32_t>(p.o_t);
  fa->loss = h->st<float>(p.o_loss);
  fa->score = h->st<float>(p.o_score);
  fa->stride = p.lay.stride;
  fa->P = c.P; fa->B = c.batch; fa->n_layers = c.n_layers;
  for (int l = 0; l <= c.n_layers; ++l) fa->dims[l] = c.dims[l];
  for (int l = 0; l < c.n_layers; ++l) { fa->w_off[l] = (int)p.lay.w_off[l]; fa->b_off[l] = (int)p.lay.b_off[l]; }
  fa->act = c.act; fa->optimizer = c.optimizer; fa->n_hyper = c.n_hyper;
  fa->col_lr = p.col_lr; fa->col_beta1 = p.col_beta1; fa->col_wd = p.col_wd;
  fa->c0 = c.opt_const[0]; fa->c1 = c.opt_const[1]; fa->c2 = c.opt_const[2]; fa->c3 = c.opt_const[3];
  fa->seed = c.seed;
}

// One population step on the bf16 path: the kernel sequence of forward, loss, backward, update.
pbt_status step_bf16(pbt_handle* h, const float* train_x, const int32_t* train_y, uint32_t step, hipStream_t s) {
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  const int L = c.n_layers, P = c.P, B = c.batch;
  const int64_t S = p.lay.stride;
  float* W32 = h->st<float>(p.o_w32);
  bf16_t* W16 = h->st<bf16_t>(p.o_w16);
  float* G = h->sc<float>(p.o_grad);
  int32_t* Y = h->sc<int32_t>(p.o_y);
  bf16_t* dlogits = h->sc<bf16_t>(p.o_dlogits);
  float* rowloss = h->sc<float>(p.o_rowloss);

  PBT_LAUNCH(h, PBT_K_FETCH, s, gather_batch(train_x, train_y, c.n_train, c.dims[0], P, B, step, c.seed,
                                             h->sc<bf16_t>(p.o_act[0]), nullptr, Y, h->st<int32_t>(p.o_t), s));
  for (int l = 0; l < L - 1; ++l) {
    GemmOperands o{h->sc<bf16_t>(p.o_act[l]), c.dims[l], (int64_t)B * c.dims[l], false,
                   W16 + p.lay.w_off[l], c.dims[l + 1], S, false, B, c.dims[l + 1], c.dims[l], P};
    PBT_LAUNCH(h, PBT_K_GEMM_FWD, s, gemm_bias_act(o, W32 + p.lay.b_off[l], S, h->sc<bf16_t>(p.o_z[l]),
                                                   h->sc<bf16_t>(p.o_act[l + 1]), c.dims[l + 1],
                                                   (int64_t)B * c.dims[l + 1], c.act, s));
  }
  const int Kh = c.dims[L - 1], C = c.dims[L];
  PBT_LAUNCH(h, PBT_K_HEAD, s, head_fwd_loss(h->sc<bf16_t>(p.o_act[L - 1]), (int64_t)B * Kh, W16 + p.lay.w_off[L - 1], S,
                                             W32 + p.lay.b_off[L - 1], S, Y, B, P, B, Kh, C, 1.f / (float)B, -1, dlogits,
                                             rowloss, B, s));
  PBT_LAUNCH(h, PBT_K_HEAD, s, row_reduce(rowloss, B, P, B, 1.f / (float)B, h->st<float>(p.o_loss), 1, s));
  {
    // dW_head[Kh][C] = X^T dlogits (contraction over the B rows), db_head = column sums
    GemmOperands wg{h->sc<bf16_t>(p.o_act[L - 1]), Kh, (int64_t)B * Kh, true, dlogits, 32, (int64_t)B * 32, false,
                    Kh, C, B, P};
    wg.colsum = G + p.lay.b_off[L - 1]; wg.colsum_stride = S;   // db_head, a by-product of the same launch
    PBT_LAUNCH(h, PBT_K_HEAD, s, gemm_store_f32(wg, G + p.lay.w_off[L - 1], C, S, s));
  }
  if (L >= 2)
    PBT_LAUNCH(h, PBT_K_HEAD, s, head_dgrad(dlogits, W16 + p.lay.w_off[L - 1], S, h->sc<bf16_t>(p.o_z[L - 2]),
                                            h->sc<bf16_t>(p.o_dz[L - 2]), P, B, Kh, C, c.act, s));
  OptArgs oa{W32, h->st<float>(p.o_opt0), c.optimizer == PBT_OPT_ADAM ? h->st<float>(p.o_opt1) : nullptr, W16, G,
             0, S, h->st<float>(p.o_hyper), h->st<int32_t>(p.o_t), S, P, c.n_hyper, c.optimizer, p.col_lr, p.col_beta1, p.col_wd,
             c.opt_const[0], c.opt_const[1], c.opt_const[2], c.opt_const[3]};
  const bool fused = c.fuse_optimizer != 0;
  for (int l = L - 2; l >= 0; --l) {
    const int K = c.dims[l], N = c.dims[l + 1];
    if (l > 0) {
      // dZ_{l-1}[B][K] = (dZ_l W_l^T) * act'(Z_{l-1}); before the weight gradient, whose fused
      // epilogue rewrites the bf16 weights read here
      GemmOperands dg{h->sc<bf16_t>(p.o_dz[l]), N, (int64_t)B * N, false, W16 + p.lay.w_off[l], N, S, true, B, K, N, P};
      PBT_LAUNCH(h, PBT_K_GEMM_DGRAD, s, gemm_dgrad_act(dg, h->sc<bf16_t>(p.o_z[l - 1]), h->sc<bf16_t>(p.o_dz[l - 1]), K,
                                                        (int64_t)B * K, c.act, s));
    }
    // dW_l[K][N] = X_l^T dZ_l (contraction over the B rows); db_l = column sums of dZ_l from the same launch
    GemmOperands wg{h->sc<bf16_t>(p.o_act[l]), K, (int64_t)B * K, true, h->sc<bf16_t>(p.o_dz[l]), N, (int64_t)B * N, false,
                    K, N, B, P};
    wg.colsum = G + p.lay.b_off[l]; wg.colsum_stride = S;
    if (fused)
      PBT_LAUNCH(h, PBT_K_GEMM_WGRAD, s, gemm_wgrad_optimizer(wg, oa, p.lay.w_off[l], N, s));
    else
      PBT_LAUNCH(h, PBT_K_GEMM_WGRAD, s, gemm_store_f32(wg, G + p.lay.w_off[l], N, S, s));
  }
  if (fused) return optimizer_rest(h, oa, 0, L, L - 1, S, s);
  PBT_LAUNCH(h, PBT_K_OPTIMIZER, s, optimizer_step(oa, s));
  return PBT_OK;
}

pbt_status eval_bf16(pbt_handle* h, const float* eval_x, const int32_t* eval_y, hipStream_t s) {
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  const int L = c.n_layers, P = c.P;
  const int64_t S = p.lay.stride;
  float* W32 = h->st<float>(p.o_w32);
  bf16_t* W16 = h->st<bf16_t>(p.o_w16);
  bf16_t* ex = h->sc<bf16_t>(p.o_evalx);
  float* rowloss = h->sc<float>(p.o_evalrow);
  PBT_HIP(h, f32_to_bf16(eval_x, ex, (int64_t)c.n_eval * c.dims[0], s));
  for (int r0 = 0; r0 < c.n_eval; r0 += p.eval_chunk) {
    const int rows = c.n_eval - r0 < p.eval_chunk ? c.n_eval - r0 : p.eval_chunk;
    const bf16_t* in = ex + (int64_t)r0 * c.dims[0];
    int64_t in_stride = 0;  // the held-out rows are shared by all members
    for (int l = 0; l < L - 1; ++l) {
      bf16_t* out = h->sc<bf16_t>(p.o_evala[l & 1]);
      GemmOperands o{in, c.dims[l], in_stride, false, W16 + p.lay.w_off[l], c.dims[l + 1], S, false,
                     rows, c.dims[l + 1], c.dims[l], P};
      PBT_HIP(h, gemm_bias_act(o, W32 + p.lay.b_off[l], S, nullptr, out, c.dims[l + 1], (int64_t)rows * c.dims[l + 1],
                               c.act, s));
      in = out;
      in_stride = (int64_t)rows * c.dims[l + 1];
    }
    PBT_HIP(h, head_fwd_loss(in, in_stride, W16 + p.lay.w_off[L - 1], S, W32 + p.lay.b_off[L - 1], S, eval_y + r0, 0, P,
                             rows, c.dims[L - 1], c.dims[L], 0.f, -1, nullptr, rowloss + r0, c.n_eval, s));
  }
  PBT_HIP(h, row_reduce(rowloss, c.n_eval, P, c.n_eval, -1.f / (float)c.n_eval, h->st<float>(p.o_score), 1, s));
  return PBT_OK;
}

}  // namespace

static hipError_t reset_store(pbt_handle* h, hipStream_t s);

extern "C" {

pbt_status pbt_query_sizes(const pbt_config* cfg, size_t* state_bytes, size_t* scratch_bytes, pbt_layout* layout) {
  Plan pl;
  pbt_status st = make_plan(cfg, &pl);
  if (st != PBT_OK) return st;
  if (state_bytes) *state_bytes = pl.state_bytes;
  if (scratch_bytes) *scratch_bytes = pl.scratch_bytes;
  if (layout) *layout = pl.lay;
  return PBT_OK;
}

pbt_status pbt_init(const pbt_config* cfg, void* d_state, size_t state_bytes, void* d_scratch, size_t scratch_bytes,
                    void* hip_stream, pbt_handle** out) {
  if (!out) return fail(nullptr, PBT_EINVAL, "out is NULL");
  *out = nullptr;
  Plan pl;
  pbt_status st = make_plan(cfg, &pl);
  if (st != PBT_OK) return st;
  if (!d_state || !d_scratch) return fail(nullptr, PBT_EINVAL, "device buffers must not be NULL");
  if (((uintptr_t)d_state | (uintptr_t)d_scratch) % BUF_ALIGN) return fail(nullptr, PBT_EINVAL, "device buffers must be 256-byte aligned");
  if (state_bytes < pl.state_bytes) return fail(nullptr, PBT_ENOMEM, "state buffer: %zu bytes given, %zu needed", state_bytes, pl.state_bytes);
  if (scratch_bytes < pl.scratch_bytes) return fail(nullptr, PBT_ENOMEM, "scratch buffer: %zu bytes given, %zu needed", scratch_bytes, pl.scratch_bytes);
  pbt_handle* h = new (std::nothrow) pbt_handle();
  if (!h) return fail(nullptr, PBT_ENOMEM, "out of host memory");
  h->cfg = *cfg;
  h->plan = pl;
  h->state = static_cast<char*>(d_state);
  h->scratch = static_cast<char*>(d_scratch);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = reset_store(h, s);
  if (e != hipSuccess) {
    delete h;
    return fail(nullptr, PBT_EDEVICE, "initialising the population store failed: %s", hipGetErrorString(e));
  }
  // set-up is the place for the one symbol lookup pbt_step_static needs on this GPU (a failure here only
  // surfaces if that entry point is used)
  char* unused = nullptr;
  (void)static_scratch_ptr(&unused);
  *out = h;
  return PBT_OK;
}

static hipError_t reset_store(pbt_handle* h, hipStream_t s) {
  const Plan& pl = h->plan;
  const int P = h->cfg.P;
  hipError_t e = fill_u32(h->st<uint32_t>(0), 0u, (int64_t)(pl.state_bytes / 4), s);
  if (e == hipSuccess) e = fill_u32(h->sc<uint32_t>(pl.o_grad), 0u, (int64_t)P * pl.lay.stride, s);
  if (e == hipSuccess) e = fill_u32(h->st<uint32_t>(pl.o_score), 0xff800000u, P, s);  // -inf
  if (e == hipSuccess) e = fill_u32(h->st<uint32_t>(pl.o_donor), 0xffffffffu, P, s);  // -1
  if (e == hipSuccess) e = iota_i32(h->st<int32_t>(pl.o_parent), P, s);
  if (e == hipSuccess) e = iota_i32(h->st<int32_t>(pl.o_order), P, s);
  return e;
}

static pbt_status check_priors(pbt_handle* h, const pbt_prior* priors) {
  if (!priors) return fail(h, PBT_EINVAL, "priors is NULL");
  for (int k = 0; k < h->cfg.n_hyper; ++k) {
    const pbt_prior& pr = priors[k];
    if (pr.kind != 0 && pr.kind != 1) return fail(h, PBT_EINVAL, "prior %d: kind must be 0 (uniform) or 1 (log-uniform)", k);
    if (!(pr.lo <= pr.hi) || !std::isfinite(pr.lo) || !std::isfinite(pr.hi)) return fail(h, PBT_EINVAL, "prior %d: need finite lo <= hi", k);
    if (pr.kind == 1 && !(pr.lo > 0.0)) return fail(h, PBT_EINVAL, "prior %d: log-uniform needs lo > 0", k);
  }
  return PBT_OK;
}

pbt_status pbt_set_priors(pbt_handle* h, const pbt_prior* priors) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  pbt_status st = check_priors(h, priors);
  if (st != PBT_OK) return st;
  for (int k = 0; k < h->cfg.n_hyper; ++k) h->priors[k] = priors[k];
  h->have_priors = true;
  return PBT_OK;
}

pbt_status pbt_init_population(pbt_handle* h, const pbt_prior* priors, void* hip_stream) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  if (!priors) return fail(h, PBT_EINVAL, "priors is NULL");
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  InitArgs a;
  std::memset(&a, 0, sizeof a);
  for (int k = 0; k < c.n_hyper; ++k) {
    const pbt_prior& pr = priors[k];
    if (pr.kind != 0 && pr.kind != 1) return fail(h, PBT_EINVAL, "prior %d: kind must be 0 (uniform) or 1 (log-uniform)", k);
    if (!(pr.lo <= pr.hi) || !std::isfinite(pr.lo) || !std::isfinite(pr.hi)) return fail(h, PBT_EINVAL, "prior %d: need finite lo <= hi", k);
    if (pr.kind == 1 && !(pr.lo > 0.0)) return fail(h, PBT_EINVAL, "prior %d: log-uniform needs lo > 0", k);
    a.prior_kind[k] = pr.kind;
    a.prior_a[k] = pr.kind == 1 ? std::log(pr.lo) : pr.lo;
    a.prior_b[k] = pr.kind == 1 ? std::log(pr.hi) : pr.hi;
  }
  for (int k = 0; k < c.n_hyper; ++k) h->priors[k] = priors[k];
  h->have_priors = true;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  PBT_HIP(h, reset_store(h, s));
  a.W32 = h->st<float>(p.o_w32);
  a.W16 = c.compute_dtype == PBT_DTYPE_BF16 ? h->st<bf16_t>(p.o_w16) : nullptr;
  a.H = h->st<float>(p.o_hyper);
  a.stride = p.lay.stride; a.P = c.P; a.n_hyper = c.n_hyper;
  a.n_seg = p.lay.n_seg;
  for (int k = 0; k < a.n_seg; ++k) { a.seg_off[k] = p.lay.seg_off[k]; a.seg_len[k] = p.lay.seg_len[k]; a.seg_fan[k] = 0; a.seg_const[k] = 0.f; }
  if (c.workload == PBT_WL_TRANSFORMER) {
    // embeddings and matrices uniform in +-1/sqrt(fan_in) (fan_in = d_model for the two tables), LayerNorm gains 1, every bias 0
    const int d = c.tf_d_model, f = c.tf_d_ff;
    a.seg_fan[0] = a.seg_fan[1] = d;
    for (int l = 0; l < c.n_layers; ++l) {
      const int b0 = 2 + 12 * l;
      a.seg_const[b0 + 0] = 1.f; a.seg_fan[b0 + 2] = d; a.seg_fan[b0 + 4] = d;
      a.seg_const[b0 + 6] = 1.f; a.seg_fan[b0 + 8] = d; a.seg_fan[b0 + 10] = f;
    }
    a.seg_const[a.n_seg - 4] = 1.f; a.seg_fan[a.n_seg - 2] = d;
  } else {
    // dense layers: weights and biases of a layer uniform in +-1/sqrt(fan_in)
    const int n_layers = c.n_layers + (c.workload == PBT_WL_GAN ? c.n_layers2 : 0);
    for (int l = 0; l < n_layers; ++l) a.seg_fan[2 * l] = a.seg_fan[2 * l + 1] = l < c.n_layers ? c.dims[l] : c.dims2[l - c.n_layers];
  }
  a.seed = c.seed;
  PBT_HIP(h, init_population(a, s));
  return PBT_OK;
}

pbt_status pbt_step(pbt_handle* h, const void* const* d_inputs, int32_t n_inputs, int64_t step_index, int32_t n_steps,
                    void* hip_stream) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  if (h->cfg.workload == PBT_WL_A2C) {
    if (n_steps < 0 || step_index < 0 || step_index + n_steps > 0xffffffffLL) return fail(h, PBT_EINVAL, "step range outside 0..2^32-1");
    if (h->cfg.on_policy) {
      if (!d_inputs || n_inputs != 5 || !d_inputs[0] || !d_inputs[1] || !d_inputs[2] || !d_inputs[3] || !d_inputs[4])
        return fail(h, PBT_EINVAL, "on-policy actor-critic step needs 5 inputs: A, B, C, w, noise scales (double arrays)");
      const A2CEnv env{static_cast<const double*>(d_inputs[0]), static_cast<const double*>(d_inputs[1]), static_cast<const double*>(d_inputs[2]),
                       static_cast<const double*>(d_inputs[3]), static_cast<const double*>(d_inputs[4])};
      for (int k = 0; k < n_steps; ++k) {
        pbt_status st = a2c_step_on_policy(h, env, (uint32_t)(step_index + k), static_cast<hipStream_t>(hip_stream));
        if (st != PBT_OK) return st;
      }
      return PBT_OK;
    }
    if (!d_inputs || n_inputs != 3 || !d_inputs[0] || !d_inputs[1] || !d_inputs[2])
      return fail(h, PBT_EINVAL, "actor-critic step needs 3 inputs: observations, actions, rewards");
    for (int k = 0; k < n_steps; ++k) {
      pbt_status st = a2c_step(h, static_cast<const float*>(d_inputs[0]), static_cast<const int32_t*>(d_inputs[1]),
                               static_cast<const float*>(d_inputs[2]), (uint32_t)(step_index + k), static_cast<hipStream_t>(hip_stream));
      if (st != PBT_OK) return st;
    }
    return PBT_OK;
  }
  if (h->cfg.workload == PBT_WL_TRANSFORMER) {
    if (!d_inputs || n_inputs != 1 || !d_inputs[0]) return fail(h, PBT_EINVAL, "transformer step needs 1 input: the token pool");
    if (n_steps < 0 || step_index < 0 || step_index + n_steps > 0xffffffffLL) return fail(h, PBT_EINVAL, "step range outside 0..2^32-1");
    for (int k = 0; k < n_steps; ++k) {
      pbt_status st = tf_step(h, static_cast<const int32_t*>(d_inputs[0]), (uint32_t)(step_index + k), static_cast<hipStream_t>(hip_stream));
      if (st != PBT_OK) return st;
    }
    return PBT_OK;
  }
  if (h->cfg.workload == PBT_WL_GAN) {
    if (!d_inputs || n_inputs != 1 || !d_inputs[0]) return fail(h, PBT_EINVAL, "GAN step needs 1 input: train_x");
    if (n_steps < 0 || step_index < 0 || step_index + n_steps > 0xffffffffLL) return fail(h, PBT_EINVAL, "step range outside 0..2^32-1");
    for (int k = 0; k < n_steps; ++k) {
      pbt_status st = gan_step(h, static_cast<const float*>(d_inputs[0]), (uint32_t)(step_index + k), static_cast<hipStream_t>(hip_stream));
      if (st != PBT_OK) return st;
    }
    return PBT_OK;
  }
  if (!d_inputs || n_inputs != 2 || !d_inputs[0] || !d_inputs[1])
    return fail(h, PBT_EINVAL, "classifier step needs 2 inputs: train_x, train_y");
  if (n_steps < 0 || step_index < 0 || step_index + n_steps > 0xffffffffLL) return fail(h, PBT_EINVAL, "step range outside 0..2^32-1");
  if (n_steps == 0) return PBT_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const float* x = static_cast<const float*>(d_inputs[0]);
  const int32_t* y = static_cast<const int32_t*>(d_inputs[1]);
  if (h->plan.fused_small) {
    FusedSmallArgs fa;
    fill_fused(h, &fa);
    fa.x = x; fa.y = y; fa.n_rows = h->cfg.n_train;
    fa.step0 = (uint32_t)step_index; fa.n_steps = n_steps;
    fused_small_plan(fa, false);
    PBT_LAUNCH(h, PBT_K_FUSED_STEP, s, fused_small_step(fa, s));
    return PBT_OK;
  }
  for (int k = 0; k < n_steps; ++k) {
    pbt_status st = step_bf16(h, x, y, (uint32_t)(step_index + k), s);
    if (st != PBT_OK) return st;
  }
  return PBT_OK;
}

pbt_status pbt_step_static(pbt_handle* h, const void* const* d_inputs, int32_t n_inputs, int64_t step_index, int32_t n_steps,
                           void* hip_stream) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  if (h->plan.scratch_bytes > STATIC_SCRATCH_BYTES)
    return fail(h, PBT_ENOMEM, "pbt_step_static: this configuration needs %zu bytes of working memory, the library's static array holds %zu; use pbt_step",
                h->plan.scratch_bytes, (size_t)STATIC_SCRATCH_BYTES);
  char* ptr = nullptr;
  hipError_t e = static_scratch_ptr(&ptr);
  if (e != hipSuccess) return fail(h, PBT_EDEVICE, "pbt_step_static: looking up the static working memory failed: %s", hipGetErrorString(e));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char* const callers = h->scratch;
  h->scratch = ptr;
  // the array keeps what the last call (of any handle) left: the gradient buffer must start at zero, because
  // its padding elements are never written and the optimiser reads them (a fill kernel, which a stream
  // capture records faithfully)
  e = fill_u32(h->sc<uint32_t>(h->plan.o_grad), 0u, (int64_t)h->cfg.P * h->plan.lay.stride, s);
  pbt_status st = e == hipSuccess ? pbt_step(h, d_inputs, n_inputs, step_index, n_steps, hip_stream)
                                  : fail(h, PBT_EDEVICE, "pbt_step_static: clearing the gradient buffer failed: %s", hipGetErrorString(e));
  h->scratch = callers;
  return st;
}

pbt_status pbt_eval(pbt_handle* h, const void* const* d_inputs, int32_t n_inputs, void* hip_stream) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  if (h->cfg.workload == PBT_WL_A2C) return a2c_eval(h, static_cast<hipStream_t>(hip_stream));
  if (h->cfg.workload == PBT_WL_TRANSFORMER) {
    if (!d_inputs || n_inputs != 1 || !d_inputs[0]) return fail(h, PBT_EINVAL, "transformer eval needs 1 input: the held-out tokens");
    return tf_eval(h, static_cast<const int32_t*>(d_inputs[0]), static_cast<hipStream_t>(hip_stream));
  }
  if (h->cfg.workload == PBT_WL_GAN) {
    if (!d_inputs || n_inputs != 1 || !d_inputs[0]) return fail(h, PBT_EINVAL, "GAN eval needs 1 input: eval_x");
    return gan_eval(h, static_cast<const float*>(d_inputs[0]), static_cast<hipStream_t>(hip_stream));
  }
  if (!d_inputs || n_inputs != 2 || !d_inputs[0] || !d_inputs[1])
    return fail(h, PBT_EINVAL, "classifier eval needs 2 inputs: eval_x, eval_y");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const float* x = static_cast<const float*>(d_inputs[0]);
  const int32_t* y = static_cast<const int32_t*>(d_inputs[1]);
  if (h->plan.fused_small) {
    FusedSmallArgs fa;
    fill_fused(h, &fa);
    fa.x = x; fa.y = y; fa.n_rows = h->cfg.n_eval;
    fused_small_plan(fa, true);
    PBT_HIP(h, fused_small_eval(fa, s));
    return PBT_OK;
  }
  return eval_bf16(h, x, y, s);
}

pbt_status pbt_exploit_explore(pbt_handle* h, int64_t round_index, const float* d_scores_override, void* hip_stream) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  if (round_index < 0 || round_index > 0xffffffffLL) return fail(h, PBT_EINVAL, "round index outside 0..2^32-1");
  const pbt_config& c = h->cfg;
  const Plan& p = h->plan;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  ExploitArgs a;
  a.score = h->st<float>(p.o_score);
  a.score_override = d_scores_override;
  a.H = h->st<float>(p.o_hyper);
  a.t = h->st<int32_t>(p.o_t);
  a.order = h->st<int32_t>(p.o_order);
  a.donor = h->st<int32_t>(p.o_donor);
  a.parent = h->st<int32_t>(p.o_parent);
  a.recip = h->st<int32_t>(p.o_recip);
  a.n_recip = h->st<int32_t>(p.o_nrecip);
  a.tournament = c.exploit_mode != PBT_EXPLOIT_TRUNCATION;
  a.ttest = c.exploit_mode == PBT_EXPLOIT_TTEST;
  a.ttest_alpha = (double)c.ttest_alpha;
  a.hist = a.ttest ? h->st<float>(p.o_hist) : nullptr;
  a.resample = c.explore_mode == PBT_EXPLORE_RESAMPLE;
  a.keep_weights = c.keep_weights; a.keep_hypers = c.keep_hypers;
  a.resample_always = c.resample_prob >= 1.f;
  a.resample_thr = a.resample_always ? 0xffffffffu : (uint32_t)std::floor((double)c.resample_prob * 4294967296.0);
  for (int k = 0; k < 8; ++k) { a.prior_kind[k] = 0; a.prior_a[k] = a.prior_b[k] = 0.0; }
  if (a.resample && !c.keep_hypers) {
    if (!h->have_priors) return fail(h, PBT_ESTATE, "resample explore needs priors: call pbt_set_priors or pbt_init_population first");
    for (int k = 0; k < c.n_hyper; ++k) {
      const pbt_prior& pr = h->priors[k];
      a.prior_kind[k] = pr.kind;
      a.prior_a[k] = pr.kind == 1 ? std::log(pr.lo) : pr.lo;
      a.prior_b[k] = pr.kind == 1 ? std::log(pr.hi) : pr.hi;
    }
  }
  a.P = c.P; a.n_trunc = c.n_trunc; a.n_hyper = c.n_hyper;
  a.f_lo = c.perturb_lo; a.f_hi = c.perturb_hi;
  for (int k = 0; k < 8; ++k) a.h_max[k] = k < c.n_hyper ? c.hyper_max[k] : INFINITY;
  a.round = (uint32_t)round_index; a.seed = c.seed;
  PBT_LAUNCH(h, PBT_K_RANK, s, rank_select_explore(a, s));
  if (c.keep_weights) return PBT_OK;  // hyperparameters only: nothing to copy
  CopyArrays ca;
  ca.n = 0;
  for (int k = 0; k < 6; ++k) ca.stage[k] = a.tournament ? h->sc<char>(p.o_stage[k]) : nullptr;
  const int64_t S = p.lay.stride;
  ca.base[ca.n] = h->st<char>(p.o_w32); ca.row_bytes[ca.n++] = S * 4;
  ca.base[ca.n] = h->st<char>(p.o_opt0); ca.row_bytes[ca.n++] = S * 4;
  if (c.optimizer == PBT_OPT_ADAM) { ca.base[ca.n] = h->st<char>(p.o_opt1); ca.row_bytes[ca.n++] = S * 4; }
  if (c.compute_dtype == PBT_DTYPE_BF16) { ca.base[ca.n] = h->st<char>(p.o_w16); ca.row_bytes[ca.n++] = S * 2; }
  if (c.workload == PBT_WL_A2C) { ca.base[ca.n] = h->st<char>(p.o_hist); ca.row_bytes[ca.n++] = 12 * 4; }
  PBT_LAUNCH(h, PBT_K_COPY, s, gather_copy(ca, a.recip, a.donor, a.tournament ? c.P : c.n_trunc, a.n_recip, a.tournament, s));
  return PBT_OK;
}

static pbt_status xfer(pbt_handle* h, int32_t which, int32_t member, void* host, size_t bytes, void* hip_stream, bool to_host) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  if (!host) return fail(h, PBT_EINVAL, "host pointer is NULL");
  ArrInfo ai;
  pbt_status st = arr_info(h, which, &ai);
  if (st != PBT_OK) return st;
  if (member < -1 || member >= h->cfg.P) return fail(h, PBT_EINVAL, "member %d outside -1..P-1", member);
  const size_t row = ai.elem * (size_t)ai.cols;
  const size_t want = member < 0 ? row * h->cfg.P : row;
  if (bytes != want) return fail(h, PBT_EINVAL, "buffer is %zu bytes, the selection is %zu", bytes, want);
  char* dev = (ai.in_scratch ? h->scratch : h->state) + ai.off + (member < 0 ? 0 : row * (size_t)member);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (to_host) {
    PBT_HIP(h, hipMemcpyAsync(host, dev, want, hipMemcpyDeviceToHost, s));
  } else {
    PBT_HIP(h, hipMemcpyAsync(dev, host, want, hipMemcpyHostToDevice, s));
    if (which == PBT_ARR_W32 && h->cfg.compute_dtype == PBT_DTYPE_BF16) {
      const size_t eoff = (size_t)(dev - (h->state + h->plan.o_w32)) / 4;
      PBT_HIP(h, f32_to_bf16(reinterpret_cast<const float*>(dev), h->st<bf16_t>(h->plan.o_w16) + eoff, (int64_t)(want / 4), s));
    }
  }
  PBT_HIP(h, hipStreamSynchronize(s));
  return PBT_OK;
}

pbt_status pbt_get_state(pbt_handle* h, int32_t which, int32_t member, void* h_dst, size_t dst_bytes, void* hip_stream) {
  return xfer(h, which, member, h_dst, dst_bytes, hip_stream, true);
}

pbt_status pbt_set_state(pbt_handle* h, int32_t which, int32_t member, const void* h_src, size_t src_bytes,
                         void* hip_stream) {
  if (which == PBT_ARR_GRAD || which == PBT_ARR_ORDER || which == PBT_ARR_DONOR || which == PBT_ARR_LOSS ||
      which == PBT_ARR_TRAJ_OBS || which == PBT_ARR_TRAJ_ACT || which == PBT_ARR_TRAJ_REW)
    return fail(h, PBT_EINVAL, "array %d is an output and cannot be set", which);
  return xfer(h, which, member, const_cast<void*>(h_src), src_bytes, hip_stream, false);
}

pbt_status pbt_state_ptr(pbt_handle* h, int32_t which, void** d_ptr, size_t* bytes) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  ArrInfo ai;
  pbt_status st = arr_info(h, which, &ai);
  if (st != PBT_OK) return st;
  if (d_ptr) *d_ptr = (ai.in_scratch ? h->scratch : h->state) + ai.off;
  if (bytes) *bytes = ai.elem * (size_t)ai.cols * h->cfg.P;
  return PBT_OK;
}

static void drop_events(pbt_handle* h) {
  for (hipEvent_t e : h->ev_start) (void)hipEventDestroy(e);
  for (hipEvent_t e : h->ev_stop) (void)hipEventDestroy(e);
  h->ev_start.clear();
  h->ev_stop.clear();
  h->ev_class.clear();
  h->ev_used = 0;
  h->timed_mask = 0;
  h->timed_stride = 1;
  for (size_t& n : h->timed_seen) n = 0;
}

pbt_status pbt_timing_enable_classes(pbt_handle* h, uint32_t class_mask, int32_t max_launches) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  if (class_mask >> PBT_K_COUNT) return fail(h, PBT_EINVAL, "class mask 0x%x names a class beyond %d", class_mask, PBT_K_COUNT - 1);
  drop_events(h);
  if (class_mask == 0) return PBT_OK;
  if (max_launches < 1 || max_launches > (1 << 20)) return fail(h, PBT_EINVAL, "max_launches outside 1..2^20");
  for (int k = 0; k < max_launches; ++k) {
    hipEvent_t a, b;
    PBT_HIP(h, hipEventCreate(&a));
    h->ev_start.push_back(a);
    PBT_HIP(h, hipEventCreate(&b));
    h->ev_stop.push_back(b);
  }
  h->ev_class.assign((size_t)max_launches, PBT_K_NONE);
  h->timed_mask = class_mask;
  return PBT_OK;
}

pbt_status pbt_timing_enable(pbt_handle* h, int32_t kernel_class, int32_t max_launches) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  if (kernel_class < PBT_K_NONE || kernel_class >= PBT_K_COUNT) return fail(h, PBT_EINVAL, "unknown kernel class %d", kernel_class);
  return pbt_timing_enable_classes(h, kernel_class == PBT_K_NONE ? 0u : 1u << kernel_class, max_launches);
}

pbt_status pbt_timing_stride(pbt_handle* h, int32_t stride) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  if (stride < 1) return fail(h, PBT_EINVAL, "stride must be at least 1");
  h->timed_stride = stride;
  for (size_t& n : h->timed_seen) n = 0;
  return PBT_OK;
}

// Sums the recorded pairs of one class (PBT_K_NONE: of all classes).
static pbt_status sum_events(pbt_handle* h, int klass, double* total_ms, int64_t* launches) {
  double sum = 0.0;
  int64_t n = 0;
  for (size_t k = 0; k < h->ev_used; ++k) {
    if (klass != PBT_K_NONE && h->ev_class[k] != klass) continue;
    PBT_HIP(h, hipEventSynchronize(h->ev_stop[k]));
    float ms = 0.f;
    PBT_HIP(h, hipEventElapsedTime(&ms, h->ev_start[k], h->ev_stop[k]));
    sum += ms;
    ++n;
  }
  if (total_ms) *total_ms = sum;
  if (launches) *launches = n;
  return PBT_OK;
}

pbt_status pbt_timing_read_class(pbt_handle* h, int32_t kernel_class, double* total_ms, int64_t* launches) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  if (kernel_class < 0 || kernel_class >= PBT_K_COUNT) return fail(h, PBT_EINVAL, "unknown kernel class %d", kernel_class);
  return sum_events(h, kernel_class, total_ms, launches);
}

pbt_status pbt_timing_read(pbt_handle* h, double* total_ms, int64_t* launches) {
  if (!h) return fail(nullptr, PBT_EINVAL, "handle is NULL");
  pbt_status st = sum_events(h, PBT_K_NONE, total_ms, launches);
  if (st == PBT_OK) h->ev_used = 0;
  return st;
}

pbt_status pbt_destroy(pbt_handle* h) {
  if (h) drop_events(h);
  delete h;
  return PBT_OK;
}

const char* pbt_last_error(const pbt_handle* h) { return h ? h->err.c_str() : g_last_error.c_str(); }

pbt_status pbt_batched_gemm_bf16(const void* d_a, int64_t lda, int64_t stride_a, int32_t a_m_contig, const void* d_b,
                                 int64_t ldb, int64_t stride_b, int32_t b_k_contig, void* d_c, int64_t ldc,
                                 int64_t stride_c, int32_t c_is_bf16, int32_t M, int32_t N, int32_t K, int32_t batch,
                                 void* hip_stream) {
  if (!d_a || !d_b || !d_c) return fail(nullptr, PBT_EINVAL, "NULL operand");
  if (M < 1 || N < 1 || K < 1 || batch < 1) return fail(nullptr, PBT_EINVAL, "M, N, K, batch must be positive");
  if (lda % 8 || ldb % 8 || stride_a % 8 || stride_b % 8 || ((uintptr_t)d_a | (uintptr_t)d_b) % 16)
    return fail(nullptr, PBT_EINVAL, "operand pitches / strides must be multiples of 8 elements and bases 16-byte aligned");
  if (lda < (a_m_contig ? M : K) || ldb < (b_k_contig ? K : N) || ldc < N) return fail(nullptr, PBT_EINVAL, "pitch smaller than the row");
  GemmOperands o{static_cast<const bf16_t*>(d_a), lda, stride_a, a_m_contig != 0,
                 static_cast<const bf16_t*>(d_b), ldb, stride_b, b_k_contig != 0, M, N, K, batch};
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = c_is_bf16 ? gemm_store_bf16(o, static_cast<bf16_t*>(d_c), ldc, stride_c, s)
                           : gemm_store_f32(o, static_cast<float*>(d_c), ldc, stride_c, s);
  if (e != hipSuccess) return fail(nullptr, PBT_EDEVICE, "GEMM launch failed: %s", hipGetErrorString(e));
  return PBT_OK;
}

}  // extern "C"
