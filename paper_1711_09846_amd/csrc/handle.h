// Host-side state behind a pbt_handle: the validated configuration, the carve-up of the caller's
// two device buffers, error reporting and the launch macros shared by the workload files.
#pragma once
#include "../../include/pbt.h"

#include <cstdarg>
#include <cstdio>
#include <string>
#include <vector>

#include "internal.h"

namespace pbt {

constexpr int64_t SEG_ALIGN = 64;      // elements: start of every W_l and b_l
constexpr int64_t STRIDE_ALIGN = 256;  // elements: per-member stride
constexpr size_t BUF_ALIGN = 256;      // bytes: every carved array

inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

struct Carver {
  size_t off = 0;
  size_t take(size_t bytes) {
    const size_t o = off;
    off += (bytes + BUF_ALIGN - 1) / BUF_ALIGN * BUF_ALIGN;
    return o;
  }
};

struct GanPlan {
  int n_g, n_d;                       // layers of generator / discriminator; layer l of D is layout index n_g + l
  int64_t g_count, d_begin, d_count;  // ranges of the flat parameter vector
  int col_lr_g, col_lr_d;
  int eval_rows;
  // scratch offsets (bytes)
  size_t o_zin, o_ga[PBT_MAX_DIMS], o_gz[PBT_MAX_DIMS], o_gdz[PBT_MAX_DIMS];
  size_t o_dx, o_da[PBT_MAX_DIMS], o_dz[PBT_MAX_DIMS], o_ddz[PBT_MAX_DIMS];
  size_t o_dlogits, o_rowloss;
  size_t o_hout, o_gin;   // WGAN-GP: the critic's outputs (float [P][rows][32]) and its input gradient on the interpolated rows (float [P][batch][width])
  size_t o_ez, o_ea[2], o_ex, o_ey, o_nx, o_ny, o_pxx, o_pyy, o_pxy;
};

struct A2CPlan {
  int rows, col_ent;
  size_t o_a[PBT_MAX_DIMS], o_z[PBT_MAX_DIMS], o_dz[PBT_MAX_DIMS], o_out, o_dout, o_act, o_rew;
  // on-policy generation: latent states (double [P][batch][latent_dim]), the policy's hidden activations and
  // head outputs for one time step ([P][batch][width])
  size_t o_lat, o_ga[PBT_MAX_DIMS], o_gout;
};

struct TfBlockOff { int64_t ln1g, ln1b, wqkv, bqkv, wo, bo, ln2g, ln2b, w1, b1, w2, b2; };
struct TfPlan {
  int col_drop, col_ls;
  int64_t tok, pos, lnfg, lnfb, whead, bhead;   // parameter offsets (elements)
  TfBlockOff blk[PBT_MAX_DIMS];
  // scratch offsets (bytes); activations are [P][batch*seq][width]
  size_t o_tokens, o_targets, o_h[PBT_MAX_DIMS + 1], o_hmid[PBT_MAX_DIMS];
  size_t o_mean1[PBT_MAX_DIMS], o_rstd1[PBT_MAX_DIMS], o_mean2[PBT_MAX_DIMS], o_rstd2[PBT_MAX_DIMS], o_meanf, o_rstdf;
  size_t o_u[PBT_MAX_DIMS], o_qkv[PBT_MAX_DIMS], o_pq[PBT_MAX_DIMS], o_pd[PBT_MAX_DIMS], o_o[PBT_MAX_DIMS];
  size_t o_u2[PBT_MAX_DIMS], o_z1[PBT_MAX_DIMS], o_fd[PBT_MAX_DIMS];
  size_t o_mask[PBT_MAX_DIMS][3];   // keep bits of the block's three dropout sites outside attention
  bool fused_attn;                  // one attention kernel per pass: no score / probability arrays, o_keep instead
  size_t o_keep[PBT_MAX_DIMS];      // keep bits of the attention dropout site (fused attention only)
  size_t o_attn_stats;              // softmax row statistics between the two backward kernels (fused attention only)
  size_t o_wpart, o_wcolpart;       // partial weight gradients of contractions cut into pieces (transformer_host.hip: wgrad)
  int64_t wpart_elems, wcol_elems;  // elements per (member, piece) these buffers hold (0: no matrix of this workload is cut)
  size_t o_score, o_tmp_d[3], o_tmp_f[2], o_dqkv, o_uf, o_logits, o_dlogits, o_rowloss, o_evalrow, o_tokstart, o_tokcursor, o_tokorder, o_lnpart;
};

struct Plan {
  pbt_layout lay;
  int n_loss;
  // offsets in bytes inside d_state
  size_t o_w32, o_opt0, o_opt1, o_w16, o_hyper, o_score, o_loss, o_t, o_order, o_donor, o_parent, o_recip, o_nrecip, o_hist;
  size_t state_bytes;
  // offsets in bytes inside d_scratch
  size_t o_grad, o_y, o_dlogits, o_rowloss, o_x32;
  size_t o_act[PBT_MAX_DIMS], o_z[PBT_MAX_DIMS], o_dz[PBT_MAX_DIMS];
  size_t o_evalx, o_evala[2], o_evalrow;
  size_t o_stage[6];  // tournament exploit: staging rows of the copied arrays
  size_t scratch_bytes;
  int eval_chunk;
  bool fused_small;  // fp32: the whole step runs in one LDS-resident kernel
  int col_lr, col_beta1, col_wd;
  GanPlan gan;
  A2CPlan a2c;
  TfPlan tf;
};

}  // namespace pbt

struct pbt_handle {
  pbt_config cfg;
  pbt::Plan plan;
  char* state;
  char* scratch;
  std::string err;
  pbt_prior priors[PBT_MAX_HYPER];  // for resample explore (pbt_set_priors / pbt_init_population)
  bool have_priors = false;
  // optional event timing of kernel classes
  uint32_t timed_mask = 0;  // bit k set: launches of class k are bracketed
  std::vector<hipEvent_t> ev_start, ev_stop;
  std::vector<int> ev_class;  // class of every recorded pair
  size_t ev_used = 0;
  int timed_stride = 1;                    // every timed_stride-th launch of a class is recorded
  size_t timed_seen[PBT_K_COUNT] = {};     // launches of each class since timing was enabled
  template <class T> T* st(size_t off) const { return reinterpret_cast<T*>(state + off); }
  template <class T> T* sc(size_t off) const { return reinterpret_cast<T*>(scratch + off); }
};

namespace pbt {

// Records the message on the handle (when there is one) and per thread; returns `code`.
pbt_status fail(pbt_handle* h, pbt_status code, const char* fmt, ...);

#define PBT_HIP(h, call)                                                                        \
  do {                                                                                          \
    hipError_t e_ = (call);                                                                     \
    if (e_ != hipSuccess) return pbt::fail(h, PBT_EDEVICE, "%s failed: %s", #call, hipGetErrorString(e_)); \
  } while (0)

// Runs `call` (a launcher returning hipError_t); when its class is the timed one, brackets it
// with an event pair on the same stream.
#define PBT_LAUNCH(h, klass, s, call)                                                           \
  do {                                                                                          \
    const bool timed_ = (((h)->timed_mask >> (klass)) & 1u) && (h)->ev_used < (h)->ev_start.size() && \
                        ((h)->timed_seen[klass]++ % (size_t)(h)->timed_stride) == 0;            \
    if (timed_) PBT_HIP(h, hipEventRecord((h)->ev_start[(h)->ev_used], s));                     \
    PBT_HIP(h, call);                                                                           \
    if (timed_) {                                                                               \
      PBT_HIP(h, hipEventRecord((h)->ev_stop[(h)->ev_used], s));                                \
      (h)->ev_class[(h)->ev_used] = (klass);                                                    \
      ++(h)->ev_used;                                                                           \
    }                                                                                           \
  } while (0)

// gan_host.hip: the GAN workload (Section 4.3.1)
pbt_status gan_check_and_plan(const pbt_config* c, Plan* pl, Carver* scratch);
pbt_status gan_step(pbt_handle* h, const float* train_x, uint32_t step, hipStream_t s);
pbt_status gan_eval(pbt_handle* h, const float* eval_x, hipStream_t s);

// a2c_host.hip: the actor-critic workload (Section 4.1.1)
pbt_status a2c_check_and_plan(const pbt_config* c, Plan* pl, Carver* scratch);
pbt_status a2c_step(pbt_handle* h, const float* obs, const int32_t* actions, const float* rewards, uint32_t step, hipStream_t s);
struct A2CEnv { const double *A, *B, *C, *w, *noise; };   // the latent system, device arrays
pbt_status a2c_step_on_policy(pbt_handle* h, const A2CEnv& env, uint32_t step, hipStream_t s);
pbt_status a2c_eval(pbt_handle* h, hipStream_t s);

// transformer_host.hip: the language-model workload (Section 4.2.1)
pbt_status tf_layout(const pbt_config* c, Plan* pl);
pbt_status tf_check_and_plan(const pbt_config* c, Plan* pl, Carver* scratch);
pbt_status tf_step(pbt_handle* h, const int32_t* pool, uint32_t step, hipStream_t s);
pbt_status tf_eval(pbt_handle* h, const int32_t* eval_tokens, hipStream_t s);

}  // namespace pbt
