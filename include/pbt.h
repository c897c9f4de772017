/*
 * pbt.h -- C ABI of the MI355X population step of Population Based Training
 * (Jaderberg et al., "Population Based Training of Neural Networks").
 *
 * The entry points follow the paper's decomposition of the method (Section 3,
 * Algorithm 1): `step` (one gradient update of every member under its own
 * hyperparameters, Eq. 2), `eval` (the score of every member, Eq. 1), `ready`
 * (stays with the caller: a test on the step count), and `exploit` + `explore`
 * (truncation selection and perturb, Section 4.1.1), executed for the whole
 * population in lock-step as in the partially synchronous scheme of
 * Appendix A.1.  The population store (theta, h, p, t) of Algorithm 1 lives
 * in device memory for the whole run.
 *
 * Conventions
 *   memory    Every pointer named d_* is DEVICE memory, h_* is HOST memory.
 *             The caller allocates and owns all device memory; the library
 *             owns only the host-side handle.  pbt_step, pbt_eval and
 *             pbt_exploit_explore allocate nothing and never synchronise:
 *             they enqueue kernels on `hip_stream` (a hipStream_t passed as
 *             void*, NULL = the null stream) and return.
 *   errors    Every call returns a pbt_status; 0 is success.  Arguments are
 *             validated before anything is launched.  pbt_last_error()
 *             returns a human-readable description of the most recent failure.
 *   determinism  All results are a pure function of (state, inputs, step or
 *             round index, seed): no atomics, fixed reduction orders.
 *   layout    A member's parameters are one flat vector: for every dense
 *             layer l the matrix W_l[fan_in][fan_out] (row-major) followed by
 *             the bias b_l[fan_out]; each of the two starts at a multiple of
 *             64 elements; the per-member stride is a multiple of 256 elements.
 *             Padding elements are zero and stay zero.  pbt_query_sizes()
 *             reports the offsets.  Population arrays are member-major:
 *             X[P][stride].
 *   random numbers  Philox4x32-10, key = (seed low word, seed high word),
 *             counter = (step or round index, member, domain tag, element):
 *             domain 1 = mini-batch row -> data-set row floor(x*n_train/2^32);
 *             domain 2 = donor -> position floor(x*n_trunc/2^32) in the top set;
 *             domain 3 = explore, element = hyperparameter k, bit 0 of word 0:
 *             0 -> perturb_lo, 1 -> perturb_hi.
 */
#ifndef PBT_H
#define PBT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PBT_MAX_DIMS 16
#define PBT_MAX_HYPER 8
#define PBT_MAX_P 1024

typedef struct pbt_handle pbt_handle; /* opaque; host memory owned by the library */

typedef enum {
  PBT_OK = 0,
  PBT_EINVAL = -1,       /* bad argument or inconsistent configuration */
  PBT_ENOMEM = -2,       /* a caller-provided buffer is too small */
  PBT_EDEVICE = -3,      /* a HIP call or kernel launch failed */
  PBT_ESTATE = -4,       /* call not valid in the handle's current state */
  PBT_EUNSUPPORTED = -5  /* valid request that the library has no kernel for */
} pbt_status;

enum { PBT_EXPLOIT_TRUNCATION = 0, PBT_EXPLOIT_TOURNAMENT = 1, PBT_EXPLOIT_TTEST = 2 };
enum { PBT_EXPLORE_PERTURB = 0, PBT_EXPLORE_RESAMPLE = 1 };
enum { PBT_WL_CLASSIFIER = 1, PBT_WL_GAN = 3, PBT_WL_TRANSFORMER = 4, PBT_WL_A2C = 5 }; /* workload families */
enum { PBT_ACT_NONE = 0, PBT_ACT_RELU = 1, PBT_ACT_GELU = 2, PBT_ACT_LEAKY_RELU = 3, PBT_ACT_TANH = 4 };
enum { PBT_OPT_SGD_MOMENTUM = 0, PBT_OPT_ADAM = 1, PBT_OPT_RMSPROP = 2 };
enum { PBT_DTYPE_FP32 = 0, PBT_DTYPE_BF16 = 1 };      /* BF16 = bf16 operands, fp32 accumulate, fp32 master weights */
enum { PBT_ROLE_LR = 0, PBT_ROLE_BETA1 = 1, PBT_ROLE_WD = 2, /* meaning of a hyperparameter column */
       PBT_ROLE_LR_G = 3, PBT_ROLE_LR_D = 4,                  /* GAN: generator / discriminator learning rate */
       PBT_ROLE_ENTROPY_COST = 5,                             /* actor-critic: weight of the entropy bonus */
       PBT_ROLE_DROPOUT = 6, PBT_ROLE_LABEL_SMOOTH = 7 };     /* transformer: dropout rate, label smoothing */

/* Arrays of the population store that pbt_get_state / pbt_set_state address. */
enum {
  PBT_ARR_W32 = 0,    /* float  [P][stride]  master weights theta                     */
  PBT_ARR_OPT0 = 1,   /* float  [P][stride]  momentum / Adam m / RMSProp mean square  */
  PBT_ARR_OPT1 = 2,   /* float  [P][stride]  Adam v (Adam only)                       */
  PBT_ARR_W16 = 3,    /* bf16   [P][stride]  shadow of theta (BF16 only)              */
  PBT_ARR_GRAD = 4,   /* float  [P][stride]  gradient of the last step (scratch)      */
  PBT_ARR_HYPER = 5,  /* float  [P][n_hyper] hyperparameters h                        */
  PBT_ARR_SCORE = 6,  /* float  [P]          p, written by pbt_eval                   */
  PBT_ARR_LOSS = 7,   /* float  [P][n_loss]  training loss(es) of the last step; n_loss = 1, GAN: 2 = {L_D, L_G} */
  PBT_ARR_T = 8,      /* int32  [P]          optimiser updates applied (travels with theta) */
  PBT_ARR_ORDER = 9,  /* int32  [P]          members from best to worst, last exploit */
  PBT_ARR_DONOR = 10, /* int32  [P]          donor of the last exploit, -1 = kept     */
  PBT_ARR_PARENT = 11,/* int32  [P]          member last copied from (initially self) */
  PBT_ARR_HIST = 12,  /* float  [P][12]      actor-critic: ring of the last 10 unroll returns, slot 10 = number of
                                             unrolls so far (int32 bits), slot 11 unused; travels with theta */
  /* actor-critic: the unroll the last step was taken on (scratch; read-only): observations as the network saw
     them, bf16 [P][batch * (unroll + 1)][dims[0]] (trajectory-major, unroll + 1 rows per trajectory), actions
     int32 [P][batch * unroll], rewards float [P][batch * unroll] */
  PBT_ARR_TRAJ_OBS = 13,
  PBT_ARR_TRAJ_ACT = 14,
  PBT_ARR_TRAJ_REW = 15,
  PBT_ARR_COUNT = 16
};

typedef struct {
  int32_t workload;                 /* PBT_WL_* */
  int32_t P;                        /* population size, 1..PBT_MAX_P */
  int32_t batch;                    /* rows per member per step */
  int32_t n_layers;                 /* dense layers; dims[0..n_layers] are the widths */
  int32_t dims[PBT_MAX_DIMS];
  int32_t act;                      /* hidden activation, PBT_ACT_* (the output layer is linear) */
  int32_t optimizer;                /* PBT_OPT_* */
  int32_t compute_dtype;            /* PBT_DTYPE_* */
  int32_t n_hyper;                  /* columns of h, 1..PBT_MAX_HYPER */
  int32_t hyper_role[PBT_MAX_HYPER];/* PBT_ROLE_* of each column */
  float hyper_max[PBT_MAX_HYPER];   /* upper clamp applied after explore; INFINITY = none */
  int32_t n_trunc;                  /* size of top and of bottom set; 0 disables exploit; 2*n_trunc <= P */
  float perturb_lo, perturb_hi;     /* explore factors, 0.8f and 1.2f in the paper's RL and translation runs */
  float opt_const[4];               /* SGD: {momentum}.  Adam: {beta1, beta2, eps, weight decay} (beta1 / decay are
                                       defaults for when no column has that role).  RMSProp: {rho, eps}. */
  /* PBT_WL_GAN only: dims/n_layers/act describe the generator (latent -> data), the fields below
     the discriminator (data -> 1 logit).  Both networks live in one flat parameter vector per
     member, generator layers first, so an exploit copies both (Section 4.3.1). */
  int32_t act_out;                  /* generator output activation (PBT_ACT_TANH) */
  int32_t n_layers2;                /* discriminator layers; dims2[0] = dims[n_layers], dims2[n_layers2] = 1 */
  int32_t dims2[PBT_MAX_DIMS];
  int32_t act2;                     /* discriminator hidden activation */
  /* PBT_WL_A2C only: dims describe torso + one head of dims[n_layers] = n_actions + 1 outputs
     (policy logits, then the value); `batch` trajectories of `unroll` transitions per step. */
  int32_t unroll;
  float gamma, value_cost;          /* discount; weight of the squared value error (0.5) */
  /* PBT_WL_TRANSFORMER only: decoder-only transformer with n_layers pre-LayerNorm blocks; `batch`
     sequences of tf_seq tokens per step (the pool rows hold tf_seq + 1 tokens: inputs and next-token
     targets); dims[] unused.  Limits (PBT_EUNSUPPORTED otherwise): tf_d_model, the head width tf_d_model / tf_heads,
     tf_d_ff, tf_vocab and tf_seq multiples of 8; tf_seq <= 4096; batch * tf_seq <= 16000. */
  int32_t tf_vocab, tf_d_model, tf_heads, tf_d_ff, tf_seq;
  int32_t n_train, n_eval;          /* rows (classifier, GAN) or trajectories (actor-critic) of the training set; rows of the held-out set */
  int32_t eval_chunk;               /* rows of the held-out set scored per pass (bounds scratch); 0 = library picks */
  int32_t fuse_optimizer;           /* bf16 compute: 1 = apply the optimiser inside the weight-gradient GEMMs (the gradient of
                                       those matrices is then never stored: PBT_ARR_GRAD holds only bias / output-layer
                                       gradients); 0 = separate optimiser pass over a complete gradient */
  /* Variants of exploit and explore (all 0 = truncation selection + perturb on weights and hyperparameters).
     exploit_mode 1: binary tournament (Section 4.3.1, Exploit (b)): every member draws one other member
     uniformly (j = floor(x (P-1) / 2^32) from Philox counter (round, i, domain 2, 0), j += 1 if j >= i) and
     copies it if that member ranks above it; n_trunc is ignored; every recipient receives its donor's state
     as it was before the pass.
     exploit_mode 2: t-test selection (Section 4.1.1, Exploit (a); actor-critic workload only): the opponent is
     drawn as in the tournament; the member copies it if the opponent's score history (the last up to 10 unroll
     returns) has the higher mean and Welch's one-sided test gives p < ttest_alpha (Student t with the
     Welch-Satterthwaite degrees of freedom, evaluated in double; zero variance on both sides counts as
     significant); histories with fewer than two entries neither copy nor are copied.
     explore_mode 1: resample (Section 4.1.1, Explore (b)): hyperparameter k of an overwritten member is drawn
     afresh from its prior (pbt_set_priors) iff word 1 of Philox counter (round, i, domain 3, k) is below
     floor(resample_prob 2^32) (always when resample_prob >= 1), from u = (word 2 + 0.5) / 2^32; otherwise the
     copied value stays; the upper clamp hyper_max applies.
     keep_weights / keep_hypers: the subsets of Section 4.4 ("PBT targets"): keep_weights = 1 copies (and
     explores) hyperparameters only, the recipient keeps its weights, optimiser state, update count, score
     and history; keep_hypers = 1 copies the weights and leaves the recipient's hyperparameters untouched. */
  int32_t exploit_mode, explore_mode;
  float resample_prob;
  int32_t keep_weights, keep_hypers;
  float ttest_alpha;                /* exploit_mode 2: significance level, 0 < alpha <= 1 */
  /* PBT_WL_A2C only.  on_policy = 1: every step first generates its unroll on the device from the member's
     current policy in a linear-Gaussian latent system of dimension latent_dim (see pbt_step), so that the
     score depends on the member's weights as in Section 4.1.1; 0: trajectories are drawn from a recorded pool. */
  int32_t on_policy, latent_dim;
  /* PBT_WL_GAN only.  gan_objective 0: non-saturating logistic GAN, one discriminator and one generator update per
     step.  1: the paper's own step (Section 4.3.1): n_critic updates of the discriminator, then one of the
     generator, on the WGAN-GP objective L_D = mean D(G(z)) - mean D(x) + gp_weight mean (|grad D(xhat)| - 1)^2,
     xhat = eps x + (1 - eps) G(z), L_G = -mean D(G(z')).  Critic update k of a step draws its rows from Philox
     counters (step, member, 1, k batch + r), its latents from sub-stream 3 + k, eps_r = (word 0 + 0.5) / 2^32 of
     counter (step, member, 14, k batch + r); its Adam bias correction counts n_critic (t - 1) + k + 1 updates.
     loss[i] = {L_D of the last critic update, L_G}. */
  int32_t gan_objective, n_critic;
  float gp_weight;
  uint64_t seed;                    /* Philox key */
} pbt_config;

/* Offsets (in elements) inside one member's flat parameter vector. */
#define PBT_MAX_SEGMENTS 96
typedef struct {
  int64_t stride;                   /* elements per member */
  int64_t n_params;                 /* elements that are parameters (rest is padding) */
  int64_t w_off[PBT_MAX_DIMS];      /* start of W_l (dense-layer workloads) */
  int64_t b_off[PBT_MAX_DIMS];      /* start of b_l */
  /* every parameter array in order of appearance (dense workloads: W_0, b_0, W_1, ...; transformer:
     token embedding [V][d], position embedding [S][d], per block {ln1 gain, ln1 bias, Wqkv [d][3d],
     bqkv, Wo [d][d], bo, ln2 gain, ln2 bias, W1 [d][f], b1, W2 [f][d], b2}, final gain, final bias,
     Whead [d][V], bhead) */
  int32_t n_seg;
  int64_t seg_off[PBT_MAX_SEGMENTS];
  int64_t seg_len[PBT_MAX_SEGMENTS];
} pbt_layout;

/* Sizes of the two device buffers pbt_init needs, and the parameter layout.
 * Any output pointer may be NULL.  Host-only; touches no device. */
pbt_status pbt_query_sizes(const pbt_config* cfg, size_t* state_bytes, size_t* scratch_bytes, pbt_layout* layout);

/* Algorithm 1, initial population.  Carves the population store out of
 * d_state (>= state_bytes, 256-byte aligned) and working buffers out of
 * d_scratch, zero-fills the store with kernels on hip_stream, sets t = 0,
 * parent[i] = i, score = -inf.  Weights and hyperparameters are then uploaded
 * with pbt_set_state.  *out is a new handle (free with pbt_destroy); on
 * failure *out is NULL.  The two buffers must outlive the handle. */
pbt_status pbt_init(const pbt_config* cfg, void* d_state, size_t state_bytes, void* d_scratch, size_t scratch_bytes,
                    void* hip_stream, pbt_handle** out);

/* A prior over one hyperparameter column: uniform on [lo, hi] or log-uniform (exp of a uniform
 * draw on [ln lo, ln hi]; needs 0 < lo). */
typedef struct {
  int32_t kind; /* 0 = uniform, 1 = log-uniform */
  double lo, hi;
} pbt_prior;

/* Figure 1(c) / Algorithm 1, initial population drawn on the device: every member gets independent
 * random weights (dense layers: uniform in +-1/sqrt(fan_in), biases included; transformer: tables and
 * matrices uniform in +-1/sqrt(fan_in) with fan_in = d_model for the two tables, LayerNorm gains 1,
 * biases 0) and hyperparameters drawn from priors[0..n_hyper-1] (HOST array).  Random words: Philox counter (0, member, domain 4,
 * position / 4) word position % 4 for the value at `position` of the member's flat parameter vector;
 * counter (0, member, domain 5, column) word 0 for a hyperparameter; u = (x + 0.5) / 2^32, evaluated
 * in double precision and rounded once to float.  Optimiser state, t and scores are reset as in
 * pbt_init.  Enqueues on hip_stream; no synchronisation. */
pbt_status pbt_init_population(pbt_handle* h, const pbt_prior* priors, void* hip_stream);

/* Section 4.1.1, Explore (b): the priors that resample-explore draws from (HOST array of n_hyper
 * entries, copied into the handle; pbt_init_population stores its priors the same way).  Host-only call.
 * PBT_EINVAL for a bad prior (as in pbt_init_population). */
pbt_status pbt_set_priors(pbt_handle* h, const pbt_prior* priors);

/* Section 3, Eq. 2: theta_i <- step(theta_i | h_i) for every member i, n_steps
 * times (step indices step_index .. step_index + n_steps - 1).  One step:
 * draw the member's mini-batch rows (Philox domain 1), forward, loss,
 * backward, optimiser update with lr / beta1 / weight decay read from h_i on
 * the device, t_i += 1.  Writes loss[P] (mean mini-batch loss before the last
 * update).  d_inputs for PBT_WL_CLASSIFIER: {train_x float[n_train][dims[0]],
 * train_y int32[n_train]}, device pointers in a HOST array of n_inputs = 2.
 * PBT_WL_A2C with on_policy = 0: {observations float[n_train][unroll + 1][dims[0]], actions
 * int32[n_train][unroll], rewards float[n_train][unroll]}; `batch` trajectories are drawn per member
 * (Philox domain 1).  With on_policy = 1 (Section 4.1.1: agents act with their current policy and are
 * evaluated by their last 10 episodic returns): d_inputs = {A double[nz][nz], B double[nz][n_actions],
 * C double[dims[0]][nz], w double[nz], noise double[3] = {observation, reward, transition scale}},
 * nz = latent_dim; the step first generates `batch` trajectories per member,
 *   z_0 ~ N(0, I); o_t = C z_t + noise[0] xi_t (rounded to float, then to bf16); a_t ~ softmax(policy
 *   logits of the member's network on o_t); r_t = w.z_t + noise[1] nu_t (float);
 *   z_{t+1} = A z_t + B[:, a_t] + noise[2] zeta_t,
 * the latent and every sum in double.  Philox counters (step, member, 32 + k, e / 4): k = 0 z_0 (element
 * e = r nz + j), 1 xi (e = (r (unroll + 1) + t) dims[0] + j), 3 nu (e = r unroll + t), 4 zeta
 * (e = (r unroll + t) nz + j), normals by Box-Muller from word pairs (0,1), (2,3) of a counter (cosine for
 * even e, sine for odd e, evaluated in double); k = 2: u = (word 0 + 0.5) / 2^32 of counter element
 * r unroll + t.  a_t = the number of actions k with cdf_k <= u (at most n_actions - 1), cdf the running
 * sum of the softmax probabilities, evaluated in double from the float logits. */
pbt_status pbt_step(pbt_handle* h, const void* const* d_inputs, int32_t n_inputs, int64_t step_index, int32_t n_steps,
                    void* hip_stream);

/* For callers that cannot allocate device memory or hold a working buffer per handle (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): pbt_step with its working
 * memory (the d_scratch of pbt_init: gradients, activations, per-row losses) taken from an array of
 * PBT_STATIC_SCRATCH_BYTES bytes that lives inside the library, one copy per GPU, held until the process
 * ends.  Same arguments, same kernels and bit-identical results as pbt_step; the population store stays
 * in the caller's d_state.  Calls no hipMalloc / hipFree and nothing that allocates.  PBT_ENOMEM when the
 * handle's configuration needs more working memory than the array holds (pbt_query_sizes reports the
 * need).  Every call on a GPU, from any handle, shares that GPU's array: it keeps the previous call's
 * contents (the call clears the part that must start at zero, with a fill kernel), and calls that overlap
 * in time on one GPU race.  PBT_ARR_GRAD of the handle (which lives in d_scratch) is not written. */
#define PBT_STATIC_SCRATCH_BYTES ((size_t)8 << 20)
pbt_status pbt_step_static(pbt_handle* h, const void* const* d_inputs, int32_t n_inputs, int64_t step_index,
                           int32_t n_steps, void* hip_stream);

/* Section 3, Eq. 1: p_i <- eval(theta_i) for every member; writes score[P].
 * PBT_WL_CLASSIFIER: minus the mean cross-entropy over the held-out set,
 * d_inputs = {eval_x float[n_eval][dims[0]], eval_y int32[n_eval]}.
 * PBT_WL_GAN: minus the biased squared maximum mean discrepancy, RBF kernel exp(-|a-b|^2 / (2 d)),
 * d = dims2[0], between n_eval generated rows (latents: Philox domain 6 + 2, step index 0) and the
 * n_eval held-out rows; d_inputs = {eval_x float[n_eval][dims2[0]]}.
 * PBT_WL_A2C (Section 4.1.1, Eval): the mean of the member's last (up to) 10 unroll returns, -inf
 * before the first step; n_inputs = 0.
 * PBT_WL_TRANSFORMER: minus the perplexity exp(mean next-token cross-entropy) over the n_eval
 * held-out sequences, no dropout, no smoothing; d_inputs = {tokens int32[n_eval][tf_seq + 1]}. */
pbt_status pbt_eval(pbt_handle* h, const void* const* d_inputs, int32_t n_inputs, void* hip_stream);

/* Section 4.1.1, Exploit (b) + Explore (a), for the whole population at once
 * (Appendix A.1).  Ranks score[P] (descending; ties: lower index first; -inf
 * then NaN last); every member of the bottom n_trunc draws a donor from the
 * top n_trunc (Philox domain 2) and receives a byte copy of the donor's
 * weights, optimiser state, bf16 shadow, update count and score; its
 * hyperparameters become the donor's times perturb_lo or perturb_hi per
 * column (Philox domain 3; one IEEE float multiply, then min with hyper_max).
 * All other members are left untouched.  d_scores_override (float[P], device)
 * replaces score[P] first when not NULL.  Writes order[P], donor[P], parent. */
pbt_status pbt_exploit_explore(pbt_handle* h, int64_t round_index, const float* d_scores_override, void* hip_stream);

/* Copies one array of the population store (PBT_ARR_*) to host memory.
 * member = -1: the whole array, else that member's row.  Synchronises
 * hip_stream.  dst_bytes must equal the size of what is copied. */
pbt_status pbt_get_state(pbt_handle* h, int32_t which, int32_t member, void* h_dst, size_t dst_bytes, void* hip_stream);

/* Inverse of pbt_get_state (used to upload an initial population or to resume
 * from a dump).  Writing PBT_ARR_W32 with BF16 compute also refreshes the bf16
 * shadow.  Synchronises hip_stream. */
pbt_status pbt_set_state(pbt_handle* h, int32_t which, int32_t member, const void* h_src, size_t src_bytes,
                         void* hip_stream);

/* Device address and size in bytes of one array of the store (no copy, no
 * sync), for callers that read results on the device. */
pbt_status pbt_state_ptr(pbt_handle* h, int32_t which, void** d_ptr, size_t* bytes);

/* Frees the handle (not the device buffers).  NULL is allowed. */
pbt_status pbt_destroy(pbt_handle* h);

/* Message for the most recent failure on this handle; with h = NULL, of the
 * most recent failed call that had no handle (per thread).  Never NULL; owned
 * by the library; valid until the next failing call. */
const char* pbt_last_error(const pbt_handle* h);

/* The population-batched GEMM used for every dense contraction of forward and
 * backward (Section 3, `step`), exposed for measurement and unit tests:
 *   C_i[M][N] = op(A_i) * op(B_i)   for i = 0..batch-1, bf16 operands, fp32 accumulate.
 * a_m_contig = 0: A_i is stored [M][K] with K contiguous (lda = row pitch);
 * 1: A_i is stored [K][M] with M contiguous.  b_k_contig = 0: B_i is stored
 * [K][N] with N contiguous; 1: B_i is stored [N][K] with K contiguous.
 * Pitches and batch strides are in elements and must be multiples of 8 (every
 * row 16-byte aligned, base pointers too); a batch stride of 0 shares the
 * operand between members.  c_is_bf16 selects bf16 or float output (ldc, stride_c
 * in elements of that type).  All pointers are device memory; M, N, K, batch > 0. */
pbt_status pbt_batched_gemm_bf16(const void* d_a, int64_t lda, int64_t stride_a, int32_t a_m_contig, const void* d_b,
                                 int64_t ldb, int64_t stride_b, int32_t b_k_contig, void* d_c, int64_t ldc,
                                 int64_t stride_c, int32_t c_is_bf16, int32_t M, int32_t N, int32_t K, int32_t batch,
                                 void* hip_stream);

/* Kernel classes for pbt_timing_enable. */
enum {
  PBT_K_NONE = -1,
  PBT_K_FETCH = 0,      /* mini-batch fetch                                  */
  PBT_K_GEMM_FWD = 1,   /* forward GEMMs (bias + activation fused)           */
  PBT_K_HEAD = 2,       /* output layer + loss + its backward kernels        */
  PBT_K_GEMM_WGRAD = 3, /* weight-gradient GEMMs                             */
  PBT_K_GEMM_DGRAD = 4, /* input-gradient GEMMs                              */
  PBT_K_BIAS_GRAD = 5,  /* (no launches of their own any more: bias gradients are column sums taken inside the weight-gradient GEMMs) */
  PBT_K_OPTIMIZER = 6,  /* fused per-member optimiser                        */
  PBT_K_RANK = 7,       /* rank + truncation select + perturb                */
  PBT_K_COPY = 8,       /* exploit gather-copy                               */
  PBT_K_FUSED_STEP = 9, /* LDS-resident fp32 step (small networks)           */
  PBT_K_COUNT = 10
};

/* Measurement aid (for benchmarks; not part of the method): brackets every launch of one kernel
 * class with a pair of HIP events on the stream it is launched on.  max_launches event pairs are
 * created here, on the host; launches beyond that are not recorded.  kernel_class = PBT_K_NONE
 * switches timing off and destroys the events.  Off by default. */
pbt_status pbt_timing_enable(pbt_handle* h, int32_t kernel_class, int32_t max_launches);

/* As pbt_timing_enable for several classes at once: bit k of class_mask selects class k (0 switches timing
 * off).  Every recorded pair remembers its class; pbt_timing_read_class sums one class without rearming,
 * pbt_timing_read sums all of them and rearms. */
pbt_status pbt_timing_enable_classes(pbt_handle* h, uint32_t class_mask, int32_t max_launches);
pbt_status pbt_timing_read_class(pbt_handle* h, int32_t kernel_class, double* total_ms, int64_t* launches);

/* Records only every stride-th launch of each timed class (stride >= 1; 1, the default, records all;
 * pbt_timing_enable resets it to 1).  An event pair costs the stream a few microseconds around the
 * launch it brackets, so a benchmark that also reports whole-run throughput samples the launches; an odd
 * stride visits the launches of a step in turn when a class has two per step. */
pbt_status pbt_timing_stride(pbt_handle* h, int32_t stride);

/* Synchronises the recorded events, returns the summed device time in milliseconds and the
 * number of recorded launches since the last read, and rearms the event pool. */
pbt_status pbt_timing_read(pbt_handle* h, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* PBT_H */
