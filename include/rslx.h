/*
 * rslx — single-GPU (gfx950) library for the data-parallel hot path of a GPU-only PPO
 * training loop: batched actor-critic inference (act), the GAE / returns reverse scan,
 * the multi-epoch minibatch PPO update, the DAgger-style behaviour-cloning update,
 * symmetry augmentation and the RND curiosity reward.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Plain C ABI.  Every function returns an int32 status (RSLX_OK = 0); on failure nothing
 *    has been launched unless stated, and rslx_last_error() gives a thread-local message.
 *  - "device" pointers are HIP device memory owned by the caller.  The library never
 *    allocates, frees or keeps them.  Scratch memory comes from the caller's workspace
 *    (`ws`, `ws_bytes`), sized by the matching *_workspace_bytes() query; a workspace that is
 *    too small gives RSLX_ERR_WORKSPACE.  Device pointers must be 16-byte aligned.
 *  - "host" pointers are ordinary host memory, read (or written) before the call returns.
 *  - All matrices are dense row-major fp32 unless said otherwise.
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = default stream).
 *    No entry point synchronises with the host; outputs are valid once the stream reaches
 *    the end of the enqueued work.  Calls that share a workspace must be stream-ordered.
 *  - Flat parameter layout of a network (struct rslx_mlp): for each linear layer l in order,
 *    W_l as [dims[l], dims[l+1]] row-major (y = x W + b), then b_l [dims[l+1]]; an actor's
 *    buffer ends with log_std[dims[n_layers]].  grads / adam_m / adam_v mirror this layout.
 *    Hidden layers use ELU with parameter elu_alpha; the last layer is linear.
 */
#ifndef RSLX_H
#define RSLX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RSLX_OK 0
#define RSLX_ERR_INVALID_ARG 1
#define RSLX_ERR_SHAPE 2
#define RSLX_ERR_WORKSPACE 3
#define RSLX_ERR_HIP 4
#define RSLX_ERR_UNSUPPORTED 5

#define RSLX_MAX_LAYERS 8
#define RSLX_MAX_ACTIONS 64

/* Columns of the per-minibatch statistics rows written by the update calls. */
#define RSLX_NSTATS 8
#define RSLX_STAT_SURROGATE 0
#define RSLX_STAT_VALUE_LOSS 1
#define RSLX_STAT_ENTROPY 2
#define RSLX_STAT_KL 3
#define RSLX_STAT_GRAD_NORM 4 /* before clipping */
#define RSLX_STAT_CLIP_FRAC 5
#define RSLX_STAT_MIRROR_LOSS 6
#define RSLX_STAT_RND_LOSS 7
/* rslx_bc_update uses column 0 for the MSE loss and column 4 for the gradient norm. */

/* rslx_act flags */
#define RSLX_ACT_DETERMINISTIC 1u /* actions := mu (no noise) */
#define RSLX_ACT_VALUES_ONLY 2u   /* only the critic runs; only `values` is written */

/* A multi-layer perceptron over caller-owned device buffers (paper Sec. 3, "Network"). */
typedef struct rslx_mlp {
  int32_t n_layers;                  /* number of linear layers, 1..RSLX_MAX_LAYERS */
  int32_t dims[RSLX_MAX_LAYERS + 1]; /* dims[0] = input width, dims[n_layers] = output width */
  float elu_alpha;                   /* ELU parameter of the hidden layers (workloads use 1) */
  int32_t has_log_std;               /* 1: params end with log_std[dims[n_layers]] (actor) */
  float* params;                     /* device, flat layout above */
  float* grads;                      /* device, same layout; NULL for frozen networks */
  float* adam_m;                     /* device, same layout; NULL for frozen networks */
  float* adam_v;                     /* device, same layout; NULL for frozen networks */
} rslx_mlp;

/* Rollout storage [T, N, .] flattened to B = T*N rows, flat row b = t*N + n (paper Sec. 3:
 * the Runner stores what act() and the environment return; all device, read-only). */
typedef struct rslx_rollout {
  int32_t T, N;            /* steps per rollout, parallel environments */
  int32_t Da, Dc, A;       /* actor obs width, critic obs width, action width */
  const float* obs_actor;  /* [B, Da] */
  const float* obs_critic; /* [B, Dc] (may alias obs_actor) */
  const float* actions;    /* [B, A] */
  const float* logp;       /* [B]  log-density of actions under the collecting policy */
  const float* values;     /* [B]  critic values at collection */
  const float* mu;         /* [B, A] collecting policy mean (KL statistic) */
  const float* sigma;      /* [B, A] collecting policy std  (KL statistic) */
  const float* advantages; /* [B]  (normalised) advantages from rslx_gae */
  const float* returns;    /* [B]  returns from rslx_gae */
} rslx_rollout;

/* Hyper-parameters of the PPO update (paper Sec. 2.1; Schulman et al. 2017). */
typedef struct rslx_ppo_cfg {
  float clip;          /* epsilon of the ratio clip and of the value clip */
  float value_coef;    /* c_v */
  float entropy_coef;  /* c_e */
  float max_grad_norm; /* global L2 clip; <= 0 or inf disables */
  float lr, beta1, beta2, adam_eps;
  int32_t epochs;      /* E */
  int32_t minibatches; /* M; B % M must be 0 */
  int32_t use_clipped_value_loss;
  uint64_t seed;        /* permutation stream */
  uint64_t call_index;  /* permutation stream: which update call */
  int32_t epoch_offset; /* permutation of epoch e uses e + epoch_offset (resume mid-update) */
} rslx_ppo_cfg;

/* Mirror maps (paper Sec. 2.2): mirror(x)[j] = sign[j] * x[perm[j]].  The host copies are
 * validated (each must be a signed permutation with mirror o mirror = id).  The device copies are
 * what the kernels read.  rslx_ppo_update accepts all six device pointers NULL: it then uploads
 * the validated host copies into its workspace itself (hipMemcpyAsync from the caller's host arrays
 * on the call's stream: not under stream capture, where device copies must be passed).  Where
 * device copies are passed they must hold the same values as the host copies; the library cannot
 * check that.  rslx_sym_augment has no workspace and needs the device copies. */
typedef struct rslx_sym {
  const int32_t* perm_obs_a_host; const float* sign_obs_a_host; /* [Da] */
  const int32_t* perm_obs_c_host; const float* sign_obs_c_host; /* [Dc] */
  const int32_t* perm_act_host;   const float* sign_act_host;   /* [A]  */
  const int32_t* perm_obs_a; const float* sign_obs_a;           /* device copies */
  const int32_t* perm_obs_c; const float* sign_obs_c;
  const int32_t* perm_act;   const float* sign_act;
  float mirror_loss_coef; /* c_sym; 0 keeps the augmentation and drops the loss term */
} rslx_sym;

/* RND predictor training inside the PPO update (paper Sec. 2.2). */
typedef struct rslx_rnd_train {
  const rslx_mlp* target;    /* frozen */
  rslx_mlp* predictor;       /* trained: params, grads, adam_m, adam_v required */
  const int32_t* subset_idx; /* device [n_subset] columns of obs_actor fed to both nets, or NULL = all */
  int32_t n_subset;          /* must equal target->dims[0]; Da when subset_idx is NULL */
  float lr;                  /* predictor's own Adam learning rate (betas/eps as in the PPO cfg) */
  int64_t* adam_step;        /* host, in-out: predictor's own step counter */
} rslx_rnd_train;

/* Hyper-parameters of the behaviour-cloning update (paper Sec. 2.1, DAgger-style BC). */
typedef struct rslx_bc_cfg {
  float lr, beta1, beta2, adam_eps;
  float max_grad_norm; /* <= 0 disables clipping */
  int32_t epochs, minibatches;
  uint64_t seed, call_index;
  int32_t epoch_offset;
} rslx_bc_cfg;

/* ---- housekeeping ------------------------------------------------------------------- */

/* Library version as major*10000 + minor*100 + patch. */
int32_t rslx_version(void);
/* Message of the last failure on the calling thread ("" if none).  Never NULL. */
const char* rslx_last_error(void);
/* RSLX_OK if the current HIP device is a gfx950 part, RSLX_ERR_UNSUPPORTED / RSLX_ERR_HIP otherwise. */
int32_t rslx_device_check(void);

/* ---- launch trace (measurement aid) ---------------------------------------------------------- */

/* While a trace is open, every kernel launch of the library is bracketed by a pair of HIP events on
 * its stream and tagged with its algorithmic work.  rslx_trace_begin clears any earlier trace and
 * keeps at most max_records launches.  rslx_trace_end stops recording, WAITS on the host for the
 * recorded events, and copies up to `cap` records (launch order) to `out` (host); *n_out receives the
 * number recorded.  Calling it with out == NULL only reports the count and keeps the records for a
 * second call.  Launches beyond max_records are counted, not recorded: rslx_trace_end then still
 * delivers the records it has and returns RSLX_ERR_WORKSPACE.  `kernel` names a launch site: "gemm_<fwd|dx|dw>_<BM>x<BN>" are the matrix-core
 * kernels (flops = 2 M N K summed over the grouped problems), the others are streaming kernels
 * (bytes = algorithmic HBM bytes).  Not thread-safe; tracing costs two event records per launch. */
typedef struct rslx_trace_record {
  char kernel[48];
  double flops;
  double bytes;
  float ms;
} rslx_trace_record;
int32_t rslx_trace_begin(int32_t max_records);
int32_t rslx_trace_end(rslx_trace_record* out, int32_t cap, int32_t* n_out);

/* ---- permutation of one epoch (first step of the update: minibatch order) -------------- */

/* Shuffled minibatch order (paper Sec. 2.1: multi-epoch minibatch updates; the generator is this
 * library's own):  mix64 = SplitMix64 output function,
 *   key_i = mix64(mix64(mix64(mix64(seed) ^ call_index) ^ epoch) ^ i),  i in [0, B)
 *   perm  = indices sorted ascending by (key_i, i).
 * perm_out: device int32 [B].  Result is bit-exact and independent of scheduling. */
size_t rslx_permutation_workspace_bytes(int32_t B);
int32_t rslx_permutation(uint64_t seed, uint64_t call_index, int32_t epoch, int32_t B,
                         int32_t* perm_out, void* ws, size_t ws_bytes, void* stream);

/* ---- act(): one rollout step (paper Sec. 2.1 / Sec. 3: Runner -> Algorithm.act) ------ */

/* mu = actor(obs_actor), V = critic(obs_critic); sigma = exp(log_std);
 * a = mu + sigma * eps;  logp = -1/2 sum ((a-mu)/sigma)^2 - sum log sigma - A/2 log(2 pi).
 * eps: device [N, A] standard-normal noise, or NULL to draw it from the counter generator
 *   h = mix64(mix64(mix64(seed ^ 0xAC7) ^ step) ^ (n*A + j)); u1 = ((h>>40)+1) 2^-24;
 *   u2 = ((h>>8) & 0xFFFFFF) 2^-24; eps = sqrt(-2 ln u1) cos(2 pi u2).
 * Outputs (device): actions [N,A], logp [N], values [N], mu [N,A], sigma [N,A]; typically
 * pointers into slot t of the rollout storage.  With RSLX_ACT_VALUES_ONLY only `values` is
 * written and actor / actor outputs may be NULL. */
size_t rslx_act_workspace_bytes(const rslx_mlp* actor, const rslx_mlp* critic, int32_t N);
int32_t rslx_act(const rslx_mlp* actor, const rslx_mlp* critic, const float* obs_actor,
                 const float* obs_critic, int32_t N, uint64_t seed, uint64_t step,
                 const float* eps_or_null, float* actions, float* logp, float* values, float* mu,
                 float* sigma, uint32_t flags, void* ws, size_t ws_bytes, void* stream);

/* ---- GAE / returns (paper Sec. 2.1; time-limit handling Sec. 3) ---------------------- */

/* With V_T = last_values and A_T = 0, for t = T-1..0:
 *   delta = r_t + gamma (1-d_t) V_{t+1} - V_t;  A_t = delta + gamma lam (1-d_t) A_{t+1};
 *   R_t = A_t + V_t.   If timeouts != NULL, r_t is first replaced by r_t + gamma V_t timeout_t.
 * If normalize_adv != 0, advantages are then replaced by (A - mean) / (std + 1e-8) with the
 * mean and the unbiased (n-1) std taken over all T*N entries; returns use the raw A.
 * rewards, values [T,N]; last_values [N]; dones, timeouts uint8 [T,N]; outputs [T,N]. All device. */
size_t rslx_gae_workspace_bytes(int32_t T, int32_t N);
int32_t rslx_gae(const float* rewards, const float* values, const float* last_values,
                 const uint8_t* dones, const uint8_t* timeouts_or_null, int32_t T, int32_t N,
                 float gamma, float lam, int32_t normalize_adv, float* advantages, float* returns,
                 void* ws, size_t ws_bytes, void* stream);

/* rslx_gae for callers that cannot allocate or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc).  Same arguments, layouts,
 * results (bit for bit) and error behaviour as rslx_gae, without ws / ws_bytes: the partial sums
 * of the advantage normalisation live in a 65 600-byte array inside the library's device image,
 * of which every GPU the library runs on holds its own copy until the process ends.  The call
 * allocates and frees nothing (with rslx_trace_begin active the trace still creates events).
 * Limit: N <= RSLX_GAE_NOALLOC_MAX_ENVS, else RSLX_ERR_SHAPE and nothing is launched (T is not
 * limited).  All calls on one GPU share that GPU's array: calls that overlap on one GPU (two
 * streams, two host threads) race on it and must be serialised by the caller; calls on one
 * stream, and replays of a graph that holds one, are ordered and need no clearing in between. */
#define RSLX_GAE_NOALLOC_MAX_ENVS (1 << 20)
int32_t rslx_gae_noalloc(const float* rewards, const float* values, const float* last_values,
                         const uint8_t* dones, const uint8_t* timeouts_or_null, int32_t T,
                         int32_t N, float gamma, float lam, int32_t normalize_adv,
                         float* advantages, float* returns, void* stream);

/* ---- fused gradient-clip + Adam over one flat buffer (last steps of the update) -------- */

/* s = min(1, max_grad_norm / (||g||_2 + 1e-6)) (1 when max_grad_norm <= 0), then Adam
 * (Kingma & Ba 2015) with g*s:  m,v moments in place, bias correction with step t = *adam_step+1,
 * theta -= lr * m_hat / (sqrt(v_hat) + eps).  *adam_step (host) is incremented.
 * params, grads, m, v: device [n].  grad_norm_out: device float[1] or NULL. */
size_t rslx_adam_workspace_bytes(int64_t n);
int32_t rslx_adam_step(float* params, const float* grads, float* m, float* v, int64_t n, float lr,
                       float beta1, float beta2, float eps, float max_grad_norm, int64_t* adam_step,
                       float* grad_norm_out, void* ws, size_t ws_bytes, void* stream);

/* ---- PPO update (paper Sec. 2.1, 2.2, 3) ---------------------------------------------- */

/* E epochs x M minibatches over the B = T*N rollout rows.  For every minibatch (rows
 * perm_e[m*mb : (m+1)*mb], mb = B/M): forward of actor and critic, Gaussian log-density and
 * entropy, ratio = exp(logp_new - logp_old),
 *   L_pi = mean max(-A ratio, -A clamp(ratio, 1-clip, 1+clip))
 *   L_V  = mean max((V-R)^2, (V_old + clamp(V-V_old, -clip, clip) - R)^2)   (or mean (R-V)^2)
 *   L    = L_pi + c_v L_V - c_e mean(entropy) [+ c_sym L_mirror]
 * backward, one global gradient norm over actor (with log_std) and critic, clip, Adam.
 * With `sym`: every minibatch is followed by its mirrored copy (2*mb rows; obs and actions
 * mirrored, advantages / returns / old values / old log-densities copied), means run over
 * 2*mb rows, and L_mirror = mean over mb rows and A dims of
 * (mu(mirror(o)) - stopgrad(mirror_a(mu(o))))^2.
 * With `rnd`: the predictor is trained on the same rows with its own Adam on
 * mean((pred(x) - target(x))^2), outside the PPO gradient norm.
 * In-out: actor/critic params, adam_m, adam_v (device), *adam_step (host, shared by both nets).
 * Out: grads hold the last minibatch's unclipped gradient; stats: device [E*M, RSLX_NSTATS].
 * Action widths up to RSLX_MAX_ACTIONS; the fused output-layer + loss launch covers A <= 32 with
 * a last hidden width of 32, 64, 128 or 256, everything else runs the same arithmetic unfused. */
size_t rslx_ppo_update_workspace_bytes(const rslx_mlp* actor, const rslx_mlp* critic,
                                       const rslx_rollout* ro, const rslx_ppo_cfg* cfg,
                                       const rslx_sym* sym_or_null, const rslx_rnd_train* rnd_or_null);
int32_t rslx_ppo_update(rslx_mlp* actor, rslx_mlp* critic, const rslx_rollout* ro,
                        const rslx_ppo_cfg* cfg, const rslx_sym* sym_or_null,
                        const rslx_rnd_train* rnd_or_null, int64_t* adam_step, float* stats,
                        void* ws, size_t ws_bytes, void* stream);

/* ---- replayable variants: call-to-call counters in device memory ----------------------- */

/* The iteration of paper Sec. 3 (T x act, advantage estimation, update) is a fixed sequence of
 * launches; a caller that records it once (HIP graph) and replays it needs every value that
 * changes between iterations to live in device memory.  rslx_dev_counters (device, 32 bytes)
 * holds them; the *_dc entry points read it in their kernels and advance it with a kernel of
 * their own, so host arguments are the same for every replay:
 *   act_step       noise stream position: rslx_act_dc draws with step = act_step, then act_step += 1
 *                  (not with RSLX_ACT_VALUES_ONLY, which draws nothing)
 *   call_index     permutation stream of rslx_ppo_update_dc (cfg->call_index is ignored), += 1 per call
 *   adam_step      optimiser steps of actor + critic so far, += epochs * minibatches per call
 *   rnd_adam_step  the same for the RND predictor (rnd->adam_step is ignored)
 * Everything else is as in rslx_act / rslx_ppo_update; the bias corrections 1 - beta^t are formed
 * in fp64 on the device.  The caller initialises the struct (e.g. zeros) and must not run two
 * calls that share it concurrently. */
typedef struct rslx_dev_counters {
  int64_t act_step;
  uint64_t call_index;
  int64_t adam_step;
  int64_t rnd_adam_step;
} rslx_dev_counters;

int32_t rslx_act_dc(const rslx_mlp* actor, const rslx_mlp* critic, const float* obs_actor,
                    const float* obs_critic, int32_t N, uint64_t seed, rslx_dev_counters* counters,
                    const float* eps_or_null, float* actions, float* logp, float* values, float* mu,
                    float* sigma, uint32_t flags, void* ws, size_t ws_bytes, void* stream);
int32_t rslx_ppo_update_dc(rslx_mlp* actor, rslx_mlp* critic, const rslx_rollout* ro,
                           const rslx_ppo_cfg* cfg, const rslx_sym* sym_or_null,
                           const rslx_rnd_train* rnd_or_null, rslx_dev_counters* counters,
                           float* stats, void* ws, size_t ws_bytes, void* stream);

/* ---- recurrent actor-critic (paper Sec. 3: hidden states managed across roll-outs, BPTT) ---- */

/* A recurrent memory in front of an MLP, one of two cells over one flat device buffer
 *   W_ih [in_dim, G*H] row-major, b_ih [G*H], W_hh [H, G*H] row-major, b_hh [G*H]      (H = hidden)
 * RSLX_CELL_GRU (G = 3, gate order r, z, n; Cho et al. 2014 with the reset gate on the hidden-side
 * candidate term, bias included), state per row: h [H]
 *   gi = x W_ih + b_ih,  gh = h W_hh + b_hh
 *   r = sigmoid(gi_r + gh_r), z = sigmoid(gi_z + gh_z), n = tanh(gi_n + r gh_n), h' = (1-z) n + z h
 * RSLX_CELL_LSTM (G = 4, gate order i, f, g, o; forget gate, no peepholes), state per row: [h | c] [2H]
 *   a = x W_ih + b_ih + h W_hh + b_hh
 *   i = sigmoid(a_i), f = sigmoid(a_f), g = tanh(a_g), o = sigmoid(a_o), c' = f c + i g, h' = o tanh(c')
 * "State" below always means the packed row of width S = H (GRU) or 2H (LSTM); the MLP reads h.
 * hidden must be a multiple of 4; buffers 16-byte aligned; grads/adam_* NULL for inference. */
#define RSLX_CELL_GRU 0
#define RSLX_CELL_LSTM 1
typedef struct rslx_memory {
  int32_t cell;
  int32_t in_dim, hidden;
  float* params;
  float* grads;
  float* adam_m;
  float* adam_v;
} rslx_memory;

/* One roll-out step of a recurrent actor-critic: each network is a memory whose new hidden state
 * feeds its MLP (mlp.dims[0] == memory.hidden).  For every environment n:
 *   sin = reset[n] ? 0 : s[n];   s[n] <- cell(obs[n], sin);   mu, V = MLPs(h of s[n]);  then as rslx_act.
 * reset_or_null (device uint8 [N]) carries the previous step's episode-end flags.  h_actor
 * [N, S_a] and h_critic [N, S_c] (device, packed states) are updated in place; when h0_actor_out / h0_critic_out
 * are not NULL they receive sin, the state the step started from - the roll-out's first step
 * stores it for rslx_ppo_update_recurrent.  With RSLX_ACT_VALUES_ONLY only the critic runs and
 * NO state is written (the bootstrap value of the observation that opens the next roll-out).
 * Everything else (noise, outputs, flags, errors) is as in rslx_act. */
size_t rslx_act_recurrent_workspace_bytes(const rslx_memory* mem_actor, const rslx_mlp* actor,
                                          const rslx_memory* mem_critic, const rslx_mlp* critic, int32_t N);
int32_t rslx_act_recurrent(const rslx_memory* mem_actor, const rslx_mlp* actor, const rslx_memory* mem_critic,
                           const rslx_mlp* critic, const float* obs_actor, const float* obs_critic,
                           int32_t N, float* h_actor, float* h_critic, const uint8_t* reset_or_null,
                           float* h0_actor_out, float* h0_critic_out, uint64_t seed, uint64_t step,
                           const float* eps_or_null, float* actions, float* logp, float* values,
                           float* mu, float* sigma, uint32_t flags, void* ws, size_t ws_bytes,
                           void* stream);

/* PPO update of a recurrent actor-critic with back-propagation through time.  Minibatches are
 * whole environment columns: per epoch the N environments are shuffled (the permutation stream of
 * rslx_ppo_update, over N instead of T*N) and minibatch m takes the m-th slice of N / minibatches
 * environments with all T steps, rows ordered step-major.  Each minibatch is re-run through both
 * memories from h0 (the packed states the roll-out's first step started from, [N, S]) with the state
 * zeroed after every step whose `dones` flag is set; the loss of rslx_ppo_update (means over the
 * T * N / minibatches samples) is back-propagated through the MLPs into the hidden states and
 * through time, truncated at the roll-out start and never across an episode end.  One gradient
 * norm over the four parameter sets, one Adam step counter.  ro->Da / ro->Dc are the memories' input
 * widths; both memories use the same cell.  dones: device uint8 [T, N].  N % minibatches != 0 is RSLX_ERR_SHAPE.  Symmetry and RND
 * are not available here.  grads of all four hold the last minibatch's gradient on return. */
size_t rslx_ppo_update_recurrent_workspace_bytes(const rslx_memory* mem_actor, const rslx_mlp* actor,
                                                 const rslx_memory* mem_critic, const rslx_mlp* critic,
                                                 const rslx_rollout* ro, const rslx_ppo_cfg* cfg);
int32_t rslx_ppo_update_recurrent(rslx_memory* mem_actor, rslx_mlp* actor, rslx_memory* mem_critic,
                                  rslx_mlp* critic, const rslx_rollout* ro, const uint8_t* dones,
                                  const float* h0_actor, const float* h0_critic, const rslx_ppo_cfg* cfg,
                                  int64_t* adam_step, float* stats, void* ws, size_t ws_bytes,
                                  void* stream);

/* Replayable variants (see rslx_dev_counters): the noise position / permutation stream / optimiser
 * step count come from device memory and are advanced by the calls' own kernels, so a recurrent
 * iteration can be recorded as a HIP graph like a feed-forward one. */
int32_t rslx_act_recurrent_dc(const rslx_memory* mem_actor, const rslx_mlp* actor, const rslx_memory* mem_critic,
                              const rslx_mlp* critic, const float* obs_actor, const float* obs_critic,
                              int32_t N, float* h_actor, float* h_critic, const uint8_t* reset_or_null,
                              float* h0_actor_out, float* h0_critic_out, uint64_t seed,
                              rslx_dev_counters* counters, const float* eps_or_null, float* actions,
                              float* logp, float* values, float* mu, float* sigma, uint32_t flags,
                              void* ws, size_t ws_bytes, void* stream);
int32_t rslx_ppo_update_recurrent_dc(rslx_memory* mem_actor, rslx_mlp* actor, rslx_memory* mem_critic,
                                     rslx_mlp* critic, const rslx_rollout* ro, const uint8_t* dones,
                                     const float* h0_actor, const float* h0_critic, const rslx_ppo_cfg* cfg,
                                     rslx_dev_counters* counters, float* stats, void* ws, size_t ws_bytes,
                                     void* stream);

/* One step of a single memory (the recurrent student of the distillation loop, paper Sec. 2.1 with
 * Sec. 3): sin = reset[n] ? 0 : s[n];  s[n] <- cell(obs[n], sin), in place on the packed state
 * s [N, S]; s0_out (optional, [N, S]) receives sin; h_dense_out (optional, [N, H]) receives the
 * new hidden state as a dense matrix (for a GRU the state itself is that matrix).  The student's
 * action and the expert's label then come from
 * rslx_bc_collect(student_mlp, teacher, hidden state, obs_teacher, ...). */
size_t rslx_memory_step_workspace_bytes(const rslx_memory* mem, int32_t N);
int32_t rslx_memory_step(const rslx_memory* mem, const float* obs, int32_t N, float* s,
                         const uint8_t* reset_or_null, float* s0_out, float* h_dense_out, void* ws,
                         size_t ws_bytes, void* stream);

/* Behaviour cloning of a recurrent student (memory + MLP, student->dims[0] == mem->hidden) on
 * a roll-out: obs_student [T, N, Ds], targets [T, N, A] (the expert's actions on the visited
 * states), dones uint8 [T, N], h0 [N, S] (the packed state the roll-out's first step started from); all
 * device.  Minibatches are whole environment columns as in rslx_ppo_update_recurrent (cfg's
 * permutation stream over N; N % minibatches != 0 is RSLX_ERR_SHAPE); per minibatch
 * L = mean over the T * N / minibatches rows and the A action dims of (student - target)^2,
 * back-propagated through the MLP and through time, optional clip, Adam (one step counter for
 * memory and MLP).  stats as in rslx_bc_update. */
size_t rslx_bc_update_recurrent_workspace_bytes(const rslx_memory* mem, const rslx_mlp* student, int32_t T,
                                                int32_t N, const rslx_bc_cfg* cfg);
int32_t rslx_bc_update_recurrent(rslx_memory* mem, rslx_mlp* student, const float* obs_student,
                                 const float* targets, const uint8_t* dones, const float* h0, int32_t T,
                                 int32_t N, const rslx_bc_cfg* cfg, int64_t* adam_step, float* stats,
                                 void* ws, size_t ws_bytes, void* stream);

/* ---- behaviour cloning update (paper Sec. 2.1) ---------------------------------------- */

/* targets = teacher(obs_teacher) (once; or the caller's precomputed `targets_or_null` [B, A]);
 * per minibatch L = mean over rows and action dims of (student(obs_student) - target)^2,
 * backward, optional clip, Adam.  obs_student [B, Ds], obs_teacher [B, Dt] device.
 * stats: device [E*M, RSLX_NSTATS] (column 0 loss, column 4 gradient norm, others 0). */
size_t rslx_bc_update_workspace_bytes(const rslx_mlp* student, const rslx_mlp* teacher, int32_t B,
                                      const rslx_bc_cfg* cfg);
int32_t rslx_bc_update(rslx_mlp* student, const rslx_mlp* teacher, const float* obs_student,
                       const float* obs_teacher, const float* targets_or_null, int32_t B,
                       const rslx_bc_cfg* cfg, int64_t* adam_step, float* stats, void* ws,
                       size_t ws_bytes, void* stream);

/* As rslx_bc_update with the permutation stream (counters->call_index, += 1) and the optimiser step
 * count (counters->adam_step, += epochs * minibatches) in device memory; cfg->call_index is ignored.
 * See rslx_dev_counters. */
int32_t rslx_bc_update_dc(rslx_mlp* student, const rslx_mlp* teacher, const float* obs_student,
                          const float* obs_teacher, const float* targets_or_null, int32_t B,
                          const rslx_bc_cfg* cfg, rslx_dev_counters* counters, float* stats, void* ws,
                          size_t ws_bytes, void* stream);

/* One collection step of the distillation loop (paper Sec. 2.1: the student is rolled out, the
 * expert relabels what it visits): actions = student(obs_student) (mean action, no noise) and
 * targets = teacher(obs_teacher) for the same N states, one launch for both networks.
 * obs_student [N, Ds], obs_teacher [N, Dt], actions [N, A], targets [N, A]; all device.  The
 * targets written over a rollout are what rslx_bc_update takes as `targets_or_null`.
 * RSLX_ERR_SHAPE if the two networks' output widths differ. */
size_t rslx_bc_collect_workspace_bytes(const rslx_mlp* student, const rslx_mlp* teacher, int32_t N);
int32_t rslx_bc_collect(const rslx_mlp* student, const rslx_mlp* teacher, const float* obs_student,
                        const float* obs_teacher, int32_t N, float* actions, float* targets, void* ws,
                        size_t ws_bytes, void* stream);

/* ---- symmetry augmentation (paper Sec. 2.2) -------------------------------------------- */

/* obs_out[0:B] = obs_in, obs_out[B:2B][:, j] = sign_obs_a[j] * obs_in[:, perm_obs_a[j]]; the same
 * for actions with perm_act / sign_act.  Uses the *_obs_a and *_act maps of `sym` (host copies
 * validated, device copies read by the kernel).  obs_in [B, D], act_in [B, A] (either may be
 * NULL to skip it), outputs [2B, D], [2B, A]; all device.  RSLX_ERR_INVALID_ARG if a map is not
 * an involutive signed permutation. */
int32_t rslx_sym_augment(const rslx_sym* sym, const float* obs_in, const float* act_in, int32_t B,
                         int32_t D, int32_t A, float* obs_out, float* act_out, void* stream);

/* ---- RND intrinsic reward (paper Sec. 2.2) --------------------------------------------- */

/* x = obs[:, subset]; r_raw_n = sum_k (predictor(x_n) - target(x_n))_k^2.  If update_stats,
 * running = {mean, var, count} (device float[3], population variance) is merged with the N new
 * values (Chan et al. pairwise update) before use.  r_int = r_raw / sqrt(var + 1e-8) is written
 * to r_int_out [N]; if rewards_inout != NULL, rewards_inout[n] += weight * r_int[n]. */
size_t rslx_rnd_workspace_bytes(const rslx_mlp* target, int32_t N);
int32_t rslx_rnd(const rslx_mlp* target, const rslx_mlp* predictor, const float* obs, int32_t N,
                 int32_t D, const int32_t* subset_idx_or_null, int32_t n_subset, float* running,
                 float weight, int32_t update_stats, float* r_int_out, float* rewards_inout_or_null,
                 void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RSLX_H */
