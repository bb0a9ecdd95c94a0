// Entry points of the recurrent paths of librslx (memories in front of the MLPs, back-propagation through time):
// argument validation, workspace carving and launch sequencing.  Shares the host helpers of api.hip (host.h).
#include "host.h"

namespace {
using namespace rslx;
using namespace rslx::host;
}  // namespace

// ======================================================================================================
// Recurrent actor-critic: GRU or LSTM memories in front of the MLPs, back-propagation through time.
// ======================================================================================================
namespace {

int gates(const rslx_memory& g) { return g.cell == RSLX_CELL_LSTM ? 4 : 3; }
int gate_width(const rslx_memory& g) { return gates(g) * g.hidden; }                              // G H
int state_width(const rslx_memory& g) { return g.cell == RSLX_CELL_LSTM ? 2 * g.hidden : g.hidden; }   // S
int64_t gru_off_bih(const rslx_memory& g) { return (int64_t)g.in_dim * gate_width(g); }
int64_t gru_off_whh(const rslx_memory& g) { return gru_off_bih(g) + gate_width(g); }
int64_t gru_off_bhh(const rslx_memory& g) { return gru_off_whh(g) + (int64_t)g.hidden * gate_width(g); }
int64_t gru_count(const rslx_memory& g) { return gru_off_bhh(g) + gate_width(g); }

int32_t check_gru(const rslx_memory* g, const char* name, bool trainable) {
  if (!g) return fail(RSLX_ERR_INVALID_ARG, "%s: null memory", name);
  if (g->cell != RSLX_CELL_GRU && g->cell != RSLX_CELL_LSTM) return fail(RSLX_ERR_INVALID_ARG, "%s: unknown cell %d", name, g->cell);
  if (g->in_dim < 1 || g->in_dim > (1 << 20) || g->hidden < 4 || g->hidden > (1 << 16) || g->hidden % 4 != 0)
    return fail(RSLX_ERR_SHAPE, "%s: in_dim = %d, hidden = %d (hidden must be a multiple of 4)", name, g->in_dim, g->hidden);
  if (!g->params || !aligned16(g->params)) return fail(RSLX_ERR_INVALID_ARG, "%s: params null or not 16-byte aligned", name);
  if (trainable) {
    if (!g->grads || !g->adam_m || !g->adam_v) return fail(RSLX_ERR_INVALID_ARG, "%s: grads / adam_m / adam_v required", name);
    if (!aligned16(g->grads) || !aligned16(g->adam_m) || !aligned16(g->adam_v))
      return fail(RSLX_ERR_INVALID_ARG, "%s: optimiser buffers not 16-byte aligned", name);
  }
  return RSLX_OK;
}

// C[M, G H] = X W + b for one side of a memory's gates (X given as a view or as a plain matrix).
GemmProblem gate_problem(const XView& x, int K, const float* W, const float* b, float* C, int M, int H3) {
  GemmProblem p = blank_problem();
  set_x(p, x);
  p.B = W; p.ldb = H3; p.aux = b;
  p.C = C; p.ldc = H3;
  p.M = M; p.N = H3; p.K = K;
  p.elu = 0; p.alpha = 1.f;
  p.a_vec = (K % 4 == 0 && p.lda % 4 == 0 && aligned16(p.A) && p.col_map == nullptr) ? 1 : 0;
  p.b_vec = (H3 % 4 == 0 && aligned16(W)) ? 1 : 0;
  return p;
}

XView plain_view(const float* base, int ld) {
  XView x;
  x.base = base; x.ld = ld;
  return x;
}

struct StepBufs {     // one memory's buffers of a single act step
  float* hin = nullptr;     // [N, S] state the step starts from (after reset)
  float* gi = nullptr;      // [N, G H]
  float* hnew = nullptr;    // [N, S] values-only: the state is not written back
};

size_t act_recurrent_carve(Carver& c, const rslx_memory* ga, const rslx_memory* gc, int32_t N, StepBufs* ba, StepBufs* bc) {
  const rslx_memory* g[2] = {ga, gc};
  StepBufs* b[2] = {ba, bc};
  for (int k = 0; k < 2; ++k) {
    if (!g[k]) continue;
    StepBufs t;
    t.hin = c.take<float>((size_t)N * state_width(*g[k]));
    t.gi = c.take<float>((size_t)N * gate_width(*g[k]));
    t.hnew = c.take<float>((size_t)N * state_width(*g[k]));
    if (b[k]) *b[k] = t;
  }
  return c.off;
}

// hin -> gi -> new state (hidden-side contraction fused with the gates), for the memories listed (1 or 2), each with its own input matrix.
int32_t gru_step(const rslx_memory* const* g, const float* const* obs, const StepBufs* b, float* const* h_out, int count,
                 int32_t N, hipStream_t s) {
  GemmBatch bi;
  bi.count = count;
  StepFwdArgs sa;
  memset(&sa, 0, sizeof sa);
  sa.n_nets = count; sa.nb = N; sa.cell = g[0]->cell;
  for (int k = 0; k < count; ++k) {
    const rslx_memory& m = *g[k];
    bi.p[k] = gate_problem(plain_view(obs[k], m.in_dim), m.in_dim, m.params, m.params + gru_off_bih(m), b[k].gi, N, gate_width(m));
    // the new packed state goes to h_out[k] ([N, S]): h in its first H columns, an LSTM's c behind it
    sa.net[k] = StepFwdNet{b[k].gi, b[k].hin, h_out[k], m.cell == RSLX_CELL_LSTM ? h_out[k] + m.hidden : nullptr, nullptr,
                           m.params + gru_off_whh(m), m.params + gru_off_bhh(m), nullptr, m.hidden, state_width(m)};
  }
  RSLX_HIP(launch_gemm(GEMM_FWD, bi, s));
  RSLX_HIP(launch_step_fwd(sa, s));
  return RSLX_OK;
}

int32_t act_recurrent_validate(const rslx_memory* ga, const rslx_mlp* actor, const rslx_memory* gc, const rslx_mlp* critic,
                               bool values_only) {
  RSLX_TRY(check_gru(gc, "rslx_act_recurrent critic memory", false));
  RSLX_TRY(check_mlp(critic, "rslx_act_recurrent critic", false));
  if (critic->dims[0] != gc->hidden) return fail(RSLX_ERR_SHAPE, "rslx_act_recurrent: critic input width != memory width");
  if (!values_only) {
    RSLX_TRY(check_gru(ga, "rslx_act_recurrent actor memory", false));
    RSLX_TRY(check_mlp(actor, "rslx_act_recurrent actor", false));
    if (actor->dims[0] != ga->hidden) return fail(RSLX_ERR_SHAPE, "rslx_act_recurrent: actor input width != memory width");
    if (ga->cell != gc->cell) return fail(RSLX_ERR_UNSUPPORTED, "rslx_act_recurrent: the two memories use different cells");
  }
  return RSLX_OK;
}

}  // namespace

extern "C" {

size_t rslx_act_recurrent_workspace_bytes(const rslx_memory* gru_actor, const rslx_mlp* actor, const rslx_memory* gru_critic,
                                          const rslx_mlp* critic, int32_t N) {
  if (N <= 0 || !gru_critic || !critic) return 256;
  Carver c(nullptr);
  act_recurrent_carve(c, gru_actor, gru_critic, N, nullptr, nullptr);
  return (c.off + 255) / 256 * 256 + rslx_act_workspace_bytes(actor, critic, N);
}

}  // extern "C"

namespace {
// Shared body of rslx_act_recurrent and rslx_act_recurrent_dc (noise position from device memory).
int32_t act_recurrent_impl(const rslx_memory* gru_actor, const rslx_mlp* actor, const rslx_memory* gru_critic,
                           const rslx_mlp* critic, const float* obs_actor, const float* obs_critic, int32_t N,
                           float* h_actor, float* h_critic, const uint8_t* reset_or_null, float* h0_actor_out,
                           float* h0_critic_out, uint64_t seed, uint64_t step, rslx_dev_counters* counters,
                           const float* eps_or_null, float* actions, float* logp, float* values, float* mu, float* sigma,
                           uint32_t flags, void* ws, size_t ws_bytes, void* stream) {
  const bool values_only = (flags & RSLX_ACT_VALUES_ONLY) != 0;
  if (N < 0) return fail(RSLX_ERR_SHAPE, "rslx_act_recurrent: N = %d", N);
  RSLX_TRY(act_recurrent_validate(gru_actor, actor, gru_critic, critic, values_only));
  if (!obs_critic || !h_critic || !values) return fail(RSLX_ERR_INVALID_ARG, "rslx_act_recurrent: null critic input / state / output");
  if (!values_only && (!obs_actor || !h_actor)) return fail(RSLX_ERR_INVALID_ARG, "rslx_act_recurrent: null actor input / state");
  // everything the MLP stage would reject is rejected here, before the memories advance the caller's states
  if (!values_only && (!actions || !logp || !mu || !sigma)) return fail(RSLX_ERR_INVALID_ARG, "rslx_act_recurrent: null actor output");
  if (!values_only && !actor->has_log_std) return fail(RSLX_ERR_INVALID_ARG, "rslx_act_recurrent: actor needs log_std");
  if (critic->dims[critic->n_layers] != 1) return fail(RSLX_ERR_SHAPE, "rslx_act_recurrent: critic output width must be 1");
  if (!values_only && actor->dims[actor->n_layers] > RSLX_MAX_ACTIONS)
    return fail(RSLX_ERR_SHAPE, "rslx_act_recurrent: action width > %d", RSLX_MAX_ACTIONS);
  if (!aligned16(h_critic) || (!values_only && !aligned16(h_actor)) || (h0_actor_out && !aligned16(h0_actor_out)) ||
      (h0_critic_out && !aligned16(h0_critic_out)))
    return fail(RSLX_ERR_INVALID_ARG, "rslx_act_recurrent: state buffers not 16-byte aligned");
  if (N == 0) return RSLX_OK;
  const rslx_memory* ga = values_only ? nullptr : gru_actor;
  const rslx_mlp* a = values_only ? nullptr : actor;
  if (!ws || ws_bytes < rslx_act_recurrent_workspace_bytes(ga, a, gru_critic, critic, N))
    return fail(RSLX_ERR_WORKSPACE, "rslx_act_recurrent: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  StepBufs ba, bc;
  act_recurrent_carve(c, ga, gru_critic, N, &ba, &bc);
  const size_t used = (c.off + 255) / 256 * 256;

  RowGatherArgs rg;
  memset(&rg, 0, sizeof rg);
  rg.nb = N; rg.reset = reset_or_null;
  if (ga) rg.job[rg.n_jobs++] = RowGatherJob{h_actor, ba.hin, values_only ? nullptr : h0_actor_out, state_width(*ga)};
  rg.job[rg.n_jobs++] = RowGatherJob{h_critic, bc.hin, values_only ? nullptr : h0_critic_out, state_width(*gru_critic)};
  RSLX_HIP(launch_row_gather(rg, s));

  const float* h_in_actor_mlp = h_actor;
  const float* h_in_critic_mlp = values_only ? bc.hnew : h_critic;
  if (ga) {
    const rslx_memory* g[2] = {ga, gru_critic};
    const float* obs[2] = {obs_actor, obs_critic};
    const StepBufs b[2] = {ba, bc};
    float* out[2] = {h_actor, h_critic};
    RSLX_TRY(gru_step(g, obs, b, out, 2, N, s));
  } else {
    const rslx_memory* g[1] = {gru_critic};
    const float* obs[1] = {obs_critic};
    const StepBufs b[1] = {bc};
    float* out[1] = {bc.hnew};
    RSLX_TRY(gru_step(g, obs, b, out, 1, N, s));
  }
  return act_impl(a, critic, h_in_actor_mlp, h_in_critic_mlp, N, seed, step, counters, eps_or_null, actions, logp, values,
                  mu, sigma, flags, static_cast<char*>(ws) + used, ws_bytes - used, stream, ga ? state_width(*ga) : 0,
                  state_width(*gru_critic));
}
}  // namespace

extern "C" {

int32_t rslx_act_recurrent(const rslx_memory* mem_actor, const rslx_mlp* actor, const rslx_memory* mem_critic,
                           const rslx_mlp* critic, const float* obs_actor, const float* obs_critic, int32_t N,
                           float* h_actor, float* h_critic, const uint8_t* reset_or_null, float* h0_actor_out,
                           float* h0_critic_out, uint64_t seed, uint64_t step, const float* eps_or_null, float* actions,
                           float* logp, float* values, float* mu, float* sigma, uint32_t flags, void* ws, size_t ws_bytes,
                           void* stream) {
  return act_recurrent_impl(mem_actor, actor, mem_critic, critic, obs_actor, obs_critic, N, h_actor, h_critic, reset_or_null,
                            h0_actor_out, h0_critic_out, seed, step, nullptr, eps_or_null, actions, logp, values, mu, sigma,
                            flags, ws, ws_bytes, stream);
}

int32_t rslx_act_recurrent_dc(const rslx_memory* mem_actor, const rslx_mlp* actor, const rslx_memory* mem_critic,
                              const rslx_mlp* critic, const float* obs_actor, const float* obs_critic, int32_t N,
                              float* h_actor, float* h_critic, const uint8_t* reset_or_null, float* h0_actor_out,
                              float* h0_critic_out, uint64_t seed, rslx_dev_counters* counters, const float* eps_or_null,
                              float* actions, float* logp, float* values, float* mu, float* sigma, uint32_t flags, void* ws,
                              size_t ws_bytes, void* stream) {
  if (!counters) return fail(RSLX_ERR_INVALID_ARG, "rslx_act_recurrent_dc: null counters");
  return act_recurrent_impl(mem_actor, actor, mem_critic, critic, obs_actor, obs_critic, N, h_actor, h_critic, reset_or_null,
                            h0_actor_out, h0_critic_out, seed, 0, counters, eps_or_null, actions, logp, values, mu, sigma,
                            flags, ws, ws_bytes, stream);
}

}  // extern "C"

namespace {

struct RnnBufs {          // per memory, one column-wise minibatch (rows = T * nb)
  float* gi = nullptr;    // [rows, G H] input-side gate terms
  float* gh = nullptr;    // [rows, G H] what the forward steps store for the backward pass (GRU: gh, LSTM: a)
  float* dgi = nullptr;   // [rows, G H] GRU only: gradient w.r.t. gi
  float* dgh = nullptr;   // [rows, G H] gradient w.r.t. the hidden-side terms (LSTM: w.r.t. a, serves both sides)
  float* hin = nullptr;   // [rows, S] packed state every step starts from
  float* hs = nullptr;    // [rows, H] new hidden states = input of the MLP
  float* dh = nullptr;    // [rows, H] gradient from the MLP
  float* direct = nullptr;  // [nb, H] carried between backward steps (GRU: dh z, LSTM: gradient w.r.t. c)
  SplitPlan plan;           // layer 0: W_ih / b_ih, layer 1: W_hh / b_hh
  float* partials = nullptr;
};

struct RnnPlan {
  int32_t T, N, nb, rows;
  bool fused_head = false;
  int32_t loss_blocks = 0;
  int32_t* perms = nullptr;      // [E, N]
  void* perm_ws = nullptr;
  int32_t* rows_all = nullptr;   // [E, M, T, nb] roll-out rows of every minibatch
  TrainBufs actor, critic;
  RnnBufs ma, mc;
  double* sumsq_all = nullptr;
  int32_t n_sumsq = 0;
  double* loss_partials = nullptr;
  size_t bytes = 0;
};

void carve_memory(Carver& c, const rslx_memory& g, int32_t rows, int32_t nb, RnnBufs& b, int group = 2) {
  const size_t H = g.hidden, GH = gate_width(g), S = state_width(g);
  b.gi = c.take<float>(rows * GH); b.gh = c.take<float>(rows * GH);
  b.dgi = g.cell == RSLX_CELL_GRU ? c.take<float>(rows * GH) : nullptr;
  b.dgh = c.take<float>(rows * GH);
  b.hin = c.take<float>(rows * S); b.hs = c.take<float>(rows * H); b.dh = c.take<float>(rows * H);
  b.direct = c.take<float>(nb * H);
  plan_layer(b.plan, 0, g.in_dim, (int)GH, rows, group, false);
  plan_layer(b.plan, 1, g.hidden, (int)GH, rows, group, false);
  b.partials = c.take<float>((size_t)b.plan.total);
}

void rnn_plan(Carver& c, const rslx_memory* ga, const rslx_mlp* actor, const rslx_memory* gc, const rslx_mlp* critic,
              const rslx_rollout* ro, const rslx_ppo_cfg* cfg, RnnPlan& p) {
  p.T = ro->T; p.N = ro->N;
  p.nb = ro->N / cfg->minibatches;
  p.rows = p.T * p.nb;
  p.perms = c.take<int32_t>((size_t)cfg->epochs * p.N);
  p.perm_ws = c.take<char>(perm_workspace_bytes(p.N));
  p.rows_all = c.take<int32_t>((size_t)cfg->epochs * p.T * p.N);
  carve_train(c, *actor, p.rows, 2, p.actor, true);
  carve_train(c, *critic, p.rows, 2, p.critic, true);
  carve_memory(c, *ga, p.rows, p.nb, p.ma);
  carve_memory(c, *gc, p.rows, p.nb, p.mc);
  p.n_sumsq = p.actor.n_sumsq + p.critic.n_sumsq + p.ma.plan.blocks + p.mc.plan.blocks + 1;
  p.sumsq_all = c.take<double>((size_t)p.n_sumsq + 1);
  p.fused_head = actor->n_layers >= 2 && critic->n_layers >= 2 &&
                 ppo_head_supported(actor->dims[actor->n_layers - 1], critic->dims[critic->n_layers - 1], ro->A);
  p.loss_blocks = p.fused_head ? ppo_head_num_blocks(p.rows, false) : ppo_loss_num_blocks(p.rows);
  p.loss_partials = c.take<double>((size_t)p.loss_blocks * (PPO_NPART_FIXED + ro->A));
  p.bytes = c.off + 256;
}

int32_t rnn_validate(const rslx_memory* ga, const rslx_mlp* actor, const rslx_memory* gc, const rslx_mlp* critic,
                     const rslx_rollout* ro, const rslx_ppo_cfg* cfg, bool need_buffers) {
  if (!ro || !cfg) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent: null rollout or cfg");
  RSLX_TRY(check_gru(ga, "rslx_ppo_update_recurrent actor memory", need_buffers));
  RSLX_TRY(check_gru(gc, "rslx_ppo_update_recurrent critic memory", need_buffers));
  RSLX_TRY(check_mlp(actor, "rslx_ppo_update_recurrent actor", need_buffers));
  RSLX_TRY(check_mlp(critic, "rslx_ppo_update_recurrent critic", need_buffers));
  if (!actor->has_log_std) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent: actor needs log_std");
  if (ro->T < 1 || ro->N < 1 || (int64_t)ro->T * ro->N > (1 << 30))
    return fail(RSLX_ERR_SHAPE, "rslx_ppo_update_recurrent: T = %d, N = %d", ro->T, ro->N);
  if (ro->Da != ga->in_dim || ro->Dc != gc->in_dim || actor->dims[0] != ga->hidden || critic->dims[0] != gc->hidden ||
      ro->A != actor->dims[actor->n_layers] || critic->dims[critic->n_layers] != 1)
    return fail(RSLX_ERR_SHAPE, "rslx_ppo_update_recurrent: rollout, memory and network widths do not match");
  if (ga->cell != gc->cell) return fail(RSLX_ERR_UNSUPPORTED, "rslx_ppo_update_recurrent: the two memories use different cells");
  if (ro->A > RSLX_MAX_ACTIONS) return fail(RSLX_ERR_SHAPE, "rslx_ppo_update_recurrent: action width %d > %d", ro->A, RSLX_MAX_ACTIONS);
  if (actor->n_layers + critic->n_layers + 4 > 16)
    return fail(RSLX_ERR_UNSUPPORTED, "rslx_ppo_update_recurrent: more than 12 MLP layers in total");
  if (cfg->epochs < 0 || cfg->minibatches < 1) return fail(RSLX_ERR_SHAPE, "rslx_ppo_update_recurrent: epochs / minibatches");
  if (ro->N % cfg->minibatches != 0)
    return fail(RSLX_ERR_SHAPE, "rslx_ppo_update_recurrent: N = %d is not a multiple of minibatches = %d", ro->N, cfg->minibatches);
  if (need_buffers && (!ro->obs_actor || !ro->obs_critic || !ro->actions || !ro->logp || !ro->values || !ro->mu ||
                       !ro->sigma || !ro->advantages || !ro->returns))
    return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent: null rollout buffer");
  return RSLX_OK;
}

// Weight-gradient problem of one side of a memory's gates: partials[l] = X^T dG over the row splits.
GemmProblem gate_dw_problem(const XView& x, int M, const float* dG, int H3, int32_t rows, const RnnBufs& b, int l) {
  GemmProblem p = blank_problem();
  set_x(p, x);
  p.B = dG; p.ldb = H3;
  p.C = b.partials + b.plan.part_off[l]; p.ldc = H3;
  p.M = M; p.N = H3; p.K = rows;
  p.n_split = b.plan.split[l];
  p.k_chunk = b.plan.chunk[l];
  p.split_stride = b.plan.pitch[l];
  p.bias_off = M * H3;
  p.dw_big = b.plan.big[l];
  p.a_vec = (M % 4 == 0 && p.lda % 4 == 0 && aligned16(p.A) && p.col_map == nullptr) ? 1 : 0;
  p.b_vec = (H3 % 4 == 0 && aligned16(dG)) ? 1 : 0;
  return p;
}

// Memories forward over one column-wise minibatch: the input-side gates of all T steps in one GEMM (rows gathered
// from the roll-out through ridx), then one fused step launch per time step for all `count` memories.
int32_t memories_forward(const rslx_memory* const* mem, RnnBufs* const* mb, int count, const float* const* obs,
                         const float* const* h0, const int32_t* envs, const int32_t* ridx, const uint8_t* dones, int T,
                         int nb, int N, hipStream_t s) {
  const int rows = T * nb;
  RowGatherArgs rg;
  memset(&rg, 0, sizeof rg);
  rg.n_jobs = count; rg.nb = nb; rg.idx = envs;
  for (int k = 0; k < count; ++k) rg.job[k] = RowGatherJob{h0[k], mb[k]->hin, nullptr, state_width(*mem[k])};
  RSLX_HIP(launch_row_gather(rg, s));
  GemmBatch bi;
  bi.count = count;
  for (int k = 0; k < count; ++k) {
    XView x;
    x.base = obs[k]; x.ld = mem[k]->in_dim; x.row_idx = ridx; x.src_rows = (int64_t)T * N;
    bi.p[k] = gate_problem(x, mem[k]->in_dim, mem[k]->params, mem[k]->params + gru_off_bih(*mem[k]), mb[k]->gi, rows,
                           gate_width(*mem[k]));
  }
  RSLX_HIP(launch_gemm(GEMM_FWD, bi, s));
  for (int t = 0; t < T; ++t) {
    StepFwdArgs sa;
    memset(&sa, 0, sizeof sa);
    sa.n_nets = count; sa.nb = nb; sa.cell = mem[0]->cell; sa.done = dones; sa.done_idx = ridx + (size_t)t * nb;
    for (int k = 0; k < count; ++k) {
      const rslx_memory& g = *mem[k];
      const size_t H = g.hidden, GH = gate_width(g), S = state_width(g), r0 = (size_t)t * nb;
      sa.net[k] = StepFwdNet{mb[k]->gi + r0 * GH, mb[k]->hin + r0 * S, mb[k]->hs + r0 * H, nullptr,
                             t + 1 < T ? mb[k]->hin + (r0 + nb) * S : nullptr, g.params + gru_off_whh(g),
                             g.params + gru_off_bhh(g), mb[k]->gh + r0 * GH, g.hidden, g.hidden};
    }
    RSLX_HIP(launch_step_fwd(sa, s));
  }
  return RSLX_OK;
}

// Back-propagation through time from mb[k]->dh (the gradient w.r.t. every step's new hidden state): one fused step
// launch per time step, last to first, then the weight gradients of both sides of the gates over all steps at once
// (split partials, to be summed by the caller's reduction).
int32_t memories_backward(const rslx_memory* const* mem, RnnBufs* const* mb, int count, const float* const* obs,
                          const int32_t* ridx, const uint8_t* dones, int T, int nb, int N, hipStream_t s) {
  const int rows = T * nb;
  for (int t = T - 1; t >= 0; --t) {
    StepBwdArgs sb;
    memset(&sb, 0, sizeof sb);
    sb.n_nets = count; sb.nb = nb; sb.cell = mem[0]->cell; sb.done = dones; sb.done_idx = ridx + (size_t)t * nb;
    for (int k = 0; k < count; ++k) {
      const rslx_memory& g = *mem[k];
      const size_t H = g.hidden, GH = gate_width(g), S = state_width(g), r0 = (size_t)t * nb;
      const bool last = t == T - 1;
      sb.net[k] = StepBwdNet{mb[k]->dh + r0 * H, last ? nullptr : mb[k]->dgh + (r0 + nb) * GH, mb[k]->direct,
                             g.params + gru_off_whh(g), mb[k]->gi + r0 * GH, mb[k]->gh + r0 * GH, mb[k]->hin + r0 * S,
                             mb[k]->dgi ? mb[k]->dgi + r0 * GH : nullptr, mb[k]->dgh + r0 * GH, g.hidden};
    }
    RSLX_HIP(launch_step_bwd(sb, s));
  }
  GemmBatch bwi, bwh;
  bwi.count = bwh.count = count;
  for (int k = 0; k < count; ++k) {
    const rslx_memory& g = *mem[k];
    XView x;
    x.base = obs[k]; x.ld = g.in_dim; x.row_idx = ridx; x.src_rows = (int64_t)T * N;
    // an LSTM's two sides of the gates share one gradient
    bwi.p[k] = gate_dw_problem(x, g.in_dim, mb[k]->dgi ? mb[k]->dgi : mb[k]->dgh, gate_width(g), rows, *mb[k], 0);
    bwh.p[k] = gate_dw_problem(plain_view(mb[k]->hin, state_width(g)), g.hidden, mb[k]->dgh, gate_width(g), rows, *mb[k], 1);
  }
  RSLX_HIP(launch_gemm(GEMM_DW, bwi, s));
  RSLX_HIP(launch_gemm(GEMM_DW, bwh, s));
  return RSLX_OK;
}

void reduce_add_memory(ReduceArgs& a, const rslx_memory& g, const RnnBufs& b) {
  for (int l = 0; l < 2; ++l) {
    ReduceSeg& sg = a.seg[a.n_seg++];
    sg.partials = b.partials + b.plan.part_off[l];
    sg.grads = g.grads + (l == 0 ? 0 : gru_off_whh(g));
    sg.size = b.plan.size[l];
    sg.pitch = b.plan.pitch[l];
    sg.split = b.plan.split[l];
    sg.block_start = a.blocks;
    a.blocks += (int)((b.plan.size[l] + REDUCE_BLOCK_FLOATS - 1) / REDUCE_BLOCK_FLOATS);
  }
}

}  // namespace

extern "C" {

size_t rslx_ppo_update_recurrent_workspace_bytes(const rslx_memory* gru_actor, const rslx_mlp* actor, const rslx_memory* gru_critic,
                                                 const rslx_mlp* critic, const rslx_rollout* ro, const rslx_ppo_cfg* cfg) {
  if (rnn_validate(gru_actor, actor, gru_critic, critic, ro, cfg, false) != RSLX_OK) return 0;
  Carver c(nullptr);
  RnnPlan p;
  rnn_plan(c, gru_actor, actor, gru_critic, critic, ro, cfg, p);
  return p.bytes;
}

}  // extern "C"

namespace {
// Shared body of rslx_ppo_update_recurrent and its device-counter variant.
int32_t ppo_update_recurrent_impl(rslx_memory* gru_actor, rslx_mlp* actor, rslx_memory* gru_critic, rslx_mlp* critic,
                                  const rslx_rollout* ro, const uint8_t* dones, const float* h0_actor, const float* h0_critic,
                                  const rslx_ppo_cfg* cfg, int64_t* adam_step, rslx_dev_counters* counters, float* stats,
                                  void* ws, size_t ws_bytes, void* stream) {
  RSLX_TRY(rnn_validate(gru_actor, actor, gru_critic, critic, ro, cfg, true));
  int64_t host_step = 0;
  if (counters) adam_step = &host_step;
  if (!dones || !h0_actor || !h0_critic || !adam_step || !stats)
    return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent: null dones, h0, adam_step or stats");
  if (!aligned16(h0_actor) || !aligned16(h0_critic)) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent: h0 not 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  RnnPlan p;
  rnn_plan(c, gru_actor, actor, gru_critic, critic, ro, cfg, p);
  if (!ws || ws_bytes < p.bytes) return fail(RSLX_ERR_WORKSPACE, "rslx_ppo_update_recurrent: workspace %zu < %zu bytes", ws_bytes, p.bytes);
  const int A = ro->A, L_a = actor->n_layers, L_c = critic->n_layers;
  const int T = p.T, nb = p.nb, rows = p.rows;
  const rslx_memory* mem[2] = {gru_actor, gru_critic};
  RnnBufs* mb[2] = {&p.ma, &p.mc};
  const float* obs[2] = {ro->obs_actor, ro->obs_critic};
  const float* h0[2] = {h0_actor, h0_critic};

  {
    std::vector<uint64_t> bases(cfg->epochs);
    for (int e = 0; e < cfg->epochs; ++e)
      bases[e] = mix64_host(mix64_host(mix64_host(cfg->seed) ^ cfg->call_index) ^ (uint64_t)(e + cfg->epoch_offset));
    RSLX_HIP(launch_permutations(bases.data(), cfg->epochs, p.N, p.perms, p.perm_ws, s, mix64_host(cfg->seed),
                                 counters ? &counters->call_index : nullptr, cfg->epoch_offset));
    RSLX_HIP(launch_column_rows(p.perms, cfg->epochs, cfg->minibatches, T, p.N, p.rows_all, s));
  }

  for (int e = 0; e < cfg->epochs; ++e) {
    for (int m = 0; m < cfg->minibatches; ++m) {
      const int32_t* envs = p.perms + (size_t)e * p.N + (size_t)m * nb;
      const int32_t* ridx = p.rows_all + ((size_t)e * cfg->minibatches + m) * rows;
      float* stats_row = stats + ((size_t)e * cfg->minibatches + m) * RSLX_NSTATS;

      RSLX_TRY(memories_forward(mem, mb, 2, obs, h0, envs, ridx, dones, T, nb, p.N, s));

      // ---- MLPs on the hidden states, loss head, MLP backward down to the hidden states ----
      XView xa = plain_view(p.ma.hs, gru_actor->hidden), xc = plain_view(p.mc.hs, gru_critic->hidden);
      NetJob fj[2] = {NetJob{actor, xa, rows, &p.actor.act}, NetJob{critic, xc, rows, &p.critic.act}};
      RSLX_TRY(forward_nets(fj, 2, s, p.fused_head));
      PpoLossArgs la;
      memset(&la, 0, sizeof la);
      la.mu = p.actor.act.out[L_a - 1];
      la.v = p.critic.act.out[L_c - 1];
      la.log_std = actor->params + weight_count(*actor);
      la.idx = ridx;
      la.actions = ro->actions; la.logp_old = ro->logp; la.adv = ro->advantages; la.returns = ro->returns;
      la.v_old = ro->values; la.mu_old = ro->mu; la.sigma_old = ro->sigma;
      la.mb = rows; la.rows = rows; la.A = A;
      la.clip = cfg->clip; la.value_coef = cfg->value_coef; la.entropy_coef = cfg->entropy_coef;
      la.clipped_value = cfg->use_clipped_value_loss;
      la.d_mu = p.actor.d_out; la.d_v = p.critic.d_out;
      la.partials = p.loss_partials;
      if (p.fused_head) {
        PpoHeadArgs ha;
        ha.loss = la;
        ha.h_a = p.actor.act.out[L_a - 2]; ha.h_c = p.critic.act.out[L_c - 2];
        ha.w_a = actor->params + layer_offset(*actor, L_a - 1); ha.w_c = critic->params + layer_offset(*critic, L_c - 1);
        ha.dz_a = p.actor.act.dz[L_a - 2]; ha.dz_c = p.critic.act.dz[L_c - 2];
        ha.Ha = actor->dims[L_a - 1]; ha.Hc = critic->dims[L_c - 1];
        ha.alpha_a = actor->elu_alpha; ha.alpha_c = critic->elu_alpha;
        RSLX_HIP(launch_ppo_head(ha, s));
      } else {
        RSLX_HIP(launch_ppo_loss(la, s));
      }
      BwdJob bj[2] = {BwdJob{actor, xa, rows, &p.actor.act, p.actor.d_out, p.actor.wt, p.actor.partials, &p.actor.plan, p.ma.dh},
                      BwdJob{critic, xc, rows, &p.critic.act, p.critic.d_out, p.critic.wt, p.critic.partials, &p.critic.plan, p.mc.dh}};
      RSLX_TRY(backward_nets(bj, 2, s, p.fused_head));

      RSLX_TRY(memories_backward(mem, mb, 2, obs, ridx, dones, T, nb, p.N, s));
      {   // one launch: every split sum and the loss head's sums
        ReduceArgs ra;
        memset(&ra, 0, sizeof ra);
        ra.sumsq_blocks = p.sumsq_all;
        reduce_add_net(ra, *actor, p.actor);
        reduce_add_net(ra, *critic, p.critic);
        reduce_add_memory(ra, *gru_actor, p.ma);
        reduce_add_memory(ra, *gru_critic, p.mc);
        ra.finish.partials = p.loss_partials; ra.finish.blocks = p.loss_blocks;
        ra.finish.rows = rows; ra.finish.mb = rows; ra.finish.A = A;
        ra.finish.log_std = la.log_std; ra.finish.entropy_coef = cfg->entropy_coef;
        ra.finish.d_log_std = actor->grads + weight_count(*actor);
        ra.finish.stats_row = stats_row;
        ra.finish.sumsq_slot = p.sumsq_all + (p.n_sumsq - 1);
        RSLX_HIP(launch_reduce_partials(ra, s));
      }
      const int64_t t1 = *adam_step + 1;
      AdamArgs aa;
      memset(&aa, 0, sizeof aa);
      aa.seg[0] = AdamSegment{actor->params, actor->grads, actor->adam_m, actor->adam_v, param_count(*actor)};
      aa.seg[1] = AdamSegment{critic->params, critic->grads, critic->adam_m, critic->adam_v, param_count(*critic)};
      aa.seg[2] = AdamSegment{gru_actor->params, gru_actor->grads, gru_actor->adam_m, gru_actor->adam_v, gru_count(*gru_actor)};
      aa.seg[3] = AdamSegment{gru_critic->params, gru_critic->grads, gru_critic->adam_m, gru_critic->adam_v, gru_count(*gru_critic)};
      aa.n_seg = 4;
      aa.sumsq_blocks = p.sumsq_all; aa.n_sumsq = p.n_sumsq;
      aa.max_grad_norm = cfg->max_grad_norm;
      aa.lr = cfg->lr; aa.beta1 = cfg->beta1; aa.beta2 = cfg->beta2; aa.eps = cfg->adam_eps;
      aa.bc1 = bias_correction(cfg->beta1, t1); aa.bc2 = bias_correction(cfg->beta2, t1);
      if (counters) { aa.step_dev = &counters->adam_step; aa.step_off = (int32_t)t1; }
      aa.grad_norm_out = stats_row + RSLX_STAT_GRAD_NORM;
      RSLX_HIP(launch_adam(aa, s));
      *adam_step = t1;
    }
  }
  if (counters) RSLX_HIP(advance_counters(counters, 0, 1, host_step, 0, s));
  return RSLX_OK;
}
}  // namespace

extern "C" {

int32_t rslx_ppo_update_recurrent(rslx_memory* mem_actor, rslx_mlp* actor, rslx_memory* mem_critic, rslx_mlp* critic,
                                  const rslx_rollout* ro, const uint8_t* dones, const float* h0_actor, const float* h0_critic,
                                  const rslx_ppo_cfg* cfg, int64_t* adam_step, float* stats, void* ws, size_t ws_bytes,
                                  void* stream) {
  if (!adam_step) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent: null adam_step");
  return ppo_update_recurrent_impl(mem_actor, actor, mem_critic, critic, ro, dones, h0_actor, h0_critic, cfg, adam_step, nullptr,
                                   stats, ws, ws_bytes, stream);
}

int32_t rslx_ppo_update_recurrent_dc(rslx_memory* mem_actor, rslx_mlp* actor, rslx_memory* mem_critic, rslx_mlp* critic,
                                     const rslx_rollout* ro, const uint8_t* dones, const float* h0_actor,
                                     const float* h0_critic, const rslx_ppo_cfg* cfg, rslx_dev_counters* counters,
                                     float* stats, void* ws, size_t ws_bytes, void* stream) {
  if (!counters) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_recurrent_dc: null counters");
  return ppo_update_recurrent_impl(mem_actor, actor, mem_critic, critic, ro, dones, h0_actor, h0_critic, cfg, nullptr, counters,
                                   stats, ws, ws_bytes, stream);
}

}  // extern "C"

// ---- a single memory: one step, and behaviour cloning of a recurrent student ---------------------------------
namespace {

struct RnnBcPlan {
  int32_t nb, rows;
  int32_t* perms = nullptr;      // [E, N]
  void* perm_ws = nullptr;
  int32_t* rows_all = nullptr;   // [E, M, T, nb]
  TrainBufs student;
  RnnBufs mem;
  double* sumsq_all = nullptr;
  int32_t n_sumsq = 0;
  double* mse_partials = nullptr;
  size_t bytes = 0;
};

void rnn_bc_plan(Carver& c, const rslx_memory* g, const rslx_mlp* student, int32_t T, int32_t N, const rslx_bc_cfg* cfg, RnnBcPlan& p) {
  p.nb = N / cfg->minibatches;
  p.rows = T * p.nb;
  p.perms = c.take<int32_t>((size_t)cfg->epochs * N);
  p.perm_ws = c.take<char>(perm_workspace_bytes(N));
  p.rows_all = c.take<int32_t>((size_t)cfg->epochs * T * N);
  carve_train(c, *student, p.rows, 1, p.student, true);
  carve_memory(c, *g, p.rows, p.nb, p.mem, 1);
  p.n_sumsq = p.student.n_sumsq + p.mem.plan.blocks;
  p.sumsq_all = c.take<double>((size_t)p.n_sumsq + 1);
  p.mse_partials = c.take<double>(mse_num_blocks((int64_t)p.rows * student->dims[student->n_layers]));
  p.bytes = c.off + 256;
}

int32_t rnn_bc_validate(const rslx_memory* g, const rslx_mlp* student, int32_t T, int32_t N, const rslx_bc_cfg* cfg, bool need_buffers) {
  if (!cfg) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update_recurrent: null cfg");
  RSLX_TRY(check_gru(g, "rslx_bc_update_recurrent memory", need_buffers));
  RSLX_TRY(check_mlp(student, "rslx_bc_update_recurrent student", need_buffers));
  if (student->dims[0] != g->hidden) return fail(RSLX_ERR_SHAPE, "rslx_bc_update_recurrent: student input width != memory width");
  if (student->n_layers + 2 > 16) return fail(RSLX_ERR_UNSUPPORTED, "rslx_bc_update_recurrent: too many layers");
  if (T < 1 || N < 1 || (int64_t)T * N > (1 << 30)) return fail(RSLX_ERR_SHAPE, "rslx_bc_update_recurrent: T = %d, N = %d", T, N);
  if (cfg->minibatches < 1 || cfg->epochs < 0 || N % cfg->minibatches != 0)
    return fail(RSLX_ERR_SHAPE, "rslx_bc_update_recurrent: N = %d is not a multiple of minibatches = %d", N, cfg->minibatches);
  return RSLX_OK;
}

}  // namespace

extern "C" {

size_t rslx_memory_step_workspace_bytes(const rslx_memory* mem, int32_t N) {
  if (!mem || N <= 0) return 256;
  Carver c(nullptr);
  act_recurrent_carve(c, mem, nullptr, N, nullptr, nullptr);
  return c.off + 256;
}

int32_t rslx_memory_step(const rslx_memory* mem, const float* obs, int32_t N, float* state, const uint8_t* reset_or_null,
                         float* s0_out, float* h_dense_out, void* ws, size_t ws_bytes, void* stream) {
  if (N < 0) return fail(RSLX_ERR_SHAPE, "rslx_memory_step: N = %d", N);
  RSLX_TRY(check_gru(mem, "rslx_memory_step memory", false));
  if (!obs || !state) return fail(RSLX_ERR_INVALID_ARG, "rslx_memory_step: null input or state");
  if (!aligned16(state) || (s0_out && !aligned16(s0_out)) || (h_dense_out && !aligned16(h_dense_out)))
    return fail(RSLX_ERR_INVALID_ARG, "rslx_memory_step: state buffers not 16-byte aligned");
  if (N == 0) return RSLX_OK;
  if (!ws || ws_bytes < rslx_memory_step_workspace_bytes(mem, N)) return fail(RSLX_ERR_WORKSPACE, "rslx_memory_step: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  StepBufs b;
  act_recurrent_carve(c, mem, nullptr, N, &b, nullptr);
  RowGatherArgs rg;
  memset(&rg, 0, sizeof rg);
  rg.n_jobs = 1; rg.nb = N; rg.reset = reset_or_null;
  rg.job[0] = RowGatherJob{state, b.hin, s0_out, state_width(*mem)};
  RSLX_HIP(launch_row_gather(rg, s));
  const rslx_memory* g[1] = {mem};
  const float* o[1] = {obs};
  const StepBufs bb[1] = {b};
  float* out[1] = {state};
  RSLX_TRY(gru_step(g, o, bb, out, 1, N, s));
  if (h_dense_out) RSLX_HIP(launch_copy_matrix(state, state_width(*mem), N, mem->hidden, h_dense_out, s));
  return RSLX_OK;
}

size_t rslx_bc_update_recurrent_workspace_bytes(const rslx_memory* gru, const rslx_mlp* student, int32_t T, int32_t N,
                                                const rslx_bc_cfg* cfg) {
  if (rnn_bc_validate(gru, student, T, N, cfg, false) != RSLX_OK) return 0;
  Carver c(nullptr);
  RnnBcPlan p;
  rnn_bc_plan(c, gru, student, T, N, cfg, p);
  return p.bytes;
}

int32_t rslx_bc_update_recurrent(rslx_memory* gru, rslx_mlp* student, const float* obs_student, const float* targets,
                                 const uint8_t* dones, const float* h0, int32_t T, int32_t N, const rslx_bc_cfg* cfg,
                                 int64_t* adam_step, float* stats, void* ws, size_t ws_bytes, void* stream) {
  RSLX_TRY(rnn_bc_validate(gru, student, T, N, cfg, true));
  if (!obs_student || !targets || !dones || !h0 || !adam_step || !stats)
    return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update_recurrent: null pointer");
  if (!aligned16(h0)) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update_recurrent: h0 not 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  RnnBcPlan p;
  rnn_bc_plan(c, gru, student, T, N, cfg, p);
  if (!ws || ws_bytes < p.bytes) return fail(RSLX_ERR_WORKSPACE, "rslx_bc_update_recurrent: workspace %zu < %zu bytes", ws_bytes, p.bytes);
  const int A = student->dims[student->n_layers], Ls = student->n_layers;
  const int nb = p.nb, rows = p.rows;
  const rslx_memory* mem[1] = {gru};
  RnnBufs* mb[1] = {&p.mem};
  const float* obs[1] = {obs_student};
  const float* h0s[1] = {h0};
  {
    std::vector<uint64_t> bases(cfg->epochs);
    for (int e = 0; e < cfg->epochs; ++e)
      bases[e] = mix64_host(mix64_host(mix64_host(cfg->seed) ^ cfg->call_index) ^ (uint64_t)(e + cfg->epoch_offset));
    RSLX_HIP(launch_permutations(bases.data(), cfg->epochs, N, p.perms, p.perm_ws, s));
    RSLX_HIP(launch_column_rows(p.perms, cfg->epochs, cfg->minibatches, T, N, p.rows_all, s));
  }
  const int nbm = mse_num_blocks((int64_t)rows * A);
  for (int e = 0; e < cfg->epochs; ++e) {
    for (int m = 0; m < cfg->minibatches; ++m) {
      const int32_t* envs = p.perms + (size_t)e * N + (size_t)m * nb;
      const int32_t* ridx = p.rows_all + ((size_t)e * cfg->minibatches + m) * rows;
      float* stats_row = stats + ((size_t)e * cfg->minibatches + m) * RSLX_NSTATS;
      RSLX_HIP(launch_fill(stats_row, RSLX_NSTATS, 0.f, s));
      RSLX_TRY(memories_forward(mem, mb, 1, obs, h0s, envs, ridx, dones, T, nb, N, s));
      XView xs = plain_view(p.mem.hs, gru->hidden);
      NetJob fj{student, xs, rows, &p.student.act};
      RSLX_TRY(forward_nets(&fj, 1, s));
      RSLX_HIP(launch_mse(p.student.act.out[Ls - 1], targets, ridx, rows, A, p.student.d_out, p.mse_partials, s));
      RSLX_HIP(launch_mse_finish(p.mse_partials, nbm, (int64_t)rows * A, stats_row, s));
      BwdJob bj{student, xs, rows, &p.student.act, p.student.d_out, p.student.wt, p.student.partials, &p.student.plan, p.mem.dh};
      RSLX_TRY(backward_nets(&bj, 1, s));
      RSLX_TRY(memories_backward(mem, mb, 1, obs, ridx, dones, T, nb, N, s));
      {
        ReduceArgs ra;
        memset(&ra, 0, sizeof ra);
        ra.sumsq_blocks = p.sumsq_all;
        reduce_add_net(ra, *student, p.student);
        reduce_add_memory(ra, *gru, p.mem);
        RSLX_HIP(launch_reduce_partials(ra, s));
      }
      const int64_t t1 = *adam_step + 1;
      AdamArgs aa;
      memset(&aa, 0, sizeof aa);
      aa.seg[0] = AdamSegment{student->params, student->grads, student->adam_m, student->adam_v, weight_count(*student)};
      aa.seg[1] = AdamSegment{gru->params, gru->grads, gru->adam_m, gru->adam_v, gru_count(*gru)};
      aa.n_seg = 2;
      aa.sumsq_blocks = p.sumsq_all; aa.n_sumsq = p.n_sumsq;
      aa.max_grad_norm = cfg->max_grad_norm;
      aa.lr = cfg->lr; aa.beta1 = cfg->beta1; aa.beta2 = cfg->beta2; aa.eps = cfg->adam_eps;
      aa.bc1 = bias_correction(cfg->beta1, t1); aa.bc2 = bias_correction(cfg->beta2, t1);
      aa.grad_norm_out = stats_row + RSLX_STAT_GRAD_NORM;
      RSLX_HIP(launch_adam(aa, s));
      *adam_step = t1;
    }
  }
  return RSLX_OK;
}

}  // extern "C"
