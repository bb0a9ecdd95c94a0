// Host side of librslx: argument validation, workspace carving and launch sequencing for the C ABI
// declared in include/rslx.h.  No entry point synchronises with the host or allocates device memory.
#include "host.h"

#include <mutex>

namespace {

using namespace rslx;
using namespace rslx::host;

struct TraceRec {
  hipEvent_t a, b;
  char kernel[48];
  double flops, bytes;
};
bool g_trace_on = false;
size_t g_trace_cap = 0;
long g_trace_dropped = 0;      // launches seen while the trace was on that got no record
std::vector<TraceRec> g_trace;

// Scratch of rslx_gae_noalloc: the per-workgroup partial sums of the advantage normalisation, then the mean and
// the inverse deviation, for up to RSLX_GAE_NOALLOC_MAX_ENVS environments.  Every device the library runs on
// holds its own copy of the array at its own address; host code never uses the array's name as an address, only
// the per-device pointer resolved below.
constexpr int kGaeScratchDoubles = 2 * (RSLX_GAE_NOALLOC_MAX_ENVS / 256) + 2 + 6;     // 8200 doubles = 65 600 bytes
static __device__ __align__(256) double scratch[kGaeScratchDoubles];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, resolved once per device.
int32_t gae_scratch(double** out) {
  int dev = 0;
  RSLX_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(RSLX_ERR_UNSUPPORTED, "rslx_gae_noalloc: device index %d", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    double* p = nullptr;
    RSLX_HIP(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(RSLX_ERR_HIP, "rslx_gae_noalloc: no device address for the scratch array on device %d", dev);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return RSLX_OK;
}

}  // namespace

namespace rslx {
int trace_open(hipStream_t stream, const char* kernel, double flops, double bytes) {
  if (!g_trace_on) return -1;
  if (g_trace.size() >= g_trace_cap) { ++g_trace_dropped; return -1; }
  TraceRec r;
  if (hipEventCreate(&r.a) != hipSuccess) { ++g_trace_dropped; return -1; }
  if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); ++g_trace_dropped; return -1; }
  snprintf(r.kernel, sizeof r.kernel, "%s", kernel);
  r.flops = flops; r.bytes = bytes;
  (void)hipEventRecord(r.a, stream);
  g_trace.push_back(r);
  return (int)g_trace.size() - 1;
}
void trace_close(hipStream_t stream, int record) {
  if (record < 0 || (size_t)record >= g_trace.size()) return;
  (void)hipEventRecord(g_trace[record].b, stream);
}
}  // namespace rslx

// ======================================================================================================
extern "C" {

int32_t rslx_trace_begin(int32_t max_records) {
  if (max_records < 1) return fail(RSLX_ERR_INVALID_ARG, "rslx_trace_begin: max_records = %d", max_records);
  for (TraceRec& r : g_trace) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  g_trace.clear();
  g_trace.reserve(max_records);
  g_trace_cap = (size_t)max_records;
  g_trace_dropped = 0;
  g_trace_on = true;
  return RSLX_OK;
}

int32_t rslx_trace_end(rslx_trace_record* out, int32_t cap, int32_t* n_out) {
  g_trace_on = false;
  if (!n_out) return fail(RSLX_ERR_INVALID_ARG, "rslx_trace_end: null n_out");
  int32_t n = 0;
  for (TraceRec& r : g_trace) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(r.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
    if (e != hipSuccess) return fail(RSLX_ERR_HIP, "rslx_trace_end: %s", hipGetErrorString(e));
    if (out && n < cap) {
      memcpy(out[n].kernel, r.kernel, sizeof r.kernel);
      out[n].flops = r.flops; out[n].bytes = r.bytes; out[n].ms = ms;
    }
    ++n;
  }
  *n_out = n;
  if (out) {
    for (TraceRec& r : g_trace) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    g_trace.clear();
  }
  if (g_trace_dropped > 0)
    return fail(RSLX_ERR_WORKSPACE, "rslx_trace_end: %ld launches were not recorded (max_records = %zu too small, or no event could be created)",
                g_trace_dropped, g_trace_cap);
  return RSLX_OK;
}

int32_t rslx_version(void) { return 100; }

const char* rslx_last_error(void) { return g_last_error.c_str(); }

int32_t rslx_device_check(void) {
  int dev = 0;
  RSLX_HIP(hipGetDevice(&dev));
  hipDeviceProp_t prop;
  RSLX_HIP(hipGetDeviceProperties(&prop, dev));
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
    return fail(RSLX_ERR_UNSUPPORTED, "device %d is %s, this library is built for gfx950", dev, prop.gcnArchName);
  return RSLX_OK;
}

// ---- permutation ---------------------------------------------------------------------------------------
size_t rslx_permutation_workspace_bytes(int32_t B) { return B > 0 ? perm_workspace_bytes(B) + 256 : 256; }

int32_t rslx_permutation(uint64_t seed, uint64_t call_index, int32_t epoch, int32_t B, int32_t* perm_out, void* ws,
                         size_t ws_bytes, void* stream) {
  if (B < 0 || epoch < 0) return fail(RSLX_ERR_SHAPE, "rslx_permutation: B = %d, epoch = %d", B, epoch);
  if (B == 0) return RSLX_OK;
  if (!perm_out || !ws) return fail(RSLX_ERR_INVALID_ARG, "rslx_permutation: null pointer");
  if (ws_bytes < rslx_permutation_workspace_bytes(B)) return fail(RSLX_ERR_WORKSPACE, "rslx_permutation: workspace too small");
  Carver c(ws);
  void* w = c.take<char>(perm_workspace_bytes(B));
  const uint64_t base = mix64_host(mix64_host(mix64_host(seed) ^ call_index) ^ (uint64_t)epoch);
  RSLX_HIP(launch_permutations(&base, 1, B, perm_out, w, (hipStream_t)stream));
  return RSLX_OK;
}

// ---- act ---------------------------------------------------------------------------------------------------
// A workspace query reads the layer table before any other check has run: a depth outside the table must not be
// walked (the entry point proper rejects it with a message; the query answers 0).
static bool depth_ok(const rslx_mlp* n) { return n == nullptr || (n->n_layers >= 1 && n->n_layers <= RSLX_MAX_LAYERS); }

static size_t act_carve(Carver& c, const rslx_mlp* actor, const rslx_mlp* critic, int32_t N, NetBufs* ba, NetBufs* bc) {
  NetBufs ta, tc;
  if (actor) carve_net(c, *actor, N, false, ta);
  if (critic) carve_net(c, *critic, N, false, tc);
  if (ba) *ba = ta;
  if (bc) *bc = tc;
  return c.off + 256;
}

size_t rslx_act_workspace_bytes(const rslx_mlp* actor, const rslx_mlp* critic, int32_t N) {
  if (!depth_ok(actor) || !depth_ok(critic)) return 0;
  if (N <= 0) return 256;
  Carver c(nullptr);
  return act_carve(c, actor, critic, N, nullptr, nullptr);
}

}  // extern "C"

namespace rslx {
namespace host {
// Shared body of rslx_act and rslx_act_dc: with `counters` the noise position comes from device memory.
int32_t act_impl(const rslx_mlp* actor, const rslx_mlp* critic, const float* obs_actor, const float* obs_critic,
                 int32_t N, uint64_t seed, uint64_t step, rslx_dev_counters* counters, const float* eps_or_null,
                 float* actions, float* logp, float* values, float* mu, float* sigma, uint32_t flags, void* ws,
                 size_t ws_bytes, void* stream, int32_t ld_actor, int32_t ld_critic) {
  const bool values_only = (flags & RSLX_ACT_VALUES_ONLY) != 0;
  const int64_t* step_dev = counters ? &counters->act_step : nullptr;
  const uint64_t noise_pre = mix64_host(seed ^ 0xAC7ull);
  if (N < 0) return fail(RSLX_ERR_SHAPE, "rslx_act: N = %d", N);
  RSLX_TRY(check_mlp(critic, "rslx_act critic", false));
  if (critic->dims[critic->n_layers] != 1) return fail(RSLX_ERR_SHAPE, "rslx_act: critic output width must be 1");
  if (!values_only) {
    RSLX_TRY(check_mlp(actor, "rslx_act actor", false));
    if (!actor->has_log_std) return fail(RSLX_ERR_INVALID_ARG, "rslx_act: actor needs log_std");
    if (actor->dims[actor->n_layers] > RSLX_MAX_ACTIONS) return fail(RSLX_ERR_SHAPE, "rslx_act: action width > %d", RSLX_MAX_ACTIONS);
    if (!obs_actor || !actions || !logp || !mu || !sigma) return fail(RSLX_ERR_INVALID_ARG, "rslx_act: null actor input / output");
  }
  if (!obs_critic || !values) return fail(RSLX_ERR_INVALID_ARG, "rslx_act: null critic input / output");
  if (N == 0) return RSLX_OK;
  const rslx_mlp* a = values_only ? nullptr : actor;
  if (!ws || ws_bytes < rslx_act_workspace_bytes(a, critic, N)) return fail(RSLX_ERR_WORKSPACE, "rslx_act: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  // Fast path: one layer-fused launch for both networks and the Gaussian head.
  {
    FusedForwardArgs fa;
    memset(&fa, 0, sizeof fa);
    fa.n_rows = N;
    fa.max_dim = max_dim_of(*critic);
    if (a) {
      fa.net[fa.n_nets++] = fused_net(*a, obs_actor, ld_actor ? ld_actor : a->dims[0], nullptr, mu, true);
      fa.max_dim = max_dim_of(*a) > fa.max_dim ? max_dim_of(*a) : fa.max_dim;
    }
    fa.net[fa.n_nets++] = fused_net(*critic, obs_critic, ld_critic ? ld_critic : critic->dims[0], nullptr, values, false);
    fa.deterministic = (flags & RSLX_ACT_DETERMINISTIC) ? 1 : 0;
    fa.eps = eps_or_null;
    fa.noise_base = mix64_host(noise_pre ^ step);
    fa.step_dev = step_dev; fa.noise_pre = noise_pre;
    fa.actions = actions; fa.logp = logp; fa.sigma = sigma;
    if (fused_forward_pays(fa)) {
      RSLX_HIP(launch_fused_forward(fa, s));
      if (counters && !values_only) RSLX_HIP(advance_counters(counters, 1, 0, 0, 0, s));
      return RSLX_OK;
    }
  }
  // General path (layers wider than the fused kernel's LDS budget): one grouped launch per layer.
  Carver c(ws);
  NetBufs ba, bc;
  act_carve(c, a, critic, N, &ba, &bc);
  bc.out[critic->n_layers - 1] = values;              // [N, 1] lands directly in the caller's buffer
  NetJob jobs[2];
  int nj = 0;
  if (a) {
    ba.out[a->n_layers - 1] = mu;
    XView xa; xa.base = obs_actor; xa.ld = ld_actor ? ld_actor : a->dims[0];
    jobs[nj++] = NetJob{a, xa, N, &ba};
  }
  XView xc; xc.base = obs_critic; xc.ld = ld_critic ? ld_critic : critic->dims[0];
  jobs[nj++] = NetJob{critic, xc, N, &bc};
  RSLX_TRY(forward_nets(jobs, nj, s));
  if (a) {
    const int A = a->dims[a->n_layers];
    const uint64_t base = mix64_host(noise_pre ^ step);
    RSLX_HIP(launch_act_head(mu, a->params + weight_count(*a), eps_or_null, base, N, A,
                             (flags & RSLX_ACT_DETERMINISTIC) ? 1 : 0, actions, logp, mu, sigma, s, step_dev, noise_pre));
    if (counters) RSLX_HIP(advance_counters(counters, 1, 0, 0, 0, s));
  }
  return RSLX_OK;
}
}  // namespace host
}  // namespace rslx

extern "C" {

int32_t rslx_act(const rslx_mlp* actor, const rslx_mlp* critic, const float* obs_actor, const float* obs_critic,
                 int32_t N, uint64_t seed, uint64_t step, const float* eps_or_null, float* actions, float* logp,
                 float* values, float* mu, float* sigma, uint32_t flags, void* ws, size_t ws_bytes, void* stream) {
  return act_impl(actor, critic, obs_actor, obs_critic, N, seed, step, nullptr, eps_or_null, actions, logp, values, mu,
                  sigma, flags, ws, ws_bytes, stream);
}

int32_t rslx_act_dc(const rslx_mlp* actor, const rslx_mlp* critic, const float* obs_actor, const float* obs_critic,
                    int32_t N, uint64_t seed, rslx_dev_counters* counters, const float* eps_or_null, float* actions,
                    float* logp, float* values, float* mu, float* sigma, uint32_t flags, void* ws, size_t ws_bytes,
                    void* stream) {
  if (!counters) return fail(RSLX_ERR_INVALID_ARG, "rslx_act_dc: null counters");
  return act_impl(actor, critic, obs_actor, obs_critic, N, seed, 0, counters, eps_or_null, actions, logp, values, mu,
                  sigma, flags, ws, ws_bytes, stream);
}

// ---- GAE -----------------------------------------------------------------------------------------------------
size_t rslx_gae_workspace_bytes(int32_t T, int32_t N) {
  (void)T;
  if (N <= 0) return 256;
  return (size_t)gae_num_blocks(N) * 16 + 16 + 512;
}

int32_t rslx_gae(const float* rewards, const float* values, const float* last_values, const uint8_t* dones,
                 const uint8_t* timeouts_or_null, int32_t T, int32_t N, float gamma, float lam, int32_t normalize_adv,
                 float* advantages, float* returns, void* ws, size_t ws_bytes, void* stream) {
  if (T < 0 || N < 0) return fail(RSLX_ERR_SHAPE, "rslx_gae: T = %d, N = %d", T, N);
  if (T == 0 || N == 0) return RSLX_OK;
  if (!rewards || !values || !last_values || !dones || !advantages || !returns)
    return fail(RSLX_ERR_INVALID_ARG, "rslx_gae: null pointer");
  if (!aligned16(advantages)) return fail(RSLX_ERR_INVALID_ARG, "rslx_gae: advantages not 16-byte aligned");
  if ((int64_t)T * N > (int64_t)INT_MAX * 4) return fail(RSLX_ERR_SHAPE, "rslx_gae: T*N too large");
  double* partials = nullptr;
  if (normalize_adv) {
    if (!ws || ws_bytes < rslx_gae_workspace_bytes(T, N)) return fail(RSLX_ERR_WORKSPACE, "rslx_gae: workspace too small");
    Carver c(ws);
    partials = c.take<double>((size_t)gae_num_blocks(N) * 2 + 2);
  }
  RSLX_HIP(launch_gae(rewards, values, last_values, dones, timeouts_or_null, T, N, gamma, lam, normalize_adv ? 1 : 0,
                      advantages, returns, partials, (hipStream_t)stream));
  return RSLX_OK;
}

int32_t rslx_gae_noalloc(const float* rewards, const float* values, const float* last_values, const uint8_t* dones,
                         const uint8_t* timeouts_or_null, int32_t T, int32_t N, float gamma, float lam,
                         int32_t normalize_adv, float* advantages, float* returns, void* stream) {
  if (T < 0 || N < 0) return fail(RSLX_ERR_SHAPE, "rslx_gae_noalloc: T = %d, N = %d", T, N);
  if (N > RSLX_GAE_NOALLOC_MAX_ENVS)
    return fail(RSLX_ERR_SHAPE, "rslx_gae_noalloc: N = %d exceeds the built-in scratch (at most %d environments); use rslx_gae",
                N, RSLX_GAE_NOALLOC_MAX_ENVS);
  if (T == 0 || N == 0) return RSLX_OK;
  if (!rewards || !values || !last_values || !dones || !advantages || !returns)
    return fail(RSLX_ERR_INVALID_ARG, "rslx_gae_noalloc: null pointer");
  if (!aligned16(advantages)) return fail(RSLX_ERR_INVALID_ARG, "rslx_gae_noalloc: advantages not 16-byte aligned");
  if ((int64_t)T * N > (int64_t)INT_MAX * 4) return fail(RSLX_ERR_SHAPE, "rslx_gae_noalloc: T*N too large");
  double* partials = nullptr;
  if (normalize_adv) {
    if ((size_t)gae_num_blocks(N) * 2 + 2 > (size_t)kGaeScratchDoubles)
      return fail(RSLX_ERR_SHAPE, "rslx_gae_noalloc: N = %d needs more partial sums than the built-in scratch holds", N);
    RSLX_TRY(gae_scratch(&partials));
  }
  // every slot the kernels read is written by the same call first, so the previous call's contents need no clearing
  RSLX_HIP(launch_gae(rewards, values, last_values, dones, timeouts_or_null, T, N, gamma, lam, normalize_adv ? 1 : 0,
                      advantages, returns, partials, (hipStream_t)stream));
  return RSLX_OK;
}

// ---- Adam ----------------------------------------------------------------------------------------------------
size_t rslx_adam_workspace_bytes(int64_t n) { return n > 0 ? ((size_t)reduce_num_blocks(n) + 1) * 8 + 512 : 256; }

int32_t rslx_adam_step(float* params, const float* grads, float* m, float* v, int64_t n, float lr, float beta1,
                       float beta2, float eps, float max_grad_norm, int64_t* adam_step, float* grad_norm_out, void* ws,
                       size_t ws_bytes, void* stream) {
  if (n < 0) return fail(RSLX_ERR_SHAPE, "rslx_adam_step: n = %lld", (long long)n);
  if (!adam_step) return fail(RSLX_ERR_INVALID_ARG, "rslx_adam_step: null adam_step");
  if (n == 0) { ++*adam_step; return RSLX_OK; }
  if (!params || !grads || !m || !v) return fail(RSLX_ERR_INVALID_ARG, "rslx_adam_step: null pointer");
  if (!aligned16(params) || !aligned16(grads) || !aligned16(m) || !aligned16(v))
    return fail(RSLX_ERR_INVALID_ARG, "rslx_adam_step: buffers not 16-byte aligned");
  if (!ws || ws_bytes < rslx_adam_workspace_bytes(n)) return fail(RSLX_ERR_WORKSPACE, "rslx_adam_step: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  const int nb = reduce_num_blocks(n);
  double* sumsq = c.take<double>((size_t)nb + 1);
  RSLX_HIP(launch_sumsq(grads, n, sumsq, s));
  const int64_t t = *adam_step + 1;
  AdamArgs a;
  memset(&a, 0, sizeof a);
  a.seg[0] = AdamSegment{params, grads, m, v, n};
  a.n_seg = 1;
  a.sumsq_blocks = sumsq; a.n_sumsq = nb;
  a.max_grad_norm = max_grad_norm;
  a.lr = lr; a.beta1 = beta1; a.beta2 = beta2; a.eps = eps;
  a.bc1 = bias_correction(beta1, t); a.bc2 = bias_correction(beta2, t);
  a.grad_norm_out = grad_norm_out;
  RSLX_HIP(launch_adam(a, s));
  *adam_step = t;
  return RSLX_OK;
}

// ---- PPO update ------------------------------------------------------------------------------------------------
namespace {

struct PpoPlan {
  int32_t B, mb, rows;
  bool fused_head = false;           // output layers + loss + their input gradient in one launch
  int32_t loss_blocks = 0;
  int32_t* perms = nullptr;          // [E, B]
  void* perm_ws = nullptr;
  TrainBufs actor, critic, pred;
  NetBufs targ;
  float* stage_a = nullptr;          // staged (padded, mirrored) network inputs, when worth it (see staged_width)
  float* stage_c = nullptr;
  int dp_a = 0, dp_c = 0;            // their row widths, 0 = not staged
  int32_t* sym_perm = nullptr;       // device copies of the mirror maps made by the call when the caller passes none:
  float* sym_sign = nullptr;         // [Da + Dc + A] each
  double* sumsq_all = nullptr;       // actor blocks, critic blocks, log_std slot
  double* loss_partials = nullptr;
  double* mse_partials = nullptr;
  size_t bytes = 0;
};

void ppo_plan(Carver& c, const rslx_mlp* actor, const rslx_mlp* critic, const rslx_rollout* ro, const rslx_ppo_cfg* cfg,
              const rslx_sym* sym, const rslx_rnd_train* rnd, PpoPlan& p) {
  p.B = ro->T * ro->N;
  p.mb = p.B / cfg->minibatches;
  p.rows = sym ? 2 * p.mb : p.mb;
  p.perms = c.take<int32_t>((size_t)cfg->epochs * p.B);
  p.perm_ws = c.take<char>(perm_workspace_bytes(p.B));
  p.dp_a = staged_width(*actor, ro->Da, sym != nullptr);
  p.dp_c = staged_width(*critic, ro->Dc, sym != nullptr);
  if (p.dp_a) p.stage_a = c.take<float>((size_t)(sym ? 2 : 1) * p.B * p.dp_a);
  if (p.dp_c) p.stage_c = c.take<float>((size_t)(sym ? 2 : 1) * p.B * p.dp_c);
  carve_train(c, *actor, p.rows, 2, p.actor);
  carve_train(c, *critic, p.rows, 2, p.critic);
  if (sym) {
    p.sym_perm = c.take<int32_t>((size_t)ro->Da + ro->Dc + ro->A);
    p.sym_sign = c.take<float>((size_t)ro->Da + ro->Dc + ro->A);
  }
  p.sumsq_all = c.take<double>((size_t)p.actor.n_sumsq + p.critic.n_sumsq + 2);
  p.actor.sumsq = p.sumsq_all;
  p.critic.sumsq = p.sumsq_all ? p.sumsq_all + p.actor.n_sumsq : nullptr;      // null while only sizing the workspace
  p.fused_head = actor->n_layers >= 2 && critic->n_layers >= 2 &&
                 ppo_head_supported(actor->dims[actor->n_layers - 1], critic->dims[critic->n_layers - 1], ro->A);
  p.loss_blocks = p.fused_head ? ppo_head_num_blocks(p.mb, sym != nullptr) : ppo_loss_num_blocks(p.mb);
  p.loss_partials = c.take<double>((size_t)p.loss_blocks * (PPO_NPART_FIXED + ro->A));
  if (rnd) {
    carve_train(c, *rnd->predictor, p.mb, 1, p.pred);
    p.pred.sumsq = c.take<double>((size_t)p.pred.n_sumsq + 1);
    carve_net(c, *rnd->target, p.mb, false, p.targ);
    const int K = rnd->target->dims[rnd->target->n_layers];
    p.mse_partials = c.take<double>(mse_num_blocks((int64_t)p.mb * K));
  }
  p.bytes = c.off + 256;
}

int32_t ppo_validate(const rslx_mlp* actor, const rslx_mlp* critic, const rslx_rollout* ro, const rslx_ppo_cfg* cfg,
                     const rslx_sym* sym, const rslx_rnd_train* rnd, bool need_buffers) {
  if (!ro || !cfg) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: null rollout or cfg");
  RSLX_TRY(check_mlp(actor, "rslx_ppo_update actor", need_buffers));
  RSLX_TRY(check_mlp(critic, "rslx_ppo_update critic", need_buffers));
  if (!actor->has_log_std) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: actor needs log_std");
  if (ro->T < 1 || ro->N < 1 || (int64_t)ro->T * ro->N > (1 << 30)) return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: T = %d, N = %d", ro->T, ro->N);
  if (ro->Da != actor->dims[0] || ro->Dc != critic->dims[0] || ro->A != actor->dims[actor->n_layers] ||
      critic->dims[critic->n_layers] != 1)
    return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: rollout widths do not match the networks");
  if (ro->A > RSLX_MAX_ACTIONS) return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: action width %d > %d", ro->A, RSLX_MAX_ACTIONS);
  if (cfg->epochs < 0 || cfg->minibatches < 1) return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: epochs / minibatches");
  if ((ro->T * ro->N) % cfg->minibatches != 0)
    return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: T*N = %d is not a multiple of minibatches = %d", ro->T * ro->N, cfg->minibatches);
  if (need_buffers) {
    if (!ro->obs_actor || !ro->obs_critic || !ro->actions || !ro->logp || !ro->values || !ro->mu || !ro->sigma ||
        !ro->advantages || !ro->returns)
      return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: null rollout buffer");
  }
  if (sym) {
    if (!involution_ok(sym->perm_obs_a_host, sym->sign_obs_a_host, ro->Da) ||
        !involution_ok(sym->perm_obs_c_host, sym->sign_obs_c_host, ro->Dc) ||
        !involution_ok(sym->perm_act_host, sym->sign_act_host, ro->A))
      return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: mirror map is not an involutive signed permutation");
    const int n_dev = (sym->perm_obs_a != nullptr) + (sym->sign_obs_a != nullptr) + (sym->perm_obs_c != nullptr) +
                      (sym->sign_obs_c != nullptr) + (sym->perm_act != nullptr) + (sym->sign_act != nullptr);
    if (need_buffers && n_dev != 0 && n_dev != 6)
      return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: device mirror maps must be given all or not at all");
  }
  if (rnd) {
    RSLX_TRY(check_mlp(rnd->target, "rslx_ppo_update rnd target", false));
    RSLX_TRY(check_mlp(rnd->predictor, "rslx_ppo_update rnd predictor", need_buffers));
    if (rnd->target->n_layers != rnd->predictor->n_layers) return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: rnd nets differ in depth");
    for (int i = 0; i <= rnd->target->n_layers; ++i)
      if (rnd->target->dims[i] != rnd->predictor->dims[i]) return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: rnd nets differ in shape");
    if (rnd->n_subset != rnd->target->dims[0] || (!rnd->subset_idx && rnd->n_subset != ro->Da))
      return fail(RSLX_ERR_SHAPE, "rslx_ppo_update: rnd subset width");
  }
  return RSLX_OK;
}

}  // namespace

size_t rslx_ppo_update_workspace_bytes(const rslx_mlp* actor, const rslx_mlp* critic, const rslx_rollout* ro,
                                       const rslx_ppo_cfg* cfg, const rslx_sym* sym, const rslx_rnd_train* rnd) {
  if (ppo_validate(actor, critic, ro, cfg, sym, rnd, false) != RSLX_OK) return 0;
  Carver c(nullptr);
  PpoPlan p;
  ppo_plan(c, actor, critic, ro, cfg, sym, rnd, p);
  return p.bytes;
}

}  // extern "C"

namespace {
// Shared body of rslx_ppo_update and rslx_ppo_update_dc: with `counters` the permutation stream index and the
// optimiser step counts are read from device memory by the kernels and advanced at the end of the call.
int32_t ppo_update_impl(rslx_mlp* actor, rslx_mlp* critic, const rslx_rollout* ro, const rslx_ppo_cfg* cfg,
                        const rslx_sym* sym, const rslx_rnd_train* rnd, int64_t* adam_step, rslx_dev_counters* counters,
                        float* stats, void* ws, size_t ws_bytes, void* stream) {
  RSLX_TRY(ppo_validate(actor, critic, ro, cfg, sym, rnd, true));
  if ((!adam_step && !counters) || !stats) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: null adam_step or stats");
  int64_t host_step = 0, host_rnd_step = 0;      // stand-ins for the host counters in the device-counter variant
  if (counters) adam_step = &host_step;
  int64_t* rnd_step = rnd ? (counters ? &host_rnd_step : rnd->adam_step) : nullptr;
  if (rnd && !rnd_step) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: rnd adam_step null");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  PpoPlan p;
  ppo_plan(c, actor, critic, ro, cfg, sym, rnd, p);
  if (!ws || ws_bytes < p.bytes) return fail(RSLX_ERR_WORKSPACE, "rslx_ppo_update: workspace %zu < %zu bytes", ws_bytes, p.bytes);
  const int A = ro->A, L_a = actor->n_layers, L_c = critic->n_layers;

  // Mirror maps without device copies: the validated host copies are uploaded into the workspace, so the kernels
  // cannot see other values than the ones that were checked.
  rslx_sym sym_dev;
  if (sym && sym->perm_obs_a == nullptr) {
    sym_dev = *sym;
    const int Da = ro->Da, Dc = ro->Dc;
    RSLX_HIP(hipMemcpyAsync(p.sym_perm, sym->perm_obs_a_host, sizeof(int32_t) * Da, hipMemcpyHostToDevice, s));
    RSLX_HIP(hipMemcpyAsync(p.sym_perm + Da, sym->perm_obs_c_host, sizeof(int32_t) * Dc, hipMemcpyHostToDevice, s));
    RSLX_HIP(hipMemcpyAsync(p.sym_perm + Da + Dc, sym->perm_act_host, sizeof(int32_t) * A, hipMemcpyHostToDevice, s));
    RSLX_HIP(hipMemcpyAsync(p.sym_sign, sym->sign_obs_a_host, sizeof(float) * Da, hipMemcpyHostToDevice, s));
    RSLX_HIP(hipMemcpyAsync(p.sym_sign + Da, sym->sign_obs_c_host, sizeof(float) * Dc, hipMemcpyHostToDevice, s));
    RSLX_HIP(hipMemcpyAsync(p.sym_sign + Da + Dc, sym->sign_act_host, sizeof(float) * A, hipMemcpyHostToDevice, s));
    sym_dev.perm_obs_a = p.sym_perm; sym_dev.perm_obs_c = p.sym_perm + Da; sym_dev.perm_act = p.sym_perm + Da + Dc;
    sym_dev.sign_obs_a = p.sym_sign; sym_dev.sign_obs_c = p.sym_sign + Da; sym_dev.sign_act = p.sym_sign + Da + Dc;
    sym = &sym_dev;
  }

  {
    std::vector<uint64_t> bases(cfg->epochs);
    for (int e = 0; e < cfg->epochs; ++e)
      bases[e] = mix64_host(mix64_host(mix64_host(cfg->seed) ^ cfg->call_index) ^ (uint64_t)(e + cfg->epoch_offset));
    RSLX_HIP(launch_permutations(bases.data(), cfg->epochs, p.B, p.perms, p.perm_ws, s, mix64_host(cfg->seed),
                                 counters ? &counters->call_index : nullptr, cfg->epoch_offset));
  }

  // The observations do not change during the call: where the 16-byte operand paths cannot read them in place,
  // a padded copy (with the mirrored rows below the originals) is made once and serves every minibatch.
  if (p.dp_a)
    RSLX_HIP(launch_stage_input(ro->obs_actor, ro->Da, (int32_t)p.B, ro->Da, p.dp_a, sym ? sym->perm_obs_a : nullptr,
                                sym ? sym->sign_obs_a : nullptr, p.stage_a, s));
  if (p.dp_c)
    RSLX_HIP(launch_stage_input(ro->obs_critic, ro->Dc, (int32_t)p.B, ro->Dc, p.dp_c, sym ? sym->perm_obs_c : nullptr,
                                sym ? sym->sign_obs_c : nullptr, p.stage_c, s));
  auto obs_view = [&](const float* obs, int D, const float* staged, int dp, const int32_t* col_map, const float* col_sign,
                      const int32_t* idx) {
    XView x;
    x.row_idx = idx;
    if (sym) x.idx_mod = p.mb;
    if (dp) {
      x.base = staged; x.ld = dp; x.cols = dp;
      x.src_rows = (sym ? 2 : 1) * (int64_t)p.B;
      if (sym) x.wrap_add = (int)p.B;
    } else {
      x.base = obs; x.ld = D; x.src_rows = p.B;
      if (sym) { x.map_from = p.mb; x.col_map = col_map; x.col_sign = col_sign; }
    }
    return x;
  };

  {   // transposed weights once per call; every Adam launch below keeps them current
    const XView none;
    BwdJob tj[2] = {BwdJob{actor, none, p.rows, &p.actor.act, p.actor.d_out, p.actor.wt, p.actor.partials, &p.actor.plan},
                    BwdJob{critic, none, p.rows, &p.critic.act, p.critic.d_out, p.critic.wt, p.critic.partials, &p.critic.plan}};
    if (cfg->epochs > 0) RSLX_TRY(transpose_weights(tj, 2, s, false));
  }
  for (int e = 0; e < cfg->epochs; ++e) {
    for (int m = 0; m < cfg->minibatches; ++m) {
      const int32_t* idx = p.perms + (size_t)e * p.B + (size_t)m * p.mb;
      float* stats_row = stats + ((size_t)e * cfg->minibatches + m) * RSLX_NSTATS;

      const XView xa = obs_view(ro->obs_actor, ro->Da, p.stage_a, p.dp_a, sym ? sym->perm_obs_a : nullptr,
                                sym ? sym->sign_obs_a : nullptr, idx);
      const XView xc = obs_view(ro->obs_critic, ro->Dc, p.stage_c, p.dp_c, sym ? sym->perm_obs_c : nullptr,
                                sym ? sym->sign_obs_c : nullptr, idx);
      NetJob fj[2] = {NetJob{actor, xa, p.rows, &p.actor.act}, NetJob{critic, xc, p.rows, &p.critic.act}};
      RSLX_TRY(forward_nets(fj, 2, s, p.fused_head));

      PpoLossArgs la;
      memset(&la, 0, sizeof la);
      la.mu = p.actor.act.out[L_a - 1];
      la.v = p.critic.act.out[L_c - 1];
      la.log_std = actor->params + weight_count(*actor);
      la.idx = idx;
      la.actions = ro->actions; la.logp_old = ro->logp; la.adv = ro->advantages; la.returns = ro->returns;
      la.v_old = ro->values; la.mu_old = ro->mu; la.sigma_old = ro->sigma;
      la.perm_act = sym ? sym->perm_act : nullptr;
      la.sign_act = sym ? sym->sign_act : nullptr;
      la.mb = p.mb; la.rows = p.rows; la.A = A;
      la.clip = cfg->clip; la.value_coef = cfg->value_coef; la.entropy_coef = cfg->entropy_coef;
      la.mirror_coef = sym ? sym->mirror_loss_coef : 0.f;
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
      BwdJob bj[2] = {BwdJob{actor, xa, p.rows, &p.actor.act, p.actor.d_out, p.actor.wt, p.actor.partials, &p.actor.plan},
                      BwdJob{critic, xc, p.rows, &p.critic.act, p.critic.d_out, p.critic.wt, p.critic.partials, &p.critic.plan}};
      RSLX_TRY(backward_nets(bj, 2, s, p.fused_head, true));
      {   // one launch: both networks' split sums and the loss head's sums
        ReduceArgs ra;
        memset(&ra, 0, sizeof ra);
        ra.sumsq_blocks = p.sumsq_all;
        reduce_add_net(ra, *actor, p.actor);
        reduce_add_net(ra, *critic, p.critic);
        ra.finish.partials = p.loss_partials; ra.finish.blocks = p.loss_blocks;
        ra.finish.rows = p.rows; ra.finish.mb = p.mb; ra.finish.A = A;
        ra.finish.log_std = la.log_std; ra.finish.entropy_coef = cfg->entropy_coef;
        ra.finish.d_log_std = actor->grads + weight_count(*actor);
        ra.finish.stats_row = stats_row;
        ra.finish.sumsq_slot = p.sumsq_all + p.actor.n_sumsq + p.critic.n_sumsq;
        RSLX_HIP(launch_reduce_partials(ra, s));
      }

      const int64_t t = *adam_step + 1;
      AdamArgs aa;
      memset(&aa, 0, sizeof aa);
      aa.seg[0] = AdamSegment{actor->params, actor->grads, actor->adam_m, actor->adam_v, param_count(*actor)};
      aa.seg[1] = AdamSegment{critic->params, critic->grads, critic->adam_m, critic->adam_v, param_count(*critic)};
      aa.n_seg = 2;
      adam_keeps_transposed(aa.seg[0], *actor, p.actor.wt);
      adam_keeps_transposed(aa.seg[1], *critic, p.critic.wt);
      aa.sumsq_blocks = p.sumsq_all; aa.n_sumsq = p.actor.n_sumsq + p.critic.n_sumsq + 1;
      aa.max_grad_norm = cfg->max_grad_norm;
      aa.lr = cfg->lr; aa.beta1 = cfg->beta1; aa.beta2 = cfg->beta2; aa.eps = cfg->adam_eps;
      aa.bc1 = bias_correction(cfg->beta1, t); aa.bc2 = bias_correction(cfg->beta2, t);
      if (counters) { aa.step_dev = &counters->adam_step; aa.step_off = (int32_t)t; }
      aa.grad_norm_out = stats_row + RSLX_STAT_GRAD_NORM;
      RSLX_HIP(launch_adam(aa, s));
      *adam_step = t;

      if (rnd) {
        const rslx_mlp& pr = *rnd->predictor;
        const int K = pr.dims[pr.n_layers];
        XView xr;
        xr.base = ro->obs_actor; xr.ld = ro->Da; xr.row_idx = idx; xr.src_rows = p.B;
        if (rnd->subset_idx) { xr.col_map = rnd->subset_idx; xr.map_from = 0; }
        NetJob rj[2] = {NetJob{&pr, xr, p.mb, &p.pred.act}, NetJob{rnd->target, xr, p.mb, &p.targ}};
        RSLX_TRY(forward_nets(rj, 2, s));
        const int nbm = mse_num_blocks((int64_t)p.mb * K);
        RSLX_HIP(launch_mse(p.pred.act.out[pr.n_layers - 1], p.targ.out[pr.n_layers - 1], nullptr, p.mb, K,
                            p.pred.d_out, p.mse_partials, s));
        RSLX_HIP(launch_mse_finish(p.mse_partials, nbm, (int64_t)p.mb * K, stats_row + RSLX_STAT_RND_LOSS, s));
        BwdJob rb{&pr, xr, p.mb, &p.pred.act, p.pred.d_out, p.pred.wt, p.pred.partials, &p.pred.plan};
        RSLX_TRY(backward_nets(&rb, 1, s));
        RSLX_TRY(reduce_net(pr, p.pred, s));
        const int64_t tr = *rnd_step + 1;
        AdamArgs ar;
        memset(&ar, 0, sizeof ar);
        ar.seg[0] = AdamSegment{pr.params, pr.grads, pr.adam_m, pr.adam_v, param_count(pr)};
        ar.n_seg = 1;
        ar.sumsq_blocks = p.pred.sumsq; ar.n_sumsq = 0;
        ar.max_grad_norm = 0.f;
        ar.lr = rnd->lr; ar.beta1 = cfg->beta1; ar.beta2 = cfg->beta2; ar.eps = cfg->adam_eps;
        ar.bc1 = bias_correction(cfg->beta1, tr); ar.bc2 = bias_correction(cfg->beta2, tr);
        if (counters) { ar.step_dev = &counters->rnd_adam_step; ar.step_off = (int32_t)tr; }
        RSLX_HIP(launch_adam(ar, s));
        *rnd_step = tr;
      }
    }
  }
  if (counters) RSLX_HIP(advance_counters(counters, 0, 1, host_step, host_rnd_step, s));
  return RSLX_OK;
}
}  // namespace

extern "C" {

int32_t rslx_ppo_update(rslx_mlp* actor, rslx_mlp* critic, const rslx_rollout* ro, const rslx_ppo_cfg* cfg,
                        const rslx_sym* sym, const rslx_rnd_train* rnd, int64_t* adam_step, float* stats, void* ws,
                        size_t ws_bytes, void* stream) {
  if (!adam_step) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update: null adam_step or stats");
  return ppo_update_impl(actor, critic, ro, cfg, sym, rnd, adam_step, nullptr, stats, ws, ws_bytes, stream);
}

int32_t rslx_ppo_update_dc(rslx_mlp* actor, rslx_mlp* critic, const rslx_rollout* ro, const rslx_ppo_cfg* cfg,
                           const rslx_sym* sym, const rslx_rnd_train* rnd, rslx_dev_counters* counters, float* stats,
                           void* ws, size_t ws_bytes, void* stream) {
  if (!counters) return fail(RSLX_ERR_INVALID_ARG, "rslx_ppo_update_dc: null counters");
  return ppo_update_impl(actor, critic, ro, cfg, sym, rnd, nullptr, counters, stats, ws, ws_bytes, stream);
}

// ---- behaviour cloning ---------------------------------------------------------------------------------------------
namespace {
struct BcPlan {
  int32_t mb;
  int32_t* perms = nullptr;
  void* perm_ws = nullptr;
  TrainBufs student;
  NetBufs teacher;
  float* targets = nullptr;
  double* mse_partials = nullptr;
  size_t bytes = 0;
};

void bc_plan(Carver& c, const rslx_mlp* student, const rslx_mlp* teacher, int32_t B, const rslx_bc_cfg* cfg, BcPlan& p) {
  p.mb = B / cfg->minibatches;
  p.perms = c.take<int32_t>((size_t)cfg->epochs * B);
  p.perm_ws = c.take<char>(perm_workspace_bytes(B));
  carve_train(c, *student, p.mb, 1, p.student);
  p.student.sumsq = c.take<double>((size_t)p.student.n_sumsq + 1);
  const int A = student->dims[student->n_layers];
  if (teacher) {
    carve_net(c, *teacher, p.mb, false, p.teacher);
    p.targets = c.take<float>((size_t)B * A);
  }
  p.mse_partials = c.take<double>(mse_num_blocks((int64_t)p.mb * A));
  p.bytes = c.off + 256;
}

int32_t bc_validate(const rslx_mlp* student, const rslx_mlp* teacher, int32_t B, const rslx_bc_cfg* cfg, bool need_buffers) {
  if (!cfg) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update: null cfg");
  RSLX_TRY(check_mlp(student, "rslx_bc_update student", need_buffers));
  if (teacher) {
    RSLX_TRY(check_mlp(teacher, "rslx_bc_update teacher", false));
    if (teacher->dims[teacher->n_layers] != student->dims[student->n_layers])
      return fail(RSLX_ERR_SHAPE, "rslx_bc_update: teacher and student action widths differ");
  }
  if (B < 1 || cfg->minibatches < 1 || cfg->epochs < 0 || B % cfg->minibatches != 0)
    return fail(RSLX_ERR_SHAPE, "rslx_bc_update: B = %d is not a positive multiple of minibatches = %d", B, cfg->minibatches);
  return RSLX_OK;
}
}  // namespace

size_t rslx_bc_update_workspace_bytes(const rslx_mlp* student, const rslx_mlp* teacher, int32_t B, const rslx_bc_cfg* cfg) {
  if (bc_validate(student, teacher, B, cfg, false) != RSLX_OK) return 0;
  Carver c(nullptr);
  BcPlan p;
  bc_plan(c, student, teacher, B, cfg, p);
  return p.bytes;
}

}  // extern "C"

namespace {
// Shared body of rslx_bc_update and rslx_bc_update_dc (permutation stream and Adam step count from device memory).
int32_t bc_update_impl(rslx_mlp* student, const rslx_mlp* teacher, const float* obs_student, const float* obs_teacher,
                       const float* targets_or_null, int32_t B, const rslx_bc_cfg* cfg, int64_t* adam_step,
                       rslx_dev_counters* counters, float* stats, void* ws, size_t ws_bytes, void* stream) {
  int64_t host_step = 0;
  if (counters) adam_step = &host_step;
  const rslx_mlp* tch = targets_or_null ? nullptr : teacher;
  if (!targets_or_null && !teacher) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update: need a teacher or precomputed targets");
  RSLX_TRY(bc_validate(student, tch, B, cfg, true));
  if (!obs_student || !stats) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update: null pointer");
  if (tch && !obs_teacher) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update: null teacher observations");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  BcPlan p;
  bc_plan(c, student, tch, B, cfg, p);
  if (!ws || ws_bytes < p.bytes) return fail(RSLX_ERR_WORKSPACE, "rslx_bc_update: workspace %zu < %zu bytes", ws_bytes, p.bytes);
  const int A = student->dims[student->n_layers];
  const int Ls = student->n_layers;

  const float* targets = targets_or_null;
  if (tch) {                           // teacher means for every row, one minibatch-sized slab at a time
    for (int k = 0; k < cfg->minibatches; ++k) {
      NetBufs tb = p.teacher;
      tb.out[tch->n_layers - 1] = p.targets + (size_t)k * p.mb * A;
      XView xt; xt.base = obs_teacher + (size_t)k * p.mb * tch->dims[0]; xt.ld = tch->dims[0];
      NetJob j{tch, xt, p.mb, &tb};
      RSLX_TRY(forward_nets(&j, 1, s));
    }
    targets = p.targets;
  }
  {
    std::vector<uint64_t> bases(cfg->epochs);
    for (int e = 0; e < cfg->epochs; ++e)
      bases[e] = mix64_host(mix64_host(mix64_host(cfg->seed) ^ cfg->call_index) ^ (uint64_t)(e + cfg->epoch_offset));
    RSLX_HIP(launch_permutations(bases.data(), cfg->epochs, B, p.perms, p.perm_ws, s, mix64_host(cfg->seed),
                                 counters ? &counters->call_index : nullptr, cfg->epoch_offset));
  }
  const int nbm = mse_num_blocks((int64_t)p.mb * A);
  if (cfg->epochs > 0) {
    // once per call: the statistics rows start at zero (each step then writes its loss and gradient norm), and the
    // transposed weights are formed; every Adam launch below keeps them current
    RSLX_HIP(launch_fill(stats, (int64_t)cfg->epochs * cfg->minibatches * RSLX_NSTATS, 0.f, s));
    const XView none;
    BwdJob tj{student, none, p.mb, &p.student.act, p.student.d_out, p.student.wt, p.student.partials, &p.student.plan};
    RSLX_TRY(transpose_weights(&tj, 1, s, false));
  }
  for (int e = 0; e < cfg->epochs; ++e) {
    for (int m = 0; m < cfg->minibatches; ++m) {
      const int32_t* idx = p.perms + (size_t)e * B + (size_t)m * p.mb;
      float* stats_row = stats + ((size_t)e * cfg->minibatches + m) * RSLX_NSTATS;
      XView xs; xs.base = obs_student; xs.ld = student->dims[0]; xs.row_idx = idx; xs.src_rows = B;
      NetJob fj{student, xs, p.mb, &p.student.act};
      RSLX_TRY(forward_nets(&fj, 1, s));
      RSLX_HIP(launch_mse(p.student.act.out[Ls - 1], targets, idx, p.mb, A, p.student.d_out, p.mse_partials, s));
      RSLX_HIP(launch_mse_finish(p.mse_partials, nbm, (int64_t)p.mb * A, stats_row, s));
      BwdJob bj{student, xs, p.mb, &p.student.act, p.student.d_out, p.student.wt, p.student.partials, &p.student.plan};
      RSLX_TRY(backward_nets(&bj, 1, s, false, true));
      RSLX_TRY(reduce_net(*student, p.student, s));
      const int64_t t = *adam_step + 1;
      AdamArgs aa;
      memset(&aa, 0, sizeof aa);
      aa.seg[0] = AdamSegment{student->params, student->grads, student->adam_m, student->adam_v, weight_count(*student)};
      adam_keeps_transposed(aa.seg[0], *student, p.student.wt);
      aa.n_seg = 1;
      aa.sumsq_blocks = p.student.sumsq; aa.n_sumsq = p.student.n_sumsq;
      aa.max_grad_norm = cfg->max_grad_norm;
      aa.lr = cfg->lr; aa.beta1 = cfg->beta1; aa.beta2 = cfg->beta2; aa.eps = cfg->adam_eps;
      aa.bc1 = bias_correction(cfg->beta1, t); aa.bc2 = bias_correction(cfg->beta2, t);
      if (counters) { aa.step_dev = &counters->adam_step; aa.step_off = (int32_t)t; }
      aa.grad_norm_out = stats_row + RSLX_STAT_GRAD_NORM;
      RSLX_HIP(launch_adam(aa, s));
      *adam_step = t;
    }
  }
  if (counters) RSLX_HIP(advance_counters(counters, 0, 1, host_step, 0, s));
  return RSLX_OK;
}
}  // namespace

extern "C" {

int32_t rslx_bc_update(rslx_mlp* student, const rslx_mlp* teacher, const float* obs_student, const float* obs_teacher,
                       const float* targets_or_null, int32_t B, const rslx_bc_cfg* cfg, int64_t* adam_step, float* stats,
                       void* ws, size_t ws_bytes, void* stream) {
  if (!adam_step) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update: null pointer");
  return bc_update_impl(student, teacher, obs_student, obs_teacher, targets_or_null, B, cfg, adam_step, nullptr, stats, ws,
                        ws_bytes, stream);
}

int32_t rslx_bc_update_dc(rslx_mlp* student, const rslx_mlp* teacher, const float* obs_student, const float* obs_teacher,
                          const float* targets_or_null, int32_t B, const rslx_bc_cfg* cfg, rslx_dev_counters* counters,
                          float* stats, void* ws, size_t ws_bytes, void* stream) {
  if (!counters) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_update_dc: null counters");
  return bc_update_impl(student, teacher, obs_student, obs_teacher, targets_or_null, B, cfg, nullptr, counters, stats, ws,
                        ws_bytes, stream);
}

// ---- one collection step of the distillation loop ---------------------------------------------------------------------
size_t rslx_bc_collect_workspace_bytes(const rslx_mlp* student, const rslx_mlp* teacher, int32_t N) {
  if (!depth_ok(student) || !depth_ok(teacher)) return 0;
  if (N <= 0 || !student || !teacher) return 256;
  Carver c(nullptr);
  return act_carve(c, student, teacher, N, nullptr, nullptr);
}

int32_t rslx_bc_collect(const rslx_mlp* student, const rslx_mlp* teacher, const float* obs_student, const float* obs_teacher,
                        int32_t N, float* actions, float* targets, void* ws, size_t ws_bytes, void* stream) {
  if (N < 0) return fail(RSLX_ERR_SHAPE, "rslx_bc_collect: N = %d", N);
  RSLX_TRY(check_mlp(student, "rslx_bc_collect student", false));
  RSLX_TRY(check_mlp(teacher, "rslx_bc_collect teacher", false));
  if (student->dims[student->n_layers] != teacher->dims[teacher->n_layers])
    return fail(RSLX_ERR_SHAPE, "rslx_bc_collect: student and teacher action widths differ");
  if (!obs_student || !obs_teacher || !actions || !targets) return fail(RSLX_ERR_INVALID_ARG, "rslx_bc_collect: null pointer");
  if (N == 0) return RSLX_OK;
  if (!ws || ws_bytes < rslx_bc_collect_workspace_bytes(student, teacher, N))
    return fail(RSLX_ERR_WORKSPACE, "rslx_bc_collect: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  {
    FusedForwardArgs fa;
    memset(&fa, 0, sizeof fa);
    fa.n_rows = N;
    fa.n_nets = 2;
    fa.max_dim = max_dim_of(*student) > max_dim_of(*teacher) ? max_dim_of(*student) : max_dim_of(*teacher);
    fa.net[0] = fused_net(*student, obs_student, student->dims[0], nullptr, actions, false);
    fa.net[1] = fused_net(*teacher, obs_teacher, teacher->dims[0], nullptr, targets, false);
    if (fused_forward_pays(fa)) {
      RSLX_HIP(launch_fused_forward(fa, s));
      return RSLX_OK;
    }
  }
  Carver c(ws);
  NetBufs bs, bt;
  act_carve(c, student, teacher, N, &bs, &bt);
  bs.out[student->n_layers - 1] = actions;
  bt.out[teacher->n_layers - 1] = targets;
  XView xs; xs.base = obs_student; xs.ld = student->dims[0];
  XView xt; xt.base = obs_teacher; xt.ld = teacher->dims[0];
  NetJob jobs[2] = {NetJob{student, xs, N, &bs}, NetJob{teacher, xt, N, &bt}};
  RSLX_TRY(forward_nets(jobs, 2, s));
  return RSLX_OK;
}


// ---- symmetry augmentation ---------------------------------------------------------------------------------------------
int32_t rslx_sym_augment(const rslx_sym* sym, const float* obs_in, const float* act_in, int32_t B, int32_t D, int32_t A,
                         float* obs_out, float* act_out, void* stream) {
  if (!sym) return fail(RSLX_ERR_INVALID_ARG, "rslx_sym_augment: null sym");
  if (B < 0 || D < 0 || A < 0) return fail(RSLX_ERR_SHAPE, "rslx_sym_augment: negative size");
  hipStream_t s = (hipStream_t)stream;
  if (obs_in) {
    if (!involution_ok(sym->perm_obs_a_host, sym->sign_obs_a_host, D))
      return fail(RSLX_ERR_INVALID_ARG, "rslx_sym_augment: observation map is not an involutive signed permutation");
    if (!obs_out || !sym->perm_obs_a || !sym->sign_obs_a) return fail(RSLX_ERR_INVALID_ARG, "rslx_sym_augment: null pointer");
  }
  if (act_in) {
    if (!involution_ok(sym->perm_act_host, sym->sign_act_host, A))
      return fail(RSLX_ERR_INVALID_ARG, "rslx_sym_augment: action map is not an involutive signed permutation");
    if (!act_out || !sym->perm_act || !sym->sign_act) return fail(RSLX_ERR_INVALID_ARG, "rslx_sym_augment: null pointer");
  }
  if (obs_in) RSLX_HIP(launch_sym_augment(obs_in, B, D, sym->perm_obs_a, sym->sign_obs_a, obs_out, s));
  if (act_in) RSLX_HIP(launch_sym_augment(act_in, B, A, sym->perm_act, sym->sign_act, act_out, s));
  return RSLX_OK;
}

// ---- RND reward -----------------------------------------------------------------------------------------------------
static size_t rnd_carve(Carver& c, const rslx_mlp* net, int32_t N, NetBufs* bp, NetBufs* bt, double** partials) {
  NetBufs p, t;
  carve_net(c, *net, N, false, p);
  carve_net(c, *net, N, false, t);
  double* pp = c.take<double>((size_t)rnd_num_blocks(N) * 2 + 2);
  if (bp) *bp = p;
  if (bt) *bt = t;
  if (partials) *partials = pp;
  return c.off + 256;
}

size_t rslx_rnd_workspace_bytes(const rslx_mlp* target, int32_t N) {
  if (!target || N <= 0 || target->n_layers < 1 || target->n_layers > RSLX_MAX_LAYERS) return 256;
  Carver c(nullptr);
  return rnd_carve(c, target, N, nullptr, nullptr, nullptr);
}

int32_t rslx_rnd(const rslx_mlp* target, const rslx_mlp* predictor, const float* obs, int32_t N, int32_t D,
                 const int32_t* subset_idx_or_null, int32_t n_subset, float* running, float weight, int32_t update_stats,
                 float* r_int_out, float* rewards_inout_or_null, void* ws, size_t ws_bytes, void* stream) {
  RSLX_TRY(check_mlp(target, "rslx_rnd target", false));
  RSLX_TRY(check_mlp(predictor, "rslx_rnd predictor", false));
  if (target->n_layers != predictor->n_layers) return fail(RSLX_ERR_SHAPE, "rslx_rnd: networks differ in depth");
  for (int i = 0; i <= target->n_layers; ++i)
    if (target->dims[i] != predictor->dims[i]) return fail(RSLX_ERR_SHAPE, "rslx_rnd: networks differ in shape");
  if (N < 0 || D < 1) return fail(RSLX_ERR_SHAPE, "rslx_rnd: N = %d, D = %d", N, D);
  if (n_subset != target->dims[0] || (!subset_idx_or_null && n_subset != D)) return fail(RSLX_ERR_SHAPE, "rslx_rnd: subset width");
  if (!obs || !running || !r_int_out) return fail(RSLX_ERR_INVALID_ARG, "rslx_rnd: null pointer");
  if (N == 0) return RSLX_OK;
  if (!ws || ws_bytes < rslx_rnd_workspace_bytes(target, N)) return fail(RSLX_ERR_WORKSPACE, "rslx_rnd: workspace too small");
  hipStream_t s = (hipStream_t)stream;
  Carver c(ws);
  NetBufs bp, bt;
  double* partials = nullptr;
  rnd_carve(c, target, N, &bp, &bt, &partials);
  XView x;
  x.base = obs; x.ld = D;
  if (subset_idx_or_null) { x.col_map = subset_idx_or_null; x.map_from = 0; }
  const int L = target->n_layers;
  FusedForwardArgs fa;
  memset(&fa, 0, sizeof fa);
  fa.n_rows = N; fa.n_nets = 2; fa.max_dim = max_dim_of(*target);
  fa.net[0] = fused_net(*predictor, obs, D, subset_idx_or_null, bp.out[L - 1], false);
  fa.net[1] = fused_net(*target, obs, D, subset_idx_or_null, bt.out[L - 1], false);
  if (fused_forward_pays(fa)) {
    RSLX_HIP(launch_fused_forward(fa, s));
  } else {
    NetJob jobs[2] = {NetJob{predictor, x, N, &bp}, NetJob{target, x, N, &bt}};
    RSLX_TRY(forward_nets(jobs, 2, s));
  }
  RSLX_HIP(launch_rnd_reward(bp.out[L - 1], bt.out[L - 1], N, target->dims[L], running, weight, update_stats ? 1 : 0,
                             r_int_out, rewards_inout_or_null, partials, s));
  return RSLX_OK;
}

}  // extern "C"
