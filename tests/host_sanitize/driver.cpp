// Host-only exercise of the C ABI for a sanitizer build of the library (address + undefined behaviour on the
// host code): version / error plumbing, every workspace query, and the argument checks of every entry point
// that return before anything is launched.  Needs no GPU; pointers that stand for device memory are host arrays
// that no code path reached here dereferences.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/rslx.h"

static int failures = 0;
#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) { std::printf("FAILED %s:%d: %s  (last error: %s)\n", __FILE__, __LINE__, #cond, rslx_last_error()); ++failures; } \
  } while (0)

static rslx_mlp make_mlp(std::vector<float>& store, const std::vector<int>& dims, bool log_std, bool trainable) {
  rslx_mlp n;
  std::memset(&n, 0, sizeof n);
  n.n_layers = (int32_t)dims.size() - 1;
  size_t count = 0;
  for (size_t i = 0; i < dims.size(); ++i) n.dims[i] = dims[i];
  for (size_t i = 0; i + 1 < dims.size(); ++i) count += (size_t)dims[i] * dims[i + 1] + dims[i + 1];
  if (log_std) count += dims.back();
  store.assign(4 * count + 64, 0.f);
  float* base = store.data();
  while (reinterpret_cast<uintptr_t>(base) & 15) ++base;
  count = (count + 3) / 4 * 4;
  n.elu_alpha = 1.0f;
  n.has_log_std = log_std ? 1 : 0;
  n.params = base;
  if (trainable) { n.grads = base + count; n.adam_m = base + 2 * count; n.adam_v = base + 3 * count; }
  return n;
}

int main() {
  CHECK(rslx_version() == 100);
  CHECK(rslx_last_error() != nullptr);

  std::vector<float> sa, sc, sp, st;
  rslx_mlp actor = make_mlp(sa, {48, 128, 128, 12}, true, true);
  rslx_mlp critic = make_mlp(sc, {48, 128, 128, 1}, false, true);
  rslx_mlp pred = make_mlp(sp, {48, 64, 32}, false, true);
  rslx_mlp targ = make_mlp(st, {48, 64, 32}, false, false);

  // ---- workspace queries ----
  CHECK(rslx_permutation_workspace_bytes(0) > 0 && rslx_permutation_workspace_bytes(98304) > 98304);
  CHECK(rslx_gae_workspace_bytes(24, 4096) > 0 && rslx_gae_workspace_bytes(24, 0) > 0);
  CHECK(rslx_adam_workspace_bytes(380313) > 0 && rslx_adam_workspace_bytes(0) > 0);
  CHECK(rslx_act_workspace_bytes(&actor, &critic, 4096) > 0);
  CHECK(rslx_rnd_workspace_bytes(&targ, 4096) > 0);
  CHECK(rslx_bc_collect_workspace_bytes(&actor, &actor, 4096) > 0);

  std::vector<float> buf(1 << 16, 0.f);
  float* d = buf.data();
  while (reinterpret_cast<uintptr_t>(d) & 15) ++d;
  rslx_rollout ro;
  std::memset(&ro, 0, sizeof ro);
  ro.T = 24; ro.N = 64; ro.Da = 48; ro.Dc = 48; ro.A = 12;
  ro.obs_actor = ro.obs_critic = ro.actions = ro.logp = ro.values = ro.mu = ro.sigma = ro.advantages = ro.returns = d;
  rslx_ppo_cfg cfg;
  std::memset(&cfg, 0, sizeof cfg);
  cfg.clip = 0.2f; cfg.value_coef = 1.f; cfg.entropy_coef = 0.01f; cfg.max_grad_norm = 1.f; cfg.lr = 1e-3f;
  cfg.beta1 = 0.9f; cfg.beta2 = 0.999f; cfg.adam_eps = 1e-8f; cfg.epochs = 5; cfg.minibatches = 4; cfg.use_clipped_value_loss = 1;
  const size_t ws_ppo = rslx_ppo_update_workspace_bytes(&actor, &critic, &ro, &cfg, nullptr, nullptr);
  CHECK(ws_ppo > 0);
  rslx_rnd_train rt;
  std::memset(&rt, 0, sizeof rt);
  int64_t rnd_step = 0;
  rt.target = &targ; rt.predictor = &pred; rt.n_subset = 48; rt.lr = 1e-3f; rt.adam_step = &rnd_step;
  CHECK(rslx_ppo_update_workspace_bytes(&actor, &critic, &ro, &cfg, nullptr, &rt) > ws_ppo);

  // mirror maps: an involution is accepted, a non-involutive permutation is refused
  std::vector<int32_t> perm_o(48), perm_a(12), bad(48);
  std::vector<float> sign_o(48, 1.f), sign_a(12, 1.f);
  for (int i = 0; i < 48; ++i) { perm_o[i] = i ^ 1; bad[i] = (i + 1) % 48; }
  for (int i = 0; i < 12; ++i) perm_a[i] = 11 - i;
  rslx_sym sym;
  std::memset(&sym, 0, sizeof sym);
  sym.perm_obs_a_host = sym.perm_obs_c_host = perm_o.data(); sym.sign_obs_a_host = sym.sign_obs_c_host = sign_o.data();
  sym.perm_act_host = perm_a.data(); sym.sign_act_host = sign_a.data();
  sym.perm_obs_a = sym.perm_obs_c = perm_o.data(); sym.sign_obs_a = sym.sign_obs_c = sign_o.data();
  sym.perm_act = perm_a.data(); sym.sign_act = sign_a.data();
  sym.mirror_loss_coef = 1.f;
  CHECK(rslx_ppo_update_workspace_bytes(&actor, &critic, &ro, &cfg, &sym, nullptr) > ws_ppo);
  sym.perm_obs_a_host = bad.data();
  CHECK(rslx_ppo_update_workspace_bytes(&actor, &critic, &ro, &cfg, &sym, nullptr) == 0);
  CHECK(std::strstr(rslx_last_error(), "involutive") != nullptr);
  sym.perm_obs_a_host = perm_o.data();

  // ---- argument errors: nothing is launched ----
  int64_t step = 0;
  CHECK(rslx_gae(nullptr, nullptr, nullptr, nullptr, nullptr, 3, 4, 0.9f, 0.9f, 1, nullptr, nullptr, nullptr, 0, nullptr) == RSLX_ERR_INVALID_ARG);
  CHECK(rslx_gae(nullptr, nullptr, nullptr, nullptr, nullptr, -1, 4, 0.9f, 0.9f, 1, nullptr, nullptr, nullptr, 0, nullptr) == RSLX_ERR_SHAPE);
  CHECK(rslx_gae(nullptr, nullptr, nullptr, nullptr, nullptr, 0, 4, 0.9f, 0.9f, 1, nullptr, nullptr, nullptr, 0, nullptr) == RSLX_OK);
  CHECK(rslx_gae_noalloc(nullptr, nullptr, nullptr, nullptr, nullptr, 3, RSLX_GAE_NOALLOC_MAX_ENVS + 1, 0.9f, 0.9f, 1, nullptr, nullptr, nullptr) == RSLX_ERR_SHAPE);
  CHECK(rslx_gae_noalloc(nullptr, nullptr, nullptr, nullptr, nullptr, 3, 4, 0.9f, 0.9f, 1, nullptr, nullptr, nullptr) == RSLX_ERR_INVALID_ARG);
  CHECK(rslx_permutation(1, 2, -1, 16, nullptr, nullptr, 0, nullptr) == RSLX_ERR_SHAPE);
  CHECK(rslx_permutation(1, 2, 0, 16, nullptr, nullptr, 0, nullptr) == RSLX_ERR_INVALID_ARG);
  CHECK(rslx_adam_step(nullptr, nullptr, nullptr, nullptr, -5, 1e-3f, 0.9f, 0.999f, 1e-8f, 1.f, &step, nullptr, nullptr, 0, nullptr) == RSLX_ERR_SHAPE);
  CHECK(rslx_adam_step(nullptr, nullptr, nullptr, nullptr, 8, 1e-3f, 0.9f, 0.999f, 1e-8f, 1.f, nullptr, nullptr, nullptr, 0, nullptr) == RSLX_ERR_INVALID_ARG);
  CHECK(rslx_ppo_update(&actor, &critic, &ro, &cfg, nullptr, nullptr, &step, d, nullptr, 0, nullptr) == RSLX_ERR_WORKSPACE);
  CHECK(rslx_ppo_update(&actor, &critic, &ro, &cfg, nullptr, nullptr, nullptr, d, d, 1 << 16, nullptr) == RSLX_ERR_INVALID_ARG);
  cfg.minibatches = 7;      // 24 * 64 is no multiple of 7
  CHECK(rslx_ppo_update(&actor, &critic, &ro, &cfg, nullptr, nullptr, &step, d, d, 1 << 16, nullptr) == RSLX_ERR_SHAPE);
  cfg.minibatches = 4;
  rslx_mlp wrong = critic;
  wrong.dims[wrong.n_layers] = 2;
  CHECK(rslx_ppo_update(&actor, &wrong, &ro, &cfg, nullptr, nullptr, &step, d, d, 1 << 16, nullptr) == RSLX_ERR_SHAPE);
  rslx_mlp deep = actor;
  deep.n_layers = RSLX_MAX_LAYERS + 1;
  CHECK(rslx_act_workspace_bytes(&deep, &critic, 64) == 0);
  CHECK(rslx_bc_collect_workspace_bytes(&deep, &actor, 64) == 0);
  CHECK(rslx_rnd_workspace_bytes(&deep, 64) == 256);
  rslx_bc_cfg bc;
  std::memset(&bc, 0, sizeof bc);
  bc.lr = 1e-3f; bc.beta1 = 0.9f; bc.beta2 = 0.999f; bc.adam_eps = 1e-8f; bc.epochs = 2; bc.minibatches = 4;
  CHECK(rslx_bc_update_workspace_bytes(&actor, &actor, 1536, &bc) > 0);
  CHECK(rslx_bc_update_workspace_bytes(&actor, &actor, 1537, &bc) == 0);
  CHECK(rslx_bc_update(&actor, nullptr, d, nullptr, nullptr, 1536, &bc, &step, d, d, 1 << 16, nullptr) == RSLX_ERR_INVALID_ARG);
  CHECK(rslx_sym_augment(&sym, d, d, -1, 48, 12, d, d, nullptr) != RSLX_OK);
  sym.perm_act_host = bad.data();      // wrong length / not an involution of 12 entries
  CHECK(rslx_sym_augment(&sym, d, d, 16, 48, 12, d, d, nullptr) == RSLX_ERR_INVALID_ARG);
  int32_t n_rec = -1;
  CHECK(rslx_trace_begin(0) == RSLX_ERR_INVALID_ARG);
  CHECK(rslx_trace_begin(4) == RSLX_OK);
  CHECK(rslx_trace_end(nullptr, 0, &n_rec) == RSLX_OK && n_rec == 0);
  CHECK(rslx_trace_end(nullptr, 0, nullptr) == RSLX_ERR_INVALID_ARG);

  // ---- recurrent entry points ----
  {
    std::vector<float> sm(4 * 3 * 64 * (48 + 64 + 2) + 64, 0.f), s1, s2;
    float* mb = sm.data();
    while (reinterpret_cast<uintptr_t>(mb) & 15) ++mb;
    const size_t cnt = (size_t)3 * 64 * (48 + 64 + 2);
    rslx_memory gru;
    std::memset(&gru, 0, sizeof gru);
    gru.cell = RSLX_CELL_GRU; gru.in_dim = 48; gru.hidden = 64;
    gru.params = mb; gru.grads = mb + cnt; gru.adam_m = mb + 2 * cnt; gru.adam_v = mb + 3 * cnt;
    rslx_mlp ra = make_mlp(s1, {64, 128, 12}, true, true), rc = make_mlp(s2, {64, 128, 1}, false, true);
    CHECK(rslx_memory_step_workspace_bytes(&gru, 64) > 0);
    CHECK(rslx_act_recurrent_workspace_bytes(&gru, &ra, &gru, &rc, 64) > 0);
    CHECK(rslx_ppo_update_recurrent_workspace_bytes(&gru, &ra, &gru, &rc, &ro, &cfg) > 0);
    rslx_memory lstm = gru;
    lstm.cell = RSLX_CELL_LSTM;
    CHECK(rslx_ppo_update_recurrent_workspace_bytes(&gru, &ra, &lstm, &rc, &ro, &cfg) == 0);
    CHECK(std::strstr(rslx_last_error(), "different cells") != nullptr);
    rslx_memory odd = gru;
    odd.cell = 7;
    CHECK(rslx_ppo_update_recurrent_workspace_bytes(&odd, &ra, &odd, &rc, &ro, &cfg) == 0);
    cfg.minibatches = 5;      // 64 environments are no multiple of 5
    CHECK(rslx_ppo_update_recurrent_workspace_bytes(&gru, &ra, &gru, &rc, &ro, &cfg) == 0);
    cfg.minibatches = 4;
    CHECK(rslx_bc_update_recurrent_workspace_bytes(&gru, &ra, 24, 64, &bc) > 0);
    rslx_mlp mism = make_mlp(s1, {48, 128, 12}, true, true);      // MLP input is not the memory's width
    CHECK(rslx_bc_update_recurrent_workspace_bytes(&gru, &mism, 24, 64, &bc) == 0);
    CHECK(rslx_ppo_update_recurrent(&gru, &ra, &gru, &rc, &ro, nullptr, d, d, &cfg, &step, d, d, 1 << 16, nullptr) == RSLX_ERR_INVALID_ARG);
    CHECK(rslx_memory_step(&gru, d, -3, d, nullptr, nullptr, nullptr, d, 1 << 16, nullptr) != RSLX_OK);
  }

  std::printf(failures ? "host driver: %d check(s) failed\n" : "host driver: all checks passed\n", failures);
  return failures ? 1 : 0;
}
