// C ABI entry points: argument validation on the host, then the launchers.
#include <mutex>
#include <vector>

#include "common.h"

namespace marl {

namespace {
struct TimerState {
  bool on = false;
  std::vector<hipEvent_t> pool;       // reused across reads
  size_t used = 0;
  struct Pair { int cls; size_t begin, end; double work; };
  std::vector<Pair> pairs;
  hipEvent_t get() {
    if (used == pool.size()) {
      hipEvent_t e;
      (void)hipEventCreate(&e);
      pool.push_back(e);
    }
    return pool[used++];
  }
};
TimerState g_timer;
}  // namespace

bool timing_on() { return g_timer.on; }

// ---- scratch of the entry point that allocates nothing ------------------------------------------------------------
// Device memory that is part of the loaded code object: every GPU the library runs on holds its own copy, at its own
// address, until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the
// kernels are given the address that call returns.
constexpr int64_t kStaticScratchBytes = MARL_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // per device, filled on the first call made with that device current

// Address of the current device's copy of `scratch` (nullptr on error).
void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

// ---- a second stream per device -----------------------------------------------------------------------------------
namespace {
struct SideState {
  bool tried = false;
  SideStream st{};
  bool ok = false;
};
std::mutex g_side_mutex;
SideState g_side[kMaxDevices];
}  // namespace

const SideStream* side_stream() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_side_mutex);
  SideState& g = g_side[dev];
  if (!g.tried) {
    g.tried = true;
    g.ok = hipStreamCreateWithFlags(&g.st.stream, hipStreamNonBlocking) == hipSuccess &&
           hipEventCreateWithFlags(&g.st.fork, hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&g.st.join, hipEventDisableTiming) == hipSuccess;
  }
  return g.ok ? &g.st : nullptr;
}

TimedLaunch::TimedLaunch(int c, double work, hipStream_t st) : cls(c), s(st), active(g_timer.on) {
  if (!active) return;
  const size_t b = g_timer.used;
  (void)hipEventRecord(g_timer.get(), s);
  g_timer.pairs.push_back({cls, b, 0, work});
}
TimedLaunch::~TimedLaunch() {
  if (!active) return;
  g_timer.pairs.back().end = g_timer.used;
  (void)hipEventRecord(g_timer.get(), s);
}

int32_t validate_config(const marl_config* c) {
  if (c == nullptr) return MARL_E_NULL;
  if (c->grid < 2 || c->grid > 64) return MARL_E_CONFIG;
  if (c->n_agents < 1 || c->n_agents > kMaxAgents) return MARL_E_CONFIG;
  if (c->n_food < 1 || c->n_food > kMaxFood) return MARL_E_CONFIG;
  if (c->n_agents + c->n_food > c->grid * c->grid) return MARL_E_CONFIG;
  if (c->max_level < 1 || c->max_level > 15) return MARL_E_CONFIG;
  if (c->episode_cap < 1) return MARL_E_CONFIG;
  if (c->view != 3 && c->view != 5 && c->view != 7) return MARL_E_CONFIG;
  if (c->n_envs < 1 || c->rollout_len < 1) return MARL_E_CONFIG;
  if (c->n_epochs < 1 || c->n_minibatches < 1) return MARL_E_CONFIG;  // before any use as a divisor
  for (int h : {c->actor_hidden, c->critic_hidden})
    if (h < 32 || h > 512 || h % 32 != 0) return MARL_E_CONFIG;
  if (c->central_critic != 0 && c->central_critic != 1) return MARL_E_CONFIG;
  if (c->precision != 0 && c->precision != 1) return MARL_E_CONFIG;
  if (c->env_kind < 0 || c->env_kind > 2) return MARL_E_CONFIG;
  if (c->env_kind != 0 && c->max_level > c->n_food) return MARL_E_CONFIG;  // requested shelves
  if (c->recurrent != 0 && c->recurrent != 1) return MARL_E_CONFIG;
  if (c->recurrent == 1 && (c->precision != 0 || c->n_envs % c->n_minibatches != 0)) return MARL_E_CONFIG;
  if (c->precision == 1 && (c->actor_hidden % 64 != 0 || c->critic_hidden % 64 != 0)) return MARL_E_CONFIG;  // bf16 k tile
  const int64_t R = (int64_t)c->n_envs * c->rollout_len;
  if (R % c->n_minibatches != 0) return MARL_E_CONFIG;
  if (R * c->n_agents >= ((int64_t)1 << 31)) return MARL_E_CONFIG;  // sample and row indices are 32-bit
  if (!(c->gamma >= 0.f && c->gamma <= 1.f) || !(c->lambda >= 0.f && c->lambda <= 1.f)) return MARL_E_CONFIG;
  if (!(c->clip_eps > 0.f) || !(c->lr > 0.f) || !(c->adam_eps > 0.f)) return MARL_E_CONFIG;
  if (!(c->beta1 >= 0.f && c->beta1 < 1.f) || !(c->beta2 >= 0.f && c->beta2 < 1.f)) return MARL_E_CONFIG;
  if (!(c->ent_coef >= 0.f) || !(c->vf_coef >= 0.f)) return MARL_E_CONFIG;
  if (c->normalize_adv != 0 && c->normalize_adv != 1) return MARL_E_CONFIG;
  if (c->clip_value != 0 && c->clip_value != 1) return MARL_E_CONFIG;
  return MARL_OK;
}

static int32_t check_state(const marl_env_state& st) {
  MARL_REQUIRE_PTR(st.agent_row); MARL_REQUIRE_PTR(st.agent_col); MARL_REQUIRE_PTR(st.agent_lvl);
  MARL_REQUIRE_PTR(st.food_row); MARL_REQUIRE_PTR(st.food_col); MARL_REQUIRE_PTR(st.food_lvl);
  MARL_REQUIRE_PTR(st.t_in_ep); MARL_REQUIRE_PTR(st.episode_id);
  return MARL_OK;
}

static int32_t check_traj(const marl_traj& t, bool need_gae_outputs) {
  MARL_REQUIRE_PTR(t.obs); MARL_REQUIRE_PTR(t.action); MARL_REQUIRE_PTR(t.logp); MARL_REQUIRE_PTR(t.value);
  MARL_REQUIRE_PTR(t.reward); MARL_REQUIRE_PTR(t.done); MARL_REQUIRE_PTR(t.last_value);
  if (need_gae_outputs) {
    MARL_REQUIRE_PTR(t.adv);
    MARL_REQUIRE_PTR(t.ret);
  }
  MARL_OPTIONAL_PTR(t.logits);
  MARL_OPTIONAL_PTR(t.sampled);
  return MARL_OK;
}

}  // namespace marl

using namespace marl;

extern "C" {

int32_t marl_query_sizes(const marl_config* cfg, marl_sizes* out) {
  if (cfg == nullptr || out == nullptr) return MARL_E_NULL;
  const int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  const Dims d = dims_of(*cfg);
  out->obs_dim = d.D;
  out->critic_in_dim = d.Dc;
  out->n_params = d.P;
  out->n_actor_params = d.Pa;
  out->state_entity_bytes_agents = (int64_t)d.A * d.N;
  out->state_entity_bytes_food = (int64_t)d.F * d.N;
  out->state_t_bytes = 4 * (int64_t)d.N;
  out->state_episode_bytes = 4 * (int64_t)d.N;
  out->obs_bytes = 4 * (int64_t)(d.T + 1) * d.NA * d.D;
  out->step_scalar_bytes = 4 * (int64_t)d.T * d.NA;
  out->done_bytes = (int64_t)d.T * d.N;
  out->last_value_bytes = 4 * d.NA;
  out->logits_bytes = 4 * (int64_t)d.T * d.NA * kActions;
  out->hidden_actor_bytes = out->hidden_critic_bytes = 0;
  if (d.recurrent) {
    out->rollout_workspace_bytes = rec_rollout_workspace_bytes(*cfg);
    out->update_workspace_bytes = rec_update_workspace_bytes(*cfg);
    out->eval_workspace_bytes = 0;
    out->hidden_actor_bytes = 4 * d.NA * d.Ha;
    out->hidden_critic_bytes = 4 * (d.central ? (int64_t)d.N : d.NA) * d.Hc;
    return MARL_OK;
  }
  out->rollout_workspace_bytes = rollout_workspace_bytes(*cfg, d.N);
  out->update_workspace_bytes = update_workspace_bytes(*cfg);
  out->eval_workspace_bytes = eval_workspace_bytes(*cfg);
  return MARL_OK;
}

int32_t marl_env_reset(const marl_config* cfg, marl_env_state st, void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  if ((rc = check_state(st)) != MARL_OK) return rc;
  return launch_env_reset(*cfg, st, (hipStream_t)stream);
}

int32_t marl_observe(const marl_config* cfg, marl_env_state st, float* obs, void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  if ((rc = check_state(st)) != MARL_OK) return rc;
  MARL_REQUIRE_PTR(obs);
  return launch_env_step(*cfg, st, nullptr, obs, nullptr, nullptr, false, (hipStream_t)stream);
}

int32_t marl_env_step(const marl_config* cfg, marl_env_state st, const int32_t* actions, float* obs, float* reward,
                      uint8_t* done, void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  if ((rc = check_state(st)) != MARL_OK) return rc;
  MARL_REQUIRE_PTR(actions); MARL_REQUIRE_PTR(reward); MARL_REQUIRE_PTR(done);
  MARL_OPTIONAL_PTR(obs);
  return launch_env_step(*cfg, st, actions, obs, reward, done, true, (hipStream_t)stream);
}

int32_t marl_policy_forward(const marl_config* cfg, const float* params, const float* obs, int64_t n_rows,
                            float* logits, float* value, void* workspace, void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  if (cfg->recurrent) return MARL_E_CONFIG;  // the recurrent networks have entry points of their own
  MARL_REQUIRE_PTR(params); MARL_REQUIRE_PTR(obs); MARL_REQUIRE_PTR(workspace);
  MARL_OPTIONAL_PTR(logits); MARL_OPTIONAL_PTR(value);
  if (n_rows < 0 || n_rows * cfg->n_agents >= ((int64_t)1 << 31)) return MARL_E_SIZE;
  if (n_rows == 0 || (logits == nullptr && value == nullptr)) return MARL_OK;
  return launch_policy_forward(*cfg, params, obs, n_rows, logits, value, workspace, (hipStream_t)stream);
}

int32_t marl_sample_actions(const marl_config* cfg, const float* logits, const float* uniforms, const int32_t* forced,
                            int64_t n, uint64_t step, int32_t* action, int32_t* sampled, float* logp, void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  MARL_REQUIRE_PTR(logits); MARL_REQUIRE_PTR(action); MARL_REQUIRE_PTR(logp);
  MARL_OPTIONAL_PTR(uniforms); MARL_OPTIONAL_PTR(forced); MARL_OPTIONAL_PTR(sampled);
  if (n < 0 || n >= ((int64_t)1 << 31)) return MARL_E_SIZE;
  if (n == 0) return MARL_OK;
  return launch_sample(*cfg, logits, uniforms, forced, n, step, action, sampled, logp, (hipStream_t)stream);
}

int32_t marl_rollout(const marl_config* cfg, marl_env_state st, const float* params, marl_traj traj,
                     uint64_t step_offset, const int32_t* forced_actions, const float* forced_uniforms,
                     void* workspace, void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  if (cfg->recurrent) return MARL_E_CONFIG;  // the recurrent networks have entry points of their own
  if ((rc = check_state(st)) != MARL_OK) return rc;
  if ((rc = check_traj(traj, false)) != MARL_OK) return rc;
  MARL_REQUIRE_PTR(params); MARL_REQUIRE_PTR(workspace);
  MARL_OPTIONAL_PTR(forced_actions); MARL_OPTIONAL_PTR(forced_uniforms);
  return launch_rollout(*cfg, st, params, traj, step_offset, forced_actions, forced_uniforms, workspace,
                        (hipStream_t)stream);
}

int32_t marl_rollout_static(const marl_config* cfg, marl_env_state st, const float* params, marl_traj traj,
                            uint64_t step_offset, const int32_t* forced_actions, const float* forced_uniforms,
                            void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  if (cfg->recurrent) return MARL_E_CONFIG;
  if ((rc = check_state(st)) != MARL_OK) return rc;
  if ((rc = check_traj(traj, false)) != MARL_OK) return rc;
  MARL_REQUIRE_PTR(params);
  MARL_OPTIONAL_PTR(forced_actions); MARL_OPTIONAL_PTR(forced_uniforms);
  if (rollout_workspace_bytes(*cfg, cfg->n_envs) > kStaticScratchBytes) return MARL_E_SIZE;
  void* ws = static_scratch();
  if (ws == nullptr) return MARL_E_LAUNCH;
  return launch_rollout(*cfg, st, params, traj, step_offset, forced_actions, forced_uniforms, ws, (hipStream_t)stream);
}

int32_t marl_compute_gae(const marl_config* cfg, marl_traj traj, void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  if ((rc = check_traj(traj, true)) != MARL_OK) return rc;
  return launch_gae(*cfg, traj, (hipStream_t)stream);
}

int32_t marl_evaluate(const marl_config* cfg, marl_env_state st, const float* params, int32_t n_episodes,
                      marl_eval_stats out, void* workspace, void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  if (cfg->recurrent) return MARL_E_CONFIG;  // the recurrent networks have entry points of their own
  if ((rc = check_state(st)) != MARL_OK) return rc;
  MARL_REQUIRE_PTR(params); MARL_REQUIRE_PTR(workspace);
  MARL_REQUIRE_PTR(out.ret_sum); MARL_REQUIRE_PTR(out.len_sum); MARL_REQUIRE_PTR(out.episodes);
  if (n_episodes < 1 || (int64_t)n_episodes * cfg->episode_cap > ((int64_t)1 << 20)) return MARL_E_SIZE;
  return launch_evaluate(*cfg, st, params, n_episodes, out, workspace, (hipStream_t)stream);
}

int32_t marl_ppo_update(const marl_config* cfg, marl_traj traj, float* params, float* adam_m, float* adam_v,
                        int64_t adam_step0, const int32_t* perm, float* stats, float* grad_dump, void* workspace,
                        void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  if (cfg->recurrent) return MARL_E_CONFIG;  // the recurrent networks have entry points of their own
  if ((rc = check_traj(traj, true)) != MARL_OK) return rc;
  MARL_REQUIRE_PTR(params); MARL_REQUIRE_PTR(adam_m); MARL_REQUIRE_PTR(adam_v); MARL_REQUIRE_PTR(stats);
  MARL_REQUIRE_PTR(workspace);
  MARL_OPTIONAL_PTR(perm); MARL_OPTIONAL_PTR(grad_dump);
  if (adam_step0 < 0) return MARL_E_SIZE;
  return launch_ppo_update(*cfg, traj, params, adam_m, adam_v, adam_step0, perm, stats, grad_dump, workspace,
                           (hipStream_t)stream);
}

int32_t marl_train_step(const marl_config* cfg, marl_env_state st, float* params, marl_traj traj, float* adam_m,
                        float* adam_v, marl_counters* counters, const int32_t* perm, float* stats,
                        void* rollout_workspace, void* update_workspace, void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  if (cfg->recurrent) return MARL_E_CONFIG;
  if ((rc = check_state(st)) != MARL_OK) return rc;
  if ((rc = check_traj(traj, true)) != MARL_OK) return rc;
  MARL_REQUIRE_PTR(params); MARL_REQUIRE_PTR(adam_m); MARL_REQUIRE_PTR(adam_v); MARL_REQUIRE_PTR(stats);
  MARL_REQUIRE_PTR(counters); MARL_REQUIRE_PTR(rollout_workspace); MARL_REQUIRE_PTR(update_workspace);
  MARL_OPTIONAL_PTR(perm);
  hipStream_t s = (hipStream_t)stream;
  if ((rc = launch_rollout(*cfg, st, params, traj, 0, nullptr, nullptr, rollout_workspace, s, &counters->step)) != MARL_OK)
    return rc;
  if ((rc = launch_gae(*cfg, traj, s)) != MARL_OK) return rc;
  if ((rc = launch_ppo_update(*cfg, traj, params, adam_m, adam_v, 0, perm, stats, nullptr, update_workspace, s,
                              &counters->adam_step)) != MARL_OK)
    return rc;
  return launch_advance_counters(counters, (uint64_t)cfg->rollout_len, (int64_t)cfg->n_epochs * cfg->n_minibatches, s);
}

static int32_t check_rec(const marl_rec_state& r) {
  MARL_REQUIRE_PTR(r.ha0); MARL_REQUIRE_PTR(r.hc0); MARL_REQUIRE_PTR(r.ha1); MARL_REQUIRE_PTR(r.hc1);
  return MARL_OK;
}

int32_t marl_rollout_recurrent(const marl_config* cfg, marl_env_state st, const float* params, marl_traj traj,
                               marl_rec_state rec, uint64_t step_offset, const int32_t* forced_actions,
                               const float* forced_uniforms, void* workspace, void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  if (!cfg->recurrent) return MARL_E_CONFIG;
  if ((rc = check_state(st)) != MARL_OK) return rc;
  if ((rc = check_traj(traj, false)) != MARL_OK) return rc;
  if ((rc = check_rec(rec)) != MARL_OK) return rc;
  MARL_REQUIRE_PTR(params); MARL_REQUIRE_PTR(workspace);
  MARL_OPTIONAL_PTR(forced_actions); MARL_OPTIONAL_PTR(forced_uniforms);
  return launch_rollout_recurrent(*cfg, st, params, traj, rec, step_offset, forced_actions, forced_uniforms, workspace,
                                  (hipStream_t)stream);
}

int32_t marl_ppo_update_recurrent(const marl_config* cfg, marl_traj traj, marl_rec_state rec, float* params,
                                  float* adam_m, float* adam_v, int64_t adam_step0, const int32_t* perm, float* stats,
                                  float* grad_dump, void* workspace, void* stream) {
  int32_t rc = validate_config(cfg);
  if (rc != MARL_OK) return rc;
  if (!cfg->recurrent) return MARL_E_CONFIG;
  if ((rc = check_traj(traj, true)) != MARL_OK) return rc;
  if ((rc = check_rec(rec)) != MARL_OK) return rc;
  MARL_REQUIRE_PTR(params); MARL_REQUIRE_PTR(adam_m); MARL_REQUIRE_PTR(adam_v); MARL_REQUIRE_PTR(stats);
  MARL_REQUIRE_PTR(workspace);
  MARL_OPTIONAL_PTR(perm); MARL_OPTIONAL_PTR(grad_dump);
  if (adam_step0 < 0) return MARL_E_SIZE;
  return launch_ppo_update_recurrent(*cfg, traj, rec, params, adam_m, adam_v, adam_step0, perm, stats, grad_dump,
                                     workspace, (hipStream_t)stream);
}

int32_t marl_timing_enable(int32_t on) {
  g_timer.on = on != 0;
  g_timer.used = 0;
  g_timer.pairs.clear();
  return MARL_OK;
}

int32_t marl_timing_read(int32_t kernel_class, double* total_ms, int64_t* launches, double* work) {
  if (total_ms == nullptr || launches == nullptr || work == nullptr) return MARL_E_NULL;
  if (kernel_class < 0 || kernel_class >= KC_COUNT) return MARL_E_SIZE;
  double ms = 0, w = 0;
  int64_t n = 0;
  for (const auto& p : g_timer.pairs) {
    if (p.cls != kernel_class) continue;
    if (hipEventSynchronize(g_timer.pool[p.end]) != hipSuccess) return MARL_E_LAUNCH;
    float t = 0.f;
    if (hipEventElapsedTime(&t, g_timer.pool[p.begin], g_timer.pool[p.end]) != hipSuccess) return MARL_E_LAUNCH;
    ms += t;
    w += p.work;
    ++n;
  }
  *total_ms = ms;
  *launches = n;
  *work = w;
  return MARL_OK;
}

const char* marl_status_string(int32_t status) {
  switch (status) {
    case MARL_OK: return "ok";
    case MARL_E_NULL: return "a required pointer is null";
    case MARL_E_ALIGN: return "a device pointer is not 16-byte aligned";
    case MARL_E_CONFIG: return "unsupported or inconsistent configuration";
    case MARL_E_LAUNCH: return "the HIP runtime reported a launch error";
    case MARL_E_SIZE: return "a size argument is out of range, or the configuration needs more than the built-in scratch";
    default: return "unknown status";
  }
}

}  // extern "C"
