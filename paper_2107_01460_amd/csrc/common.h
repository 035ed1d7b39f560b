// Internal declarations shared by the translation units of libmarl_gfx950.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "marl.h"

namespace marl {

constexpr int kActions = MARL_N_ACTIONS;
constexpr int kMaxAgents = 8;
constexpr int kMaxFood = 8;

// Sizes derived from a validated configuration.
struct Dims {
  int G, A, F, V, D, N, T;
  int Ha, Hc, Dc;
  int64_t Pa, Pc, P;   // parameter counts: actor, critic, total
  int64_t NA;          // N * A
  bool central, bf16, recurrent;
};

inline Dims dims_of(const marl_config& c) {
  Dims d;
  d.G = c.grid; d.A = c.n_agents; d.F = c.n_food; d.V = c.view; d.D = 3 * c.view * c.view;
  d.N = c.n_envs; d.T = c.rollout_len; d.Ha = c.actor_hidden; d.Hc = c.critic_hidden;
  d.central = c.central_critic != 0;
  d.bf16 = c.precision == 1;
  d.Dc = d.central ? d.A * d.D : d.D;
  d.Pa = (int64_t)d.D * d.Ha + d.Ha + (int64_t)d.Ha * d.Ha + d.Ha + (int64_t)d.Ha * kActions + kActions;
  d.Pc = (int64_t)d.Dc * d.Hc + d.Hc + (int64_t)d.Hc * d.Hc + d.Hc + d.Hc + 1;
  d.recurrent = c.recurrent != 0;
  if (d.recurrent) {  // embedding, GRU cell (input and hidden weights of three gates), output layer
    d.Pa = (int64_t)d.D * d.Ha + d.Ha + 2 * ((int64_t)d.Ha * 3 * d.Ha + 3 * d.Ha) + (int64_t)d.Ha * kActions + kActions;
    d.Pc = (int64_t)d.Dc * d.Hc + d.Hc + 2 * ((int64_t)d.Hc * 3 * d.Hc + 3 * d.Hc) + d.Hc + 1;
  }
  d.P = d.Pa + d.Pc;
  d.NA = (int64_t)d.N * d.A;
  return d;
}

// Offsets (in floats) of one network's blocks inside the flat parameter vector.
struct NetOffsets {
  int64_t W1, b1, W2, b2, W3, b3, end;
};
inline NetOffsets net_offsets(int64_t base, int Din, int H, int Dout) {
  NetOffsets o;
  o.W1 = base;
  o.b1 = o.W1 + (int64_t)Din * H;
  o.W2 = o.b1 + H;
  o.b2 = o.W2 + (int64_t)H * H;
  o.W3 = o.b2 + H;
  o.b3 = o.W3 + (int64_t)H * Dout;
  o.end = o.b3 + Dout;
  return o;
}

// The kernels read weights from a working copy of the parameter vector in which every block (W1, b1, ...)
// starts on a 64-float boundary, so that 16-byte loads of weight rows are always aligned.
struct ParamMap {
  int64_t src[13], dst[13];  // 12 blocks (actor 6, critic 6) + end
  // After the 12 blocks, per network: W1, W2 and W2 transposed once more in the order the matrix-core kernels
  // read their B operand straight from memory: element (k, n) of a [K][H] matrix at ((k / 4) * H + n) * 4 + k % 4,
  // so that the four k values a lane feeds to consecutive MFMAs are one 16-byte load, contiguous across lanes.
  // W1 is zero-padded to kpad1 rows (a multiple of 16).
  int64_t sw_w1[2], sw_w2[2], sw_w2t[2];
  int din[2], kpad1[2];
  int hidden[2];
  int64_t total;             // floats of the whole working copy
};
inline ParamMap param_map(const Dims& d) {
  ParamMap m;
  const NetOffsets a = net_offsets(0, d.D, d.Ha, kActions), c = net_offsets(d.Pa, d.Dc, d.Hc, 1);
  const int64_t src[13] = {a.W1, a.b1, a.W2, a.b2, a.W3, a.b3, c.W1, c.b1, c.W2, c.b2, c.W3, c.b3, c.end};
  int64_t off = 0;
  for (int i = 0; i < 13; ++i) {
    m.src[i] = src[i];
    m.dst[i] = off;
    if (i < 12) off += ((src[i + 1] - src[i] + 63) / 64) * 64;
  }
  m.hidden[0] = d.Ha;
  m.hidden[1] = d.Hc;
  m.din[0] = d.D;
  m.din[1] = d.Dc;
  for (int n = 0; n < 2; ++n) {
    const int64_t H = m.hidden[n];
    m.kpad1[n] = (m.din[n] + 15) / 16 * 16;
    m.sw_w1[n] = off;
    off += ((m.kpad1[n] * H + 63) / 64) * 64;
    m.sw_w2[n] = off;
    off += ((H * H + 63) / 64) * 64;
    m.sw_w2t[n] = off;
    off += ((H * H + 63) / 64) * 64;
  }
  m.total = off;
  return m;
}
inline NetOffsets padded_offsets(const ParamMap& m, int net) {
  const int64_t* o = m.dst + 6 * net;
  NetOffsets r;
  r.W1 = o[0]; r.b1 = o[1]; r.W2 = o[2]; r.b2 = o[3]; r.W3 = o[4]; r.b3 = o[5]; r.end = o[6];
  return r;
}

int32_t validate_config(const marl_config* cfg);
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

#define MARL_REQUIRE_PTR(p)                 \
  do {                                      \
    if ((p) == nullptr) return MARL_E_NULL; \
    if (marl::misaligned(p)) return MARL_E_ALIGN; \
  } while (0)
#define MARL_OPTIONAL_PTR(p)                                     \
  do {                                                           \
    if ((p) != nullptr && marl::misaligned(p)) return MARL_E_ALIGN; \
  } while (0)

inline int32_t launch_status() { return hipGetLastError() == hipSuccess ? MARL_OK : MARL_E_LAUNCH; }

// ---- Philox4x32-10 (Salmon et al., SC'11, Section 4) -------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t out[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // (one 32 x 32 -> 64 bit multiply per product: a separate high and low multiply are two quarter-rate instructions)
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}
__device__ __forceinline__ uint32_t rand_below(uint32_t x, uint32_t n) { return __umulhi(x, n); }
__device__ __forceinline__ float rand_unit(uint32_t x) { return ((float)(x >> 9) + 0.5f) * (1.0f / 8388608.0f); }
constexpr uint32_t kStreamReset = 1, kStreamSample = 2, kStreamRequest = 3;

// ---- XCD-aware tile order ---------------------------------------------------------------------
// Workgroups are dealt round-robin to the eight XCDs (each with its own L2), so consecutive workgroup ids never
// share an L2.  This maps linear workgroup id L of `total` to a logical index such that every XCD walks a
// contiguous run of logical indices: tiles that share an operand panel are made neighbours in logical order
// and therefore meet in one L2.  (A bijection for any total.)
__device__ __forceinline__ unsigned xcd_remap(unsigned L, unsigned total) {
  const unsigned q = total / 8u, r = total % 8u, x = L % 8u;
  return x * q + (x < r ? x : r) + L / 8u;
}

// ---- bfloat16: round-to-nearest-even, stored as the upper 16 bits of an fp32 -------------------
typedef uint16_t bf16_t;
__device__ __forceinline__ float round_to_bf16(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7f800000u) == 0x7f800000u) return x;
  u += 0x7fffu + ((u >> 16) & 1u);
  return __uint_as_float(u & 0xffff0000u);
}
// fp32 -> bf16 with the hardware conversion (round-to-nearest-even, two values per instruction on gfx950)
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
  uint32_t u;
  __builtin_memcpy(&u, &b, 4);
  return u;
}
__device__ __forceinline__ bf16_t to_bf16(float x) { return (bf16_t)(pack2_bf16(x, 0.f) & 0xffffu); }
__device__ __forceinline__ float from_bf16(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ float load_act(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float load_act(const bf16_t* p, int64_t i) { return from_bf16(p[i]); }

// ---- optional per-kernel timing with HIP events (measurement hook, host side) -----------------
enum KernelClass { KC_GEMM_NN = 0, KC_GEMM_NT = 1, KC_GEMM_TN = 2, KC_ENV_STEP = 3, KC_GAE = 4, KC_FUSED_TRAIN = 5, KC_ROLLOUT = 6, KC_COUNT = 7 };
bool timing_on();
// Records an event on `s` before and after the launch bracketed by the guard's lifetime and books
// `work` (flops or bytes) to the class.
struct TimedLaunch {
  int cls;
  hipStream_t s;
  bool active;
  TimedLaunch(int cls, double work, hipStream_t s);
  ~TimedLaunch();
};

// A second stream of the current device (default priority, created on the first call, kept until the process ends) with
// the two events of a fork and join: work that is independent of what follows on the caller's stream -- the second
// network of an update -- is launched there between
//   hipEventRecord(fork, s); hipStreamWaitEvent(stream, fork, 0);   and   hipEventRecord(join, stream); hipStreamWaitEvent(s, join, 0);
// so that it still starts after everything already queued on s and everything queued on s afterwards waits for it.
// One fork at a time per device: calls that overlap on one device from several host threads would share the events.
// nullptr when the stream cannot be created (the caller then stays on its own stream).
struct SideStream {
  hipStream_t stream;
  hipEvent_t fork, join;
};
const SideStream* side_stream();

// ---- launchers implemented in the kernel translation units ------------------------------------
int32_t launch_env_reset(const marl_config& c, marl_env_state st, hipStream_t s);
// do_step = false: only observe.  actions/reward/done may be null then.
int32_t launch_env_step(const marl_config& c, marl_env_state st, const int32_t* actions, float* obs, float* reward,
                        uint8_t* done, bool do_step, hipStream_t s);

struct RolloutWs;  // opaque carve-up of the rollout workspace
int64_t rollout_workspace_bytes(const marl_config& c, int64_t n_rows);
int64_t update_workspace_bytes(const marl_config& c);

int32_t launch_policy_forward(const marl_config& c, const float* params, const float* obs, int64_t n_rows,
                              float* logits, float* value, void* workspace, hipStream_t s);
int32_t launch_sample(const marl_config& c, const float* logits, const float* uniforms, const int32_t* forced,
                      int64_t n, uint64_t step, int32_t* action, int32_t* sampled, float* logp, hipStream_t s);
int32_t launch_rollout(const marl_config& c, marl_env_state st, const float* params, marl_traj tr,
                       uint64_t step_offset, const int32_t* forced_actions, const float* forced_uniforms,
                       void* workspace, hipStream_t s, const uint64_t* step_base = nullptr);
int32_t launch_gae(const marl_config& c, marl_traj tr, hipStream_t s);
int64_t eval_workspace_bytes(const marl_config& c);
int64_t rec_rollout_workspace_bytes(const marl_config& c);
int64_t rec_update_workspace_bytes(const marl_config& c);
int32_t launch_rollout_recurrent(const marl_config& c, marl_env_state st, const float* params, marl_traj tr,
                                 marl_rec_state rec, uint64_t step_offset, const int32_t* forced_actions,
                                 const float* forced_uniforms, void* workspace, hipStream_t s);
int32_t launch_ppo_update_recurrent(const marl_config& c, marl_traj tr, marl_rec_state rec, float* params, float* adam_m,
                                    float* adam_v, int64_t adam_step0, const int32_t* perm, float* stats,
                                    float* grad_dump, void* workspace, hipStream_t s);
int32_t launch_evaluate(const marl_config& c, marl_env_state st, const float* params, int32_t n_episodes,
                        marl_eval_stats out, void* workspace, hipStream_t s);
int32_t launch_ppo_update(const marl_config& c, marl_traj tr, float* params, float* adam_m, float* adam_v,
                          int64_t adam_step0, const int32_t* perm, float* stats, float* grad_dump, void* workspace,
                          hipStream_t s, const int64_t* adam_step_base = nullptr);
// step_base / adam_step_base (nullable, device memory): counters added on the device to step_offset / adam_step0, so
// that the launch sequence of a call does not depend on how many steps came before it.
int32_t launch_advance_counters(marl_counters* counters, uint64_t steps, int64_t adam_steps, hipStream_t s);

}  // namespace marl
