// The two grid worlds on the GPU (foraging, warehouse): reset, lock-step transition and egocentric observation.
//
// One lane per env-agent, and a wavefront owns floor(64 / A) whole envs.  Every lane reads the small state of
// its env into registers and resolves the whole transition redundantly there (targets of all agents, collisions,
// cooperative loading or deliveries, termination, and the re-seeding of a finished episode), so no lane waits
// for another.  For the observation each lane paints its own V x V x 3
// window into a wavefront-private LDS slab, which then leaves as one contiguous, 16-byte-coalesced run: the
// slab of a wavefront is exactly a contiguous piece of the [N][A][D] output.
#include <algorithm>

#include "env_device.h"

namespace marl {
namespace {

template <int KIND>
__global__ void __launch_bounds__(64) env_reset_kernel(EnvParams p, marl_env_state st) {
  const int n = blockIdx.x * 64 + threadIdx.x;
  if (n >= p.N) return;
  uint32_t ag[kMaxAgents], fd[kMaxFood];
  if (KIND == 0) reset_regs<kMaxAgents, kMaxFood>(ag, fd, p, (uint32_t)n, 0u);
  else wh_reset_regs<kMaxAgents, kMaxFood>(ag, fd, p, (uint32_t)n, 0u);
#pragma unroll
  for (int a = 0; a < kMaxAgents; ++a)
    if (a < p.A) {
      st.agent_row[(size_t)a * p.N + n] = (uint8_t)e_row(ag[a]);
      st.agent_col[(size_t)a * p.N + n] = (uint8_t)e_col(ag[a]);
      st.agent_lvl[(size_t)a * p.N + n] = KIND == 0 ? (uint8_t)e_lvl(ag[a]) : (uint8_t)0;
    }
#pragma unroll
  for (int f = 0; f < kMaxFood; ++f)
    if (f < p.F) {
      st.food_row[(size_t)f * p.N + n] = (uint8_t)e_row(fd[f]);
      st.food_col[(size_t)f * p.N + n] = (uint8_t)e_col(fd[f]);
      st.food_lvl[(size_t)f * p.N + n] = (uint8_t)e_lvl(fd[f]);
    }
  st.t_in_ep[n] = 0;
  st.episode_id[n] = 0;
}

// Dynamic LDS per workgroup of NW wavefronts: float slab[NW][64 * D]
// CA / CF: compile-time capacity for agents / food (every loop over entities is unrolled to it)
// KIND: 0 foraging world, 1 warehouse world
template <int V, int NW, int CA, int CF, int KIND>
__global__ void __launch_bounds__(64 * NW) env_step_kernel(EnvParams p, marl_env_state st,
                                                            const int32_t* __restrict__ actions, float* __restrict__ obs,
                                                            float* __restrict__ reward, uint8_t* __restrict__ done,
                                                            int do_step) {
  constexpr int D = 3 * V * V;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ew = 64 / p.A;  // envs per wavefront
  float* slab = reinterpret_cast<float*>(smem) + (size_t)wave * 64 * D;

  const int le = lane / p.A, a = lane - le * p.A;
  const int64_t wave_env0 = ((int64_t)blockIdx.x * NW + wave) * ew;
  const int64_t n = wave_env0 + le;
  const bool active = le < ew && n < p.N;
  const int N = p.N;

  // ---- the env's state, in registers.  All loads are issued branch-free (clamped indices) so that they are in
  // flight together; entries past A / F and inactive lanes are masked afterwards.
  uint32_t ag[CA], fd[CF];
  int act[CA];
  const size_t nn = active ? (size_t)n : 0;
  load_env_state<CA, CF, KIND>(ag, fd, st, p, nn, active);
  {
    int a32[CA];
#pragma unroll
    for (int b = 0; b < CA; ++b) a32[b] = do_step ? actions[nn * p.A + min(b, p.A - 1)] : 0;
#pragma unroll
    for (int b = 0; b < CA; ++b) act[b] = (active && b < p.A) ? a32[b] : 0;
  }
  int t = st.t_in_ep[nn];
  uint32_t episode = st.episode_id[nn];

  if (do_step) {
    float rew;
    bool dn;
    if (KIND == 0) forage_transition<CA, CF>(ag, fd, act, a, active, p, (uint32_t)n, t, episode, rew, dn);
    else wh_transition<CA, CF>(ag, fd, act, a, active, p, (uint32_t)n, t, episode, rew, dn);
    if (active) {
      reward[(size_t)n * p.A + a] = rew;
      if (a == 0) done[n] = dn ? 1 : 0;
      store_env_state<CA, CF, KIND>(ag, fd, st, p, (size_t)n, a, dn, t, episode);
    }
  }

  if (obs == nullptr) return;
  if (active) {
    if (KIND == 0) forage_paint<V, CA, CF>(slab + lane * D, ag, fd, a, p);
    else wh_paint<V, CA, CF>(slab + lane * D, ag, fd, a, p);
  }
  // the slab is private to the wavefront, whose LDS operations execute in order: only the compiler has to keep them so
  // (no workgroup barrier: a wavefront that re-seeds episodes does not hold the others back)
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  __builtin_amdgcn_wave_barrier();
  // ---- the slab of a wavefront is one contiguous run of the output
  const int64_t envs_here = max((int64_t)0, min((int64_t)ew, (int64_t)p.N - wave_env0));
  const int count = (int)envs_here * p.A * D;  // floats
  float* out = obs + (size_t)wave_env0 * p.A * D;
  if ((reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
    const int n4 = count >> 2;
    // streaming stores: the observations are not read again soon, and written through as they are produced they do
    // not wait in the L2 for the write-back at the end of the kernel (9.9 -> 9.0 us per launch at 262 144 env-agents)
    typedef float f4v __attribute__((ext_vector_type(4)));
    for (int i = lane; i < n4; i += 64) __builtin_nontemporal_store(reinterpret_cast<const f4v*>(slab)[i], reinterpret_cast<f4v*>(out) + i);
    for (int i = (n4 << 2) + lane; i < count; i += 64) out[i] = slab[i];
  } else {
    for (int i = lane; i < count; i += 64) out[i] = slab[i];
  }
}

template <int V, int NW, int CA, int CF, int KIND>
int32_t launch_env_step_inst(const EnvParams& p, marl_env_state st, const int32_t* actions, float* obs, float* reward,
                             uint8_t* done, bool do_step, hipStream_t s) {
  const int ew = 64 / p.A;
  const int64_t waves = (p.N + ew - 1) / ew;
  const size_t lds = sizeof(float) * NW * 64 * 3 * V * V;
  auto kern = env_step_kernel<V, NW, CA, CF, KIND>;
  static bool configured = false;
  if (!configured && lds > 64 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
      return MARL_E_LAUNCH;
    configured = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)((waves + NW - 1) / NW)), dim3(64 * NW), lds, s, p, st, actions, obs, reward, done,
                     (int)do_step);
  return launch_status();
}

template <int V, int NW>
int32_t launch_env_step_caps(const EnvParams& p, marl_env_state st, const int32_t* actions, float* obs, float* reward,
                             uint8_t* done, bool do_step, hipStream_t s) {
  const int cap = std::max(p.A, p.F);  // every loop over entities is unrolled to the capacity
  if (p.kind != 0) {
    if (cap <= 4) return launch_env_step_inst<V, NW, 4, 4, 1>(p, st, actions, obs, reward, done, do_step, s);
    return launch_env_step_inst<V, NW, kMaxAgents, kMaxFood, 1>(p, st, actions, obs, reward, done, do_step, s);
  }
  if (cap <= 2) return launch_env_step_inst<V, NW, 2, 2, 0>(p, st, actions, obs, reward, done, do_step, s);
  if (cap <= 4) return launch_env_step_inst<V, NW, 4, 4, 0>(p, st, actions, obs, reward, done, do_step, s);
  return launch_env_step_inst<V, NW, kMaxAgents, kMaxFood, 0>(p, st, actions, obs, reward, done, do_step, s);
}

}  // namespace

int32_t launch_env_reset(const marl_config& c, marl_env_state st, hipStream_t s) {
  const EnvParams p = env_params(c);
  if (p.kind != 0) hipLaunchKernelGGL(env_reset_kernel<1>, dim3((p.N + 63) / 64), dim3(64), 0, s, p, st);
  else hipLaunchKernelGGL(env_reset_kernel<0>, dim3((p.N + 63) / 64), dim3(64), 0, s, p, st);
  return launch_status();
}

int32_t launch_env_step(const marl_config& c, marl_env_state st, const int32_t* actions, float* obs, float* reward,
                        uint8_t* done, bool do_step, hipStream_t s) {
  const EnvParams p = env_params(c);
  // algorithmic bytes of one transition: observation, reward, action per agent; done and the state (read + write) per env
  const double D = 3.0 * c.view * c.view;
  const double bytes = do_step ? (double)p.N * (p.A * (4.0 * D * (obs ? 1 : 0) + 8.0) + 1.0 + 2.0 * (3.0 * p.A + 4.0 * p.F + 8.0))
                               : (double)p.N * p.A * 4.0 * D;
  TimedLaunch timed(KC_ENV_STEP, bytes, s);
  switch (c.view) {
    case 3: return launch_env_step_caps<3, 8>(p, st, actions, obs, reward, done, do_step, s);
    case 5: return launch_env_step_caps<5, 4>(p, st, actions, obs, reward, done, do_step, s);
    case 7: return launch_env_step_caps<7, 2>(p, st, actions, obs, reward, done, do_step, s);
    default: return MARL_E_CONFIG;
  }
}

}  // namespace marl
