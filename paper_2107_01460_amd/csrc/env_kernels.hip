// The two grid worlds on the GPU (foraging, warehouse): reset, lock-step transition and egocentric observation.
//
// One lane per env-agent, and a wavefront owns floor(64 / A) whole envs.  Every lane reads the small state of
// its env into registers and resolves the whole transition redundantly there (targets of all agents, collisions,
// cooperative loading or deliveries, termination, and the re-seeding of a finished episode), so no lane waits
// for another.  For the observation each lane paints its own V x V x 3
// window into a wavefront-private LDS slab, which then leaves as one contiguous, 16-byte-coalesced run: the
// slab of a wavefront is exactly a contiguous piece of the [N][A][D] output.
#include <algorithm>

#include "common.h"

namespace marl {
namespace {

struct EnvParams {
  int G, A, F, L, cap, N;
  int kind;  // 0 foraging; 1 warehouse; 2 warehouse with episode end on collision (L = requested shelves there)
  uint32_t k0, k1;
  uint32_t inv_g20;  // ceil(2^20 / G): (r * inv_g20) >> 20 == r / G exactly for r < G*G <= 4096
};

// Entity packed as row | col << 8 | level << 16.
__device__ __forceinline__ int e_row(uint32_t e) { return (int)(e & 0xff); }
__device__ __forceinline__ int e_col(uint32_t e) { return (int)((e >> 8) & 0xff); }
__device__ __forceinline__ int e_lvl(uint32_t e) { return (int)((e >> 16) & 0xff); }

// New episode for one env, entirely in registers (every loop is unrolled over the at most 16 entities, so the
// arrays never leave the register file).  Draw order: A agent levels, A + F cells (agents first), F food levels;
// draw j is word j % 4 of Philox call j / 4 of the stream (env, episode).
template <int CA, int CF>
__device__ __forceinline__ void reset_regs(uint32_t ag[CA], uint32_t fd[CF], const EnvParams& p,
                                           uint32_t env, uint32_t episode) {
  constexpr int kMaxEnt = CA + CF;
  uint32_t buf[4] = {0, 0, 0, 0};
  int j = 0;
  auto draw = [&]() -> uint32_t {
    if ((j & 3) == 0) philox4x32_10(env, episode, (uint32_t)(j >> 2), kStreamReset, p.k0, p.k1, buf);
    const int w = j & 3;
    ++j;
    return w == 0 ? buf[0] : (w == 1 ? buf[1] : (w == 2 ? buf[2] : buf[3]));
  };
  int lvl[CA];
#pragma unroll
  for (int a = 0; a < CA; ++a) lvl[a] = 0;
#pragma unroll
  for (int a = 0; a < CA; ++a)
    if (a < p.A) lvl[a] = 1 + (int)rand_below(draw(), (uint32_t)p.L);
  // cells without replacement: the k-th entity draws r in [0, G*G - k) and takes the r-th free cell (ascending)
  int chosen[kMaxEnt];  // ascending
#pragma unroll
  for (int q = 0; q < kMaxEnt; ++q) chosen[q] = 0x7fffffff;
  const int cells = p.G * p.G, ne = p.A + p.F;
#pragma unroll
  for (int k = 0; k < kMaxEnt; ++k) {
    if (k < ne) {
      int r = (int)rand_below(draw(), (uint32_t)(cells - k));
#pragma unroll
      for (int q = 0; q < kMaxEnt; ++q) r += (q < k && chosen[q] <= r) ? 1 : 0;
      int pos = 0;  // entries smaller than r
#pragma unroll
      for (int q = 0; q < kMaxEnt; ++q) pos += (q < k && chosen[q] < r) ? 1 : 0;
#pragma unroll
      for (int q = kMaxEnt - 1; q >= 1; --q) chosen[q] = (q > pos) ? chosen[q - 1] : chosen[q];
#pragma unroll
      for (int q = 0; q < kMaxEnt; ++q) chosen[q] = (q == pos) ? r : chosen[q];
      const uint32_t row = ((uint32_t)r * p.inv_g20) >> 20, col = (uint32_t)r - row * (uint32_t)p.G;
      const uint32_t cell = row | (col << 8);
#pragma unroll
      for (int a = 0; a < CA; ++a)
        if (k == a) ag[a] = cell | ((uint32_t)lvl[a] << 16);
#pragma unroll
      for (int f = 0; f < CF; ++f)
        if (k == p.A + f) fd[f] = cell;
    }
  }
  // food level in 1..Lsum, Lsum = summed level of the (at most four) strongest agents
  int lsum = 0;
  uint32_t used = 0;
#pragma unroll
  for (int k = 0; k < (CA < 4 ? CA : 4); ++k) {
    int best = 0, bl = 0;
#pragma unroll
    for (int a = 0; a < CA; ++a) {
      const bool better = !((used >> a) & 1u) && lvl[a] > bl;
      bl = better ? lvl[a] : bl;
      best = better ? a : best;
    }
    if (k < p.A) {
      used |= 1u << best;
      lsum += bl;
    }
  }
#pragma unroll
  for (int f = 0; f < CF; ++f)
    if (f < p.F) fd[f] |= (1u + rand_below(draw(), (uint32_t)lsum)) << 16;
}

__global__ void __launch_bounds__(64) env_reset_kernel(EnvParams p, marl_env_state st) {
  const int n = blockIdx.x * 64 + threadIdx.x;
  if (n >= p.N) return;
  uint32_t ag[kMaxAgents], fd[kMaxFood];
  reset_regs<kMaxAgents, kMaxFood>(ag, fd, p, (uint32_t)n, 0u);
#pragma unroll
  for (int a = 0; a < kMaxAgents; ++a)
    if (a < p.A) {
      st.agent_row[(size_t)a * p.N + n] = (uint8_t)e_row(ag[a]);
      st.agent_col[(size_t)a * p.N + n] = (uint8_t)e_col(ag[a]);
      st.agent_lvl[(size_t)a * p.N + n] = (uint8_t)e_lvl(ag[a]);
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
template <int V, int NW, int CA, int CF>
__global__ void __launch_bounds__(64 * NW) env_step_kernel(EnvParams p, marl_env_state st,
                                                            const int32_t* __restrict__ actions, float* __restrict__ obs,
                                                            float* __restrict__ reward, uint8_t* __restrict__ done,
                                                            int do_step) {
  constexpr int D = 3 * V * V, h = (V - 1) / 2;
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
  {
    uint32_t r8[CA], c8[CA], l8[CA], fr8[CF], fc8[CF], fl8[CF];
    int a32[CA];
#pragma unroll
    for (int b = 0; b < CA; ++b) {
      const size_t i = (size_t)min(b, p.A - 1) * N + nn;
      r8[b] = st.agent_row[i];
      c8[b] = st.agent_col[i];
      l8[b] = st.agent_lvl[i];
      a32[b] = do_step ? actions[nn * p.A + min(b, p.A - 1)] : 0;
    }
#pragma unroll
    for (int f = 0; f < CF; ++f) {
      const size_t i = (size_t)min(f, p.F - 1) * N + nn;
      fr8[f] = st.food_row[i];
      fc8[f] = st.food_col[i];
      fl8[f] = st.food_lvl[i];
    }
#pragma unroll
    for (int b = 0; b < CA; ++b) {
      const bool on = active && b < p.A;
      ag[b] = on ? (r8[b] | (c8[b] << 8) | (l8[b] << 16)) : 0xffffu;  // off-grid: never matches a cell
      act[b] = on ? a32[b] : 0;
    }
#pragma unroll
    for (int f = 0; f < CF; ++f) fd[f] = (active && f < p.F) ? (fr8[f] | (fc8[f] << 8) | (fl8[f] << 16)) : 0xffffu;  // level 0: absent
  }
  int t = st.t_in_ep[nn];
  uint32_t episode = st.episode_id[nn];

  bool dn = false;
  if (do_step) {
    // ---- targets of every agent against the start-of-step state
    uint32_t tgt[CA];  // target cell (row | col << 8), 0xffff when the agent does not move
#pragma unroll
    for (int b = 0; b < CA; ++b) {
      const int ac = act[b];
      const int nr = e_row(ag[b]) + (ac == 2) - (ac == 1), nc = e_col(ag[b]) + (ac == 4) - (ac == 3);
      bool ok = b < p.A && ac >= 1 && ac <= 4 && nr >= 0 && nr < p.G && nc >= 0 && nc < p.G;
      const uint32_t cell = (uint32_t)nr | ((uint32_t)nc << 8);
#pragma unroll
      for (int o = 0; o < CA; ++o) ok = ok && (ag[o] & 0xffffu) != cell;
#pragma unroll
      for (int f = 0; f < CF; ++f) ok = ok && !(e_lvl(fd[f]) != 0 && (fd[f] & 0xffffu) == cell);
      tgt[b] = ok ? cell : 0xffffu;
    }
    // ---- cooperative loading: summed level of the adjacent loaders of each food
    float rew = 0.f;
    uint32_t mine = 0;
#pragma unroll
    for (int b = 0; b < CA; ++b) mine = (b == a) ? ag[b] : mine;
    int my_act = 0;
#pragma unroll
    for (int b = 0; b < CA; ++b) my_act = (b == a) ? act[b] : my_act;
    bool any_food = false;
#pragma unroll
    for (int f = 0; f < CF; ++f) {
      const int fl = e_lvl(fd[f]);
      if (f < p.F && fl != 0) {
        const int fr = e_row(fd[f]), fc = e_col(fd[f]);
        int lsum = 0;
#pragma unroll
        for (int b = 0; b < CA; ++b) {
          const int dist = abs(e_row(ag[b]) - fr) + abs(e_col(ag[b]) - fc);
          lsum += (b < p.A && act[b] == 5 && dist == 1) ? e_lvl(ag[b]) : 0;
        }
        if (lsum >= fl) {
          const int mdist = abs(e_row(mine) - fr) + abs(e_col(mine) - fc);
          if (my_act == 5 && mdist == 1) rew += __fdiv_rn((float)(fl * e_lvl(mine)), (float)lsum);
          fd[f] &= 0xffffu;  // collected: level 0
        } else {
          any_food = true;
        }
      }
    }
    // ---- movement: two or more valid movers onto one cell all stay
    uint32_t moved[CA];
#pragma unroll
    for (int b = 0; b < CA; ++b) {
      bool go = tgt[b] != 0xffffu;
#pragma unroll
      for (int o = 0; o < CA; ++o) go = go && (o == b || tgt[o] != tgt[b]);
      moved[b] = go ? ((ag[b] & 0xff0000u) | tgt[b]) : ag[b];
    }
#pragma unroll
    for (int b = 0; b < CA; ++b) ag[b] = moved[b];
    // ---- termination
    t += 1;
    dn = active && (!any_food || t == p.cap);
    if (active) {
      reward[(size_t)n * p.A + a] = rew;
      if (a == 0) done[n] = dn ? 1 : 0;
    }
    // ---- auto-reset: every lane of a finished env re-seeds it in its own registers (same result in each)
    if (dn) {
      episode += 1;
      reset_regs<CA, CF>(ag, fd, p, (uint32_t)n, episode);
      t = 0;
    }
    // ---- write the state back: every lane its own agent, the env's lanes share the food
    if (active) {
      uint32_t me = 0;
#pragma unroll
      for (int b = 0; b < CA; ++b) me = (b == a) ? ag[b] : me;
      st.agent_row[(size_t)a * N + n] = (uint8_t)e_row(me);
      st.agent_col[(size_t)a * N + n] = (uint8_t)e_col(me);
      if (dn) st.agent_lvl[(size_t)a * N + n] = (uint8_t)e_lvl(me);
#pragma unroll
      for (int f = 0; f < CF; ++f)
        if (f < p.F && (f % p.A) == a) {
          st.food_lvl[(size_t)f * N + n] = (uint8_t)e_lvl(fd[f]);
          if (dn) {
            st.food_row[(size_t)f * N + n] = (uint8_t)e_row(fd[f]);
            st.food_col[(size_t)f * N + n] = (uint8_t)e_col(fd[f]);
          }
        }
      if (a == 0) {
        st.t_in_ep[n] = t;
        st.episode_id[n] = episode;
      }
    }
  }

  if (obs == nullptr) return;
  // ---- the lane's window into the slab: walls and zeros first, then the entities that fall inside it
  float* w = slab + lane * D;
  {
    uint32_t me = 0;
#pragma unroll
    for (int b = 0; b < CA; ++b) me = (b == a) ? ag[b] : me;
    const int r0 = e_row(me), c0 = e_col(me);
    if (active) {
#pragma unroll
      for (int dy = -h; dy <= h; ++dy)
#pragma unroll
        for (int dx = -h; dx <= h; ++dx) {
          const int rr = r0 + dy, cc = c0 + dx;
          const bool wall = rr < 0 || rr >= p.G || cc < 0 || cc >= p.G;
          float* o = w + ((dy + h) * V + (dx + h)) * 3;
          o[0] = 0.f;
          o[1] = 0.f;
          o[2] = wall ? 1.f : 0.f;
        }
#pragma unroll
      for (int b = 0; b < CA; ++b) {
        const int dy = e_row(ag[b]) - r0, dx = e_col(ag[b]) - c0;
        if (b < p.A && dy >= -h && dy <= h && dx >= -h && dx <= h) w[((dy + h) * V + (dx + h)) * 3 + 0] = (float)e_lvl(ag[b]);
      }
#pragma unroll
      for (int f = 0; f < CF; ++f) {
        const int dy = e_row(fd[f]) - r0, dx = e_col(fd[f]) - c0;
        if (f < p.F && e_lvl(fd[f]) != 0 && dy >= -h && dy <= h && dx >= -h && dx <= h)
          w[((dy + h) * V + (dx + h)) * 3 + 1] = (float)e_lvl(fd[f]);
      }
    }
  }
  __syncthreads();
  // ---- the slab of a wavefront is one contiguous run of the output
  const int64_t envs_here = max((int64_t)0, min((int64_t)ew, (int64_t)p.N - wave_env0));
  const int count = (int)envs_here * p.A * D;  // floats
  float* out = obs + (size_t)wave_env0 * p.A * D;
  if ((reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
    const int n4 = count >> 2;
    for (int i = lane; i < n4; i += 64) reinterpret_cast<float4*>(out)[i] = reinterpret_cast<const float4*>(slab)[i];
    for (int i = (n4 << 2) + lane; i < count; i += 64) out[i] = slab[i];
  } else {
    for (int i = lane; i < count; i += 64) out[i] = slab[i];
  }
}

// ---- warehouse world -------------------------------------------------------------------------------------------
// Same lane assignment and output path as the foraging kernel (one lane per env-agent, the whole small transition
// resolved redundantly in registers, the observation painted into a wavefront-private LDS slab that leaves as one
// contiguous run).  Robots: row | col << 8 | (carried shelf + 1) << 16; shelves: row | col << 8 | state << 16.

__device__ __forceinline__ bool wh_goal(int G, int r, int c) { return r == G - 1 && (c == G / 2 - 1 || c == G / 2); }

// New episode: A + F distinct cells (robots first), then L requested shelves.  Draw j is word j % 4 of Philox
// call j / 4 of the stream (env, episode).
template <int CA, int CF>
__device__ __forceinline__ void wh_reset_regs(uint32_t ag[CA], uint32_t fd[CF], const EnvParams& p, uint32_t env,
                                              uint32_t episode) {
  constexpr int kMaxEnt = CA + CF;
  uint32_t buf[4] = {0, 0, 0, 0};
  int j = 0;
  auto draw = [&]() -> uint32_t {
    if ((j & 3) == 0) philox4x32_10(env, episode, (uint32_t)(j >> 2), kStreamReset, p.k0, p.k1, buf);
    const int w = j & 3;
    ++j;
    return w == 0 ? buf[0] : (w == 1 ? buf[1] : (w == 2 ? buf[2] : buf[3]));
  };
  int chosen[kMaxEnt];  // ascending
#pragma unroll
  for (int q = 0; q < kMaxEnt; ++q) chosen[q] = 0x7fffffff;
  const int cells = p.G * p.G, ne = p.A + p.F;
#pragma unroll
  for (int k = 0; k < kMaxEnt; ++k) {
    if (k < ne) {
      int r = (int)rand_below(draw(), (uint32_t)(cells - k));
#pragma unroll
      for (int q = 0; q < kMaxEnt; ++q) r += (q < k && chosen[q] <= r) ? 1 : 0;
      int pos = 0;
#pragma unroll
      for (int q = 0; q < kMaxEnt; ++q) pos += (q < k && chosen[q] < r) ? 1 : 0;
#pragma unroll
      for (int q = kMaxEnt - 1; q >= 1; --q) chosen[q] = (q > pos) ? chosen[q - 1] : chosen[q];
#pragma unroll
      for (int q = 0; q < kMaxEnt; ++q) chosen[q] = (q == pos) ? r : chosen[q];
      const uint32_t row = ((uint32_t)r * p.inv_g20) >> 20, col = (uint32_t)r - row * (uint32_t)p.G;
      const uint32_t cell = row | (col << 8);
#pragma unroll
      for (int a = 0; a < CA; ++a)
        if (k == a) ag[a] = cell;  // nothing carried
#pragma unroll
      for (int f = 0; f < CF; ++f)
        if (k == p.A + f) fd[f] = cell | (1u << 16);  // idle
    }
  }
#pragma unroll
  for (int q = 0; q < CF; ++q) {
    if (q < p.L) {
      int r = (int)rand_below(draw(), (uint32_t)(p.F - q));
#pragma unroll
      for (int f = 0; f < CF; ++f) {
        const bool idle = f < p.F && e_lvl(fd[f]) == 1;
        if (idle && r == 0) fd[f] = (fd[f] & 0xffffu) | (2u << 16);
        r -= idle ? 1 : 0;  // after the hit r is negative and nothing else matches
      }
    }
  }
}

__global__ void __launch_bounds__(64) wh_reset_kernel(EnvParams p, marl_env_state st) {
  const int n = blockIdx.x * 64 + threadIdx.x;
  if (n >= p.N) return;
  uint32_t ag[kMaxAgents], fd[kMaxFood];
  wh_reset_regs<kMaxAgents, kMaxFood>(ag, fd, p, (uint32_t)n, 0u);
#pragma unroll
  for (int a = 0; a < kMaxAgents; ++a)
    if (a < p.A) {
      st.agent_row[(size_t)a * p.N + n] = (uint8_t)e_row(ag[a]);
      st.agent_col[(size_t)a * p.N + n] = (uint8_t)e_col(ag[a]);
      st.agent_lvl[(size_t)a * p.N + n] = 0;
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
template <int V, int NW, int CA, int CF>
__global__ void __launch_bounds__(64 * NW) wh_step_kernel(EnvParams p, marl_env_state st, const int32_t* __restrict__ actions,
                                                          float* __restrict__ obs, float* __restrict__ reward,
                                                          uint8_t* __restrict__ done, int do_step) {
  constexpr int D = 3 * V * V, h = (V - 1) / 2;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ew = 64 / p.A;
  float* slab = reinterpret_cast<float*>(smem) + (size_t)wave * 64 * D;
  const int le = lane / p.A, a = lane - le * p.A;
  const int64_t wave_env0 = ((int64_t)blockIdx.x * NW + wave) * ew;
  const int64_t n = wave_env0 + le;
  const bool active = le < ew && n < p.N;
  const int N = p.N;
  const size_t nn = active ? (size_t)n : 0;

  uint32_t ag[CA], fd[CF];
  int act[CA];
#pragma unroll
  for (int b = 0; b < CA; ++b) {
    const size_t i = (size_t)min(b, p.A - 1) * N + nn;
    const uint32_t e = (uint32_t)st.agent_row[i] | ((uint32_t)st.agent_col[i] << 8) | ((uint32_t)st.agent_lvl[i] << 16);
    const int ac = do_step ? actions[nn * p.A + min(b, p.A - 1)] : 0;
    const bool on = active && b < p.A;
    ag[b] = on ? e : 0xffffu;  // off-grid: never matches a cell
    act[b] = on ? ac : 0;
  }
#pragma unroll
  for (int f = 0; f < CF; ++f) {
    const size_t i = (size_t)min(f, p.F - 1) * N + nn;
    const uint32_t e = (uint32_t)st.food_row[i] | ((uint32_t)st.food_col[i] << 8) | ((uint32_t)st.food_lvl[i] << 16);
    fd[f] = (active && f < p.F) ? e : 0xfffeu;  // another off-grid cell, state 0
  }
  int t = st.t_in_ep[nn];
  uint32_t episode = st.episode_id[nn];

  if (do_step) {
    // ---- targets against the start-of-step state
    uint32_t tgt[CA];  // target cell, 0xffff when the robot does not move
    bool collided = false;
#pragma unroll
    for (int b = 0; b < CA; ++b) {
      const int ac = act[b];
      const int nr = e_row(ag[b]) + (ac == 2) - (ac == 1), nc = e_col(ag[b]) + (ac == 4) - (ac == 3);
      bool ok = b < p.A && ac >= 1 && ac <= 4 && nr >= 0 && nr < p.G && nc >= 0 && nc < p.G;
      const uint32_t cell = (uint32_t)nr | ((uint32_t)nc << 8);
      bool hit = false;
#pragma unroll
      for (int o = 0; o < CA; ++o) hit = hit || (ag[o] & 0xffffu) == cell;
      collided = collided || (ok && hit);
      ok = ok && !hit;
      if (e_lvl(ag[b]) != 0) {
#pragma unroll
        for (int f = 0; f < CF; ++f) ok = ok && (fd[f] & 0xffffu) != cell;
      }
      tgt[b] = ok ? cell : 0xffffu;
    }
    // ---- contested cells; movement, carried shelves with their robots
    uint32_t moved[CA];
#pragma unroll
    for (int b = 0; b < CA; ++b) {
      bool go = tgt[b] != 0xffffu;
      bool contested = false;
#pragma unroll
      for (int o = 0; o < CA; ++o) contested = contested || (o != b && tgt[o] == tgt[b]);
      collided = collided || (go && contested);
      go = go && !contested;
      moved[b] = go ? ((ag[b] & 0xff0000u) | tgt[b]) : ag[b];
    }
    uint32_t fd0[CF];  // start-of-step shelves, for the toggle
#pragma unroll
    for (int f = 0; f < CF; ++f) fd0[f] = fd[f];
#pragma unroll
    for (int b = 0; b < CA; ++b) {
      const int cy = e_lvl(ag[b]);
#pragma unroll
      for (int f = 0; f < CF; ++f)
        if (cy == f + 1) fd[f] = (fd[f] & 0xff0000u) | (moved[b] & 0xffffu);
    }
    // ---- toggle (togglers have not moved)
    uint32_t carried_mask = 0;
#pragma unroll
    for (int b = 0; b < CA; ++b) carried_mask |= e_lvl(ag[b]) != 0 ? (1u << (e_lvl(ag[b]) - 1)) : 0u;
#pragma unroll
    for (int b = 0; b < CA; ++b) {
      if (b < p.A && act[b] == 5) {
        uint32_t cy = 0;
        if (e_lvl(ag[b]) == 0) {
#pragma unroll
          for (int f = 0; f < CF; ++f)
            if ((fd0[f] & 0xffffu) == (ag[b] & 0xffffu) && !((carried_mask >> f) & 1u)) cy = (uint32_t)(f + 1);
        }
        moved[b] = (moved[b] & 0xffffu) | (cy << 16);
      }
    }
#pragma unroll
    for (int b = 0; b < CA; ++b) ag[b] = moved[b];
    // ---- delivery, robots in ascending index
    float rew = 0.f;
    uint32_t words[4] = {0, 0, 0, 0};
    int ordinal = 0;
#pragma unroll
    for (int b = 0; b < CA; ++b) {
      const int cy = e_lvl(ag[b]);
      bool deliver = false;
      int fsel = 0;
#pragma unroll
      for (int f = 0; f < CF; ++f) {
        const bool mine = cy == f + 1 && e_lvl(fd[f]) == 2;
        deliver = deliver || mine;
        fsel = mine ? f : fsel;
      }
      deliver = deliver && b < p.A && wh_goal(p.G, e_row(ag[b]), e_col(ag[b]));
      if (deliver) {
        if (b == a) rew = 1.0f;
        int n_cand = 0;
#pragma unroll
        for (int f = 0; f < CF; ++f) {
          if (f == fsel) fd[f] = (fd[f] & 0xffffu) | (1u << 16);
          n_cand += (f < p.F && f != fsel && e_lvl(fd[f]) == 1) ? 1 : 0;
        }
        if ((ordinal & 3) == 0) philox4x32_10((uint32_t)n, episode, (uint32_t)t * 2u + (uint32_t)(ordinal >> 2), kStreamRequest, p.k0, p.k1, words);
        const int w = ordinal & 3;
        const uint32_t word = w == 0 ? words[0] : (w == 1 ? words[1] : (w == 2 ? words[2] : words[3]));
        if (n_cand == 0) {
#pragma unroll
          for (int f = 0; f < CF; ++f)
            if (f == fsel) fd[f] = (fd[f] & 0xffffu) | (2u << 16);
        } else {
          int r = (int)rand_below(word, (uint32_t)n_cand);
#pragma unroll
          for (int f = 0; f < CF; ++f) {
            const bool cand = f < p.F && f != fsel && e_lvl(fd[f]) == 1;
            if (cand && r == 0) fd[f] = (fd[f] & 0xffffu) | (2u << 16);
            r -= cand ? 1 : 0;
          }
        }
        ++ordinal;
      }
    }
    // ---- termination, auto-reset
    t += 1;
    const bool dn = active && (t == p.cap || (p.kind == 2 && collided));
    if (active) {
      reward[(size_t)n * p.A + a] = rew;
      if (a == 0) done[n] = dn ? 1 : 0;
    }
    if (dn) {
      episode += 1;
      wh_reset_regs<CA, CF>(ag, fd, p, (uint32_t)n, episode);
      t = 0;
    }
    if (active) {
      uint32_t me = 0;
#pragma unroll
      for (int b = 0; b < CA; ++b) me = (b == a) ? ag[b] : me;
      st.agent_row[(size_t)a * N + n] = (uint8_t)e_row(me);
      st.agent_col[(size_t)a * N + n] = (uint8_t)e_col(me);
      st.agent_lvl[(size_t)a * N + n] = (uint8_t)e_lvl(me);
#pragma unroll
      for (int f = 0; f < CF; ++f)
        if (f < p.F && (f % p.A) == a) {
          st.food_row[(size_t)f * N + n] = (uint8_t)e_row(fd[f]);
          st.food_col[(size_t)f * N + n] = (uint8_t)e_col(fd[f]);
          st.food_lvl[(size_t)f * N + n] = (uint8_t)e_lvl(fd[f]);
        }
      if (a == 0) {
        st.t_in_ep[n] = t;
        st.episode_id[n] = episode;
      }
    }
  }

  if (obs == nullptr) return;
  float* w = slab + lane * D;
  if (active) {
    uint32_t me = 0;
#pragma unroll
    for (int b = 0; b < CA; ++b) me = (b == a) ? ag[b] : me;
    const int r0 = e_row(me), c0 = e_col(me);
#pragma unroll
    for (int dy = -h; dy <= h; ++dy)
#pragma unroll
      for (int dx = -h; dx <= h; ++dx) {
        const int rr = r0 + dy, cc = c0 + dx;
        const bool wall = rr < 0 || rr >= p.G || cc < 0 || cc >= p.G;
        float* o = w + ((dy + h) * V + (dx + h)) * 3;
        o[0] = 0.f;
        o[1] = 0.f;
        o[2] = wall ? 1.f : (wh_goal(p.G, rr, cc) ? 0.5f : 0.f);
      }
#pragma unroll
    for (int b = 0; b < CA; ++b) {
      const int dy = e_row(ag[b]) - r0, dx = e_col(ag[b]) - c0;
      if (b < p.A && dy >= -h && dy <= h && dx >= -h && dx <= h)
        w[((dy + h) * V + (dx + h)) * 3 + 0] = e_lvl(ag[b]) != 0 ? 2.f : 1.f;
    }
#pragma unroll
    for (int f = 0; f < CF; ++f) {
      const int dy = e_row(fd[f]) - r0, dx = e_col(fd[f]) - c0;
      if (f < p.F && dy >= -h && dy <= h && dx >= -h && dx <= h) {
        float* o = &w[((dy + h) * V + (dx + h)) * 3 + 1];
        *o = fmaxf(*o, (float)e_lvl(fd[f]));
      }
    }
  }
  __syncthreads();
  const int64_t envs_here = max((int64_t)0, min((int64_t)ew, (int64_t)p.N - wave_env0));
  const int count = (int)envs_here * p.A * D;
  float* out = obs + (size_t)wave_env0 * p.A * D;
  if ((reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
    const int n4 = count >> 2;
    for (int i = lane; i < n4; i += 64) reinterpret_cast<float4*>(out)[i] = reinterpret_cast<const float4*>(slab)[i];
    for (int i = (n4 << 2) + lane; i < count; i += 64) out[i] = slab[i];
  } else {
    for (int i = lane; i < count; i += 64) out[i] = slab[i];
  }
}

template <int V, int NW, int CA, int CF>
int32_t launch_wh_step_inst(const EnvParams& p, marl_env_state st, const int32_t* actions, float* obs, float* reward,
                            uint8_t* done, bool do_step, hipStream_t s) {
  const int ew = 64 / p.A;
  const int64_t waves = (p.N + ew - 1) / ew;
  const size_t lds = sizeof(float) * NW * 64 * 3 * V * V;
  auto kern = wh_step_kernel<V, NW, CA, CF>;
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
int32_t launch_wh_step_caps(const EnvParams& p, marl_env_state st, const int32_t* actions, float* obs, float* reward,
                            uint8_t* done, bool do_step, hipStream_t s) {
  const int cap = std::max(p.A, p.F);  // every loop over entities is unrolled to the capacity
  if (cap <= 4) return launch_wh_step_inst<V, NW, 4, 4>(p, st, actions, obs, reward, done, do_step, s);
  return launch_wh_step_inst<V, NW, kMaxAgents, kMaxFood>(p, st, actions, obs, reward, done, do_step, s);
}

EnvParams env_params(const marl_config& c) {
  EnvParams p;
  p.G = c.grid; p.A = c.n_agents; p.F = c.n_food; p.L = c.max_level; p.cap = c.episode_cap; p.N = c.n_envs;
  p.kind = c.env_kind;
  p.k0 = (uint32_t)(c.seed & 0xffffffffu);
  p.k1 = (uint32_t)(c.seed >> 32);
  p.inv_g20 = ((1u << 20) + (uint32_t)c.grid - 1u) / (uint32_t)c.grid;
  return p;
}

}  // namespace

int32_t launch_env_reset(const marl_config& c, marl_env_state st, hipStream_t s) {
  const EnvParams p = env_params(c);
  if (p.kind != 0) {
    hipLaunchKernelGGL(wh_reset_kernel, dim3((p.N + 63) / 64), dim3(64), 0, s, p, st);
    return launch_status();
  }
  hipLaunchKernelGGL(env_reset_kernel, dim3((p.N + 63) / 64), dim3(64), 0, s, p, st);
  return launch_status();
}

template <int V, int NW, int CA, int CF>
static int32_t launch_env_step_inst(const EnvParams& p, marl_env_state st, const int32_t* actions, float* obs,
                                    float* reward, uint8_t* done, bool do_step, hipStream_t s) {
  const int ew = 64 / p.A;
  const int64_t waves = (p.N + ew - 1) / ew;
  const size_t lds = sizeof(float) * NW * 64 * 3 * V * V;
  auto kern = env_step_kernel<V, NW, CA, CF>;
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
static int32_t launch_env_step_caps(const EnvParams& p, marl_env_state st, const int32_t* actions, float* obs,
                                    float* reward, uint8_t* done, bool do_step, hipStream_t s) {
  const int cap = std::max(p.A, p.F);
  if (cap <= 2) return launch_env_step_inst<V, NW, 2, 2>(p, st, actions, obs, reward, done, do_step, s);
  if (cap <= 4) return launch_env_step_inst<V, NW, 4, 4>(p, st, actions, obs, reward, done, do_step, s);
  return launch_env_step_inst<V, NW, kMaxAgents, kMaxFood>(p, st, actions, obs, reward, done, do_step, s);
}

int32_t launch_env_step(const marl_config& c, marl_env_state st, const int32_t* actions, float* obs, float* reward,
                        uint8_t* done, bool do_step, hipStream_t s) {
  const EnvParams p = env_params(c);
  // algorithmic bytes of one transition: observation, reward, action per agent; done and the state (read + write) per env
  const double D = 3.0 * c.view * c.view;
  const double bytes = do_step ? (double)p.N * (p.A * (4.0 * D * (obs ? 1 : 0) + 8.0) + 1.0 + 2.0 * (3.0 * p.A + 4.0 * p.F + 8.0))
                               : (double)p.N * p.A * 4.0 * D;
  TimedLaunch timed(KC_ENV_STEP, bytes, s);
  if (p.kind != 0) {
    switch (c.view) {
      case 3: return launch_wh_step_caps<3, 4>(p, st, actions, obs, reward, done, do_step, s);
      case 5: return launch_wh_step_caps<5, 4>(p, st, actions, obs, reward, done, do_step, s);
      case 7: return launch_wh_step_caps<7, 2>(p, st, actions, obs, reward, done, do_step, s);
      default: return MARL_E_CONFIG;
    }
  }
  switch (c.view) {
    case 3: return launch_env_step_caps<3, 4>(p, st, actions, obs, reward, done, do_step, s);
    case 5: return launch_env_step_caps<5, 4>(p, st, actions, obs, reward, done, do_step, s);
    case 7: return launch_env_step_caps<7, 2>(p, st, actions, obs, reward, done, do_step, s);
    default: return MARL_E_CONFIG;
  }
}

}  // namespace marl
