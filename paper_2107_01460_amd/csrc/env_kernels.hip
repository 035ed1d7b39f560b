// Grid-foraging environment on the GPU: reset, lock-step transition and egocentric observation.
//
// One lane per env-agent.  A workgroup owns a contiguous block of envs; their state is staged in
// LDS, every lane resolves its own agent (target, collision, reward), lane 0 of an env settles
// food removal, termination and the re-seeding of a finished episode.  For the observation the
// workgroup paints one G x G occupancy grid per env into LDS and all lanes then emit window cells
// in output order, so the stores of a wavefront are one contiguous run of 12-byte cells.
#include <algorithm>

#include "common.h"

namespace marl {
namespace {

struct EnvParams {
  int G, A, F, L, cap, N;
  uint32_t k0, k1;
};

// LDS image of one env.
struct __attribute__((aligned(8))) EnvLds {
  uint8_t ar[kMaxAgents], ac[kMaxAgents], al[kMaxAgents];   // agent row / col / level
  uint8_t fr[kMaxFood], fc[kMaxFood], fl[kMaxFood];         // food row / col / level (0 = gone)
  uint8_t tr[kMaxAgents], tc[kMaxAgents], mv[kMaxAgents];   // target cell, move-is-valid
  uint8_t act[kMaxAgents], ld[kMaxAgents];                  // action, bitmask of foods this agent loads
  uint16_t chosen[kMaxAgents + kMaxFood];                   // sorted cells already taken (reset only)
  int32_t t;
  uint32_t episode;
  int32_t done;
};

// New episode for one env, executed by a single lane on the env's LDS image.
__device__ void reset_one(EnvLds& e, const EnvParams& p, uint32_t env) {
  uint32_t buf[4];
  int have = -1;
  int j = 0;
  auto draw = [&](int idx) -> uint32_t {
    const int call = idx >> 2;
    if (call != have) {
      philox4x32_10(env, e.episode, (uint32_t)call, kStreamReset, p.k0, p.k1, buf);
      have = call;
    }
    return buf[idx & 3];
  };
  for (int a = 0; a < p.A; ++a) e.al[a] = (uint8_t)(1u + rand_below(draw(j++), (uint32_t)p.L));
  const int cells = p.G * p.G;
  int cnt = 0;
  for (int k = 0; k < p.A + p.F; ++k) {
    int r = (int)rand_below(draw(j++), (uint32_t)(cells - k));
    for (int q = 0; q < cnt; ++q)
      if ((int)e.chosen[q] <= r) ++r;
    int pos = cnt;  // insert keeping ascending order
    while (pos > 0 && (int)e.chosen[pos - 1] > r) {
      e.chosen[pos] = e.chosen[pos - 1];
      --pos;
    }
    e.chosen[pos] = (uint16_t)r;
    ++cnt;
    const uint8_t row = (uint8_t)(r / p.G), col = (uint8_t)(r - (r / p.G) * p.G);
    if (k < p.A) {
      e.ar[k] = row;
      e.ac[k] = col;
    } else {
      e.fr[k - p.A] = row;
      e.fc[k - p.A] = col;
    }
  }
  // summed level of the (at most four) strongest agents
  int lsum = 0;
  uint32_t used = 0;
  const int take = p.A < 4 ? p.A : 4;
  for (int k = 0; k < take; ++k) {
    int best = -1, bl = 0;
    for (int a = 0; a < p.A; ++a)
      if (!((used >> a) & 1u) && (int)e.al[a] > bl) {
        bl = e.al[a];
        best = a;
      }
    used |= 1u << best;
    lsum += bl;
  }
  for (int f = 0; f < p.F; ++f) e.fl[f] = (uint8_t)(1u + rand_below(draw(j++), (uint32_t)lsum));
  e.t = 0;
}

__global__ void __launch_bounds__(64) env_reset_kernel(EnvParams p, marl_env_state st) {
  __shared__ EnvLds lds[64];
  const int n = blockIdx.x * 64 + threadIdx.x;
  if (n >= p.N) return;
  EnvLds& e = lds[threadIdx.x];
  e.episode = 0;
  reset_one(e, p, (uint32_t)n);
  for (int a = 0; a < p.A; ++a) {
    st.agent_row[(size_t)a * p.N + n] = e.ar[a];
    st.agent_col[(size_t)a * p.N + n] = e.ac[a];
    st.agent_lvl[(size_t)a * p.N + n] = e.al[a];
  }
  for (int f = 0; f < p.F; ++f) {
    st.food_row[(size_t)f * p.N + n] = e.fr[f];
    st.food_col[(size_t)f * p.N + n] = e.fc[f];
    st.food_lvl[(size_t)f * p.N + n] = e.fl[f];
  }
  st.t_in_ep[n] = 0;
  st.episode_id[n] = 0;
}

// Dynamic LDS: EnvLds[epb] | uint32 sample_info[epb*A] | uint16 grid[epb][G*G]
template <int V>
__global__ void __launch_bounds__(256) env_step_kernel(EnvParams p, marl_env_state st, const int32_t* __restrict__ actions,
                                                       float* __restrict__ obs, float* __restrict__ reward,
                                                       uint8_t* __restrict__ done, int epb, int do_step) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  EnvLds* envs = reinterpret_cast<EnvLds*>(smem);
  uint32_t* sample_info = reinterpret_cast<uint32_t*>(smem + sizeof(EnvLds) * epb);
  uint16_t* grid = reinterpret_cast<uint16_t*>(sample_info + epb * p.A);

  const int tid = threadIdx.x;
  const int n0 = blockIdx.x * epb;
  const int nenv = min(epb, p.N - n0);
  const int le = tid / p.A, a = tid - le * p.A;
  const bool active = le < nenv;
  const int n = n0 + le;

  // ---- stage state in LDS
  if (active) {
    EnvLds& e = envs[le];
    e.ar[a] = st.agent_row[(size_t)a * p.N + n];
    e.ac[a] = st.agent_col[(size_t)a * p.N + n];
    e.al[a] = st.agent_lvl[(size_t)a * p.N + n];
    for (int f = a; f < p.F; f += p.A) {
      e.fr[f] = st.food_row[(size_t)f * p.N + n];
      e.fc[f] = st.food_col[(size_t)f * p.N + n];
      e.fl[f] = st.food_lvl[(size_t)f * p.N + n];
    }
    if (do_step) e.act[a] = (uint8_t)actions[(size_t)n * p.A + a];
    if (a == 0) {
      e.t = st.t_in_ep[n];
      e.episode = st.episode_id[n];
      e.done = 0;
    }
  }
  __syncthreads();

  if (do_step) {
    int r0 = 0, c0 = 0, act = 0;
    // ---- targets against the start-of-step state, loader flags
    if (active) {
      EnvLds& e = envs[le];
      r0 = e.ar[a]; c0 = e.ac[a]; act = e.act[a];
      int nr = r0 + (act == 2) - (act == 1), nc = c0 + (act == 4) - (act == 3);
      bool ok = (act >= 1 && act <= 4) && nr >= 0 && nr < p.G && nc >= 0 && nc < p.G;
      for (int b = 0; b < p.A; ++b) ok = ok && !((int)e.ar[b] == nr && (int)e.ac[b] == nc);
      uint32_t ldmask = 0;
      for (int f = 0; f < p.F; ++f) {
        const int fl = e.fl[f], fr = e.fr[f], fc = e.fc[f];
        ok = ok && !(fl != 0 && fr == nr && fc == nc);
        const int dist = abs(r0 - fr) + abs(c0 - fc);
        if (fl != 0 && act == 5 && dist == 1) ldmask |= 1u << f;
      }
      e.mv[a] = ok;
      e.tr[a] = (uint8_t)(ok ? nr : r0);
      e.tc[a] = (uint8_t)(ok ? nc : c0);
      e.ld[a] = (uint8_t)ldmask;
    }
    __syncthreads();
    // ---- collisions and rewards (read-only on the LDS image)
    int new_r = r0, new_c = c0;
    uint32_t eaten = 0;
    if (active) {
      const EnvLds& e = envs[le];
      bool go = e.mv[a];
      for (int b = 0; b < p.A; ++b)
        if (b != a && e.mv[b] && e.tr[b] == e.tr[a] && e.tc[b] == e.tc[a]) go = false;
      if (go) {
        new_r = e.tr[a];
        new_c = e.tc[a];
      }
      float rew = 0.0f;
      const int my_lvl = e.al[a];
      const uint32_t my_ld = e.ld[a];
      for (int f = 0; f < p.F; ++f) {
        const int fl = e.fl[f];
        if (fl == 0) continue;
        int lsum = 0;
        for (int b = 0; b < p.A; ++b) lsum += ((e.ld[b] >> f) & 1) ? (int)e.al[b] : 0;
        if (lsum >= fl) {
          eaten |= 1u << f;
          if ((my_ld >> f) & 1u) rew += __fdiv_rn((float)(fl * my_lvl), (float)lsum);
        }
      }
      reward[(size_t)n * p.A + a] = rew;
    }
    __syncthreads();
    if (active) {
      EnvLds& e = envs[le];
      e.ar[a] = (uint8_t)new_r;
      e.ac[a] = (uint8_t)new_c;
    }
    __syncthreads();
    // ---- food removal, termination, auto-reset: one lane per env
    if (active && a == 0) {
      EnvLds& e = envs[le];
      bool any = false;
      for (int f = 0; f < p.F; ++f) {
        if ((eaten >> f) & 1u) e.fl[f] = 0;
        any = any || e.fl[f] != 0;
      }
      e.t += 1;
      const bool dn = !any || e.t == p.cap;
      done[n] = dn ? 1 : 0;
      if (dn) {
        e.episode += 1;
        reset_one(e, p, (uint32_t)n);
      }
      e.done = dn;
    }
    __syncthreads();
    // ---- write the state back
    if (active) {
      const EnvLds& e = envs[le];
      st.agent_row[(size_t)a * p.N + n] = e.ar[a];
      st.agent_col[(size_t)a * p.N + n] = e.ac[a];
      if (e.done) st.agent_lvl[(size_t)a * p.N + n] = e.al[a];
      for (int f = a; f < p.F; f += p.A) {
        st.food_lvl[(size_t)f * p.N + n] = e.fl[f];
        if (e.done) {
          st.food_row[(size_t)f * p.N + n] = e.fr[f];
          st.food_col[(size_t)f * p.N + n] = e.fc[f];
        }
      }
      if (a == 0) {
        st.t_in_ep[n] = e.t;
        st.episode_id[n] = e.episode;
      }
    }
  }

  if (obs == nullptr) return;
  // ---- paint the occupancy grids: low byte agent level, high byte food level
  const int cells = p.G * p.G;
  {
    uint32_t* g32 = reinterpret_cast<uint32_t*>(grid);
    const int words = (nenv * cells + 1) / 2;
    for (int i = tid; i < words; i += blockDim.x) g32[i] = 0;
  }
  __syncthreads();
  if (active) {
    const EnvLds& e = envs[le];
    const int r = e.ar[a], c = e.ac[a];
    grid[le * cells + r * p.G + c] = (uint16_t)e.al[a];
    sample_info[tid] = ((uint32_t)le << 16) | ((uint32_t)r << 8) | (uint32_t)c;
    for (int f = a; f < p.F; f += p.A)
      if (e.fl[f] != 0) grid[le * cells + e.fr[f] * p.G + e.fc[f]] = (uint16_t)((uint32_t)e.fl[f] << 8);
  }
  __syncthreads();
  // ---- emit window cells in output order: cell index i of the block <-> 3 consecutive floats
  constexpr int VV = V * V, h = (V - 1) / 2;
  const int total = nenv * p.A * VV;
  float* out = obs + (size_t)n0 * p.A * VV * 3;
  for (int i = tid; i < total; i += blockDim.x) {
    const int smp = i / VV, cell = i - smp * VV;
    const int dy = cell / V - h, dx = cell % V - h;
    const uint32_t info = sample_info[smp];
    const int rr = (int)((info >> 8) & 0xff) + dy, cc = (int)(info & 0xff) + dx;
    float v0 = 0.f, v1 = 0.f, v2 = 0.f;
    if (rr < 0 || rr >= p.G || cc < 0 || cc >= p.G) {
      v2 = 1.f;
    } else {
      const uint32_t g = grid[(info >> 16) * cells + rr * p.G + cc];
      v0 = (float)(g & 0xff);
      v1 = (float)(g >> 8);
    }
    float* o = out + (size_t)i * 3;
    o[0] = v0; o[1] = v1; o[2] = v2;
  }
}

EnvParams env_params(const marl_config& c) {
  EnvParams p;
  p.G = c.grid; p.A = c.n_agents; p.F = c.n_food; p.L = c.max_level; p.cap = c.episode_cap; p.N = c.n_envs;
  p.k0 = (uint32_t)(c.seed & 0xffffffffu);
  p.k1 = (uint32_t)(c.seed >> 32);
  return p;
}

}  // namespace

int32_t launch_env_reset(const marl_config& c, marl_env_state st, hipStream_t s) {
  const EnvParams p = env_params(c);
  hipLaunchKernelGGL(env_reset_kernel, dim3((p.N + 63) / 64), dim3(64), 0, s, p, st);
  return launch_status();
}

int32_t launch_env_step(const marl_config& c, marl_env_state st, const int32_t* actions, float* obs, float* reward,
                        uint8_t* done, bool do_step, hipStream_t s) {
  const EnvParams p = env_params(c);
  // envs per workgroup: at most 256 lanes, and the occupancy grids must fit in ~48 KB of LDS
  int epb = 256 / p.A;
  const int grid_bytes = 2 * p.G * p.G;
  epb = std::min(epb, std::max(1, 49152 / grid_bytes));
  epb = std::min(epb, p.N);
  while (epb * p.A > 64 && p.N / epb < 1024) epb = (epb + 1) / 2;  // enough workgroups to cover 256 CUs
  auto lds_bytes = [&](int e) { return sizeof(EnvLds) * e + 4 * (size_t)e * p.A + (size_t)grid_bytes * e + 16; };
  while (epb > 1 && lds_bytes(epb) > 60 * 1024) epb = (epb + 1) / 2;
  int threads = ((epb * p.A + 63) / 64) * 64;
  const size_t lds = lds_bytes(epb);
  const dim3 grid((p.N + epb - 1) / epb), block(threads);
  // algorithmic bytes of one transition: observation, reward, action per agent; done and the state (read + write) per env
  const double D = 3.0 * c.view * c.view;
  const double bytes = do_step ? (double)p.N * (p.A * (4.0 * D * (obs ? 1 : 0) + 8.0) + 1.0 + 2.0 * (3.0 * p.A + 4.0 * p.F + 8.0))
                               : (double)p.N * p.A * 4.0 * D;
  TimedLaunch timed(KC_ENV_STEP, bytes, s);
  switch (c.view) {
    case 3: hipLaunchKernelGGL(env_step_kernel<3>, grid, block, lds, s, p, st, actions, obs, reward, done, epb, (int)do_step); break;
    case 5: hipLaunchKernelGGL(env_step_kernel<5>, grid, block, lds, s, p, st, actions, obs, reward, done, epb, (int)do_step); break;
    case 7: hipLaunchKernelGGL(env_step_kernel<7>, grid, block, lds, s, p, st, actions, obs, reward, done, epb, (int)do_step); break;
    default: return MARL_E_CONFIG;
  }
  return launch_status();
}

}  // namespace marl
