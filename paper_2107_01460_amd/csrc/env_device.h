// Device-side pieces of the two grid worlds (foraging, warehouse), shared by the standalone env-step kernels and by
// the fused rollout kernel: the new-episode draw, the lock-step transition of one env resolved redundantly in the
// registers of each of its agents' lanes, and the painting of a lane's egocentric window.
#pragma once
#include "common.h"

namespace marl {

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

// The draws of a new episode: draw j is word j % 4 of Philox call j / 4 of the stream (env, episode).
// SHARE = false: the lane computes every call itself.  SHARE = true: the A lanes of the env's agents (consecutive lanes
// of one wavefront, this one being agent a_idx, all of them in here together because the episode ended for the env)
// split the calls -- lane a computes calls a, a + A, ... -- and fetch the others' words across lanes: a call is forty
// quarter-rate multiplies, and every lane of an env computing all of them was a quarter of the env step's time.
template <int NC, bool SHARE>
struct ResetDraws {
  uint32_t buf[4];
  uint32_t mine[SHARE ? NC : 1][4];
  int j, A, base;
  uint32_t env, episode, k0, k1;
  __device__ __forceinline__ void init(const EnvParams& p, uint32_t env_, uint32_t episode_, int ncalls, int a_idx) {
    j = 0; A = p.A; env = env_; episode = episode_; k0 = p.k0; k1 = p.k1;
    buf[0] = buf[1] = buf[2] = buf[3] = 0;
    base = (int)(threadIdx.x & 63) - a_idx;
    if (SHARE) {
#pragma unroll
      for (int s = 0; s < NC; ++s) {
        mine[s][0] = mine[s][1] = mine[s][2] = mine[s][3] = 0;
        const int c = a_idx + s * A;
        if (c < ncalls) philox4x32_10(env, episode, (uint32_t)c, kStreamReset, k0, k1, mine[s]);
      }
    }
  }
  __device__ __forceinline__ uint32_t draw() {
    if ((j & 3) == 0) {
      const int c = j >> 2;
      if (SHARE) {
        int own = c, slot = 0;  // call c was computed by agent c % A as its call number c / A (uniform values)
#pragma unroll
        for (int q = 0; q < NC; ++q) {
          const bool more = own >= A;
          own -= more ? A : 0;
          slot += more ? 1 : 0;
        }
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          uint32_t v = mine[0][w];
#pragma unroll
          for (int s = 1; s < NC; ++s) v = (slot == s) ? mine[s][w] : v;
          buf[w] = (uint32_t)__shfl((int)v, base + own);
        }
      } else {
        philox4x32_10(env, episode, (uint32_t)c, kStreamReset, k0, k1, buf);
      }
    }
    const int w = j & 3;
    ++j;
    return w == 0 ? buf[0] : (w == 1 ? buf[1] : (w == 2 ? buf[2] : buf[3]));
  }
};

// New episode for one env, entirely in registers (every loop is unrolled over the at most 16 entities, so the
// arrays never leave the register file).  Draw order: A agent levels, A + F cells (agents first), F food levels;
// draw j is word j % 4 of Philox call j / 4 of the stream (env, episode).
template <int CA, int CF, bool SHARE = false>
__device__ __forceinline__ void reset_regs(uint32_t ag[CA], uint32_t fd[CF], const EnvParams& p,
                                           uint32_t env, uint32_t episode, int a_idx = 0) {
  constexpr int kMaxEnt = CA + CF;
  ResetDraws<(2 * kMaxEnt + 3) / 4, SHARE> rd;
  rd.init(p, env, episode, (2 * (p.A + p.F) + 3) >> 2, a_idx);
  auto draw = [&]() -> uint32_t { return rd.draw(); };
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
        if (k == a && a < p.A) ag[a] = cell | ((uint32_t)lvl[a] << 16);  // slots past A keep their off-grid marker
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

// The env's entities into registers.  All loads are issued branch-free (clamped indices) so that they are in flight
// together; entries past A / F and inactive lanes are masked afterwards (off-grid cells that never match a cell).
// (Indices are 32-bit: the entity arrays hold at most 8 N < 2^31 elements, and a uniform base plus a 32-bit lane offset
// is an address the hardware forms by itself, where a 64-bit index costs several instructions per access.)
template <int CA, int CF, int KIND>
__device__ __forceinline__ void load_env_state(uint32_t (&ag)[CA], uint32_t (&fd)[CF], const marl_env_state& st,
                                               const EnvParams& p, size_t nn, bool active) {
  const unsigned N = (unsigned)p.N, n = (unsigned)nn;
  uint32_t r8[CA], c8[CA], l8[CA], fr8[CF], fc8[CF], fl8[CF];
#pragma unroll
  for (int b = 0; b < CA; ++b) {
    const unsigned i = (unsigned)min(b, p.A - 1) * N + n;
    r8[b] = st.agent_row[i];
    c8[b] = st.agent_col[i];
    l8[b] = st.agent_lvl[i];
  }
#pragma unroll
  for (int f = 0; f < CF; ++f) {
    const unsigned i = (unsigned)min(f, p.F - 1) * N + n;
    fr8[f] = st.food_row[i];
    fc8[f] = st.food_col[i];
    fl8[f] = st.food_lvl[i];
  }
#pragma unroll
  for (int b = 0; b < CA; ++b) ag[b] = (active && b < p.A) ? (r8[b] | (c8[b] << 8) | (l8[b] << 16)) : 0xffffu;
#pragma unroll
  for (int f = 0; f < CF; ++f)  // foraging: level 0 = absent; warehouse: another off-grid cell, state 0
    fd[f] = (active && f < p.F) ? (fr8[f] | (fc8[f] << 8) | (fl8[f] << 16)) : (KIND == 0 ? 0xffffu : 0xfffeu);
}

// The state back to memory: every lane its own agent, the env's lanes share the food.  In the foraging world the
// levels and the food cells change only when a new episode starts (dn).
template <int CA, int CF, int KIND>
__device__ __forceinline__ void store_env_state(const uint32_t (&ag)[CA], const uint32_t (&fd)[CF], const marl_env_state& st,
                                                const EnvParams& p, size_t n_, int a, bool dn, int t, uint32_t episode) {
  const unsigned N = (unsigned)p.N, n = (unsigned)n_;
  const bool all = dn || KIND != 0;
  uint32_t me = 0;
#pragma unroll
  for (int b = 0; b < CA; ++b) me = (b == a) ? ag[b] : me;
  const unsigned ia = (unsigned)a * N + n;
  st.agent_row[ia] = (uint8_t)e_row(me);
  st.agent_col[ia] = (uint8_t)e_col(me);
  if (all) st.agent_lvl[ia] = (uint8_t)e_lvl(me);
#pragma unroll
  for (int f = 0; f < CF; ++f)
    if (f < p.F && (f % p.A) == a) {
      const unsigned i = (unsigned)f * N + n;
      st.food_lvl[i] = (uint8_t)e_lvl(fd[f]);
      if (all) {
        st.food_row[i] = (uint8_t)e_row(fd[f]);
        st.food_col[i] = (uint8_t)e_col(fd[f]);
      }
    }
  if (a == 0) {
    st.t_in_ep[n] = t;
    st.episode_id[n] = episode;
  }
}

// One transition of the foraging world for the lane of agent `a` of env `env`: act[] holds the actions of all agents of
// the env, ag / fd the start-of-step entities.  Leaves the post-step (after an auto-reset: the new episode's) entities,
// step count and episode id in place; rew = this agent's reward, dn = the env finished its episode in this step.
template <int CA, int CF>
__device__ __forceinline__ void forage_transition(uint32_t (&ag)[CA], uint32_t (&fd)[CF], const int (&act)[CA], int a,
                                                  bool active, const EnvParams& p, uint32_t env, int& t,
                                                  uint32_t& episode, float& rew_out, bool& dn_out) {
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
  const bool dn = active && (!any_food || t == p.cap);
  // ---- auto-reset: every lane of a finished env re-seeds it in its own registers (same result in each)
  if (dn) {
    episode += 1;
    reset_regs<CA, CF, true>(ag, fd, p, env, episode, a);
    t = 0;
  }
  rew_out = rew;
  dn_out = dn;
}

// The lane's V x V x 3 window into w[0 .. 3 V V): walls and zeros first, then the entities that fall inside it.
template <int V, int CA, int CF>
__device__ __forceinline__ void forage_paint(float* w, const uint32_t (&ag)[CA], const uint32_t (&fd)[CF], int a,
                                             const EnvParams& p) {
  constexpr int h = (V - 1) / 2;
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

__device__ __forceinline__ bool wh_goal(int G, int r, int c) { return r == G - 1 && (c == G / 2 - 1 || c == G / 2); }

// New episode: A + F distinct cells (robots first), then L requested shelves.  Draw j is word j % 4 of Philox
// call j / 4 of the stream (env, episode).
template <int CA, int CF, bool SHARE = false>
__device__ __forceinline__ void wh_reset_regs(uint32_t ag[CA], uint32_t fd[CF], const EnvParams& p, uint32_t env,
                                              uint32_t episode, int a_idx = 0) {
  constexpr int kMaxEnt = CA + CF;
  ResetDraws<(kMaxEnt + CF + 3) / 4, SHARE> rd;
  rd.init(p, env, episode, (p.A + p.F + p.L + 3) >> 2, a_idx);
  auto draw = [&]() -> uint32_t { return rd.draw(); };
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
        if (k == a && a < p.A) ag[a] = cell;  // nothing carried; slots past A keep their off-grid marker
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

// One transition of the warehouse world, arguments as forage_transition.
template <int CA, int CF>
__device__ __forceinline__ void wh_transition(uint32_t (&ag)[CA], uint32_t (&fd)[CF], const int (&act)[CA], int a,
                                              bool active, const EnvParams& p, uint32_t env, int& t, uint32_t& episode,
                                              float& rew_out, bool& dn_out) {
  const uint32_t n = env;
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
  if (dn) {
    episode += 1;
    wh_reset_regs<CA, CF, true>(ag, fd, p, env, episode, a);
    t = 0;
  }
  rew_out = rew;
  dn_out = dn;
}

template <int V, int CA, int CF>
__device__ __forceinline__ void wh_paint(float* w, const uint32_t (&ag)[CA], const uint32_t (&fd)[CF], int a,
                                         const EnvParams& p) {
  constexpr int h = (V - 1) / 2;
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

inline EnvParams env_params(const marl_config& c) {
  EnvParams p;
  p.G = c.grid; p.A = c.n_agents; p.F = c.n_food; p.L = c.max_level; p.cap = c.episode_cap; p.N = c.n_envs;
  p.kind = c.env_kind;
  p.k0 = (uint32_t)(c.seed & 0xffffffffu);
  p.k1 = (uint32_t)(c.seed >> 32);
  p.inv_g20 = ((1u << 20) + (uint32_t)c.grid - 1u) / (uint32_t)c.grid;
  return p;
}

}  // namespace marl
