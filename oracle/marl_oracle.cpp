// CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, single-threaded reference of the fused multi-agent PPO training step
// (vectorised grid-foraging environments -> parameter-shared actor/critic MLP ->
// Gumbel-max sampling -> GAE -> clipped-PPO minibatch update with Adam) that the paper's
// Fig. 2 ("Anakin" update function: roll out N environment copies, feed the experience to
// a loss, take the gradient, produce new parameters) and Section 2 (feed-forward IPPO with
// decentralised critics, MAPPO with a centralised critic) describe structurally.
//
// Only tests, the smoke check and the benchmark's cpu_baseline leg may call this code.
// It shares nothing with the HIP library: no header, no table, no helper.  It never
// includes or links anything from the product package.
//
// Arithmetic: the environment is integer-only except for the reward (IEEE fp32, one
// division per loader and food, accumulated in ascending food index).  All network, loss,
// GAE and optimiser arithmetic is carried out in fp64 and rounded to fp32 only where a
// result is stored in an fp32 buffer.  The bf16 configuration rounds the weights to bf16
// (precision 1) and, in a second mode (precision 2, oracle only), also the inputs of every
// matrix product where the method rounds them; see mlp_forward.
//
// Parity status of each function is listed in tests/test_oracle_*.py; every function here
// has at least one pin that is not itself (known-answer vectors for Philox, hand-built
// grids and a brute-force set-based stepper for the environment, brute-force discounted
// sums for GAE, finite differences and float64 autograd for the loss gradients,
// torch.optim.Adam for the optimiser; closed forms and a step-by-step restatement for the
// evaluation block; torch's GRUCell, float64 autograd through time and the feed-forward
// special case for the recurrent networks; hand-built cases, invariants and an
// independent set-based restatement for the warehouse world).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <vector>

extern "C" {

typedef struct orc_config {
  int32_t grid, n_agents, n_food, max_level, episode_cap, view;
  int32_t n_envs, rollout_len;
  int32_t actor_hidden, critic_hidden, central_critic, precision;
  int32_t n_epochs, n_minibatches, normalize_adv, clip_value;
  float gamma, lambda, clip_eps, ent_coef, vf_coef, max_grad_norm;
  float lr, beta1, beta2, adam_eps;
  uint64_t seed;
  int32_t recurrent;  // 0: feed-forward networks; 1: a GRU cell in place of the second hidden layer
  int32_t env_kind;   // 0: foraging world; 1: warehouse world; 2: warehouse world whose episodes end on a collision
} orc_config;

// Environment state, structure of arrays, entity-major: x[e * n_envs + env].
typedef struct orc_env_state {
  uint8_t *agent_row, *agent_col, *agent_lvl;  // [A][N]
  uint8_t *food_row, *food_col, *food_lvl;     // [F][N]   (lvl 0 = already collected)
  int32_t* t_in_ep;                            // [N]
  uint32_t* episode_id;                        // [N]
} orc_env_state;

// Trajectory, time-major.
typedef struct orc_traj {
  float* obs;         // [T+1][N][A][D]   slab t = observation the action of step t was taken on
  int32_t* action;    // [T][N][A]
  float* logp;        // [T][N][A]
  float* value;       // [T][N][A]        (centralised critic: one value per env, broadcast over A)
  float* reward;      // [T][N][A]
  uint8_t* done;      // [T][N]
  float* last_value;  // [N][A]
  float* adv;         // [T][N][A]
  float* ret;         // [T][N][A]
  float* logits;      // nullable [T][N][A][6]
  int32_t* sampled;   // nullable [T][N][A]  action the sampler drew (differs from action only when forced)
  float* gap;         // nullable [T][N][A]  top-two gap of the Gumbel-perturbed logits (fp64 -> fp32)
} orc_traj;

// Hidden states of the recurrent networks around one rollout: h0 = state the rollout starts from (already
// zeroed where the previous step ended an episode), h1 = the same for the next rollout.
typedef struct orc_rec_state {
  float *ha0, *hc0;  // [N][A][Ha];  [N][A][Hc] (decentralised critic) or [N][Hc] (centralised)
  float *ha1, *hc1;
} orc_rec_state;

}  // extern "C"

namespace {

constexpr int kActions = 6;

// ---------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
// SC'11, Section 4 and Table 2): ten rounds of two 32x32->64 multiplications whose high
// halves are xored with the other counter words and the round key; the key is bumped by
// the Weyl constants between rounds.
// ---------------------------------------------------------------------------------------
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)M0 * c0;
    const uint64_t p1 = (uint64_t)M1 * c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n1 = lo1;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    const uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += W0; k1 += W1;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Integer in [0, n) by multiply-high.
inline uint32_t rand_below(uint32_t x, uint32_t n) { return (uint32_t)(((uint64_t)x * n) >> 32); }

// Uniform in the open interval (0,1): the top 23 bits, centred in their bucket.
inline float rand_unit(uint32_t x) { return ((float)(x >> 9) + 0.5f) * (1.0f / 8388608.0f); }

enum : uint32_t { kStreamReset = 1, kStreamSample = 2, kStreamRequest = 3 };

// j-th 32-bit draw of the reset stream of (env, episode).
struct ResetDraws {
  uint32_t key[2];
  uint32_t env, episode;
  uint32_t buf[4];
  int have_call = -1;
  uint32_t get(int j) {
    const int call = j >> 2;
    if (call != have_call) {
      const uint32_t ctr[4] = {env, episode, (uint32_t)call, kStreamReset};
      philox4x32_10(ctr, key, buf);
      have_call = call;
    }
    return buf[j & 3];
  }
};

struct Dims {
  int G, A, F, V, D, N, T, Ha, Hc, Dc, Pa, Pc, P;
  bool central;
  bool round_act;  // precision 2: the inputs of every matrix product are rounded to bf16 (see mlp_forward)
};

Dims dims_of(const orc_config& c) {
  Dims d;
  d.G = c.grid; d.A = c.n_agents; d.F = c.n_food; d.V = c.view; d.D = 3 * c.view * c.view;
  d.N = c.n_envs; d.T = c.rollout_len; d.Ha = c.actor_hidden; d.Hc = c.critic_hidden;
  d.central = c.central_critic != 0;
  d.round_act = c.precision == 2;
  d.Dc = d.central ? d.A * d.D : d.D;
  d.Pa = d.D * d.Ha + d.Ha + d.Ha * d.Ha + d.Ha + d.Ha * kActions + kActions;
  d.Pc = d.Dc * d.Hc + d.Hc + d.Hc * d.Hc + d.Hc + d.Hc + 1;
  if (c.recurrent) {  // embedding, GRU cell (input and hidden weights of three gates), output layer
    d.Pa = d.D * d.Ha + d.Ha + 2 * (d.Ha * 3 * d.Ha + 3 * d.Ha) + d.Ha * kActions + kActions;
    d.Pc = d.Dc * d.Hc + d.Hc + 2 * (d.Hc * 3 * d.Hc + 3 * d.Hc) + d.Hc + 1;
  }
  d.P = d.Pa + d.Pc;
  return d;
}

// ---------------------------------------------------------------------------------------
// Environment
// ---------------------------------------------------------------------------------------

void wh_reset_one(const orc_config& c, const orc_env_state& s, int env);
void wh_step_one(const orc_config& c, const orc_env_state& s, int env, const int32_t* actions, float* reward, uint8_t* done);
void wh_observe_one(const orc_config& c, const orc_env_state& s, int env, float* obs);

// New episode for one env: levels, then A+F distinct cells, then food levels.
void reset_one(const orc_config& c, const orc_env_state& s, int env) {
  if (c.env_kind != 0) return wh_reset_one(c, s, env);
  const Dims d = dims_of(c);
  ResetDraws rng;
  rng.key[0] = (uint32_t)(c.seed & 0xffffffffu);
  rng.key[1] = (uint32_t)(c.seed >> 32);
  rng.env = (uint32_t)env;
  rng.episode = s.episode_id[env];
  int j = 0;
  std::vector<int> lv(d.A);
  for (int a = 0; a < d.A; ++a) {
    lv[a] = 1 + (int)rand_below(rng.get(j++), (uint32_t)c.max_level);
    s.agent_lvl[a * d.N + env] = (uint8_t)lv[a];
  }
  // Cells without replacement: the j-th entity draws r in [0, G*G - j) and takes the r-th
  // free cell in ascending cell order.
  std::vector<int> chosen;  // kept sorted ascending
  for (int e = 0; e < d.A + d.F; ++e) {
    int r = (int)rand_below(rng.get(j++), (uint32_t)(d.G * d.G - e));
    for (size_t q = 0; q < chosen.size(); ++q)
      if (chosen[q] <= r) ++r;
    chosen.insert(std::upper_bound(chosen.begin(), chosen.end(), r), r);
    const uint8_t row = (uint8_t)(r / d.G), col = (uint8_t)(r % d.G);
    if (e < d.A) {
      s.agent_row[e * d.N + env] = row;
      s.agent_col[e * d.N + env] = col;
    } else {
      s.food_row[(e - d.A) * d.N + env] = row;
      s.food_col[(e - d.A) * d.N + env] = col;
    }
  }
  // Food level in 1..Lsum, Lsum = summed level of the (at most four) strongest agents:
  // at most four agents can stand next to one food.
  std::vector<int> sorted = lv;
  std::sort(sorted.begin(), sorted.end(), [](int x, int y) { return x > y; });
  int lsum = 0;
  for (int a = 0; a < std::min(d.A, 4); ++a) lsum += sorted[a];
  for (int f = 0; f < d.F; ++f)
    s.food_lvl[f * d.N + env] = (uint8_t)(1 + rand_below(rng.get(j++), (uint32_t)lsum));
  s.t_in_ep[env] = 0;
}

// One env, one step; actions[a]; writes reward[a] and *done; auto-resets.
void step_one(const orc_config& c, const orc_env_state& s, int env, const int32_t* actions,
              float* reward, uint8_t* done) {
  if (c.env_kind != 0) return wh_step_one(c, s, env, actions, reward, done);
  const Dims d = dims_of(c);
  const int N = d.N;
  std::vector<int> r0(d.A), c0(d.A), tr(d.A), tc(d.A);
  std::vector<char> moves(d.A, 0);
  for (int a = 0; a < d.A; ++a) {
    r0[a] = s.agent_row[a * N + env];
    c0[a] = s.agent_col[a * N + env];
  }
  // 1. targets against the start-of-step state
  for (int a = 0; a < d.A; ++a) {
    int nr = r0[a], nc = c0[a];
    switch (actions[a]) {
      case 1: nr -= 1; break;  // north
      case 2: nr += 1; break;  // south
      case 3: nc -= 1; break;  // west
      case 4: nc += 1; break;  // east
      default: break;          // 0 noop, 5 load
    }
    bool ok = (nr != r0[a] || nc != c0[a]) && nr >= 0 && nr < d.G && nc >= 0 && nc < d.G;
    if (ok)
      for (int b = 0; b < d.A; ++b)
        if (r0[b] == nr && c0[b] == nc) ok = false;
    if (ok)
      for (int f = 0; f < d.F; ++f)
        if (s.food_lvl[f * N + env] != 0 && s.food_row[f * N + env] == nr &&
            s.food_col[f * N + env] == nc)
          ok = false;
    moves[a] = ok;
    tr[a] = ok ? nr : r0[a];
    tc[a] = ok ? nc : c0[a];
  }
  // 2. two or more valid movers onto one cell all stay
  std::vector<char> blocked(d.A, 0);
  for (int a = 0; a < d.A; ++a)
    for (int b = 0; b < d.A; ++b)
      if (a != b && moves[a] && moves[b] && tr[a] == tr[b] && tc[a] == tc[b]) blocked[a] = 1;
  // 3. loading (positions at start of step; loaders do not move)
  for (int a = 0; a < d.A; ++a) reward[a] = 0.0f;
  for (int f = 0; f < d.F; ++f) {
    const int fl = s.food_lvl[f * N + env];
    if (fl == 0) continue;
    const int fr = s.food_row[f * N + env], fc = s.food_col[f * N + env];
    int lsum = 0;
    std::vector<char> loader(d.A, 0);
    for (int a = 0; a < d.A; ++a) {
      const int dist = std::abs(r0[a] - fr) + std::abs(c0[a] - fc);
      if (actions[a] == 5 && dist == 1) {
        loader[a] = 1;
        lsum += s.agent_lvl[a * N + env];
      }
    }
    if (lsum >= fl) {  // lsum >= 1 follows since fl >= 1
      for (int a = 0; a < d.A; ++a)
        if (loader[a])
          reward[a] += (float)(fl * (int)s.agent_lvl[a * N + env]) / (float)lsum;
      s.food_lvl[f * N + env] = 0;
    }
  }
  // commit movement
  for (int a = 0; a < d.A; ++a) {
    if (moves[a] && !blocked[a]) {
      s.agent_row[a * N + env] = (uint8_t)tr[a];
      s.agent_col[a * N + env] = (uint8_t)tc[a];
    }
  }
  // 4. termination
  s.t_in_ep[env] += 1;
  bool any_food = false;
  for (int f = 0; f < d.F; ++f) any_food |= (s.food_lvl[f * N + env] != 0);
  const bool dn = !any_food || s.t_in_ep[env] == c.episode_cap;
  *done = dn ? 1 : 0;
  // 5. auto-reset
  if (dn) {
    s.episode_id[env] += 1;
    reset_one(c, s, env);
  }
}

// Egocentric V x V x 3 view of every agent of one env: (agent level, food level, wall).
void observe_one(const orc_config& c, const orc_env_state& s, int env, float* obs /*[A][D]*/) {
  if (c.env_kind != 0) return wh_observe_one(c, s, env, obs);
  const Dims d = dims_of(c);
  const int N = d.N, h = (d.V - 1) / 2;
  for (int a = 0; a < d.A; ++a) {
    const int r = s.agent_row[a * N + env], col = s.agent_col[a * N + env];
    float* o = obs + (size_t)a * d.D;
    for (int dy = -h; dy <= h; ++dy)
      for (int dx = -h; dx <= h; ++dx) {
        const int rr = r + dy, cc = col + dx;
        float al = 0.f, fl = 0.f, wall = 0.f;
        if (rr < 0 || rr >= d.G || cc < 0 || cc >= d.G) {
          wall = 1.f;
        } else {
          for (int b = 0; b < d.A; ++b)
            if (s.agent_row[b * N + env] == rr && s.agent_col[b * N + env] == cc)
              al = (float)s.agent_lvl[b * N + env];
          for (int f = 0; f < d.F; ++f)
            if (s.food_lvl[f * N + env] != 0 && s.food_row[f * N + env] == rr &&
                s.food_col[f * N + env] == cc)
              fl = (float)s.food_lvl[f * N + env];
        }
        const int cell = (dy + h) * d.V + (dx + h);
        o[cell * 3 + 0] = al;
        o[cell * 3 + 1] = fl;
        o[cell * 3 + 2] = wall;
      }
  }
}

// ---------------------------------------------------------------------------------------
// Warehouse world (a second grid workload in the spirit of the multi-robot warehouse task the paper trains on in
// Section 4; the paper gives no rules, and says only that the variant it uses ends the episode on collisions and
// that it reports results with and without that feature.  The rules below are this build's own.)
//
// The same buffers as the foraging world: A robots (agent_row / agent_col), F shelves (food_row / food_col).
// agent_lvl[a] = 0 when robot a carries nothing, else 1 + the index of the shelf it carries; food_lvl[f] = 1 for an
// idle shelf, 2 for a requested one.  R = max_level shelves are requested at any time.  The two goal cells are
// (G-1, G/2 - 1) and (G-1, G/2).
//   Reset: A + F distinct cells as in the foraging world (robots first), then R distinct requested shelves: the
//   j-th request draws r in [0, F - j) and takes the r-th idle shelf in ascending index.  Nothing is carried.
//   Step (actions 0 stay, 1 north, 2 south, 3 west, 4 east, 5 toggle), against the start-of-step state:
//   1. a move is valid iff its target is inside the grid, holds no robot, and -- for a loaded robot -- holds no
//      shelf (a loaded robot's own shelf travels with it; unloaded robots pass under shelves);
//   2. two or more valid movers onto one cell all stay;
//   3. a robot whose in-grid move was refused because of another robot (occupied or contested cell) has collided;
//   4. movers move, carried shelves with them;
//   5. toggle: a loaded robot puts its shelf down; an unloaded robot standing on a shelf that nobody carries picks
//      it up;
//   6. delivery, robots in ascending index: a robot carrying a requested shelf on a goal cell earns 1.0, the shelf
//      becomes idle, and one idle shelf other than the delivered one (the delivered one if there is no other)
//      becomes requested: candidate r in ascending index, r = multiply-high of the candidate count with word
//      (ordinal of the delivery in the step) % 4 of Philox counter (env, episode, 2 * steps taken in the episode
//      before this one + ordinal / 4, stream 3);
//   7. the episode ends at the cap, and in kind 2 also when any robot collided; then auto-reset.
//   Observation: the same V x V x 3 window; channel 0: 0 / 1 unloaded robot / 2 loaded robot; channel 1: 0 / 1 idle
//   shelf / 2 requested shelf; channel 2: 1 outside the grid, 0.5 on a goal cell, else 0.
// ---------------------------------------------------------------------------------------
inline bool wh_is_goal(int G, int r, int col) { return r == G - 1 && (col == G / 2 - 1 || col == G / 2); }

void wh_reset_one(const orc_config& c, const orc_env_state& s, int env) {
  const Dims d = dims_of(c);
  ResetDraws rng;
  rng.key[0] = (uint32_t)(c.seed & 0xffffffffu);
  rng.key[1] = (uint32_t)(c.seed >> 32);
  rng.env = (uint32_t)env;
  rng.episode = s.episode_id[env];
  int j = 0;
  std::vector<int> chosen;  // kept sorted ascending
  for (int e = 0; e < d.A + d.F; ++e) {
    int r = (int)rand_below(rng.get(j++), (uint32_t)(d.G * d.G - e));
    for (size_t q = 0; q < chosen.size(); ++q)
      if (chosen[q] <= r) ++r;
    chosen.insert(std::upper_bound(chosen.begin(), chosen.end(), r), r);
    const uint8_t row = (uint8_t)(r / d.G), col = (uint8_t)(r % d.G);
    if (e < d.A) {
      s.agent_row[e * d.N + env] = row;
      s.agent_col[e * d.N + env] = col;
      s.agent_lvl[e * d.N + env] = 0;
    } else {
      s.food_row[(e - d.A) * d.N + env] = row;
      s.food_col[(e - d.A) * d.N + env] = col;
      s.food_lvl[(e - d.A) * d.N + env] = 1;
    }
  }
  for (int q = 0; q < c.max_level; ++q) {
    int r = (int)rand_below(rng.get(j++), (uint32_t)(d.F - q));
    for (int f = 0; f < d.F; ++f)
      if (s.food_lvl[f * d.N + env] == 1 && r-- == 0) {
        s.food_lvl[f * d.N + env] = 2;
        break;
      }
  }
  s.t_in_ep[env] = 0;
}

void wh_step_one(const orc_config& c, const orc_env_state& s, int env, const int32_t* actions, float* reward,
                 uint8_t* done) {
  const Dims d = dims_of(c);
  const int N = d.N;
  std::vector<int> r0(d.A), c0(d.A), carry(d.A), tr(d.A), tc(d.A);
  std::vector<char> moves(d.A, 0), robot_refused(d.A, 0);
  for (int a = 0; a < d.A; ++a) {
    r0[a] = s.agent_row[a * N + env];
    c0[a] = s.agent_col[a * N + env];
    carry[a] = s.agent_lvl[a * N + env];
  }
  // 1. targets against the start-of-step state
  for (int a = 0; a < d.A; ++a) {
    int nr = r0[a], nc = c0[a];
    switch (actions[a]) {
      case 1: nr -= 1; break;
      case 2: nr += 1; break;
      case 3: nc -= 1; break;
      case 4: nc += 1; break;
      default: break;
    }
    const bool wants = (nr != r0[a] || nc != c0[a]) && nr >= 0 && nr < d.G && nc >= 0 && nc < d.G;
    bool ok = wants;
    if (ok)
      for (int b = 0; b < d.A; ++b)
        if (r0[b] == nr && c0[b] == nc) {
          ok = false;
          robot_refused[a] = 1;
        }
    if (ok && carry[a] != 0)
      for (int f = 0; f < d.F; ++f)
        if (s.food_row[f * N + env] == nr && s.food_col[f * N + env] == nc) ok = false;
    moves[a] = ok;
    tr[a] = ok ? nr : r0[a];
    tc[a] = ok ? nc : c0[a];
  }
  // 2. contested cells
  std::vector<char> blocked(d.A, 0);
  for (int a = 0; a < d.A; ++a)
    for (int b = 0; b < d.A; ++b)
      if (a != b && moves[a] && moves[b] && tr[a] == tr[b] && tc[a] == tc[b]) blocked[a] = 1;
  // 3. collisions
  bool collided = false;
  for (int a = 0; a < d.A; ++a) collided |= robot_refused[a] || blocked[a];
  // 4. movement, carried shelves with their robots
  for (int a = 0; a < d.A; ++a)
    if (moves[a] && !blocked[a]) {
      s.agent_row[a * N + env] = (uint8_t)tr[a];
      s.agent_col[a * N + env] = (uint8_t)tc[a];
      if (carry[a] != 0) {
        s.food_row[(carry[a] - 1) * N + env] = (uint8_t)tr[a];
        s.food_col[(carry[a] - 1) * N + env] = (uint8_t)tc[a];
      }
    }
  // 5. toggle (togglers have not moved)
  for (int a = 0; a < d.A; ++a) {
    if (actions[a] != 5) continue;
    if (carry[a] != 0) {
      s.agent_lvl[a * N + env] = 0;
    } else {
      for (int f = 0; f < d.F; ++f) {
        if (s.food_row[f * N + env] != r0[a] || s.food_col[f * N + env] != c0[a]) continue;
        bool carried = false;
        for (int b = 0; b < d.A; ++b) carried |= (carry[b] == f + 1);
        if (!carried) s.agent_lvl[a * N + env] = (uint8_t)(f + 1);
      }
    }
  }
  // 6. delivery
  for (int a = 0; a < d.A; ++a) reward[a] = 0.0f;
  uint32_t words[4] = {0, 0, 0, 0};
  int have_call = -1;  // Philox call the words belong to: deliveries 4 q .. 4 q + 3 of the step use call q
  int ordinal = 0;
  for (int a = 0; a < d.A; ++a) {
    const int cy = s.agent_lvl[a * N + env];
    if (cy == 0) continue;
    const int f = cy - 1;
    if (s.food_lvl[f * N + env] != 2) continue;
    if (!wh_is_goal(d.G, s.agent_row[a * N + env], s.agent_col[a * N + env])) continue;
    reward[a] = 1.0f;
    s.food_lvl[f * N + env] = 1;
    int n_cand = 0;
    for (int g = 0; g < d.F; ++g) n_cand += (g != f && s.food_lvl[g * N + env] == 1);
    const int call = ordinal >> 2;
    if (call != have_call) {
      const uint32_t key[2] = {(uint32_t)(c.seed & 0xffffffffu), (uint32_t)(c.seed >> 32)};
      const uint32_t ctr[4] = {(uint32_t)env, s.episode_id[env], (uint32_t)s.t_in_ep[env] * 2u + (uint32_t)call, kStreamRequest};
      philox4x32_10(ctr, key, words);
      have_call = call;
    }
    if (n_cand == 0) {
      s.food_lvl[f * N + env] = 2;
    } else {
      int r = (int)rand_below(words[ordinal & 3], (uint32_t)n_cand);
      for (int g = 0; g < d.F; ++g)
        if (g != f && s.food_lvl[g * N + env] == 1 && r-- == 0) {
          s.food_lvl[g * N + env] = 2;
          break;
        }
    }
    ++ordinal;
  }
  // 7. termination and auto-reset
  s.t_in_ep[env] += 1;
  const bool dn = s.t_in_ep[env] == c.episode_cap || (c.env_kind == 2 && collided);
  *done = dn ? 1 : 0;
  if (dn) {
    s.episode_id[env] += 1;
    reset_one(c, s, env);
  }
}

void wh_observe_one(const orc_config& c, const orc_env_state& s, int env, float* obs /*[A][D]*/) {
  const Dims d = dims_of(c);
  const int N = d.N, h = (d.V - 1) / 2;
  for (int a = 0; a < d.A; ++a) {
    const int r = s.agent_row[a * N + env], col = s.agent_col[a * N + env];
    float* o = obs + (size_t)a * d.D;
    for (int dy = -h; dy <= h; ++dy)
      for (int dx = -h; dx <= h; ++dx) {
        const int rr = r + dy, cc = col + dx;
        float robot = 0.f, shelf = 0.f, ground = 0.f;
        if (rr < 0 || rr >= d.G || cc < 0 || cc >= d.G) {
          ground = 1.f;
        } else {
          if (wh_is_goal(d.G, rr, cc)) ground = 0.5f;
          for (int b = 0; b < d.A; ++b)
            if (s.agent_row[b * N + env] == rr && s.agent_col[b * N + env] == cc)
              robot = s.agent_lvl[b * N + env] != 0 ? 2.f : 1.f;
          for (int f = 0; f < d.F; ++f)
            if (s.food_row[f * N + env] == rr && s.food_col[f * N + env] == cc)
              shelf = std::max(shelf, (float)s.food_lvl[f * N + env]);
        }
        const int cell = (dy + h) * d.V + (dx + h);
        o[cell * 3 + 0] = robot;
        o[cell * 3 + 1] = shelf;
        o[cell * 3 + 2] = ground;
      }
  }
}

// ---------------------------------------------------------------------------------------
// Networks (fp64).  y = x W + b, W row-major [in][out].
// ---------------------------------------------------------------------------------------
struct Net {
  int Din, H, Dout;
  const double *W1, *b1, *W2, *b2, *W3, *b3;
  bool round_act;
};
struct NetGrad {
  double *W1, *b1, *W2, *b2, *W3, *b3;
};

Net net_at(const double* p, int Din, int H, int Dout, bool round_act) {
  Net n{Din, H, Dout, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, round_act};
  n.W1 = p; p += (size_t)Din * H;
  n.b1 = p; p += H;
  n.W2 = p; p += (size_t)H * H;
  n.b2 = p; p += H;
  n.W3 = p; p += (size_t)H * Dout;
  n.b3 = p;
  return n;
}
NetGrad grad_at(double* p, int Din, int H, int Dout) {
  NetGrad n;
  n.W1 = p; p += (size_t)Din * H;
  n.b1 = p; p += H;
  n.W2 = p; p += (size_t)H * H;
  n.b2 = p; p += H;
  n.W3 = p; p += (size_t)H * Dout;
  n.b3 = p;
  return n;
}

// Round-to-nearest-even to bfloat16, returned as fp32.
float round_bf16(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return x;  // inf / nan unchanged
  const uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  float y;
  std::memcpy(&y, &u, 4);
  return y;
}

// Parameters as the networks see them: fp32 master widened to fp64; in the bf16
// configuration (precision 1 and 2) every weight and bias is first rounded to bf16.
std::vector<double> effective_params(const orc_config& c, const float* params) {
  const Dims d = dims_of(c);
  std::vector<double> p(d.P);
  for (int i = 0; i < d.P; ++i) p[i] = c.precision >= 1 ? (double)round_bf16(params[i]) : (double)params[i];
  return p;
}

// The bf16 configuration of the workload list ("bf16 weights and activations with fp32 accumulation") has two
// oracle modes.  precision 1 rounds the weights only and evaluates everything else exactly: the error of the
// activation rounding is then what a comparison measures.  precision 2 also rounds every INPUT of a matrix product
// to bf16 (round to nearest even, via fp32) where the method does: the hidden activations h1 and h2 after the tanh,
// and in the backward pass dz2 and dz1, the gradients with respect to the pre-activations; tanh' is taken from the
// rounded activation, the bias gradients are sums of the rounded dz, and the sums themselves stay exact.  (The
// observations are small integers and halves, which bf16 holds exactly.)
inline double act_round(const Net& n, double v) { return n.round_act ? (double)round_bf16((float)v) : v; }

void mlp_forward(const Net& n, const double* x, double* h1, double* h2, double* out) {
  for (int j = 0; j < n.H; ++j) {
    double acc = n.b1[j];
    for (int i = 0; i < n.Din; ++i) acc += x[i] * n.W1[(size_t)i * n.H + j];
    h1[j] = act_round(n, std::tanh(acc));
  }
  for (int j = 0; j < n.H; ++j) {
    double acc = n.b2[j];
    for (int i = 0; i < n.H; ++i) acc += h1[i] * n.W2[(size_t)i * n.H + j];
    h2[j] = act_round(n, std::tanh(acc));
  }
  for (int k = 0; k < n.Dout; ++k) {
    double acc = n.b3[k];
    for (int i = 0; i < n.H; ++i) acc += h2[i] * n.W3[(size_t)i * n.Dout + k];
    out[k] = acc;
  }
}

// Accumulates parameter gradients for one sample given dL/dout.
void mlp_backward(const Net& n, const NetGrad& g, const double* x, const double* h1, const double* h2,
                  const double* dout, double* dz1, double* dz2) {
  for (int i = 0; i < n.H; ++i) {
    double acc = 0;
    for (int k = 0; k < n.Dout; ++k) {
      acc += dout[k] * n.W3[(size_t)i * n.Dout + k];
      g.W3[(size_t)i * n.Dout + k] += h2[i] * dout[k];
    }
    dz2[i] = act_round(n, acc * (1.0 - h2[i] * h2[i]));
  }
  for (int k = 0; k < n.Dout; ++k) g.b3[k] += dout[k];
  for (int i = 0; i < n.H; ++i) {
    double acc = 0;
    for (int j = 0; j < n.H; ++j) {
      acc += dz2[j] * n.W2[(size_t)i * n.H + j];
      g.W2[(size_t)i * n.H + j] += h1[i] * dz2[j];
    }
    dz1[i] = act_round(n, acc * (1.0 - h1[i] * h1[i]));
  }
  for (int j = 0; j < n.H; ++j) g.b2[j] += dz2[j];
  for (int i = 0; i < n.Din; ++i)
    for (int j = 0; j < n.H; ++j) g.W1[(size_t)i * n.H + j] += x[i] * dz1[j];
  for (int j = 0; j < n.H; ++j) g.b1[j] += dz1[j];
}

// logits / value of every agent of one (t,n) row.  obs_row = [A][D] fp32.
void policy_row(const Dims& d, const double* p, const float* obs_row, double* logits /*[A][6]*/,
                double* value /*[A]*/) {
  const Net actor = net_at(p, d.D, d.Ha, kActions, d.round_act);
  const Net critic = net_at(p + d.Pa, d.Dc, d.Hc, 1, d.round_act);
  std::vector<double> x(std::max(d.D, d.Dc)), h1(std::max(d.Ha, d.Hc)), h2(std::max(d.Ha, d.Hc));
  for (int a = 0; a < d.A; ++a) {
    for (int i = 0; i < d.D; ++i) x[i] = obs_row[(size_t)a * d.D + i];
    if (logits) mlp_forward(actor, x.data(), h1.data(), h2.data(), logits + (size_t)a * kActions);
    if (value && !d.central) mlp_forward(critic, x.data(), h1.data(), h2.data(), value + a);
  }
  if (value && d.central) {
    for (int i = 0; i < d.Dc; ++i) x[i] = obs_row[i];  // concatenation over agents = the contiguous row
    double v;
    mlp_forward(critic, x.data(), h1.data(), h2.data(), &v);
    for (int a = 0; a < d.A; ++a) value[a] = v;
  }
}

// Gumbel-max sample from fp32 logits and fp32 uniforms; log-prob of a given action.
void sample_one(const float* logits, const float* u, int32_t* action, float* gap) {
  double best = -INFINITY, second = -INFINITY;
  int arg = 0;
  for (int k = 0; k < kActions; ++k) {
    const double g = -std::log(-std::log((double)u[k]));
    const double z = (double)logits[k] + g;
    if (z > best) {  // strict: lowest index wins exact ties
      second = best;
      best = z;
      arg = k;
    } else if (z > second) {
      second = z;
    }
  }
  *action = arg;
  if (gap) *gap = (float)(best - second);
}

double log_prob(const double* logits, int a) {
  double m = logits[0];
  for (int k = 1; k < kActions; ++k) m = std::max(m, logits[k]);
  double s = 0;
  for (int k = 0; k < kActions; ++k) s += std::exp(logits[k] - m);
  return logits[a] - m - std::log(s);
}

// ---------------------------------------------------------------------------------------
// PPO minibatch: loss and gradient (fp64) over the rows [rows, rows + n_rows).
// ---------------------------------------------------------------------------------------
struct MbStats {
  double pi_loss, v_loss, entropy, approx_kl, clip_frac, total;
};

MbStats minibatch_loss_grad(const orc_config& c, const orc_traj& tr, const double* p, const int32_t* rows,
                            int n_rows, double* grad /*nullable [P], overwritten*/) {
  const Dims d = dims_of(c);
  const double B = (double)n_rows * d.A;
  // advantage normalisation over the minibatch (population std)
  double mean = 0, stdv = 1;
  if (c.normalize_adv) {
    double s = 0;
    for (int i = 0; i < n_rows; ++i)
      for (int a = 0; a < d.A; ++a) s += tr.adv[(size_t)rows[i] * d.A + a];
    mean = s / B;
    double q = 0;
    for (int i = 0; i < n_rows; ++i)
      for (int a = 0; a < d.A; ++a) {
        const double e = tr.adv[(size_t)rows[i] * d.A + a] - mean;
        q += e * e;
      }
    stdv = std::sqrt(q / B);
  }
  const Net actor = net_at(p, d.D, d.Ha, kActions, d.round_act);
  const Net critic = net_at(p + d.Pa, d.Dc, d.Hc, 1, d.round_act);
  NetGrad ga{}, gc{};
  if (grad) {
    std::fill(grad, grad + d.P, 0.0);
    ga = grad_at(grad, d.D, d.Ha, kActions);
    gc = grad_at(grad + d.Pa, d.Dc, d.Hc, 1);
  }
  const int Hm = std::max(d.Ha, d.Hc);
  std::vector<double> x(std::max(d.D, d.Dc)), h1(Hm), h2(Hm), dz1(Hm), dz2(Hm);
  MbStats st{0, 0, 0, 0, 0, 0};
  const double eps = c.clip_eps;

  auto value_term = [&](double v, double ret, double v_old, double* dv) {
    // 0.5 (v - ret)^2, optionally the pessimistic maximum with the clipped prediction
    double e = v - ret, loss = 0.5 * e * e, g = e;
    if (c.clip_value) {
      const double dvv = v - v_old;
      const double vc = v_old + std::min(std::max(dvv, -eps), eps);
      const double ec = vc - ret, lc = 0.5 * ec * ec;
      if (lc > loss) {
        loss = lc;
        g = (dvv > -eps && dvv < eps) ? ec : 0.0;
      }
    }
    *dv = g;
    return loss;
  };

  for (int i = 0; i < n_rows; ++i) {
    const size_t row = (size_t)rows[i];
    const float* obs_row = tr.obs + row * d.A * d.D;
    for (int a = 0; a < d.A; ++a) {
      const size_t s = row * d.A + a;
      for (int k = 0; k < d.D; ++k) x[k] = obs_row[(size_t)a * d.D + k];
      double logits[kActions];
      mlp_forward(actor, x.data(), h1.data(), h2.data(), logits);
      double m = logits[0];
      for (int k = 1; k < kActions; ++k) m = std::max(m, logits[k]);
      double se = 0;
      for (int k = 0; k < kActions; ++k) se += std::exp(logits[k] - m);
      const double lse = m + std::log(se);
      double pk[kActions], lpk[kActions], H = 0;
      for (int k = 0; k < kActions; ++k) {
        lpk[k] = logits[k] - lse;
        pk[k] = std::exp(lpk[k]);
        H -= pk[k] * lpk[k];
      }
      const int act = tr.action[s];
      const double logp_new = lpk[act];
      const double log_ratio = logp_new - (double)tr.logp[s];
      const double ratio = std::exp(log_ratio);
      const double advn = c.normalize_adv ? ((double)tr.adv[s] - mean) / (stdv + 1e-8) : (double)tr.adv[s];
      const double rc = std::min(std::max(ratio, 1.0 - eps), 1.0 + eps);
      const double s1 = ratio * advn, s2 = rc * advn;
      st.pi_loss += -std::min(s1, s2) / B;
      st.entropy += H / B;
      st.approx_kl += ((ratio - 1.0) - log_ratio) / B;
      st.clip_frac += (std::fabs(ratio - 1.0) > eps ? 1.0 : 0.0) / B;
      if (grad) {
        // the unclipped branch carries the gradient iff it is the minimum (ties included)
        const double dlogp = (s1 <= s2) ? -(advn * ratio) / B : 0.0;
        double dl[kActions];
        for (int k = 0; k < kActions; ++k) {
          dl[k] = dlogp * ((k == act ? 1.0 : 0.0) - pk[k]);
          dl[k] += (c.ent_coef / B) * pk[k] * (lpk[k] + H);  // -ent_coef * dH/dlogit_k / B
        }
        mlp_backward(actor, ga, x.data(), h1.data(), h2.data(), dl, dz1.data(), dz2.data());
      }
      if (!d.central) {
        double v;
        mlp_forward(critic, x.data(), h1.data(), h2.data(), &v);
        double dv;
        st.v_loss += value_term(v, tr.ret[s], tr.value[s], &dv) / B;
        if (grad) {
          dv *= c.vf_coef / B;
          mlp_backward(critic, gc, x.data(), h1.data(), h2.data(), &dv, dz1.data(), dz2.data());
        }
      }
    }
    if (d.central) {
      for (int k = 0; k < d.Dc; ++k) x[k] = obs_row[k];
      double v;
      mlp_forward(critic, x.data(), h1.data(), h2.data(), &v);
      double dv_sum = 0;
      for (int a = 0; a < d.A; ++a) {
        const size_t s = row * d.A + a;
        double dv;
        st.v_loss += value_term(v, tr.ret[s], tr.value[s], &dv) / B;
        dv_sum += dv;
      }
      if (grad) {
        dv_sum *= c.vf_coef / B;
        mlp_backward(critic, gc, x.data(), h1.data(), h2.data(), &dv_sum, dz1.data(), dz2.data());
      }
    }
  }
  st.total = st.pi_loss - c.ent_coef * st.entropy + c.vf_coef * st.v_loss;
  return st;
}

// ---------------------------------------------------------------------------------------
// Recurrent networks (the paper's Section 2 and Section 4 list recurrent IPPO and MAPPO next to the feed-forward
// systems; it gives no architecture).  Reading used here: the second hidden layer is replaced by a GRU cell.
//   e  = tanh(x We + be)
//   r  = sigma(e Wi[:, 0:H] + bi[0:H] + h Wh[:, 0:H] + bh[0:H])
//   z  = sigma(e Wi[:, H:2H] + bi[H:2H] + h Wh[:, H:2H] + bh[H:2H])
//   n  = tanh(e Wi[:, 2H:3H] + bi[2H:3H] + r * (h Wh[:, 2H:3H] + bh[2H:3H]))
//   h' = (1 - z) * n + z * h,      out = h' W3 + b3
// (the gate arrangement of Cho et al. 2014 as most libraries implement it: reset gate applied to the hidden
// product).  The hidden state entering a step is zero if the previous step ended an episode.  Parameters of a
// network, in order: We[Din][H] be[H] Wi[H][3H] bi[3H] Wh[H][3H] bh[3H] W3[H][Dout] b3[Dout].
// The PPO update treats every environment's rollout as one sequence: minibatches are sets of environments, and
// the gradient flows back through time from t = T-1 to 0, stopping at episode boundaries and at the state the
// rollout started from.
// ---------------------------------------------------------------------------------------
struct RecNet {
  int Din, H, Dout;
  const double *We, *be, *Wi, *bi, *Wh, *bh, *W3, *b3;
};
struct RecGrad {
  double *We, *be, *Wi, *bi, *Wh, *bh, *W3, *b3;
};
template <class NetT, class Ptr>
NetT rec_at(Ptr p, int Din, int H, int Dout) {
  NetT n{};
  n.We = p; p += (size_t)Din * H;
  n.be = p; p += H;
  n.Wi = p; p += (size_t)H * 3 * H;
  n.bi = p; p += 3 * H;
  n.Wh = p; p += (size_t)H * 3 * H;
  n.bh = p; p += 3 * H;
  n.W3 = p; p += (size_t)H * Dout;
  n.b3 = p;
  return n;
}
RecNet rec_net_at(const double* p, int Din, int H, int Dout) {
  RecNet n = rec_at<RecNet>(p, Din, H, Dout);
  n.Din = Din; n.H = H; n.Dout = Dout;
  return n;
}

inline double sigmoid(double x) { return 1.0 / (1.0 + std::exp(-x)); }

// Everything one step of one sequence leaves behind for the backward pass.
struct RecStep {
  std::vector<double> x, e, r, z, n, ghn, hprev, h;
  void size(int Din, int H) {
    x.resize(Din); e.resize(H); r.resize(H); z.resize(H); n.resize(H); ghn.resize(H); hprev.resize(H); h.resize(H);
  }
};

// st.x and st.hprev are inputs; fills the rest of st and out[Dout].
void rec_forward(const RecNet& w, RecStep& st, double* out) {
  const int H = w.H;
  for (int j = 0; j < H; ++j) {
    double acc = w.be[j];
    for (int i = 0; i < w.Din; ++i) acc += st.x[i] * w.We[(size_t)i * H + j];
    st.e[j] = std::tanh(acc);
  }
  for (int j = 0; j < H; ++j) {
    double gi[3], gh[3];
    for (int g = 0; g < 3; ++g) {
      gi[g] = w.bi[g * H + j];
      gh[g] = w.bh[g * H + j];
      for (int i = 0; i < H; ++i) {
        gi[g] += st.e[i] * w.Wi[(size_t)i * 3 * H + g * H + j];
        gh[g] += st.hprev[i] * w.Wh[(size_t)i * 3 * H + g * H + j];
      }
    }
    st.r[j] = sigmoid(gi[0] + gh[0]);
    st.z[j] = sigmoid(gi[1] + gh[1]);
    st.ghn[j] = gh[2];
    st.n[j] = std::tanh(gi[2] + st.r[j] * gh[2]);
    st.h[j] = (1.0 - st.z[j]) * st.n[j] + st.z[j] * st.hprev[j];
  }
  if (out)
    for (int k = 0; k < w.Dout; ++k) {
      double acc = w.b3[k];
      for (int i = 0; i < H; ++i) acc += st.h[i] * w.W3[(size_t)i * w.Dout + k];
      out[k] = acc;
    }
}

// dh[H]: on entry the gradient arriving at h' from later steps; dout[Dout] the gradient of this step's output.
// Accumulates parameter gradients; on exit dhprev[H] is the gradient with respect to the incoming hidden state.
void rec_backward(const RecNet& w, const RecGrad& g, const RecStep& st, const double* dout, const double* dh_in,
                  double* dhprev) {
  const int H = w.H;
  std::vector<double> dh(H), dgi(3 * H), dgh(3 * H), de(H);
  for (int i = 0; i < H; ++i) {
    double acc = dh_in[i];
    for (int k = 0; k < w.Dout; ++k) {
      acc += dout[k] * w.W3[(size_t)i * w.Dout + k];
      g.W3[(size_t)i * w.Dout + k] += st.h[i] * dout[k];
    }
    dh[i] = acc;
  }
  for (int k = 0; k < w.Dout; ++k) g.b3[k] += dout[k];
  for (int j = 0; j < H; ++j) {
    const double dn = dh[j] * (1.0 - st.z[j]);
    const double dz = dh[j] * (st.hprev[j] - st.n[j]);
    dhprev[j] = dh[j] * st.z[j];
    const double dpre_n = dn * (1.0 - st.n[j] * st.n[j]);
    const double dr = dpre_n * st.ghn[j];
    const double dpre_z = dz * st.z[j] * (1.0 - st.z[j]);
    const double dpre_r = dr * st.r[j] * (1.0 - st.r[j]);
    dgi[j] = dpre_r; dgi[H + j] = dpre_z; dgi[2 * H + j] = dpre_n;
    dgh[j] = dpre_r; dgh[H + j] = dpre_z; dgh[2 * H + j] = dpre_n * st.r[j];
  }
  for (int c = 0; c < 3 * H; ++c) {
    g.bi[c] += dgi[c];
    g.bh[c] += dgh[c];
  }
  for (int i = 0; i < H; ++i) {
    double ae = 0, ah = 0;
    for (int c = 0; c < 3 * H; ++c) {
      ae += dgi[c] * w.Wi[(size_t)i * 3 * H + c];
      ah += dgh[c] * w.Wh[(size_t)i * 3 * H + c];
      g.Wi[(size_t)i * 3 * H + c] += st.e[i] * dgi[c];
      g.Wh[(size_t)i * 3 * H + c] += st.hprev[i] * dgh[c];
    }
    de[i] = ae * (1.0 - st.e[i] * st.e[i]);
    dhprev[i] += ah;
  }
  for (int i = 0; i < w.Din; ++i)
    for (int j = 0; j < H; ++j) g.We[(size_t)i * H + j] += st.x[i] * de[j];
  for (int j = 0; j < H; ++j) g.be[j] += de[j];
}

// Sequence-minibatch loss and gradient over the environments envs[0 .. n_envs_mb).
MbStats rec_minibatch_loss_grad(const orc_config& c, const orc_traj& tr, const orc_rec_state& rs, const double* p,
                                const int32_t* envs, int n_envs_mb, double* grad /*nullable [P], overwritten*/) {
  const Dims d = dims_of(c);
  const double B = (double)n_envs_mb * d.T * d.A;
  const size_t NA = (size_t)d.N * d.A;
  double mean = 0, stdv = 1;
  if (c.normalize_adv) {
    double s = 0;
    for (int i = 0; i < n_envs_mb; ++i)
      for (int t = 0; t < d.T; ++t)
        for (int a = 0; a < d.A; ++a) s += tr.adv[(size_t)t * NA + (size_t)envs[i] * d.A + a];
    mean = s / B;
    double q = 0;
    for (int i = 0; i < n_envs_mb; ++i)
      for (int t = 0; t < d.T; ++t)
        for (int a = 0; a < d.A; ++a) {
          const double e = tr.adv[(size_t)t * NA + (size_t)envs[i] * d.A + a] - mean;
          q += e * e;
        }
    stdv = std::sqrt(q / B);
  }
  const RecNet actor = rec_net_at(p, d.D, d.Ha, kActions);
  const RecNet critic = rec_net_at(p + d.Pa, d.Dc, d.Hc, 1);
  RecGrad ga{}, gc{};
  if (grad) {
    std::fill(grad, grad + d.P, 0.0);
    ga = rec_at<RecGrad>(grad, d.D, d.Ha, kActions);
    gc = rec_at<RecGrad>(grad + d.Pa, d.Dc, d.Hc, 1);
  }
  MbStats st{0, 0, 0, 0, 0, 0};
  const double eps = c.clip_eps;
  auto value_term = [&](double v, double ret, double v_old, double* dv) {
    double e = v - ret, loss = 0.5 * e * e, g = e;
    if (c.clip_value) {
      const double dvv = v - v_old;
      const double vc = v_old + std::min(std::max(dvv, -eps), eps);
      const double ec = vc - ret, lc = 0.5 * ec * ec;
      if (lc > loss) {
        loss = lc;
        g = (dvv > -eps && dvv < eps) ? ec : 0.0;
      }
    }
    *dv = g;
    return loss;
  };
  std::vector<RecStep> steps(d.T);
  std::vector<double> douts((size_t)d.T * kActions);

  // one sequence of one network: forward over t storing the steps and dL/dout, then backward through time
  auto run_sequence = [&](const RecNet& w, const RecGrad& g, int env, const float* h0, int Dout,
                          const std::function<void(int, double*)>& load_x,
                          const std::function<void(int, const double*, double*)>& loss_at) {
    for (int t = 0; t < d.T; ++t) {
      RecStep& s = steps[t];
      s.size(w.Din, w.H);
      load_x(t, s.x.data());
      const bool cut = t > 0 && tr.done[(size_t)(t - 1) * d.N + env];
      for (int j = 0; j < w.H; ++j) s.hprev[j] = t == 0 ? (double)h0[j] : (cut ? 0.0 : steps[t - 1].h[j]);
      double out[kActions];
      rec_forward(w, s, out);
      loss_at(t, out, douts.data() + (size_t)t * kActions);
    }
    if (!grad) return;
    std::vector<double> carry(w.H, 0.0), dhprev(w.H);
    for (int t = d.T - 1; t >= 0; --t) {
      rec_backward(w, g, steps[t], douts.data() + (size_t)t * kActions, carry.data(), dhprev.data());
      const bool cut = t > 0 && tr.done[(size_t)(t - 1) * d.N + env];
      for (int j = 0; j < w.H; ++j) carry[j] = cut ? 0.0 : dhprev[j];
    }
    (void)Dout;
  };

  for (int i = 0; i < n_envs_mb; ++i) {
    const int env = envs[i];
    for (int a = 0; a < d.A; ++a) {
      auto load_obs = [&](int t, double* x) {
        const float* o = tr.obs + ((size_t)t * NA + (size_t)env * d.A + a) * d.D;
        for (int k = 0; k < d.D; ++k) x[k] = o[k];
      };
      run_sequence(actor, ga, env, rs.ha0 + ((size_t)env * d.A + a) * d.Ha, kActions, load_obs,
                   [&](int t, const double* logits, double* dl) {
                     const size_t s = (size_t)t * NA + (size_t)env * d.A + a;
                     double m = logits[0];
                     for (int k = 1; k < kActions; ++k) m = std::max(m, logits[k]);
                     double se = 0;
                     for (int k = 0; k < kActions; ++k) se += std::exp(logits[k] - m);
                     const double lse = m + std::log(se);
                     double pk[kActions], lpk[kActions], Hent = 0;
                     for (int k = 0; k < kActions; ++k) {
                       lpk[k] = logits[k] - lse;
                       pk[k] = std::exp(lpk[k]);
                       Hent -= pk[k] * lpk[k];
                     }
                     const int act = tr.action[s];
                     const double log_ratio = lpk[act] - (double)tr.logp[s];
                     const double ratio = std::exp(log_ratio);
                     const double advn = c.normalize_adv ? ((double)tr.adv[s] - mean) / (stdv + 1e-8) : (double)tr.adv[s];
                     const double rc = std::min(std::max(ratio, 1.0 - eps), 1.0 + eps);
                     const double s1 = ratio * advn, s2 = rc * advn;
                     st.pi_loss += -std::min(s1, s2) / B;
                     st.entropy += Hent / B;
                     st.approx_kl += ((ratio - 1.0) - log_ratio) / B;
                     st.clip_frac += (std::fabs(ratio - 1.0) > eps ? 1.0 : 0.0) / B;
                     const double dlogp = (s1 <= s2) ? -(advn * ratio) / B : 0.0;
                     for (int k = 0; k < kActions; ++k)
                       dl[k] = dlogp * ((k == act ? 1.0 : 0.0) - pk[k]) + (c.ent_coef / B) * pk[k] * (lpk[k] + Hent);
                   });
      if (!d.central)
        run_sequence(critic, gc, env, rs.hc0 + ((size_t)env * d.A + a) * d.Hc, 1, load_obs,
                     [&](int t, const double* v, double* dv) {
                       const size_t s = (size_t)t * NA + (size_t)env * d.A + a;
                       double g;
                       st.v_loss += value_term(v[0], tr.ret[s], tr.value[s], &g) / B;
                       dv[0] = g * c.vf_coef / B;
                     });
    }
    if (d.central)
      run_sequence(critic, gc, env, rs.hc0 + (size_t)env * d.Hc, 1,
                   [&](int t, double* x) {
                     const float* o = tr.obs + ((size_t)t * NA + (size_t)env * d.A) * d.D;
                     for (int k = 0; k < d.Dc; ++k) x[k] = o[k];
                   },
                   [&](int t, const double* v, double* dv) {
                     double sum = 0;
                     for (int a = 0; a < d.A; ++a) {
                       const size_t s = (size_t)t * NA + (size_t)env * d.A + a;
                       double g;
                       st.v_loss += value_term(v[0], tr.ret[s], tr.value[s], &g) / B;
                       sum += g;
                     }
                     dv[0] = sum * c.vf_coef / B;
                   });
  }
  st.total = st.pi_loss - c.ent_coef * st.entropy + c.vf_coef * st.v_loss;
  return st;
}

}  // namespace

// =========================================================================================
// C ABI
// =========================================================================================
extern "C" {

void orc_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) { philox4x32_10(ctr, key, out); }
uint32_t orc_rand_below(uint32_t x, uint32_t n) { return rand_below(x, n); }
float orc_rand_unit(uint32_t x) { return rand_unit(x); }
float orc_round_bf16(float x) { return round_bf16(x); }

int32_t orc_param_count(const orc_config* c) { return dims_of(*c).P; }
int32_t orc_actor_param_count(const orc_config* c) { return dims_of(*c).Pa; }

// Episode 0 for every env.
void orc_env_reset(const orc_config* c, orc_env_state s) {
  for (int n = 0; n < c->n_envs; ++n) {
    s.episode_id[n] = 0;
    reset_one(*c, s, n);
  }
}

void orc_observe(const orc_config* c, orc_env_state s, float* obs /*[N][A][D]*/) {
  const Dims d = dims_of(*c);
  for (int n = 0; n < d.N; ++n) observe_one(*c, s, n, obs + (size_t)n * d.A * d.D);
}

// actions [N][A]; obs (post-step, nullable) [N][A][D]; reward [N][A]; done [N].
void orc_env_step(const orc_config* c, orc_env_state s, const int32_t* actions, float* obs, float* reward,
                  uint8_t* done) {
  const Dims d = dims_of(*c);
  for (int n = 0; n < d.N; ++n) {
    step_one(*c, s, n, actions + (size_t)n * d.A, reward + (size_t)n * d.A, done + n);
    if (obs) observe_one(*c, s, n, obs + (size_t)n * d.A * d.D);
  }
}

// Actor logits [rows][A][6] and critic values [rows][A] for rows of observations [rows][A][D].
void orc_policy_forward(const orc_config* c, const float* params, const float* obs, int64_t n_rows,
                        float* logits /*nullable*/, float* value /*nullable*/) {
  const Dims d = dims_of(*c);
  const std::vector<double> p = effective_params(*c, params);
  std::vector<double> lg(d.A * kActions), v(d.A);
  for (int64_t r = 0; r < n_rows; ++r) {
    policy_row(d, p.data(), obs + (size_t)r * d.A * d.D, logits ? lg.data() : nullptr, value ? v.data() : nullptr);
    if (logits)
      for (int i = 0; i < d.A * kActions; ++i) logits[(size_t)r * d.A * kActions + i] = (float)lg[i];
    if (value)
      for (int a = 0; a < d.A; ++a) value[(size_t)r * d.A + a] = (float)v[a];
  }
}

// Gumbel-max over n samples of 6 logits with 6 uniforms each; logp of the chosen (or forced) action.
void orc_sample(const float* logits, const float* uniforms, const int32_t* forced /*nullable*/, int64_t n,
                int32_t* action, int32_t* sampled /*nullable*/, float* logp, float* gap /*nullable*/) {
  for (int64_t i = 0; i < n; ++i) {
    int32_t a;
    float g;
    sample_one(logits + i * kActions, uniforms + i * kActions, &a, &g);
    if (sampled) sampled[i] = a;
    if (gap) gap[i] = g;
    if (forced) a = forced[i];
    action[i] = a;
    double lg[kActions];
    for (int k = 0; k < kActions; ++k) lg[k] = logits[i * kActions + k];
    logp[i] = (float)log_prob(lg, a);
  }
}

// The six sampling uniforms of (step, env, agent).
void orc_sample_uniforms(const orc_config* c, uint64_t step, int32_t env, int32_t agent, float* u /*[6]*/) {
  const uint32_t key[2] = {(uint32_t)(c->seed & 0xffffffffu), (uint32_t)(c->seed >> 32)};
  const uint32_t lane = (uint32_t)(env * c->n_agents + agent);
  uint32_t out[8];
  for (uint32_t call = 0; call < 2; ++call) {
    const uint32_t ctr[4] = {(uint32_t)(step & 0xffffffffu), (uint32_t)(step >> 32), lane * 2u + call, kStreamSample};
    philox4x32_10(ctr, key, out + 4 * call);
  }
  for (int k = 0; k < kActions; ++k) u[k] = rand_unit(out[k]);
}

// T-step rollout from the current state.  forced_actions [T][N][A] and forced_uniforms
// [T][N][A][6] are nullable.
void orc_rollout(const orc_config* c, orc_env_state s, const float* params, orc_traj tr, uint64_t step_offset,
                 const int32_t* forced_actions, const float* forced_uniforms) {
  const Dims d = dims_of(*c);
  const std::vector<double> p = effective_params(*c, params);
  const size_t NA = (size_t)d.N * d.A;
  std::vector<double> lg(d.A * kActions), v(d.A);
  for (int t = 0; t < d.T; ++t) {
    float* obs_t = tr.obs + (size_t)t * NA * d.D;
    for (int n = 0; n < d.N; ++n) {
      observe_one(*c, s, n, obs_t + (size_t)n * d.A * d.D);
      policy_row(d, p.data(), obs_t + (size_t)n * d.A * d.D, lg.data(), v.data());
      for (int a = 0; a < d.A; ++a) {
        const size_t i = (size_t)t * NA + (size_t)n * d.A + a;
        float lf[kActions], u[kActions];
        for (int k = 0; k < kActions; ++k) lf[k] = (float)lg[a * kActions + k];
        if (forced_uniforms)
          std::memcpy(u, forced_uniforms + i * kActions, sizeof(u));
        else
          orc_sample_uniforms(c, step_offset + (uint64_t)t, n, a, u);
        int32_t act;
        float gp;
        sample_one(lf, u, &act, &gp);
        if (tr.sampled) tr.sampled[i] = act;
        if (tr.gap) tr.gap[i] = gp;
        if (tr.logits) std::memcpy(tr.logits + i * kActions, lf, sizeof(lf));
        if (forced_actions) act = forced_actions[i];
        tr.action[i] = act;
        tr.logp[i] = (float)log_prob(lg.data() + a * kActions, act);
        tr.value[i] = (float)v[a];
      }
      step_one(*c, s, n, tr.action + (size_t)t * NA + (size_t)n * d.A, tr.reward + (size_t)t * NA + (size_t)n * d.A,
               tr.done + (size_t)t * d.N + n);
    }
  }
  float* obs_T = tr.obs + (size_t)d.T * NA * d.D;
  for (int n = 0; n < d.N; ++n) {
    observe_one(*c, s, n, obs_T + (size_t)n * d.A * d.D);
    policy_row(d, p.data(), obs_T + (size_t)n * d.A * d.D, nullptr, v.data());
    for (int a = 0; a < d.A; ++a) tr.last_value[(size_t)n * d.A + a] = (float)v[a];
  }
}

// Greedy evaluation block (the paper's Section 2, "robust evaluation": training is frozen periodically and the
// current policy is evaluated in blocks that run on the accelerator between training blocks).  The paper fixes
// no protocol; the reading here: from the state passed in, every environment plays its first `n_episodes`
// episodes with the greedy action (largest fp32 logit, lowest index on exact ties) of every agent.  Per
// environment: ret_sum = sum over those episodes and their steps of the team reward of the step (the agents'
// rewards added in ascending agent index, then added to the running sum, both in fp32, in time order), len_sum =
// number of steps of those episodes, episodes = n_episodes.  Steps after an environment's n_episodes-th episode
// are not counted; n_episodes * episode_cap steps are taken, which covers every counted episode.  min_gap
// (nullable) = the smallest difference between the two largest logits over all counted decisions of the
// environment (how close the run came to a tie that an fp32 evaluation might break the other way).
void orc_evaluate(const orc_config* c, orc_env_state s, const float* params, int32_t n_episodes, float* ret_sum,
                  int32_t* len_sum, int32_t* episodes, float* min_gap) {
  const Dims d = dims_of(*c);
  const std::vector<double> p = effective_params(*c, params);
  std::vector<float> obs((size_t)d.A * d.D), reward(d.A);
  std::vector<double> lg((size_t)d.A * kActions);
  std::vector<int32_t> act(d.A);
  for (int n = 0; n < d.N; ++n) {
    ret_sum[n] = 0.0f;
    len_sum[n] = 0;
    episodes[n] = 0;
    if (min_gap) min_gap[n] = INFINITY;
  }
  const int64_t steps = (int64_t)n_episodes * c->episode_cap;
  for (int64_t t = 0; t < steps; ++t)
    for (int n = 0; n < d.N; ++n) {
      observe_one(*c, s, n, obs.data());
      policy_row(d, p.data(), obs.data(), lg.data(), nullptr);
      const bool counted = episodes[n] < n_episodes;
      for (int a = 0; a < d.A; ++a) {
        int best = 0;
        float top = (float)lg[(size_t)a * kActions], second = -INFINITY;
        for (int k = 1; k < kActions; ++k) {
          const float v = (float)lg[(size_t)a * kActions + k];
          if (v > top) {
            second = top;
            top = v;
            best = k;
          } else if (v > second) {
            second = v;
          }
        }
        act[a] = best;
        if (counted && min_gap) min_gap[n] = std::min(min_gap[n], top - second);
      }
      uint8_t done = 0;
      step_one(*c, s, n, act.data(), reward.data(), &done);
      if (counted) {
        float team = 0.0f;
        for (int a = 0; a < d.A; ++a) team += reward[a];
        ret_sum[n] += team;
        len_sum[n] += 1;
        if (done) episodes[n] += 1;
      }
    }
}

// Generalised advantage estimation, backwards in time per (env, agent) lane:
//   delta_t = r_t + gamma (1 - d_t) V_{t+1} - V_t,  A_t = delta_t + gamma lambda (1 - d_t) A_{t+1},
//   A_T = 0, V_T = last_value, ret_t = A_t + V_t.
void orc_compute_gae(const orc_config* c, orc_traj tr) {
  const Dims d = dims_of(*c);
  const size_t NA = (size_t)d.N * d.A;
  const double gamma = c->gamma, lambda = c->lambda;
  for (int n = 0; n < d.N; ++n)
    for (int a = 0; a < d.A; ++a) {
      const size_t lane = (size_t)n * d.A + a;
      double next_adv = 0, next_v = tr.last_value[lane];
      for (int t = d.T - 1; t >= 0; --t) {
        const size_t i = (size_t)t * NA + lane;
        const double nd = tr.done[(size_t)t * d.N + n] ? 0.0 : 1.0;
        const double v = tr.value[i];
        const double delta = (double)tr.reward[i] + gamma * nd * next_v - v;
        const double adv = delta + gamma * lambda * nd * next_adv;
        tr.adv[i] = (float)adv;
        tr.ret[i] = (float)(adv + v);
        next_adv = adv;
        next_v = v;
      }
    }
}

// Loss (and optionally gradient) of one minibatch, evaluated in fp64 at fp64 parameters:
// the function the finite-difference and autograd pins probe.  out_stats[6] =
// {policy loss, value loss (unscaled), entropy, approx KL, clip fraction, total}.
void orc_minibatch_loss_grad_f64(const orc_config* c, orc_traj tr, const double* params, const int32_t* rows,
                                 int32_t n_rows, double* out_stats, double* grad /*nullable [P]*/) {
  const MbStats st = minibatch_loss_grad(*c, tr, params, rows, n_rows, grad);
  out_stats[0] = st.pi_loss; out_stats[1] = st.v_loss; out_stats[2] = st.entropy;
  out_stats[3] = st.approx_kl; out_stats[4] = st.clip_frac; out_stats[5] = st.total;
}

// One Adam step on fp32 master parameters and moments from an fp64 gradient; k = 1-based step.
void orc_adam_step(const orc_config* c, float* params, float* m, float* v, const double* grad, int64_t k,
                   int64_t count) {
  const double b1 = c->beta1, b2 = c->beta2;
  const double bc1 = 1.0 - std::pow(b1, (double)k), bc2 = 1.0 - std::pow(b2, (double)k);
  for (int64_t i = 0; i < count; ++i) {
    const double g = grad[i];
    const double mi = b1 * (double)m[i] + (1.0 - b1) * g;
    const double vi = b2 * (double)v[i] + (1.0 - b2) * g * g;
    m[i] = (float)mi;
    v[i] = (float)vi;
    const double upd = (double)c->lr * (mi / bc1) / (std::sqrt(vi / bc2) + (double)c->adam_eps);
    params[i] = (float)((double)params[i] - upd);
  }
}

// E epochs x M minibatches.  perm nullable [E][R] (R = T*N rows); stats [E*M][8] =
// {policy loss, value loss, entropy, approx KL, clip fraction, grad norm (pre-clip), total loss,
//  non-finite flag}; grad_dump nullable [P] = gradient (after clipping) of the last minibatch.
void orc_ppo_update(const orc_config* c, orc_traj tr, float* params, float* adam_m, float* adam_v,
                    int64_t adam_step0, const int32_t* perm, float* stats, float* grad_dump) {
  const Dims d = dims_of(*c);
  const int R = d.T * d.N, M = c->n_minibatches, rows_mb = R / M;
  std::vector<int32_t> ident;
  std::vector<double> grad(d.P);
  int64_t k = adam_step0;
  for (int e = 0; e < c->n_epochs; ++e) {
    const int32_t* order;
    if (perm) {
      order = perm + (size_t)e * R;
    } else {
      if (ident.empty()) {
        ident.resize(R);
        for (int i = 0; i < R; ++i) ident[i] = i;
      }
      order = ident.data();
    }
    for (int mb = 0; mb < M; ++mb) {
      const std::vector<double> p = effective_params(*c, params);
      const MbStats st = minibatch_loss_grad(*c, tr, p.data(), order + (size_t)mb * rows_mb, rows_mb, grad.data());
      double sq = 0;
      for (int i = 0; i < d.P; ++i) sq += grad[i] * grad[i];
      const double norm = std::sqrt(sq);
      if (c->max_grad_norm > 0.f) {
        const double scale = (double)c->max_grad_norm / std::max(norm, (double)c->max_grad_norm);
        for (int i = 0; i < d.P; ++i) grad[i] *= scale;
      }
      ++k;
      orc_adam_step(c, params, adam_m, adam_v, grad.data(), k, d.P);
      float* so = stats + (size_t)(e * M + mb) * 8;
      so[0] = (float)st.pi_loss; so[1] = (float)st.v_loss; so[2] = (float)st.entropy;
      so[3] = (float)st.approx_kl; so[4] = (float)st.clip_frac; so[5] = (float)norm;
      so[6] = (float)st.total;
      so[7] = (std::isfinite(st.total) && std::isfinite(norm)) ? 0.f : 1.f;
      if (grad_dump && e == c->n_epochs - 1 && mb == M - 1)
        for (int i = 0; i < d.P; ++i) grad_dump[i] = (float)grad[i];
    }
  }
}

// ---- recurrent networks ---------------------------------------------------------------------------------

// One step of both recurrent networks on n_rows observation rows obs [n_rows][A][D] from the hidden states
// ha_in [n_rows][A][Ha], hc_in [n_rows][A][Hc] (centralised critic: [n_rows][Hc]).  Any output may be NULL.
void orc_rec_policy_step(const orc_config* c, const float* params, const float* obs, const float* ha_in,
                         const float* hc_in, int64_t n_rows, float* logits, float* value, float* ha_out,
                         float* hc_out) {
  const Dims d = dims_of(*c);
  const std::vector<double> p = effective_params(*c, params);
  const RecNet actor = rec_net_at(p.data(), d.D, d.Ha, kActions);
  const RecNet critic = rec_net_at(p.data() + d.Pa, d.Dc, d.Hc, 1);
  RecStep sa, sc;
  sa.size(d.D, d.Ha);
  sc.size(d.Dc, d.Hc);
  for (int64_t r = 0; r < n_rows; ++r) {
    const float* row = obs + (size_t)r * d.A * d.D;
    for (int a = 0; a < d.A; ++a) {
      const size_t i = (size_t)r * d.A + a;
      for (int k = 0; k < d.D; ++k) sa.x[k] = row[(size_t)a * d.D + k];
      for (int j = 0; j < d.Ha; ++j) sa.hprev[j] = ha_in[i * d.Ha + j];
      double lg[kActions];
      rec_forward(actor, sa, lg);
      if (logits)
        for (int k = 0; k < kActions; ++k) logits[i * kActions + k] = (float)lg[k];
      if (ha_out)
        for (int j = 0; j < d.Ha; ++j) ha_out[i * d.Ha + j] = (float)sa.h[j];
      if (!d.central) {
        for (int k = 0; k < d.D; ++k) sc.x[k] = sa.x[k];
        for (int j = 0; j < d.Hc; ++j) sc.hprev[j] = hc_in[i * d.Hc + j];
        double v;
        rec_forward(critic, sc, &v);
        if (value) value[i] = (float)v;
        if (hc_out)
          for (int j = 0; j < d.Hc; ++j) hc_out[i * d.Hc + j] = (float)sc.h[j];
      }
    }
    if (d.central) {
      for (int k = 0; k < d.Dc; ++k) sc.x[k] = row[k];
      for (int j = 0; j < d.Hc; ++j) sc.hprev[j] = hc_in[(size_t)r * d.Hc + j];
      double v;
      rec_forward(critic, sc, &v);
      if (value)
        for (int a = 0; a < d.A; ++a) value[(size_t)r * d.A + a] = (float)v;
      if (hc_out)
        for (int j = 0; j < d.Hc; ++j) hc_out[(size_t)r * d.Hc + j] = (float)sc.h[j];
    }
  }
}

// Rollout with the recurrent networks: as orc_rollout, the hidden states carried in fp64 from rs.h*0 through the
// T steps (zeroed where the previous step ended an episode) and left in rs.h*1 for the next rollout.
void orc_rec_rollout(const orc_config* c, orc_env_state s, const float* params, orc_traj tr, orc_rec_state rs,
                     uint64_t step_offset, const int32_t* forced_actions, const float* forced_uniforms) {
  const Dims d = dims_of(*c);
  const std::vector<double> p = effective_params(*c, params);
  const RecNet actor = rec_net_at(p.data(), d.D, d.Ha, kActions);
  const RecNet critic = rec_net_at(p.data() + d.Pa, d.Dc, d.Hc, 1);
  const size_t NA = (size_t)d.N * d.A;
  const size_t nc = d.central ? (size_t)d.N : NA;  // critic sequences
  std::vector<double> ha(NA * d.Ha), hc(nc * d.Hc);
  for (size_t i = 0; i < ha.size(); ++i) ha[i] = rs.ha0[i];
  for (size_t i = 0; i < hc.size(); ++i) hc[i] = rs.hc0[i];
  RecStep sa, sc;
  sa.size(d.D, d.Ha);
  sc.size(d.Dc, d.Hc);
  auto critic_step = [&](const float* obs_row, int n, int a, bool keep, double* v) {  // a ignored when centralised
    const size_t q = d.central ? (size_t)n : (size_t)n * d.A + a;
    const float* x = d.central ? obs_row : obs_row + (size_t)a * d.D;
    for (int k = 0; k < d.Dc; ++k) sc.x[k] = x[k];
    for (int j = 0; j < d.Hc; ++j) sc.hprev[j] = hc[q * d.Hc + j];
    rec_forward(critic, sc, v);
    if (keep)
      for (int j = 0; j < d.Hc; ++j) hc[q * d.Hc + j] = sc.h[j];
  };
  for (int t = 0; t <= d.T; ++t) {
    float* obs_t = tr.obs + (size_t)t * NA * d.D;
    for (int n = 0; n < d.N; ++n) {
      if (t > 0 && tr.done[(size_t)(t - 1) * d.N + n]) {  // a new episode starts from the zero state
        for (int a = 0; a < d.A; ++a)
          for (int j = 0; j < d.Ha; ++j) ha[((size_t)n * d.A + a) * d.Ha + j] = 0.0;
        if (d.central) {
          for (int j = 0; j < d.Hc; ++j) hc[(size_t)n * d.Hc + j] = 0.0;
        } else {
          for (int a = 0; a < d.A; ++a)
            for (int j = 0; j < d.Hc; ++j) hc[((size_t)n * d.A + a) * d.Hc + j] = 0.0;
        }
      }
      float* obs_row = obs_t + (size_t)n * d.A * d.D;
      observe_one(*c, s, n, obs_row);
      if (t == d.T) {  // bootstrap value of the post-rollout observation; the hidden states stay as they are
        double v;
        if (d.central) critic_step(obs_row, n, 0, false, &v);
        for (int a = 0; a < d.A; ++a) {
          if (!d.central) critic_step(obs_row, n, a, false, &v);
          tr.last_value[(size_t)n * d.A + a] = (float)v;
        }
        continue;
      }
      double vc = 0;
      if (d.central) critic_step(obs_row, n, 0, true, &vc);
      for (int a = 0; a < d.A; ++a) {
        const size_t i = (size_t)t * NA + (size_t)n * d.A + a, q = (size_t)n * d.A + a;
        for (int k = 0; k < d.D; ++k) sa.x[k] = obs_row[(size_t)a * d.D + k];
        for (int j = 0; j < d.Ha; ++j) sa.hprev[j] = ha[q * d.Ha + j];
        double lg[kActions];
        rec_forward(actor, sa, lg);
        for (int j = 0; j < d.Ha; ++j) ha[q * d.Ha + j] = sa.h[j];
        float lf[kActions], u[kActions];
        for (int k = 0; k < kActions; ++k) lf[k] = (float)lg[k];
        if (forced_uniforms)
          std::memcpy(u, forced_uniforms + i * kActions, sizeof(u));
        else
          orc_sample_uniforms(c, step_offset + (uint64_t)t, n, a, u);
        int32_t act;
        float gp;
        sample_one(lf, u, &act, &gp);
        if (tr.sampled) tr.sampled[i] = act;
        if (tr.gap) tr.gap[i] = gp;
        if (tr.logits) std::memcpy(tr.logits + i * kActions, lf, sizeof(lf));
        if (forced_actions) act = forced_actions[i];
        tr.action[i] = act;
        tr.logp[i] = (float)log_prob(lg, act);
        double v = vc;
        if (!d.central) critic_step(obs_row, n, a, true, &v);
        tr.value[i] = (float)v;
      }
      step_one(*c, s, n, tr.action + (size_t)t * NA + (size_t)n * d.A, tr.reward + (size_t)t * NA + (size_t)n * d.A,
               tr.done + (size_t)t * d.N + n);
    }
  }
  for (size_t i = 0; i < ha.size(); ++i) rs.ha1[i] = (float)ha[i];
  for (size_t i = 0; i < hc.size(); ++i) rs.hc1[i] = (float)hc[i];
}

void orc_rec_minibatch_loss_grad_f64(const orc_config* c, orc_traj tr, orc_rec_state rs, const double* params,
                                     const int32_t* envs, int32_t n_envs_mb, double* out_stats, double* grad) {
  const MbStats st = rec_minibatch_loss_grad(*c, tr, rs, params, envs, n_envs_mb, grad);
  out_stats[0] = st.pi_loss; out_stats[1] = st.v_loss; out_stats[2] = st.entropy;
  out_stats[3] = st.approx_kl; out_stats[4] = st.clip_frac; out_stats[5] = st.total;
}

// E epochs x M minibatches of N / M environments (whole T-step sequences).  perm nullable [E][N].
void orc_rec_ppo_update(const orc_config* c, orc_traj tr, orc_rec_state rs, float* params, float* adam_m,
                        float* adam_v, int64_t adam_step0, const int32_t* perm, float* stats, float* grad_dump) {
  const Dims d = dims_of(*c);
  const int M = c->n_minibatches, envs_mb = d.N / M;
  std::vector<int32_t> ident(d.N);
  for (int i = 0; i < d.N; ++i) ident[i] = i;
  std::vector<double> grad(d.P);
  int64_t k = adam_step0;
  for (int e = 0; e < c->n_epochs; ++e) {
    const int32_t* order = perm ? perm + (size_t)e * d.N : ident.data();
    for (int mb = 0; mb < M; ++mb) {
      const std::vector<double> p = effective_params(*c, params);
      const MbStats st = rec_minibatch_loss_grad(*c, tr, rs, p.data(), order + (size_t)mb * envs_mb, envs_mb, grad.data());
      double sq = 0;
      for (int i = 0; i < d.P; ++i) sq += grad[i] * grad[i];
      const double norm = std::sqrt(sq);
      if (c->max_grad_norm > 0.f) {
        const double scale = (double)c->max_grad_norm / std::max(norm, (double)c->max_grad_norm);
        for (int i = 0; i < d.P; ++i) grad[i] *= scale;
      }
      ++k;
      orc_adam_step(c, params, adam_m, adam_v, grad.data(), k, d.P);
      float* so = stats + (size_t)(e * M + mb) * 8;
      so[0] = (float)st.pi_loss; so[1] = (float)st.v_loss; so[2] = (float)st.entropy;
      so[3] = (float)st.approx_kl; so[4] = (float)st.clip_frac; so[5] = (float)norm;
      so[6] = (float)st.total;
      so[7] = (std::isfinite(st.total) && std::isfinite(norm)) ? 0.f : 1.f;
      if (grad_dump && e == c->n_epochs - 1 && mb == M - 1)
        for (int i = 0; i < d.P; ++i) grad_dump[i] = (float)grad[i];
    }
  }
}

}  // extern "C"

