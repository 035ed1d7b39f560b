/* marl.h -- C ABI of the MI355X (gfx950) fused multi-agent PPO training step.
 *
 * The step is the "update function" of the Anakin architecture the paper adopts (Section 2,
 * Fig. 2): N copies of the environment are rolled out on the accelerator under the current
 * parameters, the experience goes to a loss, its gradient gives new parameters; nothing leaves
 * the device in between.  The systems are the paper's feed-forward multi-agent PPO variants
 * (Section 2 and Section 4): independent PPO with decentralised critics (IPPO) and PPO with a
 * centralised critic over the joint observation (MAPPO), both with parameters shared by all
 * agents.  The environment is a synthetic level-based-foraging grid world with the shapes of
 * the paper's LBF scenarios (Section 4, Fig. 6).
 *
 * Conventions for every entry point
 *   - All array arguments are DEVICE pointers unless a comment says "host".  The library never
 *     allocates, frees or synchronises: every buffer, including workspaces, is owned by the
 *     caller, and sizes come from marl_query_sizes() (marl_rollout_static brings its own fixed scratch instead).  Device pointers must be 16-byte aligned
 *     (256 recommended); a misaligned or null required pointer is rejected before any launch.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *     asynchronous on that stream and ordered by it.
 *     The one exception is the measurement hook marl_timing_enable / marl_timing_read at the end of this header,
 *     which keeps host state, is not thread-safe and waits for events; a product caller never needs it.
 *   - Return value: MARL_OK (0) or a negative marl_status.  Validation happens on the host
 *     before anything is launched; a call that returns an error has launched nothing.
 *   - Index conventions: N envs, A agents, F food items, D = 3*view*view observation floats,
 *     T rollout length.  Trajectory arrays are time-major and densely packed; a "row" is one
 *     (t, n) pair, row index t*N + n, and carries its A agent samples.
 */
#ifndef MARL_H_
#define MARL_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MARL_N_ACTIONS 6 /* 0 noop, 1 north (row-1), 2 south (row+1), 3 west (col-1), 4 east (col+1), 5 load */
#define MARL_N_STATS 8

typedef enum marl_status {
  MARL_OK = 0,
  MARL_E_NULL = -1,   /* a required pointer is NULL */
  MARL_E_ALIGN = -2,  /* a device pointer is not 16-byte aligned */
  MARL_E_CONFIG = -3, /* unsupported or inconsistent configuration */
  MARL_E_LAUNCH = -4, /* the HIP runtime reported an error at launch */
  MARL_E_SIZE = -5    /* a size argument is out of range */
} marl_status;

/* Host struct, passed by const pointer. */
typedef struct marl_config {
  /* environment */
  int32_t grid;        /* G: side of the square grid, 2..64 */
  int32_t n_agents;    /* A: 1..8 */
  int32_t n_food;      /* F: 1..8; A + F <= G*G */
  int32_t max_level;   /* agent levels are uniform in 1..max_level; 1 <= max_level <= 15.  Warehouse world: the number of
                          shelves requested at any time, 1..n_food */
  int32_t episode_cap; /* an episode ends after this many steps at the latest */
  int32_t view;        /* V: odd side of the egocentric window, 3, 5 or 7 */
  int32_t n_envs;      /* N */
  int32_t rollout_len; /* T */
  /* networks: in-H-H-out MLPs with tanh, shared by all agents */
  int32_t actor_hidden;   /* multiple of 32, <= 512 */
  int32_t critic_hidden;  /* multiple of 32, <= 512 */
  int32_t central_critic; /* 0: critic sees one agent's D floats (IPPO); 1: the A*D joint observation (MAPPO) */
  int32_t precision;      /* 0: fp32; 1: bf16 weights/activations in the GEMMs, fp32 accumulation and master weights */
  /* PPO */
  int32_t n_epochs, n_minibatches; /* T*N must be divisible by n_minibatches */
  int32_t normalize_adv;           /* per-minibatch (adv - mean) / (std + 1e-8), population std */
  int32_t clip_value;              /* 1: pessimistic clipped value loss */
  float gamma, lambda, clip_eps, ent_coef, vf_coef;
  float max_grad_norm; /* <= 0: no global-norm clipping */
  float lr, beta1, beta2, adam_eps;
  uint64_t seed; /* Philox key */
  int32_t recurrent; /* 0: feed-forward networks; 1: a GRU cell in place of the second hidden layer (fp32 only; sequence
                        minibatches: n_envs must be divisible by n_minibatches).  Use the *_recurrent entry points. */
  int32_t env_kind;  /* 0: foraging world; 1: warehouse world (see marl_env_step); 2: warehouse world whose episodes also
                        end when robots collide */
} marl_config;

/* Environment state: entity-major structure of arrays, x[e*N + n]. */
typedef struct marl_env_state {
  uint8_t *agent_row, *agent_col, *agent_lvl; /* [A][N] */
  uint8_t *food_row, *food_col, *food_lvl;    /* [F][N]; level 0 = collected */
  int32_t* t_in_ep;                           /* [N] steps taken in the current episode */
  uint32_t* episode_id;                       /* [N] counts auto-resets; part of the layout's random key */
} marl_env_state;

/* One rollout's experience. */
typedef struct marl_traj {
  float* obs;        /* [T+1][N][A][D]; slab t is what the action of step t was chosen on, slab T the state after the rollout */
  int32_t* action;   /* [T][N][A] */
  float* logp;       /* [T][N][A] log-probability of `action` under the rollout policy */
  float* value;      /* [T][N][A] critic value (centralised critic: one value per env, stored for each agent) */
  float* reward;     /* [T][N][A] */
  uint8_t* done;     /* [T][N] 1 where the step ended the episode (all food collected, or cap reached) */
  float* last_value; /* [N][A] critic value of slab T */
  float* adv;        /* [T][N][A] written by marl_compute_gae */
  float* ret;        /* [T][N][A] written by marl_compute_gae */
  float* logits;     /* optional (may be NULL) [T][N][A][6] actor logits */
  int32_t* sampled;  /* optional (may be NULL) [T][N][A] the action the sampler drew (differs from `action` only when forced) */
} marl_traj;

/* Sizes in bytes unless named otherwise (host struct, filled by marl_query_sizes). */
typedef struct marl_sizes {
  int64_t obs_dim, critic_in_dim, n_params, n_actor_params; /* counts */
  int64_t state_entity_bytes_agents, state_entity_bytes_food, state_t_bytes, state_episode_bytes;
  int64_t obs_bytes, step_scalar_bytes /* action, logp, value, reward, adv, ret: each */, done_bytes, last_value_bytes,
      logits_bytes;
  int64_t rollout_workspace_bytes, update_workspace_bytes, eval_workspace_bytes;
  int64_t hidden_actor_bytes, hidden_critic_bytes; /* recurrent networks: one hidden-state array each (else 0) */
} marl_sizes;

/* Hidden states of the recurrent networks around one rollout (device, caller-owned, fp32): h*0 is the state the
 * rollout starts from (zero before the first rollout), h*1 the state it leaves for the next rollout (already zero
 * where the last step ended an episode).  Actor [N][A][Ha]; critic [N][A][Hc] (IPPO) or [N][Hc] (MAPPO). */
typedef struct marl_rec_state {
  float *ha0, *hc0;
  float *ha1, *hc1;
} marl_rec_state;

/* Parameter vector (fp32, one flat array, caller-owned):
 *   actor  W1[D][Ha] b1[Ha] W2[Ha][Ha] b2[Ha] W3[Ha][6] b3[6]
 *   critic W1[Dc][Hc] b1[Hc] W2[Hc][Hc] b2[Hc] W3[Hc][1] b3[1]      y = x W + b, row-major
 * Dc = D (IPPO) or A*D (MAPPO: the agents' observations in agent order, i.e. one contiguous obs row).
 * Recurrent networks (cfg.recurrent = 1), per network with H hidden units, gates in the order reset, update, new:
 *   We[Din][H] be[H] Wi[H][3H] bi[3H] Wh[H][3H] bh[3H] W3[H][Dout] b3[Dout]
 *   e = tanh(x We + be); r = sigma(e Wi_r + bi_r + h Wh_r + bh_r); z likewise; n = tanh(e Wi_n + bi_n + r (h Wh_n + bh_n));
 *   h' = (1 - z) n + z h; out = h' W3 + b3.  h is zero at the first step of an episode. */

/* Warehouse world (cfg.env_kind = 1 or 2): a second grid workload in the spirit of the multi-robot warehouse task of
 * Section 4; the rules are this library's own.  It lives in the same buffers: A robots in agent_row / agent_col,
 * F shelves in food_row / food_col; agent_lvl[a] = 0 when robot a carries nothing, else 1 + the index of the shelf
 * it carries; food_lvl[f] = 1 for an idle shelf, 2 for a requested one; max_level shelves are requested at any
 * time; the goal cells are (G-1, G/2 - 1) and (G-1, G/2).  Reset: A + F distinct cells (robots first), then the
 * requested shelves (the j-th request takes the r-th idle shelf, r drawn in [0, F - j)).  Step, actions 0 stay,
 * 1..4 north / south / west / east, 5 toggle, against the start-of-step state: a move is valid iff its target is in
 * the grid, holds no robot and -- for a loaded robot -- no shelf; two or more valid movers onto one cell all stay;
 * a robot whose in-grid move was refused because of another robot has collided; carried shelves move with their
 * robots; toggle puts a carried shelf down, or picks up the shelf the robot stands on; then, robots in ascending
 * index, a robot carrying a requested shelf on a goal cell earns 1.0, the shelf becomes idle and another idle shelf
 * (the delivered one if there is none) becomes requested, drawn from Philox keyed (seed; env, episode, step in the
 * episode, ordinal of the delivery); the episode ends at the cap and, with env_kind = 2, on a collision.
 * Observation channels: 0 / 1 unloaded / 2 loaded robot; 0 / 1 idle / 2 requested shelf; 1 outside the grid, 0.5 goal. */

/* Buffer sizes of a configuration: what the caller has to allocate for the state, one rollout's experience
 * (Section 2, Fig. 2: the experience a rollout hands to the loss) and the workspaces.  The paper gives no shapes;
 * they follow from the workload list (grid, agents, view, networks).  Fills *out; touches no GPU.
 * Errors: MARL_E_NULL, MARL_E_CONFIG. */
int32_t marl_query_sizes(const marl_config* cfg, marl_sizes* out);

/* The vectorised environment's reset (Section 2: the environments are implemented on the accelerator so that they
 * can be batched and compiled with the rest of the step; the paper names the task, Section 4, not its layout rules --
 * those are the workload's).  Starts episode 0 in every env: agent levels, then A+F distinct cells (agents first), then food
 * levels (1..sum of the <=4 highest agent levels), all drawn from Philox4x32-10 keyed by
 * (seed; env, episode).  The layout of an env depends only on (seed, env index, episode id). */
int32_t marl_env_reset(const marl_config* cfg, marl_env_state st, void* stream);

/* Egocentric observation of the current state: obs [N][A][D], element ((dy+h)*V + (dx+h))*3 + c,
 * c = 0 level of the agent in that cell (self included), 1 level of the food there, 2 = 1.0 outside the grid. */
int32_t marl_observe(const marl_config* cfg, marl_env_state st, float* obs, void* stream);

/* One lock-step transition of all envs under given actions [N][A] (values 0..5).  Rules (the
 * paper names the environment, Section 3/4, but not its rules; these are the workload's):
 * all agents act simultaneously against the start-of-step state; a move is refused if the target
 * is outside the grid or holds food or any agent at the start of the step; two or more agents
 * moving onto one cell all stay; a food is collected when the summed level of the 4-adjacent agents
 * that chose "load" reaches its level, and each such loader i earns food_level*level_i/sum (fp32,
 * accumulated in ascending food index); done = no food left or episode_cap steps taken; a finished
 * env is re-seeded at once (episode_id+1).  Writes reward [N][A], done [N] of the transition and the
 * observation obs [N][A][D] of the resulting state (after any auto-reset); obs may be NULL. */
int32_t marl_env_step(const marl_config* cfg, marl_env_state st, const int32_t* actions, float* obs, float* reward,
                      uint8_t* done, void* stream);

/* Actor logits [n_rows][A][6] and critic values [n_rows][A] for observation rows obs [n_rows][A][D]
 * (either output may be NULL).  workspace: rollout_workspace_bytes of a config with n_envs >= n_rows. */
int32_t marl_policy_forward(const marl_config* cfg, const float* params, const float* obs, int64_t n_rows,
                            float* logits, float* value, void* workspace, void* stream);

/* Gumbel-max categorical sampling of n samples (sample i = env*A + agent): action = argmax_k
 * logits[i][k] - log(-log u[i][k]), lowest k on exact ties; logp = log-softmax(logits)[action].
 * u = uniforms[i][k] if given, else the Philox draw of (seed; step, i, k).  forced (nullable) [n]
 * replaces the returned action (logp follows it); `sampled` (nullable) always gets the draw. */
int32_t marl_sample_actions(const marl_config* cfg, const float* logits, const float* uniforms, const int32_t* forced,
                            int64_t n, uint64_t step, int32_t* action, int32_t* sampled, float* logp, void* stream);

/* T environment steps from the current state under the policy in `params`: per step observe ->
 * actor/critic forward -> sample -> env step (Fig. 2's rollout).  Fills every traj array except
 * adv/ret, leaves `st` at the post-rollout state.  step_offset + t is the sampling key of step t.
 * forced_actions [T][N][A] and forced_uniforms [T][N][A][6] are nullable test hooks.
 * workspace: rollout_workspace_bytes. */
int32_t marl_rollout(const marl_config* cfg, marl_env_state st, const float* params, marl_traj traj,
                     uint64_t step_offset, const int32_t* forced_actions, const float* forced_uniforms,
                     void* workspace, void* stream);

/* marl_rollout for callers that cannot allocate or hold a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments without `workspace`, same results.  The working copy of the
 * parameters (and, for networks the fused forward kernel does not cover, one step's hidden activations) lives in a
 * device array built into the library, MARL_STATIC_SCRATCH_BYTES per GPU for the life of the process.  The call
 * allocates and frees nothing.  MARL_E_SIZE when marl_query_sizes' rollout_workspace_bytes exceeds that size (the bf16
 * configuration and unfused wide networks with many environments do), MARL_E_LAUNCH when the array's address cannot
 * be obtained.  Nothing in the array has to start at zero and nothing in it is kept between calls; every call on a
 * GPU uses that GPU's one array, so calls that overlap on one GPU (different streams, different host threads) race. */
#define MARL_STATIC_SCRATCH_BYTES (8 * 1024 * 1024)
int32_t marl_rollout_static(const marl_config* cfg, marl_env_state st, const float* params, marl_traj traj,
                            uint64_t step_offset, const int32_t* forced_actions, const float* forced_uniforms,
                            void* stream);

/* The advantage step between rollout and loss (Fig. 2: the experience is turned into a loss; the paper names PPO,
 * Section 2, without its equations -- these are the standard ones the workload list states).
 * Generalised advantage estimation per (env, agent), backwards in time:
 * delta_t = r_t + gamma (1-d_t) V_{t+1} - V_t;  adv_t = delta_t + gamma lambda (1-d_t) adv_{t+1};
 * adv_T = 0, V_T = last_value;  ret_t = adv_t + V_t.  Reads reward/value/done/last_value, writes adv/ret. */
int32_t marl_compute_gae(const marl_config* cfg, marl_traj traj, void* stream);

/* n_epochs x n_minibatches clipped-PPO steps (loss -> gradient -> new parameters, Fig. 2) on the
 * trajectory.  Epoch e visits rows in the order perm[e][0..R) (R = T*N; NULL = identity), minibatch m
 * = the m-th R/M rows of that order.  params (fp32 master), adam_m, adam_v [n_params] are updated
 * in place; adam_step0 = optimiser steps already taken.  stats [E*M][8] = {policy loss, value loss
 * (unscaled), entropy, approx KL, clip fraction, gradient norm before clipping, total loss,
 * non-finite flag}.  grad_dump (nullable) [n_params] gets the (clipped) gradient of the last
 * minibatch.  workspace: update_workspace_bytes. */
int32_t marl_ppo_update(const marl_config* cfg, marl_traj traj, float* params, float* adam_m, float* adam_v,
                        int64_t adam_step0, const int32_t* perm, float* stats, float* grad_dump, void* workspace,
                        void* stream);

/* Counters of a training run kept in device memory (caller-owned, 16 bytes, zero before the first step): the
 * sampling-key offset of the next rollout and the number of optimiser steps taken so far. */
typedef struct marl_counters {
  uint64_t step;
  int64_t adam_step;
} marl_counters;

/* One whole training iteration (Fig. 2: rollout -> loss -> gradient -> new parameters) as one call: marl_rollout
 * with step_offset = counters->step, marl_compute_gae, marl_ppo_update with adam_step0 = counters->adam_step, then
 * counters->step += rollout_len and counters->adam_step += n_epochs * n_minibatches, all on the device.  The
 * sequence of launches and their arguments do not depend on the values of the counters, the call makes no
 * allocation, no host-device copy and no synchronisation, so after one ordinary call (which sets kernel attributes)
 * a capture of it into a HIP graph can be replayed for every following iteration; the caller may rewrite the
 * contents of `perm` between replays.  Results equal those of the three separate calls, except that Adam's bias
 * corrections 1 - beta^k are evaluated in fp64 on the device instead of on the host.  `counters` is device memory;
 * the other arguments are those of the three calls.  Feed-forward networks only (MARL_E_CONFIG otherwise). */
int32_t marl_train_step(const marl_config* cfg, marl_env_state st, float* params, marl_traj traj, float* adam_m,
                        float* adam_v, marl_counters* counters, const int32_t* perm, float* stats,
                        void* rollout_workspace, void* update_workspace, void* stream);

/* Recurrent IPPO / MAPPO (Section 2 and Section 4 list them beside the feed-forward systems).  As marl_rollout, with
 * the hidden states carried from rec.h*0 through the T steps and left in rec.h*1.  workspace: rollout_workspace_bytes
 * of the recurrent configuration.  MARL_E_CONFIG unless cfg->recurrent = 1. */
int32_t marl_rollout_recurrent(const marl_config* cfg, marl_env_state st, const float* params, marl_traj traj,
                               marl_rec_state rec, uint64_t step_offset, const int32_t* forced_actions,
                               const float* forced_uniforms, void* workspace, void* stream);

/* As marl_ppo_update for the recurrent networks: every environment's T-step rollout is one sequence, a minibatch is
 * n_envs / n_minibatches environments (epoch e visits them in the order perm[e][0..N), NULL = identity), the loss
 * is the PPO loss over all steps of those sequences, and the gradient flows back through time from step T-1 to 0,
 * stopping at episode boundaries and at rec.h*0.  workspace: update_workspace_bytes of the recurrent configuration.
 * The two networks of a minibatch run side by side: the critic's kernels go to a second stream that the library creates
 * once per device (default priority, kept until the process ends), forked from `stream` and joined back into it with
 * events inside the call, so for the caller everything is still ordered on `stream` and nothing is waited for on the
 * host.  One such call at a time per device: calls that overlap on one device from several host threads would share
 * that stream's two events.  If the stream cannot be created the critic simply follows the actor on `stream`. */
int32_t marl_ppo_update_recurrent(const marl_config* cfg, marl_traj traj, marl_rec_state rec, float* params,
                                  float* adam_m, float* adam_v, int64_t adam_step0, const int32_t* perm, float* stats,
                                  float* grad_dump, void* workspace, void* stream);

/* Per-environment results of an evaluation block: device arrays of n_envs elements, caller-owned. */
typedef struct marl_eval_stats {
  float* ret_sum;    /* [N] team return (all agents' rewards) summed over the counted episodes, fp32 in time order */
  int32_t* len_sum;  /* [N] steps of the counted episodes */
  int32_t* episodes; /* [N] counted episodes completed (= n_episodes when the call returns) */
} marl_eval_stats;

/* Greedy evaluation block (Section 2: training is frozen periodically and the current policy evaluated on the
 * accelerator, between training blocks).  From the state in `st` (the caller resets it; it is left at the state
 * after the last step) every environment plays with action = argmax_k logits[k] (lowest k on exact ties) for
 * every agent; its first n_episodes episodes are counted into `out`, later steps are not.  n_episodes *
 * episode_cap steps are taken, which covers every counted episode.  Mean episode return = sum(ret_sum) /
 * sum(episodes).  workspace: eval_workspace_bytes.  Errors: MARL_E_SIZE if n_episodes < 1 or n_episodes *
 * episode_cap > 2^20. */
int32_t marl_evaluate(const marl_config* cfg, marl_env_state st, const float* params, int32_t n_episodes,
                      marl_eval_stats out, void* workspace, void* stream);

/* Measurement hook for benchmarks (host state only, not thread-safe).  While enabled, every launch of
 * the instrumented kernel classes is bracketed by two HIP events recorded on the launch's own stream.
 * Classes: 0 forward GEMM (activations x weights), 1 backward-data GEMM (gradient x weights^T),
 * 2 weight-gradient GEMM (activations^T x gradient, split over samples), 3 env step / observe, 4 GAE,
 * 5 whole-network training kernel of the small networks (forward + backward flops), 6 the fused rollout kernel
 * (all T steps of actor inference, sampling and environment transition in one launch; booked with the flops of the
 * actor's two hidden layers).  Fused forward kernels are booked under class 0 with the flops of their two hidden layers.
 * marl_timing_enable(1) clears earlier records; marl_timing_read waits for the class's events and
 * returns the summed kernel time, the number of launches and the summed algorithmic work (flops for the
 * GEMMs: 2*M*N*K of the unpadded problem; bytes for env step and GAE).  Errors: MARL_E_NULL, MARL_E_SIZE,
 * MARL_E_LAUNCH. */
int32_t marl_timing_enable(int32_t on);
int32_t marl_timing_read(int32_t kernel_class, double* total_ms, int64_t* launches, double* work);

/* Human-readable name of a status code (static storage, host).  Part of the error convention of this boundary,
 * not of the paper's method. */
const char* marl_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* MARL_H_ */
