// Actor / critic forward pass of the rollout, categorical sampling, and the rollout driver.
//
// The two hidden layers of each network are MFMA GEMMs (gemm.h); the narrow output layer
// (6 logits or 1 value) runs on the vector ALUs of the "head" kernel, which also draws the
// action by Gumbel-max from Philox uniforms and evaluates its log-probability.
#include "bf16_path.h"
#include "fused_forward.h"
#include "gemm.h"
#include "heads.h"
#include "rollout_fused.h"

namespace marl {

int64_t effective_param_floats(const marl_config& c);

namespace {

// Working copy of the parameters: blocks moved to their aligned offsets, optionally rounded to bf16, plus the
// operand-order copies of W1, W2 and W2 transposed that the fused training kernel streams from memory.
__global__ void stage_params_kernel(const float* __restrict__ src, float* __restrict__ dst, ParamMap pm, int round) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pm.src[12]) return;
#pragma unroll
  for (int net = 0; net < 2; ++net) {  // zero rows of the operand-order W1 (fewer than 16 rows: far fewer floats than parameters)
    const int H = pm.hidden[net];
    if (i < (int64_t)(pm.kpad1[net] - pm.din[net]) * H) {
      const int64_t k = pm.din[net] + i / H, n = i % H;
      dst[pm.sw_w1[net] + ((k / 4) * H + n) * 4 + k % 4] = 0.f;
    }
  }
  int b = 0;
#pragma unroll
  for (int k = 1; k < 12; ++k) b += (i >= pm.src[k]) ? 1 : 0;
  const float v = round ? round_to_bf16(src[i]) : src[i];
  const int64_t e = i - pm.src[b];
  dst[pm.dst[b] + e] = v;
  const int net = b >= 6, H = pm.hidden[net];
  const int64_t r = e / H, c = e - r * H;
  if (b == 0 || b == 6) dst[pm.sw_w1[net] + ((r / 4) * H + c) * 4 + r % 4] = v;
  if (b == 2 || b == 8) {
    dst[pm.sw_w2[net] + ((r / 4) * H + c) * 4 + r % 4] = v;
    dst[pm.sw_w2t[net] + ((c / 4) * H + r) * 4 + c % 4] = v;
  }
}

// What the rollout does with a sample's outputs.
struct ActorRolloutFinish {
  float* logits_out;  // nullable
  SampleArgs sa;
  int do_sample;
  __device__ __forceinline__ void operator()(int64_t s, const float out[kActions], float*, float*) const {
    if (logits_out) {
#pragma unroll
      for (int k = 0; k < kActions; ++k) logits_out[s * kActions + k] = out[k];
    }
    if (do_sample) sample_and_store(out, s, sa);
  }
};
// Rows below `split` go to value_out, the rest (the rows of the post-rollout observation, when one pass covers all
// T + 1 slabs) to tail_out.
struct CriticRolloutFinish {
  float* value_out;
  int broadcast;
  int64_t split;
  float* tail_out;
  __device__ __forceinline__ void operator()(int64_t s, const float out[1], float*, float*) const {
    float* const dst = s < split ? value_out + s * broadcast : tail_out + (s - split) * broadcast;
    for (int k = 0; k < broadcast; ++k) dst[k] = out[0];
  }
};

FusedFwdArgs fused_args(const RowSrc& X, int64_t S, int Din, const float* eff, const ParamMap& pm, int net) {
  const NetOffsets o = padded_offsets(pm, net);
  FusedFwdArgs a{};
  a.X = X; a.S = S; a.Din = Din;
  a.xvec = aligned16(X.base) && X.ld % 4 == 0 && Din % 4 == 0;
  if (!a.xvec && X.gather == nullptr && aligned16(X.base) && (X.nrows * X.ld) % 4 == 0) a.xvec = 2;
  a.W1 = eff + o.W1; a.b1 = eff + o.b1; a.W2 = eff + o.W2; a.b2 = eff + o.b2; a.W3 = eff + o.W3; a.b3 = eff + o.b3;
  a.W1s = eff + pm.sw_w1[net]; a.W2s = eff + pm.sw_w2[net]; a.kpad1 = pm.kpad1[net]; a.px = fused_forward_px(Din);
  return a;
}

struct RolloutWsView {
  float *eff_params, *h1a, *h2a, *h1c, *h2c;   // fp32 path
  bf16_t *xba, *bh1a, *bh2a, *xbc, *bh1c, *bh2c;  // bf16 configuration
};

int64_t align256(int64_t x) { return (x + 255) & ~(int64_t)255; }

RolloutWsView carve_rollout_ws(const marl_config& c, int64_t n_rows, void* ws, int64_t* total) {
  const Dims d = dims_of(c);
  const int64_t S = n_rows * d.A, Sc = d.central ? n_rows : S;
  char* p = static_cast<char*>(ws);
  int64_t off = 0;
  auto take = [&](int64_t bytes) {
    char* r = p + off;
    off += align256(bytes);
    return r;
  };
  RolloutWsView v{};
  v.eff_params = (float*)take(effective_param_floats(c) * 4);
  if (!d.bf16) {
    // hidden activations of one pass: only the layer-by-layer path stores them (the fused kernel keeps them on chip)
    if (!fused_forward_supported(d.Ha, d.D)) {
      v.h1a = (float*)take(S * d.Ha * 4);
      v.h2a = (float*)take(S * d.Ha * 4);
    }
    if (!fused_forward_supported(d.Hc, d.Dc)) {
      v.h1c = (float*)take(Sc * d.Hc * 4);
      v.h2c = (float*)take(Sc * d.Hc * 4);
    }
  } else {
    v.xba = (bf16_t*)take(S * round_up64(d.D) * 2);
    v.bh1a = (bf16_t*)take(S * d.Ha * 2);
    v.bh2a = (bf16_t*)take(S * d.Ha * 2);
    v.xbc = (bf16_t*)take(Sc * round_up64(d.Dc) * 2);
    v.bh1c = (bf16_t*)take(Sc * d.Hc * 2);
    v.bh2c = (bf16_t*)take(Sc * d.Hc * 2);
  }
  if (total) *total = off;
  return v;
}

}  // namespace

void mlp_hidden_forward(const RowSrc& X, int64_t S, int Din, int H, const float* W1, const float* b1, const float* W2,
                        const float* b2, float* h1, float* h2, bool bf16, hipStream_t s) {
  GemmArgs g{};
  g.A = X; g.B = W1; g.ldb = H; g.C = h1; g.ldc = H; g.aux_vec = b1;
  g.M = S; g.N = H; g.K = Din; g.round_bf16 = bf16;
  launch_gemm<GEMM_NN, EPI_BIAS_TANH>(g, s);
  GemmArgs g2{};
  g2.A = RowSrc{h1, H, nullptr, 1, S}; g2.B = W2; g2.ldb = H; g2.C = h2; g2.ldc = H; g2.aux_vec = b2;
  g2.M = S; g2.N = H; g2.K = H; g2.round_bf16 = bf16;
  launch_gemm<GEMM_NN, EPI_BIAS_TANH>(g2, s);
}

// Floats of the working copy: the aligned fp32 copy, followed (bf16 configuration) by the bf16 weight matrices.
int64_t effective_param_floats(const marl_config& c) {
  const Dims d = dims_of(c);
  int64_t n = param_map(d).total;
  if (d.bf16) n += (bf16_net_weight_elems(d.D, d.Ha) + bf16_net_weight_elems(d.Dc, d.Hc) + 1) / 2 + 192;  // + alignment slack
  return n;
}

Bf16NetWeights effective_bf16_weights(const marl_config& c, const float* eff, int net) {
  const Dims d = dims_of(c);
  bf16_t* base = reinterpret_cast<bf16_t*>(const_cast<float*>(eff) + ((param_map(d).total + 63) / 64) * 64);
  if (net == 0) return bf16_net_weights(base, d.D, d.Ha);
  return bf16_net_weights(base + ((bf16_net_weight_elems(d.D, d.Ha) + 63) / 64) * 64, d.Dc, d.Hc);
}

const float* effective_params(const marl_config& c, const float* params, float* scratch, hipStream_t s) {
  const Dims d = dims_of(c);
  hipLaunchKernelGGL(stage_params_kernel, dim3((unsigned)((d.P + 255) / 256)), dim3(256), 0, s, params, scratch,
                     param_map(d), (int)d.bf16);
  if (d.bf16) {
    const NetOffsets oa = net_offsets(0, d.D, d.Ha, kActions), oc = net_offsets(d.Pa, d.Dc, d.Hc, 1);
    stage_weights_bf16(params + oa.W1, params + oa.W2, d.D, d.Ha, effective_bf16_weights(c, scratch, 0), s);
    stage_weights_bf16(params + oc.W1, params + oc.W2, d.Dc, d.Hc, effective_bf16_weights(c, scratch, 1), s);
  }
  return scratch;
}

int64_t rollout_workspace_bytes(const marl_config& c, int64_t n_rows) {
  int64_t total = 0;
  carve_rollout_ws(c, n_rows, nullptr, &total);
  return total;
}

// One forward pass over n_rows observation rows.  Any of logits / value / sampling outputs may be absent.
// value_tail (nullable): the values of rows value_split .. n_rows go there instead (fused critic kernel only).
static int32_t forward_rows(const marl_config& c, const float* eff, const float* obs, int64_t n_rows,
                            const RolloutWsView& w, bool want_actor, float* logits_out, const SampleArgs* sample,
                            float* value_out, hipStream_t s, int64_t value_split = -1, float* value_tail = nullptr) {
  const Dims d = dims_of(c);
  const int64_t S = n_rows * d.A;
  if (d.bf16) {
    if (want_actor) {
      const NetOffsets o = padded_offsets(param_map(d), 0);
      const Bf16NetWeights bw = effective_bf16_weights(c, eff, 0);
      pack_obs_bf16(RowSrc{obs, d.D, nullptr, 1, S}, S, d.D, bw.Dp, S, w.xba, nullptr, s);
      mlp_hidden_forward_bf16(w.xba, S, S, d.Ha, bw, eff + o.b1, eff + o.b2, w.bh1a, nullptr, w.bh2a, s);
      launch_actor_head_rollout(w.bh2a, S, d.Ha, eff + o.W3, eff + o.b3, logits_out, sample, s);
    }
    if (value_out) {
      const NetOffsets o = padded_offsets(param_map(d), 1);
      const Bf16NetWeights bw = effective_bf16_weights(c, eff, 1);
      const int64_t Sc = d.central ? n_rows : S;
      // IPPO: the critic reads the rows packed for the actor (same rows, same width)
      const bool shared = want_actor && !d.central;
      if (!shared) pack_obs_bf16(RowSrc{obs, d.Dc, nullptr, 1, Sc}, Sc, d.Dc, bw.Dp, Sc, w.xbc, nullptr, s);
      mlp_hidden_forward_bf16(shared ? w.xba : w.xbc, Sc, Sc, d.Hc, bw, eff + o.b1, eff + o.b2, w.bh1c, nullptr, w.bh2c, s);
      launch_critic_head_rollout(w.bh2c, Sc, d.Hc, eff + o.W3, eff + o.b3, value_out, d.central ? d.A : 1, s);
    }
    return launch_status();
  }
  if (want_actor) {
    const NetOffsets o = padded_offsets(param_map(d), 0);
    const RowSrc X{obs, d.D, nullptr, 1, S};
    if (fused_forward_supported(d.Ha, d.D)) {
      ActorRolloutFinish fin{logits_out, sample ? *sample : SampleArgs{}, sample ? 1 : 0};
      const int32_t rc = launch_fused_forward<kActions, false>(d.Ha, fused_args(X, S, d.D, eff, param_map(d), 0), fin, s);
      if (rc != MARL_OK) return rc;
    } else {
      mlp_hidden_forward(X, S, d.D, d.Ha, eff + o.W1, eff + o.b1, eff + o.W2, eff + o.b2, w.h1a, w.h2a, d.bf16, s);
      launch_actor_head_rollout(w.h2a, S, d.Ha, eff + o.W3, eff + o.b3, logits_out, sample, s);
    }
  }
  if (value_out) {
    const NetOffsets o = padded_offsets(param_map(d), 1);
    const int64_t Sc = d.central ? n_rows : S;
    const RowSrc X{obs, d.Dc, nullptr, 1, Sc};
    if (fused_forward_supported(d.Hc, d.Dc)) {
      CriticRolloutFinish fin{value_out, d.central ? d.A : 1, value_tail ? value_split : Sc, value_tail};
      const int32_t rc = launch_fused_forward<1, false>(d.Hc, fused_args(X, Sc, d.Dc, eff, param_map(d), 1), fin, s);
      if (rc != MARL_OK) return rc;
    } else {
      mlp_hidden_forward(X, Sc, d.Dc, d.Hc, eff + o.W1, eff + o.b1, eff + o.W2, eff + o.b2, w.h1c, w.h2c, d.bf16, s);
      launch_critic_head_rollout(w.h2c, Sc, d.Hc, eff + o.W3, eff + o.b3, value_out, d.central ? d.A : 1, s);
    }
  }
  return launch_status();
}

int32_t launch_policy_forward(const marl_config& c, const float* params, const float* obs, int64_t n_rows,
                              float* logits, float* value, void* workspace, hipStream_t s) {
  const RolloutWsView w = carve_rollout_ws(c, n_rows, workspace, nullptr);
  const float* eff = effective_params(c, params, w.eff_params, s);
  return forward_rows(c, eff, obs, n_rows, w, logits != nullptr, logits, nullptr, value, s);
}

int32_t launch_sample(const marl_config& c, const float* logits, const float* uniforms, const int32_t* forced,
                      int64_t n, uint64_t step, int32_t* action, int32_t* sampled, float* logp, hipStream_t s) {
  SampleArgs a{};
  a.uniforms = uniforms; a.forced = forced; a.action = action; a.sampled = sampled; a.logp = logp;
  a.step = step; a.k0 = (uint32_t)(c.seed & 0xffffffffu); a.k1 = (uint32_t)(c.seed >> 32);
  launch_sample_only(logits, n, a, s);
  return launch_status();
}

static int32_t launch_rollout_fused(const marl_config& c, bool eval, const RolloutFusedArgs& a, hipStream_t s) {
  switch (c.view) {
    case 3: return launch_rollout_fused_v3(c.actor_hidden, eval, a, s);
    case 5: return launch_rollout_fused_v5(c.actor_hidden, eval, a, s);
    case 7: return launch_rollout_fused_v7(c.actor_hidden, eval, a, s);
    default: return MARL_E_CONFIG;
  }
}

// The actor's part of the arguments of the fused rollout kernel.
static RolloutFusedArgs rollout_fused_args(const marl_config& c, marl_env_state st, const float* eff) {
  const Dims d = dims_of(c);
  const ParamMap pm = param_map(d);
  const NetOffsets o = padded_offsets(pm, 0);
  RolloutFusedArgs a{};
  a.p = env_params(c);
  a.st = st;
  a.W1s = eff + pm.sw_w1[0]; a.W2s = eff + pm.sw_w2[0]; a.b1 = eff + o.b1; a.b2 = eff + o.b2; a.W3 = eff + o.W3; a.b3 = eff + o.b3;
  a.kpad1 = pm.kpad1[0];
  a.px = fused_forward_px(d.D);
  return a;
}

static bool use_fused_rollout(const marl_config& c) {
  const Dims d = dims_of(c);
  return !d.bf16 && rollout_fused_supported(d.Ha, d.A) && fused_forward_supported(d.Ha, d.D);
}

int32_t launch_rollout(const marl_config& c, marl_env_state st, const float* params, marl_traj tr,
                       uint64_t step_offset, const int32_t* forced_actions, const float* forced_uniforms,
                       void* workspace, hipStream_t s, const uint64_t* step_base) {
  const Dims d = dims_of(c);
  const RolloutWsView w = carve_rollout_ws(c, d.N, workspace, nullptr);
  const float* eff = effective_params(c, params, w.eff_params, s);
  const int64_t NA = d.NA, slab = NA * d.D;
  int32_t rc;
  // The values do not steer the rollout (the parameters are constant during it): where the critic's forward pass
  // needs no per-row workspace (the fused fp32 kernel), the values of all T steps and of the post-rollout observation
  // are computed in one pass over the stored observations afterwards instead of one small launch per step.
  const bool batch_values = !d.bf16 && fused_forward_supported(d.Hc, d.Dc);
  if (use_fused_rollout(c)) {
    // all T steps in one launch: a workgroup keeps its environments on chip and streams the trajectory out
    RolloutFusedArgs a = rollout_fused_args(c, st, eff);
    a.T = d.T;
    a.obs = tr.obs; a.action = tr.action; a.logp = tr.logp; a.reward = tr.reward; a.done = tr.done;
    a.logits = tr.logits; a.sampled = tr.sampled; a.uniforms = forced_uniforms; a.forced = forced_actions;
    a.step0 = step_offset; a.step_base = step_base;
    {
      // booked with the algorithmic flops of the actor's two hidden layers over all T steps
      const double flops = 2.0 * (double)d.T * NA * ((double)d.D * d.Ha + (double)d.Ha * d.Ha);
      TimedLaunch timed(KC_ROLLOUT, flops, s);
      if ((rc = launch_rollout_fused(c, false, a, s)) != MARL_OK) return rc;
    }
    if (!batch_values) {
      for (int t = 0; t < d.T; ++t)
        if ((rc = forward_rows(c, eff, tr.obs + (int64_t)t * slab, d.N, w, false, nullptr, nullptr, tr.value + (int64_t)t * NA, s)) != MARL_OK)
          return rc;
    }
  } else {
    rc = launch_env_step(c, st, nullptr, tr.obs, nullptr, nullptr, /*do_step=*/false, s);
    if (rc != MARL_OK) return rc;
    for (int t = 0; t < d.T; ++t) {
      SampleArgs a{};
      a.uniforms = forced_uniforms ? forced_uniforms + (int64_t)t * NA * kActions : nullptr;
      a.forced = forced_actions ? forced_actions + (int64_t)t * NA : nullptr;
      a.action = tr.action + (int64_t)t * NA;
      a.sampled = tr.sampled ? tr.sampled + (int64_t)t * NA : nullptr;
      a.logp = tr.logp + (int64_t)t * NA;
      a.step = step_offset + (uint64_t)t;
      a.step_base = step_base;
      a.k0 = (uint32_t)(c.seed & 0xffffffffu);
      a.k1 = (uint32_t)(c.seed >> 32);
      rc = forward_rows(c, eff, tr.obs + (int64_t)t * slab, d.N, w, true,
                        tr.logits ? tr.logits + (int64_t)t * NA * kActions : nullptr, &a,
                        batch_values ? nullptr : tr.value + (int64_t)t * NA, s);
      if (rc != MARL_OK) return rc;
      rc = launch_env_step(c, st, a.action, tr.obs + (int64_t)(t + 1) * slab, tr.reward + (int64_t)t * NA,
                           tr.done + (int64_t)t * d.N, true, s);
      if (rc != MARL_OK) return rc;
    }
  }
  if (batch_values) {  // slabs 0 .. T in one launch: rows of slab T go to last_value
    const int64_t Sc_split = (int64_t)d.T * (d.central ? d.N : NA);
    return forward_rows(c, eff, tr.obs, (int64_t)(d.T + 1) * d.N, w, false, nullptr, nullptr, tr.value, s, Sc_split, tr.last_value);
  }
  return forward_rows(c, eff, tr.obs + (int64_t)d.T * slab, d.N, w, false, nullptr, nullptr, tr.last_value, s);
}

// ---- greedy evaluation block ---------------------------------------------------------------------------

namespace {

__global__ void eval_zero_kernel(marl_eval_stats out, int N) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n < N) {
    out.ret_sum[n] = 0.f;
    out.len_sum[n] = 0;
    out.episodes[n] = 0;
  }
}

// action = index of the largest logit, lowest index on exact ties
__global__ void __launch_bounds__(256) greedy_kernel(const float* __restrict__ logits, int32_t* __restrict__ action, int64_t S) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S) return;
  int best = 0;
  float top = logits[i * kActions];
#pragma unroll
  for (int k = 1; k < kActions; ++k) {
    const float v = logits[i * kActions + k];
    if (v > top) {
      top = v;
      best = k;
    }
  }
  action[i] = best;
}

// Books one step into the statistics of the environments that are still inside their first n_episodes episodes:
// team reward = the agents' rewards added in ascending agent index, then added to the running sum (fp32).
__global__ void __launch_bounds__(256) eval_accumulate_kernel(const float* __restrict__ reward, const uint8_t* __restrict__ done,
                                                              marl_eval_stats out, int N, int A, int n_episodes) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  const int e = out.episodes[n];
  if (e >= n_episodes) return;
  float team = 0.f;
  for (int a = 0; a < A; ++a) team += reward[(int64_t)n * A + a];
  out.ret_sum[n] += team;
  out.len_sum[n] += 1;
  if (done[n]) out.episodes[n] = e + 1;
}

struct EvalWsView {
  void* rollout_ws;
  float *obs, *logits, *reward;
  int32_t* action;
  uint8_t* done;
};

EvalWsView carve_eval_ws(const marl_config& c, void* ws, int64_t* total) {
  const Dims d = dims_of(c);
  char* p = static_cast<char*>(ws);
  int64_t off = 0;
  auto take = [&](int64_t bytes) {
    char* r = p + off;
    off += align256(bytes);
    return r;
  };
  EvalWsView v;
  v.rollout_ws = take(rollout_workspace_bytes(c, d.N));
  v.obs = (float*)take(d.NA * d.D * 4);
  v.logits = (float*)take(d.NA * kActions * 4);
  v.reward = (float*)take(d.NA * 4);
  v.action = (int32_t*)take(d.NA * 4);
  v.done = (uint8_t*)take(d.N);
  if (total) *total = off;
  return v;
}

}  // namespace

int64_t eval_workspace_bytes(const marl_config& c) {
  int64_t total = 0;
  carve_eval_ws(c, nullptr, &total);
  return total;
}

int32_t launch_evaluate(const marl_config& c, marl_env_state st, const float* params, int32_t n_episodes,
                        marl_eval_stats out, void* workspace, hipStream_t s) {
  const Dims d = dims_of(c);
  const EvalWsView e = carve_eval_ws(c, workspace, nullptr);
  const RolloutWsView w = carve_rollout_ws(c, d.N, e.rollout_ws, nullptr);
  const float* eff = effective_params(c, params, w.eff_params, s);
  const int64_t steps = (int64_t)n_episodes * c.episode_cap;
  if (use_fused_rollout(c)) {  // the whole block in one launch, statistics in registers
    RolloutFusedArgs a = rollout_fused_args(c, st, eff);
    a.T = (int)steps;
    a.ev = out;
    a.n_episodes = n_episodes;
    return launch_rollout_fused(c, true, a, s);
  }
  const unsigned nb_env = (unsigned)((d.N + 255) / 256), nb_s = (unsigned)((d.NA + 255) / 256);
  hipLaunchKernelGGL(eval_zero_kernel, dim3(nb_env), dim3(256), 0, s, out, d.N);
  int32_t rc = launch_env_step(c, st, nullptr, e.obs, nullptr, nullptr, /*do_step=*/false, s);
  if (rc != MARL_OK) return rc;
  for (int64_t t = 0; t < steps; ++t) {
    rc = forward_rows(c, eff, e.obs, d.N, w, true, e.logits, nullptr, nullptr, s);
    if (rc != MARL_OK) return rc;
    hipLaunchKernelGGL(greedy_kernel, dim3(nb_s), dim3(256), 0, s, e.logits, e.action, d.NA);
    rc = launch_env_step(c, st, e.action, e.obs, e.reward, e.done, true, s);
    if (rc != MARL_OK) return rc;
    hipLaunchKernelGGL(eval_accumulate_kernel, dim3(nb_env), dim3(256), 0, s, e.reward, e.done, out, d.N, d.A, (int)n_episodes);
  }
  return launch_status();
}

}  // namespace marl
