// The whole rollout as ONE kernel: a workgroup owns a block of environments for all T time steps.
//
// Environments never interact and the parameters are constant during a rollout, so nothing has to be exchanged
// between workgroups: each keeps the state of its BM / A environments in the registers of one lane per env-agent,
// paints the agents' observation windows straight into the LDS tile that is the A operand of the actor's first
// layer, runs both hidden layers on the matrix cores (weights from the operand-order copies in L2, as in
// fused_forward_kernel), the output layer and the Gumbel-max sampling on the ALUs, hands the actions to the env lanes
// through cross-lane reads, resolves the transition in registers, and paints the next observation -- only the
// trajectory (observations, actions, log-probabilities, rewards, dones) is streamed out.  The critic's values do not
// steer the rollout and are computed in one pass over the stored observations afterwards.
//
// The same kernel with EVAL = true is the greedy evaluation block: argmax actions, no trajectory, and the
// per-environment return / length / episode counts accumulated in registers.
#pragma once
#include "env_device.h"
#include "fused_forward.h"

namespace marl {

struct RolloutFusedArgs {
  EnvParams p;
  marl_env_state st;
  const float *W1s, *W2s, *b1, *b2, *W3, *b3;  // actor: operand-order W1 / W2, aligned biases and output layer
  int kpad1, px;
  int T;  // steps to take
  // training rollout
  float* obs;  // [T+1][N][A][D]
  int32_t* action;
  float* logp;
  float* reward;
  uint8_t* done;
  float* logits;     // nullable
  int32_t* sampled;  // nullable
  const float* uniforms;  // nullable [T][N][A][6]
  const int32_t* forced;  // nullable [T][N][A]
  uint64_t step0;
  const uint64_t* step_base;  // nullable
  // evaluation block
  marl_eval_stats ev;
  int n_episodes;
};

template <int H, int BM, int V, int CA, int KIND, bool EVAL>
__global__ void __launch_bounds__(256) rollout_fused_kernel(RolloutFusedArgs a) {
  constexpr int D = 3 * V * V, PH = H + 4, GROUPS = 256 / BM, NOUT = kActions;
  constexpr int NTN = H / 32, MT = BM / 32, TILES = MT * NTN;
  static_assert(TILES == 4, "one 32x32 MFMA tile per wavefront");
  static_assert(BM <= 64, "the env lanes are lanes of the first wavefront");
  extern __shared__ __attribute__((aligned(16))) float lds[];
  const int px = a.px;
  float* const Xs = lds;                       // [BM][px]  observation windows, k-contiguous; columns D .. px stay zero
  float* const Hs = Xs + BM * px;              // [BM][PH]  h1, then h2
  float* const red = Hs + BM * PH;             // [GROUPS][BM][NOUT]
  float* const W3s = red + GROUPS * BM * NOUT; // [H][NOUT]

  const EnvParams& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = lane & 31, hi = lane >> 5;
  const int mt = wave / NTN, nt = wave % NTN;
  const int A = p.A, N = p.N;
  const int epw = BM / A;  // envs of this workgroup
  const int64_t env0 = (int64_t)blockIdx.x * epw;
  const int envs_here = (int)min((int64_t)epw, (int64_t)N - env0);
  const int samples_here = envs_here * A;
  const int64_t NA = (int64_t)N * A;
  const int64_t s_glob = env0 * A + tid;  // this env lane's sample index

  // ---- env lanes: lane tid < BM of the first wavefront is agent tid % A of env env0 + tid / A
  const int le = tid / A, ai = tid - le * A;
  const bool active = tid < samples_here;
  const int64_t n = env0 + le;
  const size_t nn = active ? (size_t)n : 0;
  uint32_t ag[CA], fd[CA];
  int t_ep = 0;
  uint32_t episode = 0;
  float ret_sum = 0.f;
  int len_sum = 0, episodes = 0;

  for (int i = tid; i < H * NOUT; i += 256) W3s[i] = a.W3[i];
  for (int i = tid; i < BM * px; i += 256) Xs[i] = 0.f;  // padding columns and unused rows stay zero for good
  if (wave == 0) {
    load_env_state<CA, CA, KIND>(ag, fd, a.st, p, nn, active);
    t_ep = a.st.t_in_ep[nn];
    episode = a.st.episode_id[nn];
  }
  __syncthreads();
  if (wave == 0 && active) {
    if (KIND == 0) forage_paint<V, CA, CA>(Xs + tid * px, ag, fd, ai, p);
    else wh_paint<V, CA, CA>(Xs + tid * px, ag, fd, ai, p);
  }
  const uint64_t step_base = (!EVAL && a.step_base != nullptr) ? *a.step_base : 0;

  for (int t = 0;; ++t) {
    __syncthreads();  // the windows of step t are complete
    if (!EVAL) {      // the tile's rows are one contiguous piece of slab t
      float* const out = a.obs + ((int64_t)t * N + env0) * A * D;
      const int count = samples_here * D;
      for (int i = tid; i < count; i += 256) {
        const int r = i / D, c = i - r * D;
        out[i] = Xs[r * px + c];
      }
    }
    if (t == a.T) break;
    // ---- layer 1: h1 = tanh(X W1 + b1) -> LDS
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    gemm_phase_regs<H>(Xs + (mt * 32 + lo) * px + 4 * hi, a.W1s + (hi * H + nt * 32 + lo) * 4, a.kpad1 / 16, acc);
    {
      const int col = nt * 32 + lo;
      const float bias = a.b1[col];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        Hs[m * PH + col] = tanh_f32(acc[r] + bias);
      }
    }
    __syncthreads();  // h1 complete; every wavefront is past its reads of the windows
    // ---- layer 2: h2 = tanh(h1 W2 + b2)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    gemm_phase_regs<H>(Hs + (mt * 32 + lo) * PH + 4 * hi, a.W2s + (hi * H + nt * 32 + lo) * 4, H / 16, acc);
    __syncthreads();  // every wavefront is past its last read of h1
    {
      const int col = nt * 32 + lo;
      const float bias = a.b2[col];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        Hs[m * PH + col] = tanh_f32(acc[r] + bias);
      }
    }
    __syncthreads();
    // ---- output layer on the ALUs: thread -> (sample tid % BM, slice tid / BM of the hidden units)
    {
      const int s = tid % BM, grp = tid / BM;
      constexpr int PER = H / GROUPS;
      static_assert(PER % 4 == 0, "hidden units are read four at a time");
      float part[NOUT];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) part[k] = 0.f;
#pragma unroll 2
      for (int i = grp * PER; i < (grp + 1) * PER; i += 4) {
        const float4 hv = *reinterpret_cast<const float4*>(&Hs[s * PH + i]);
        const float hh[4] = {hv.x, hv.y, hv.z, hv.w};
        float wv[4 * NOUT];
#pragma unroll
        for (int q = 0; q < NOUT; ++q) {
          const float4 w4 = *reinterpret_cast<const float4*>(&W3s[i * NOUT + 4 * q]);
          wv[4 * q] = w4.x; wv[4 * q + 1] = w4.y; wv[4 * q + 2] = w4.z; wv[4 * q + 3] = w4.w;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int k = 0; k < NOUT; ++k) part[k] = fmaf(hh[j], wv[j * NOUT + k], part[k]);
      }
#pragma unroll
      for (int k = 0; k < NOUT; ++k) red[(grp * BM + s) * NOUT + k] = part[k];
    }
    __syncthreads();
    // ---- the env lanes: logits -> action -> transition -> next window.  Whole first wavefront, so that the cross-lane
    // reads below find their source lanes running.
    if (wave == 0) {
      const int row = tid < BM ? tid : 0;
      float lg[NOUT];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) {
        float v = a.b3[k];
#pragma unroll
        for (int gq = 0; gq < GROUPS; ++gq) v += red[(gq * BM + row) * NOUT + k];
        lg[k] = v;
      }
      int my_act = 0;
      if (active) {
        if (EVAL) {  // largest logit, lowest index on exact ties
          float top = lg[0];
#pragma unroll
          for (int k = 1; k < NOUT; ++k)
            if (lg[k] > top) {
              top = lg[k];
              my_act = k;
            }
        } else {
          const int64_t o = (int64_t)t * NA;
          if (a.logits) {
#pragma unroll
            for (int k = 0; k < NOUT; ++k) a.logits[(o + s_glob) * NOUT + k] = lg[k];
          }
          SampleArgs sa;
          sa.uniforms = a.uniforms ? a.uniforms + o * NOUT : nullptr;
          sa.forced = a.forced ? a.forced + o : nullptr;
          sa.action = a.action + o;
          sa.sampled = a.sampled ? a.sampled + o : nullptr;
          sa.logp = a.logp + o;
          sa.step = a.step0 + step_base + (uint64_t)t;
          sa.k0 = p.k0; sa.k1 = p.k1;
          sa.step_base = nullptr;
          my_act = sample_and_store(lg, s_glob, sa);
        }
      }
      int act[CA];
#pragma unroll
      for (int b = 0; b < CA; ++b) {
        const int v = __shfl(my_act, min(le * A + b, 63));
        act[b] = (active && b < A) ? v : 0;
      }
      float rew;
      bool dn;
      if (KIND == 0) forage_transition<CA, CA>(ag, fd, act, ai, active, p, (uint32_t)n, t_ep, episode, rew, dn);
      else wh_transition<CA, CA>(ag, fd, act, ai, active, p, (uint32_t)n, t_ep, episode, rew, dn);
      if (EVAL) {
        // team reward = the agents' rewards added in ascending agent index, then added to the running sum (fp32)
        float team = 0.f;
#pragma unroll
        for (int b = 0; b < CA; ++b) {
          const float rb = __shfl(rew, min(le * A + b, 63));
          if (b < A) team += rb;
        }
        if (active && episodes < a.n_episodes) {
          ret_sum += team;
          len_sum += 1;
          if (dn) episodes += 1;
        }
      } else if (active) {
        a.reward[(int64_t)t * NA + s_glob] = rew;
        if (ai == 0) a.done[(int64_t)t * N + n] = dn ? 1 : 0;
      }
      if (active) {
        if (KIND == 0) forage_paint<V, CA, CA>(Xs + tid * px, ag, fd, ai, p);
        else wh_paint<V, CA, CA>(Xs + tid * px, ag, fd, ai, p);
      }
    }
  }
  if (wave == 0 && active) {
    store_env_state<CA, CA, KIND>(ag, fd, a.st, p, (size_t)n, ai, /*dn=*/true, t_ep, episode);
    if (EVAL && ai == 0) {
      a.ev.ret_sum[n] = ret_sum;
      a.ev.len_sum[n] = len_sum;
      a.ev.episodes[n] = episodes;
    }
  }
}

// Networks and views the kernel is instantiated for: hidden width 64 (64-sample tiles) or 128 (32-sample tiles).
inline bool rollout_fused_supported(int H, int A) { return (H == 64 || H == 128) && A <= 8; }
inline int rollout_fused_bm(int H) { return H == 64 ? 64 : 32; }

template <int H, int BM, int V, int CA, int KIND, bool EVAL>
inline int32_t launch_rollout_fused_inst(const RolloutFusedArgs& a, hipStream_t s) {
  auto kern = rollout_fused_kernel<H, BM, V, CA, KIND, EVAL>;
  const size_t bytes = ((size_t)BM * a.px + (size_t)BM * (H + 4) + 256 * (size_t)kActions + (size_t)H * kActions) * sizeof(float);
  static bool configured = false;  // per instantiation
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
      return MARL_E_LAUNCH;
    configured = true;
  }
  const int epw = BM / a.p.A;
  const unsigned grid = (unsigned)((a.p.N + epw - 1) / epw);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), bytes, s, a);
  return launch_status();
}

template <int V, int KIND, bool EVAL>
inline int32_t launch_rollout_fused_view(int H, const RolloutFusedArgs& a, hipStream_t s) {
  const int cap = a.p.A > a.p.F ? a.p.A : a.p.F;  // every loop over entities is unrolled to the capacity
  if (H == 64) {
    if (cap <= 4) return launch_rollout_fused_inst<64, 64, V, 4, KIND, EVAL>(a, s);
    return launch_rollout_fused_inst<64, 64, V, 8, KIND, EVAL>(a, s);
  }
  if (cap <= 4) return launch_rollout_fused_inst<128, 32, V, 4, KIND, EVAL>(a, s);
  return launch_rollout_fused_inst<128, 32, V, 8, KIND, EVAL>(a, s);
}

// Defined in rollout_v3.hip / rollout_v5.hip / rollout_v7.hip (one translation unit per view size).
int32_t launch_rollout_fused_v3(int H, bool eval, const RolloutFusedArgs& a, hipStream_t s);
int32_t launch_rollout_fused_v5(int H, bool eval, const RolloutFusedArgs& a, hipStream_t s);
int32_t launch_rollout_fused_v7(int H, bool eval, const RolloutFusedArgs& a, hipStream_t s);

template <int V>
inline int32_t launch_rollout_fused_tu(int H, bool eval, const RolloutFusedArgs& a, hipStream_t s) {
  if (a.p.kind == 0) {
    if (eval) return launch_rollout_fused_view<V, 0, true>(H, a, s);
    return launch_rollout_fused_view<V, 0, false>(H, a, s);
  }
  if (eval) return launch_rollout_fused_view<V, 1, true>(H, a, s);
  return launch_rollout_fused_view<V, 1, false>(H, a, s);
}

}  // namespace marl
