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

// log-softmax(lg)[a] with the hardware exp2 / log2 units (a value, not a decision: the relative error of about
// 1e-6 is far inside the tolerance of a log-probability)
__device__ __forceinline__ float log_softmax_fast(const float lg[kActions], int a) {
  float m = lg[0];
#pragma unroll
  for (int k = 1; k < kActions; ++k) m = fmaxf(m, lg[k]);
  float se = 0.f, la = 0.f;
#pragma unroll
  for (int k = 0; k < kActions; ++k) {
    se += __builtin_amdgcn_exp2f((lg[k] - m) * 1.4426950408889634f);
    la = (k == a) ? lg[k] : la;
  }
  return la - m - __builtin_amdgcn_logf(se) * 0.6931471805599453f;
}

template <int H, int BM, int V, int CA, int KIND, bool EVAL>
__global__ void __launch_bounds__(256, ((H == 64 && CA <= 2) || (CA <= 4 && V <= 5)) ? 3 : 1) rollout_fused_kernel(RolloutFusedArgs a) {
  constexpr int D = 3 * V * V, PH = H + 4, GROUPS = 256 / BM, NOUT = kActions;
  constexpr int NTN = H / 32, MT = BM / 32, TILES = MT * NTN;
  static_assert(TILES == 4, "one 32x32 MFMA tile per wavefront");
  static_assert(BM <= 64, "the env lanes are lanes of one wavefront");
  extern __shared__ __attribute__((aligned(16))) float lds[];
  const int px = a.px;
  float* const Xs2 = lds;                      // [2][BM][px]  observation windows of two consecutive steps, k-contiguous;
                                               //              columns D .. px stay zero
  float* const Hs = Xs2 + 2 * BM * px;         // [BM][PH]  h1, then h2
  float* const red = Hs + BM * PH;             // [GROUPS][BM][NOUT]
  float* const W3s = red + GROUPS * BM * NOUT; // [H][NOUT]
  float* const noise = W3s + H * NOUT;         // [2][BM][8] log(-log u) of the step's uniforms, two steps alternating

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

  // ---- env lanes: lane l < BM of ONE wavefront is agent l % A of env env0 + l / A.  Which wavefront it is rotates
  // with the workgroup index, so that the workgroups of a CU keep their serial sections on different SIMDs.
  const int env_wave = blockIdx.x & 3;
  const bool is_env_wave = wave == env_wave;
  const int le = lane / A, ai = lane - le * A;
  const bool active = is_env_wave && lane < samples_here;
  const int64_t n = env0 + le;
  const size_t nn = active ? (size_t)n : 0;
  const int64_t s_glob = env0 * A + lane;  // this env lane's sample index
  // ---- the other three wavefronts draw the sampling noise of the NEXT step while the env lanes work: it depends on
  // (step, sample) only.  Thread j of them: sample slot j % BM, Philox call j / BM (call 0: actions 0..3, call 1: 4, 5).
  const int nz_j = ((wave - env_wave - 1) & 3) * 64 + lane;
  const bool nz_on = !EVAL && !is_env_wave && nz_j < 2 * BM && (nz_j % BM) < samples_here;
  const int nz_s = nz_j % BM, nz_call = nz_j / BM;
  uint32_t ag[CA], fd[CA];
  int t_ep = 0;
  uint32_t episode = 0;
  float ret_sum = 0.f;
  int len_sum = 0, episodes = 0;
  const uint64_t step_base = (!EVAL && a.step_base != nullptr) ? *a.step_base : 0;

  auto draw_noise = [&](int t) {  // noise of step t into buffer t & 1
    if (!nz_on) return;
    float* const dst = noise + ((t & 1) * BM + nz_s) * 8 + 4 * nz_call;
    const int64_t s = env0 * A + nz_s;
    float u[4];
    if (a.uniforms) {
      const float* src = a.uniforms + ((int64_t)t * NA + s) * NOUT + 4 * nz_call;
#pragma unroll
      for (int k = 0; k < 4; ++k) u[k] = (4 * nz_call + k < NOUT) ? src[k] : 0.5f;
    } else {
      const uint64_t step = a.step0 + step_base + (uint64_t)t;
      uint32_t o[4];
      philox4x32_10((uint32_t)step, (uint32_t)(step >> 32), (uint32_t)s * 2u + (uint32_t)nz_call, kStreamSample, p.k0, p.k1, o);
#pragma unroll
      for (int k = 0; k < 4; ++k) u[k] = rand_unit(o[k]);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) dst[k] = logf(-logf(u[k]));  // the same fp32 operations as the per-step sampler
  };

  for (int i = tid; i < H * NOUT; i += 256) W3s[i] = a.W3[i];
  for (int i = tid; i < 2 * BM * px; i += 256) Xs2[i] = 0.f;  // padding columns and unused rows stay zero for good
  if (is_env_wave) {
    load_env_state<CA, CA, KIND>(ag, fd, a.st, p, nn, active);
    t_ep = a.st.t_in_ep[nn];
    episode = a.st.episode_id[nn];
  }
  __syncthreads();
  if (active) {
    if (KIND == 0) forage_paint<V, CA, CA>(Xs2 + lane * px, ag, fd, ai, p);
    else wh_paint<V, CA, CA>(Xs2 + lane * px, ag, fd, ai, p);
  }
  if (a.T > 0) draw_noise(0);
  // the biases of this lane's column and of the output layer stay in registers for all T steps
  const float bias1 = a.b1[nt * 32 + lo], bias2 = a.b2[nt * 32 + lo];
  float b3r[NOUT];
#pragma unroll
  for (int k = 0; k < NOUT; ++k) b3r[k] = a.b3[k];
  // The windows of step t sit in tile t & 1: while the env lanes paint the windows of step t + 1 into the other tile, the
  // wavefronts that are idle then copy tile t & 1 out as slab t of the trajectory.  Thread j of them (0 .. 191).
  auto store_slab = [&](int t, int j, int nthreads) {
    const float* const Xt = Xs2 + (t & 1) * BM * px;
    float* const out = a.obs + ((int64_t)t * N + env0) * A * D;
    const int count = samples_here * D;
    for (int i = j; i < count; i += nthreads) {
      const int r = i / D, c = i - r * D;
      out[i] = Xt[r * px + c];
    }
  };

  // the weights of a whole layer are requested a phase ahead (buffer loads: one descriptor, one lane offset)
  constexpr int KG1 = (D + 15) / 16, KG2 = H / 16;
  const int wlane = (hi * H + nt * 32 + lo) * 4;
  const WeightRsrc rsW1 = weight_rsrc(a.W1s, a.kpad1 * H), rsW2 = weight_rsrc(a.W2s, H * H);
  PhaseW<KG1> pw1;
  phase_w_request<H, KG1>(pw1, rsW1, wlane, a.kpad1 / 16);
  for (int t = 0;; ++t) {
    __syncthreads();  // the windows (and the noise) of step t are complete
    if (t == a.T) {
      if (!EVAL) store_slab(t, tid, 256);  // the post-rollout observation
      break;
    }
    const float* const Xs = Xs2 + (t & 1) * BM * px;
    // ---- layer 1: h1 = tanh(X W1 + b1) -> LDS
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    gemm_phase_w<KG1>(Xs + (mt * 32 + lo) * px + 4 * hi, a.kpad1 / 16, acc, pw1);
    PhaseW<KG2> pw2;  // layer 2's weights arrive during the tanh of layer 1
    phase_w_request<H, KG2>(pw2, rsW2, wlane, KG2);
    {
      const int col = nt * 32 + lo;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        Hs[m * PH + col] = tanh_f32(acc[r] + bias1);
      }
    }
    __syncthreads();  // h1 complete; every wavefront is past its reads of the windows
    // ---- layer 2: h2 = tanh(h1 W2 + b2)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    gemm_phase_w<KG2>(Hs + (mt * 32 + lo) * PH + 4 * hi, KG2, acc, pw2);
    phase_w_request<H, KG1>(pw1, rsW1, wlane, a.kpad1 / 16);  // layer 1 of the next step
    __syncthreads();  // every wavefront is past its last read of h1
    {
      const int col = nt * 32 + lo;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        Hs[m * PH + col] = tanh_f32(acc[r] + bias2);
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
    if (!is_env_wave) {
      if (t + 1 < a.T) draw_noise(t + 1);
      if (!EVAL) store_slab(t, ((wave - env_wave - 1) & 3) * 64 + lane, 192);
    } else {
      // ---- the env lanes: logits -> action -> transition -> next window.  The whole wavefront runs this, so that the
      // cross-lane reads below find their source lanes running.
      const int row = lane < BM ? lane : 0;
      float lg[NOUT];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) {
        float v = b3r[k];
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
          const int64_t o = (int64_t)t * NA + s_glob;
          if (a.logits) {
#pragma unroll
            for (int k = 0; k < NOUT; ++k) a.logits[o * NOUT + k] = lg[k];
          }
          // Gumbel-max: argmax_k lg[k] - log(-log u[k]), lowest k on exact ties
          const float* const g = noise + ((t & 1) * BM + lane) * 8;
          const float4 g0 = *reinterpret_cast<const float4*>(g);
          const float2 g1 = *reinterpret_cast<const float2*>(g + 4);
          const float gk[NOUT] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y};
          float best = -INFINITY;
#pragma unroll
          for (int k = 0; k < NOUT; ++k) {
            const float z = lg[k] - gk[k];
            if (z > best) {
              best = z;
              my_act = k;
            }
          }
          if (a.sampled) a.sampled[o] = my_act;
          if (a.forced) my_act = a.forced[o];
          a.action[o] = my_act;
          a.logp[o] = log_softmax_fast(lg, my_act);
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
      if (active) {  // the windows of step t + 1 into the other tile
        float* const Xn = Xs2 + ((t + 1) & 1) * BM * px;
        if (KIND == 0) forage_paint<V, CA, CA>(Xn + lane * px, ag, fd, ai, p);
        else wh_paint<V, CA, CA>(Xn + lane * px, ag, fd, ai, p);
      }
    }
  }
  if (active) {
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
  const size_t bytes = (2 * (size_t)BM * a.px + (size_t)BM * (H + 4) + 256 * (size_t)kActions + (size_t)H * kActions + 2 * BM * 8) * sizeof(float);
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
  if constexpr (V == 3 && KIND == 0) {  // the small foraging shape (two agents, one food): half the unrolled entity loops
    if (cap <= 2 && H == 64) return launch_rollout_fused_inst<64, 64, V, 2, KIND, EVAL>(a, s);
  }
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
