// Generalised advantage estimation: one lane per (env, agent), walking the rollout backwards.
// The loads of a step do not depend on the recurrence, so each lane keeps two register batches of
// kGaeBatch steps: the recurrence runs over one while the loads of the next are in flight.  With
// 64-thread workgroups even the small configurations spread over all CUs.
#include "common.h"

namespace marl {
namespace {

constexpr int kGaeBatch = 16;

struct GaeBatch {
  float r[kGaeBatch], v[kGaeBatch];
  uint8_t d[kGaeBatch];
};

__device__ __forceinline__ void gae_load(GaeBatch& b, const float* __restrict__ reward, const float* __restrict__ value,
                                         const uint8_t* __restrict__ done, int64_t NA, int N, int64_t lane, int n,
                                         int t_hi) {
#pragma unroll
  for (int k = 0; k < kGaeBatch; ++k) {
    const int t = t_hi - k;
    if (t >= 0) {
      const int64_t i = (int64_t)t * NA + lane;
      b.r[k] = reward[i];
      b.v[k] = value[i];
      b.d[k] = done[(int64_t)t * N + n];
    }
  }
}

__global__ void __launch_bounds__(64) gae_kernel(const float* __restrict__ reward, const float* __restrict__ value,
                                                 const uint8_t* __restrict__ done,
                                                 const float* __restrict__ last_value, float* __restrict__ adv,
                                                 float* __restrict__ ret, int T, int N, int A, float gamma,
                                                 float lambda) {
  const int64_t NA = (int64_t)N * A;
  const int64_t lane = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (lane >= NA) return;
  const int n = (int)(lane / A);
  float next_adv = 0.f, next_v = last_value[lane];
  const float gl = gamma * lambda;
  GaeBatch cur, nxt;
  gae_load(cur, reward, value, done, NA, N, lane, n, T - 1);
  for (int t_hi = T - 1; t_hi >= 0; t_hi -= kGaeBatch) {
    if (t_hi - kGaeBatch >= 0) gae_load(nxt, reward, value, done, NA, N, lane, n, t_hi - kGaeBatch);
#pragma unroll
    for (int k = 0; k < kGaeBatch; ++k) {
      const int t = t_hi - k;
      if (t >= 0) {
        const int64_t i = (int64_t)t * NA + lane;
        const float nd = cur.d[k] ? 0.f : 1.f;
        // contraction-free arithmetic in the order the definition states it
        const float delta = __fadd_rn(cur.r[k], __fmul_rn(__fmul_rn(gamma, nd), next_v)) - cur.v[k];
        const float a = __fadd_rn(delta, __fmul_rn(__fmul_rn(gl, nd), next_adv));
        adv[i] = a;
        ret[i] = a + cur.v[k];
        next_adv = a;
        next_v = cur.v[k];
      }
    }
    cur = nxt;
  }
}

}  // namespace

int32_t launch_gae(const marl_config& c, marl_traj tr, hipStream_t s) {
  const Dims d = dims_of(c);
  const int threads = 64;
  const int64_t blocks = (d.NA + threads - 1) / threads;
  // reward, value read; adv, ret written (4 B each per env-agent step); done 1 B per env step; last_value
  TimedLaunch timed(KC_GAE, (double)d.T * (16.0 * d.NA + d.N) + 4.0 * d.NA, s);
  hipLaunchKernelGGL(gae_kernel, dim3((unsigned)blocks), dim3(threads), 0, s, tr.reward, tr.value, tr.done,
                     tr.last_value, tr.adv, tr.ret, d.T, d.N, d.A, c.gamma, c.lambda);
  return launch_status();
}

}  // namespace marl
