// Generalised advantage estimation: one lane per (env, agent), walking the rollout backwards.
// The loads of a step do not depend on the recurrence, so they are issued in batches ahead of it.
#include "common.h"

namespace marl {
namespace {

constexpr int kGaeBatch = 8;

__global__ void __launch_bounds__(256) gae_kernel(const float* __restrict__ reward, const float* __restrict__ value,
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
  int t = T - 1;
  while (t >= 0) {
    float r[kGaeBatch], v[kGaeBatch], nd[kGaeBatch];
    const int cnt = min(kGaeBatch, t + 1);
#pragma unroll
    for (int k = 0; k < kGaeBatch; ++k)
      if (k < cnt) {
        const int64_t i = (int64_t)(t - k) * NA + lane;
        r[k] = reward[i];
        v[k] = value[i];
        nd[k] = done[(int64_t)(t - k) * N + n] ? 0.f : 1.f;
      }
#pragma unroll
    for (int k = 0; k < kGaeBatch; ++k)
      if (k < cnt) {
        const int64_t i = (int64_t)(t - k) * NA + lane;
        // contraction-free arithmetic in the order the definition states it
        const float delta = __fadd_rn(r[k], __fmul_rn(__fmul_rn(gamma, nd[k]), next_v)) - v[k];
        const float a = __fadd_rn(delta, __fmul_rn(__fmul_rn(gl, nd[k]), next_adv));
        adv[i] = a;
        ret[i] = a + v[k];
        next_adv = a;
        next_v = v[k];
      }
    t -= cnt;
  }
}

}  // namespace

int32_t launch_gae(const marl_config& c, marl_traj tr, hipStream_t s) {
  const Dims d = dims_of(c);
  const int threads = d.NA >= 256 * 1024 ? 256 : 64;
  const int64_t blocks = (d.NA + threads - 1) / threads;
  // reward, value read; adv, ret written (4 B each per env-agent step); done 1 B per env step; last_value
  TimedLaunch timed(KC_GAE, (double)d.T * (16.0 * d.NA + d.N) + 4.0 * d.NA, s);
  hipLaunchKernelGGL(gae_kernel, dim3((unsigned)blocks), dim3(threads), 0, s, tr.reward, tr.value, tr.done,
                     tr.last_value, tr.adv, tr.ret, d.T, d.N, d.A, c.gamma, c.lambda);
  return launch_status();
}

}  // namespace marl
