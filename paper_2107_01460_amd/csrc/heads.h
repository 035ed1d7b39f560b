// Output layers (6 logits / 1 value) on the vector ALUs, Gumbel-max sampling, log-softmax.
#pragma once
#include <type_traits>
#include "common.h"

namespace marl {

constexpr int kHeadTile = 64;    // samples per tile
constexpr int kHeadChunk = 128;  // hidden units staged in LDS at a time

struct SampleArgs {
  const float* uniforms;  // nullable [S][6]
  const int32_t* forced;  // nullable [S]
  int32_t* action;        // [S]
  int32_t* sampled;       // nullable [S]
  float* logp;            // [S]
  uint64_t step;
  uint32_t k0, k1;
  const uint64_t* step_base;  // nullable: a device-resident base that is added to `step`
};

struct HeadLds {
  float tile[kHeadTile * (kHeadChunk + 1)];
  float w3[kHeadChunk * kActions];
  float red[4 * kHeadTile * kActions];
};

// out[k] = sum_i H2[s0 + s][i] * W3[i][k] for the 64 samples of a tile; valid in threads tid < 64 (s = tid).
// Must be called by all 256 threads of the workgroup.
template <int NOUT, typename HT>
__device__ __forceinline__ void head_tile(const HT* __restrict__ H2, int64_t s0, int64_t S, int H,
                                          const float* __restrict__ W3, HeadLds& L, float out[NOUT]) {
  const int tid = threadIdx.x, lane = tid & 63, grp = tid >> 6;
  float acc[NOUT];
#pragma unroll
  for (int k = 0; k < NOUT; ++k) acc[k] = 0.f;
  for (int h0 = 0; h0 < H; h0 += kHeadChunk) {
    const int hc = min(kHeadChunk, H - h0);
    __syncthreads();
    {  // the chunk of the tile: all of a thread's elements are requested before the first is stored
      constexpr int PER = kHeadTile * kHeadChunk / 256;
      float v[PER];
#pragma unroll
      for (int q = 0; q < PER; ++q) {
        const int idx = tid + 256 * q, r = idx / kHeadChunk, c = idx % kHeadChunk;
        const int64_t s = s0 + r;
        v[q] = (s < S && c < hc) ? load_act(H2, s * H + h0 + c) : 0.f;
      }
#pragma unroll
      for (int q = 0; q < PER; ++q) {
        const int idx = tid + 256 * q, r = idx / kHeadChunk, c = idx % kHeadChunk;
        L.tile[r * (kHeadChunk + 1) + c] = v[q];
      }
    }
    for (int e = tid; e < hc * NOUT; e += 256) L.w3[e] = W3[(int64_t)h0 * NOUT + e];
    __syncthreads();
    const int per = hc / 4;
    for (int i = grp * per; i < (grp + 1) * per; ++i) {
      const float h = L.tile[lane * (kHeadChunk + 1) + i];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) acc[k] = fmaf(h, L.w3[i * NOUT + k], acc[k]);
    }
  }
#pragma unroll
  for (int k = 0; k < NOUT; ++k) L.red[(grp * kHeadTile + lane) * NOUT + k] = acc[k];
  __syncthreads();
  if (tid < kHeadTile) {
#pragma unroll
    for (int k = 0; k < NOUT; ++k)
      out[k] = (L.red[(0 * kHeadTile + tid) * NOUT + k] + L.red[(1 * kHeadTile + tid) * NOUT + k]) +
               (L.red[(2 * kHeadTile + tid) * NOUT + k] + L.red[(3 * kHeadTile + tid) * NOUT + k]);
  }
}

// The six uniforms of (step, sample): two Philox calls, counter (lo(step), hi(step), 2*sample + call, 2).
__device__ __forceinline__ void sample_uniforms(uint64_t step, uint32_t sample, uint32_t k0, uint32_t k1, float u[6]) {
  uint32_t o[8];
  philox4x32_10((uint32_t)step, (uint32_t)(step >> 32), sample * 2u, kStreamSample, k0, k1, o);
  philox4x32_10((uint32_t)step, (uint32_t)(step >> 32), sample * 2u + 1u, kStreamSample, k0, k1, o + 4);
#pragma unroll
  for (int k = 0; k < kActions; ++k) u[k] = rand_unit(o[k]);
}

__device__ __forceinline__ int gumbel_argmax(const float lg[kActions], const float u[kActions]) {
  float best = -INFINITY;
  int arg = 0;
#pragma unroll
  for (int k = 0; k < kActions; ++k) {
    const float z = lg[k] - logf(-logf(u[k]));
    if (z > best) {
      best = z;
      arg = k;
    }
  }
  return arg;
}

__device__ __forceinline__ float log_softmax_at(const float lg[kActions], int a) {
  float m = lg[0];
#pragma unroll
  for (int k = 1; k < kActions; ++k) m = fmaxf(m, lg[k]);
  float se = 0.f, la = 0.f;
#pragma unroll
  for (int k = 0; k < kActions; ++k) {
    se += expf(lg[k] - m);
    la = (k == a) ? lg[k] : la;
  }
  return la - m - logf(se);
}

// Returns the action taken (the forced one if given).
__device__ __forceinline__ int sample_and_store(const float lg[kActions], int64_t s, const SampleArgs& a) {
  float u[kActions];
  if (a.uniforms) {
#pragma unroll
    for (int k = 0; k < kActions; ++k) u[k] = a.uniforms[s * kActions + k];
  } else {
    sample_uniforms(a.step + (a.step_base != nullptr ? *a.step_base : 0), (uint32_t)s, a.k0, a.k1, u);
  }
  int act = gumbel_argmax(lg, u);
  if (a.sampled) a.sampled[s] = act;
  if (a.forced) act = a.forced[s];
  a.action[s] = act;
  a.logp[s] = log_softmax_at(lg, act);
  return act;
}

namespace heads_detail {

template <typename HT>
static __global__ void __launch_bounds__(256) actor_head_rollout_kernel(const HT* __restrict__ H2, int64_t S, int H,
                                                                 const float* __restrict__ W3,
                                                                 const float* __restrict__ b3, float* logits_out,
                                                                 SampleArgs a, int do_sample) {
  __shared__ HeadLds L;
  const int64_t s0 = (int64_t)blockIdx.x * kHeadTile;
  float lg[kActions];
  head_tile<kActions>(H2, s0, S, H, W3, L, lg);
  const int64_t s = s0 + threadIdx.x;
  if (threadIdx.x < kHeadTile && s < S) {
#pragma unroll
    for (int k = 0; k < kActions; ++k) lg[k] += b3[k];
    if (logits_out) {
#pragma unroll
      for (int k = 0; k < kActions; ++k) logits_out[s * kActions + k] = lg[k];
    }
    if (do_sample) sample_and_store(lg, s, a);
  }
}

template <typename HT>
static __global__ void __launch_bounds__(256) critic_head_rollout_kernel(const HT* __restrict__ H2, int64_t S, int H,
                                                                  const float* __restrict__ W3,
                                                                  const float* __restrict__ b3, float* value_out,
                                                                  int broadcast) {
  __shared__ HeadLds L;
  const int64_t s0 = (int64_t)blockIdx.x * kHeadTile;
  float v[1];
  head_tile<1>(H2, s0, S, H, W3, L, v);
  const int64_t s = s0 + threadIdx.x;
  if (threadIdx.x < kHeadTile && s < S) {
    const float val = v[0] + b3[0];
    for (int k = 0; k < broadcast; ++k) value_out[s * broadcast + k] = val;
  }
}

// The output layer for bf16 activations of up to 512 hidden units (a multiple of 64): the 32-sample tile goes to
// LDS with 16-byte loads and is read back 16 bytes at a time -- the element-wise tile of head_tile costs one 2-byte
// load per element.  out[k] is valid in threads tid < 32 (sample s0 + tid); all 256 threads must call.
constexpr int kHeadTileB = 32;
template <int NOUT>
struct HeadBf16Lds {
  static constexpr int PITCH = 512 + 8;  // elements; an odd number of 16-byte units
  bf16_t tile[kHeadTileB * PITCH];
  float w3[512 * NOUT];
  float red[8 * NOUT * kHeadTileB];
};
template <int NOUT>
__device__ __forceinline__ void head_tile_bf16(const bf16_t* __restrict__ H2, int64_t s0, int64_t S, int H,
                                               const float* __restrict__ W3, HeadBf16Lds<NOUT>& L, float out[NOUT]) {
  constexpr int PITCH = HeadBf16Lds<NOUT>::PITCH;
  const int tid = threadIdx.x, smp = tid & 31, grp = tid >> 5;  // output layer: sample smp, share grp (of 8) of the hidden units
  {  // thread -> rows tid / 64 + 4 q, 16-byte piece tid % 64 of the row; all loads before the first store
    const int c8 = tid & 63;
    uint4 v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int64_t r = min(s0 + (tid >> 6) + 4 * q, S - 1);  // rows past the end: the last row (their outputs are not used)
      v[q] = make_uint4(0u, 0u, 0u, 0u);
      if (8 * c8 < H) v[q] = *reinterpret_cast<const uint4*>(&H2[r * H + 8 * c8]);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q)
      if (8 * c8 < H) *reinterpret_cast<uint4*>(&L.tile[((tid >> 6) + 4 * q) * PITCH + 8 * c8]) = v[q];
  }
  for (int e = tid; e < H * NOUT; e += 256) L.w3[e] = W3[e];
  __syncthreads();
  float acc[NOUT];
#pragma unroll
  for (int k = 0; k < NOUT; ++k) acc[k] = 0.f;
  const int per = H / 8;  // a multiple of 8
#pragma unroll 2
  for (int i = grp * per; i < (grp + 1) * per; i += 8) {
    const uint4 hv = *reinterpret_cast<const uint4*>(&L.tile[smp * PITCH + i]);
    const uint32_t hw[4] = {hv.x, hv.y, hv.z, hv.w};
    float hh[8];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      hh[2 * q] = __uint_as_float(hw[q] << 16);
      hh[2 * q + 1] = __uint_as_float(hw[q] & 0xffff0000u);
    }
    float wv[8 * NOUT];
#pragma unroll
    for (int q = 0; q < 2 * NOUT; ++q) {
      const float4 t = *reinterpret_cast<const float4*>(&L.w3[i * NOUT + 4 * q]);
      wv[4 * q] = t.x; wv[4 * q + 1] = t.y; wv[4 * q + 2] = t.z; wv[4 * q + 3] = t.w;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int k = 0; k < NOUT; ++k) acc[k] = fmaf(hh[j], wv[j * NOUT + k], acc[k]);
  }
#pragma unroll
  for (int k = 0; k < NOUT; ++k) L.red[(grp * NOUT + k) * kHeadTileB + smp] = acc[k];
  __syncthreads();
  if (tid < kHeadTileB) {
#pragma unroll
    for (int k = 0; k < NOUT; ++k) {
      float v = 0.f;
#pragma unroll
      for (int gq = 0; gq < 8; ++gq) v += L.red[(gq * NOUT + k) * kHeadTileB + tid];
      out[k] = v;
    }
  }
}

static __global__ void __launch_bounds__(256) actor_head_rollout_bf16_kernel(const bf16_t* __restrict__ H2, int64_t S, int H,
                                                                           const float* __restrict__ W3,
                                                                           const float* __restrict__ b3, float* logits_out,
                                                                           SampleArgs a, int do_sample) {
  __shared__ __attribute__((aligned(16))) HeadBf16Lds<kActions> L;
  const int64_t s0 = (int64_t)blockIdx.x * kHeadTileB;
  float lg[kActions];
  head_tile_bf16<kActions>(H2, s0, S, H, W3, L, lg);
  const int64_t s = s0 + threadIdx.x;
  if (threadIdx.x < kHeadTileB && s < S) {
#pragma unroll
    for (int k = 0; k < kActions; ++k) lg[k] += b3[k];
    if (logits_out) {
#pragma unroll
      for (int k = 0; k < kActions; ++k) logits_out[s * kActions + k] = lg[k];
    }
    if (do_sample) sample_and_store(lg, s, a);
  }
}

static __global__ void __launch_bounds__(256) critic_head_rollout_bf16_kernel(const bf16_t* __restrict__ H2, int64_t S, int H,
                                                                            const float* __restrict__ W3,
                                                                            const float* __restrict__ b3, float* value_out,
                                                                            int broadcast) {
  __shared__ __attribute__((aligned(16))) HeadBf16Lds<1> L;
  const int64_t s0 = (int64_t)blockIdx.x * kHeadTileB;
  float v[1];
  head_tile_bf16<1>(H2, s0, S, H, W3, L, v);
  const int64_t s = s0 + threadIdx.x;
  if (threadIdx.x < kHeadTileB && s < S) {
    const float val = v[0] + b3[0];
    for (int k = 0; k < broadcast; ++k) value_out[s * broadcast + k] = val;
  }
}

static __global__ void __launch_bounds__(256) sample_only_kernel(const float* __restrict__ logits, int64_t S, SampleArgs a) {
  const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= S) return;
  float lg[kActions];
#pragma unroll
  for (int k = 0; k < kActions; ++k) lg[k] = logits[s * kActions + k];
  sample_and_store(lg, s, a);
}

}  // namespace heads_detail

template <typename HT>
inline void launch_actor_head_rollout(const HT* H2, int64_t S, int H, const float* W3, const float* b3,
                                      float* logits_out, const SampleArgs* a, hipStream_t s) {
  SampleArgs z{};
  if constexpr (std::is_same<HT, bf16_t>::value) {
    if (H <= 512 && H % 64 == 0) {
      hipLaunchKernelGGL(heads_detail::actor_head_rollout_bf16_kernel, dim3((unsigned)((S + heads_detail::kHeadTileB - 1) / heads_detail::kHeadTileB)),
                         dim3(256), 0, s, H2, S, H, W3, b3, logits_out, a ? *a : z, a ? 1 : 0);
      return;
    }
  }
  hipLaunchKernelGGL(heads_detail::actor_head_rollout_kernel<HT>, dim3((unsigned)((S + kHeadTile - 1) / kHeadTile)),
                     dim3(256), 0, s, H2, S, H, W3, b3, logits_out, a ? *a : z, a ? 1 : 0);
}
template <typename HT>
inline void launch_critic_head_rollout(const HT* H2, int64_t S, int H, const float* W3, const float* b3,
                                       float* value_out, int broadcast, hipStream_t s) {
  if constexpr (std::is_same<HT, bf16_t>::value) {
    if (H <= 512 && H % 64 == 0) {
      hipLaunchKernelGGL(heads_detail::critic_head_rollout_bf16_kernel, dim3((unsigned)((S + heads_detail::kHeadTileB - 1) / heads_detail::kHeadTileB)),
                         dim3(256), 0, s, H2, S, H, W3, b3, value_out, broadcast);
      return;
    }
  }
  hipLaunchKernelGGL(heads_detail::critic_head_rollout_kernel<HT>, dim3((unsigned)((S + kHeadTile - 1) / kHeadTile)),
                     dim3(256), 0, s, H2, S, H, W3, b3, value_out, broadcast);
}
inline void launch_sample_only(const float* logits, int64_t S, const SampleArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(heads_detail::sample_only_kernel, dim3((unsigned)((S + 255) / 256)), dim3(256), 0, s, logits, S,
                     a);
}

}  // namespace marl
