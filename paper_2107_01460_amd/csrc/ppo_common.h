// Pieces of the PPO update shared by the feed-forward and the recurrent drivers: per-minibatch device scalars,
// the actor and critic loss functors (loss terms and dL/d(output) of one sample), the output-layer + loss
// kernel of the layer-wise paths, advantage statistics, gradient-norm and Adam kernels.
#pragma once
#include <algorithm>
#include <cmath>

#include "gemm.h"
#include "heads.h"

namespace marl {
namespace {

constexpr int kNormBlocks = 256;

// Device scalars of one minibatch step.
struct Scalars {
  double adv_sum, adv_sq;  // sum of the minibatch's advantages, sum of their squares
  float acc[8];            // 0 policy loss, 1 value loss, 2 entropy, 3 approx KL, 4 clip fraction
  double norm_part[kNormBlocks];  // |grad|^2 summed per workgroup of grad_norm_kernel; adam_kernel adds them in order
};

struct LossCommon {
  const int32_t* rows;  // [rows_mb] trajectory row of each minibatch row
  int A;
  SmallDiv ad;          // make_small_div(A)
  int64_t rows_mb;
  float inv_B;  // 1 / (rows_mb * A)
  const Scalars* sc;
  const double* adv_stats;  // sum and sum of squares of this minibatch's advantages
  int normalize;
  float clip_eps, ent_coef, vf_coef;
  int clip_value;
};

__global__ void iota_kernel(int32_t* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = (int32_t)i;
}

// Zeroes the gradient, `nsc` sets of scalars and `nextra` doubles (nullable).
__global__ void zero_step_kernel(float* grad, int64_t P, Scalars* sc, int nsc, double* extra, int nextra) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < P) grad[i] = 0.f;
  if (i < nsc) {
    sc[i].adv_sum = 0.0;
    sc[i].adv_sq = 0.0;
    for (int k = 0; k < 8; ++k) sc[i].acc[k] = 0.f;
  }
  if (extra != nullptr)
    for (int64_t j = i; j < nextra; j += (int64_t)gridDim.x * blockDim.x) extra[j] = 0.0;
}

__device__ __forceinline__ double block_sum_f64(double v, double* red) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  double t = 0;
  if (threadIdx.x == 0)
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += red[w];
  return t;  // valid in thread 0
}

// Sum and sum of squares of the minibatch's advantages, both in fp64 (the variance is their difference: with fp32
// inputs and fp64 sums the cancellation costs nothing that matters until the spread is 1e-6 of the mean).
__global__ void __launch_bounds__(256) adv_stats_kernel(const float* __restrict__ adv, LossCommon lc, Scalars* sc) {
  __shared__ double red[2][4];
  const int64_t B = lc.rows_mb * lc.A;
  double sum = 0, sq = 0;
  for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s < B; s += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = s / lc.A;
    const int a = (int)(s - row * lc.A);
    const double x = adv[(int64_t)lc.rows[row] * lc.A + a];
    sum += x;
    sq += x * x;
  }
  const double t0 = block_sum_f64(sum, red[0]);
  const double t1 = block_sum_f64(sq, red[1]);
  if (threadIdx.x == 0) {
    atomicAdd(&sc->adv_sum, t0);
    atomicAdd(&sc->adv_sq, t1);
  }
}

// The same for every minibatch of an update in one launch: blockIdx.y = e * n_minibatches + mb; the row order of
// epoch e starts at rows + e * epoch_stride, minibatch mb takes its rows mb * rows_mb .. ; out[2 (e * n_minibatches + mb)]
// gets the sum, the next double the sum of squares (zeroed before the launch).
__global__ void __launch_bounds__(256) adv_stats_all_kernel(const float* __restrict__ adv, const int32_t* __restrict__ rows,
                                                            int64_t epoch_stride, int n_minibatches, int64_t rows_mb, int A,
                                                            double* __restrict__ out) {
  __shared__ double red[2][4];
  const int m = blockIdx.y, e = m / n_minibatches, mb = m - e * n_minibatches;
  const int32_t* const r0 = rows + e * epoch_stride + (int64_t)mb * rows_mb;
  const int64_t B = rows_mb * A;
  double sum = 0, sq = 0;
  for (int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; s < B; s += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = s / A;
    const int a = (int)(s - row * A);
    const double x = adv[(int64_t)r0[row] * A + a];
    sum += x;
    sq += x * x;
  }
  const double t0 = block_sum_f64(sum, red[0]);
  const double t1 = block_sum_f64(sq, red[1]);
  if (threadIdx.x == 0) {
    atomicAdd(&out[2 * m], t0);
    atomicAdd(&out[2 * m + 1], t1);
  }
}

// exp and log on the hardware exp2 / log2 units (1 ulp each; the arguments here are O(1))
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.4426950408889634f); }
__device__ __forceinline__ float fast_log(float x) { return __builtin_amdgcn_logf(x) * 0.6931471805599453f; }

// Per-minibatch constants of a loss, computed once per thread instead of once per sample.
struct LossPrep {
  float mean, rstd;
};

struct ActorLoss {
  LossCommon lc;
  const int32_t* action;
  const float* logp_old;
  const float* adv;
  struct In {
    int act;
    float logp_old, adv;
  };
  // the trajectory values of minibatch sample s (separate from the arithmetic so that they can be fetched early);
  // row_entry / load_with split the dependent pair of loads so that the first can be issued a phase ahead
  // (FAST: the magic-number division of SmallDiv, for callers that have checked small_div_ok(lc.ad, samples))
  template <bool FAST = false>
  __device__ __forceinline__ int32_t row_entry(int64_t s) const { return lc.rows[lc.ad.div<FAST>(s, lc.A)]; }
  template <bool FAST = false>
  __device__ __forceinline__ In load_with(int64_t s, int32_t entry) const {
    const int a = (int)(s - lc.ad.div<FAST>(s, lc.A) * lc.A);
    const int64_t src = (int64_t)entry * lc.A + a;
    return In{action[src], logp_old[src], adv[src]};
  }
  __device__ __forceinline__ In load(int64_t s) const { return load_with(s, row_entry(s)); }
  __device__ __forceinline__ LossPrep prepare() const {
    LossPrep p{0.f, 1.f};
    if (lc.normalize) {
      const double B = (double)lc.rows_mb * lc.A;
      const double mean = lc.adv_stats[0] / B;
      p.mean = (float)mean;
      p.rstd = (float)(1.0 / (sqrt(fmax(lc.adv_stats[1] / B - mean * mean, 0.0)) + 1e-8));
    }
    return p;
  }
  // returns dL/dlogits in dl; adds this sample's terms to st[0..4]
  __device__ __forceinline__ void compute(const In& in, const LossPrep& prep, const float out[kActions], float dl[kActions],
                                          float st[5]) const {
    const int act = in.act;
    float m = out[0];
#pragma unroll
    for (int k = 1; k < kActions; ++k) m = fmaxf(m, out[k]);
    float ex[kActions], se = 0.f;
#pragma unroll
    for (int k = 0; k < kActions; ++k) {
      ex[k] = fast_exp(out[k] - m);
      se += ex[k];
    }
    const float lse = m + fast_log(se), rse = __builtin_amdgcn_rcpf(se);
    float lp[kActions], p[kActions], ent = 0.f, logp_new = 0.f;
#pragma unroll
    for (int k = 0; k < kActions; ++k) {
      lp[k] = out[k] - lse;
      p[k] = ex[k] * rse;
      ent -= p[k] * lp[k];
      logp_new = (k == act) ? lp[k] : logp_new;
    }
    float advn = in.adv;
    if (lc.normalize) advn = (advn - prep.mean) * prep.rstd;
    const float log_ratio = logp_new - in.logp_old;
    const float ratio = fast_exp(log_ratio);
    const float rc = fminf(fmaxf(ratio, 1.0f - lc.clip_eps), 1.0f + lc.clip_eps);
    const float s1 = ratio * advn, s2 = rc * advn;
    st[0] += -fminf(s1, s2) * lc.inv_B;
    st[2] += ent * lc.inv_B;
    st[3] += ((ratio - 1.0f) - log_ratio) * lc.inv_B;
    st[4] += (fabsf(ratio - 1.0f) > lc.clip_eps ? 1.0f : 0.0f) * lc.inv_B;
    const float dlogp = (s1 <= s2) ? -(advn * ratio) * lc.inv_B : 0.0f;
    const float ec = lc.ent_coef * lc.inv_B;
#pragma unroll
    for (int k = 0; k < kActions; ++k) dl[k] = dlogp * ((k == act ? 1.0f : 0.0f) - p[k]) + ec * p[k] * (lp[k] + ent);
  }
  __device__ __forceinline__ void operator()(int64_t s, const float out[kActions], float dl[kActions], float st[5]) const {
    compute(load(s), prepare(), out, dl, st);
  }
};

struct CriticLoss {
  LossCommon lc;
  const float* ret;
  const float* v_old;
  int per_row;  // samples of the trajectory that share this prediction: A (central critic) or 1
  struct In {
    float ret[kMaxAgents], v_old[kMaxAgents];
  };
  template <bool FAST = false>
  __device__ __forceinline__ int32_t row_entry(int64_t s) const { return lc.rows[per_row == 1 ? lc.ad.div<FAST>(s, lc.A) : s]; }
  __device__ __forceinline__ In load(int64_t s) const { return load_with(s, row_entry(s)); }
  __device__ __forceinline__ LossPrep prepare() const { return LossPrep{0.f, 1.f}; }
  template <bool FAST = false>
  __device__ __forceinline__ In load_with(int64_t s, int32_t entry) const {
    In in;
    if (per_row == 1) {
      const int a = (int)(s - lc.ad.div<FAST>(s, lc.A) * lc.A);
      const int64_t src = (int64_t)entry * lc.A + a;
      in.ret[0] = ret[src];
      in.v_old[0] = v_old[src];
    } else {
      const int64_t src0 = (int64_t)entry * lc.A;
#pragma unroll
      for (int a = 0; a < kMaxAgents; ++a)
        if (a < lc.A) {
          in.ret[a] = ret[src0 + a];
          in.v_old[a] = v_old[src0 + a];
        }
    }
    return in;
  }
  __device__ __forceinline__ float term(float v, float r, float vo, float* loss) const {
    const float e = v - r;
    float l = 0.5f * e * e, g = e;
    if (lc.clip_value) {
      const float dvv = v - vo;
      const float vc = vo + fminf(fmaxf(dvv, -lc.clip_eps), lc.clip_eps);
      const float ec = vc - r, lcl = 0.5f * ec * ec;
      if (lcl > l) {
        l = lcl;
        g = (dvv > -lc.clip_eps && dvv < lc.clip_eps) ? ec : 0.0f;
      }
    }
    *loss += l * lc.inv_B;
    return g;
  }
  __device__ __forceinline__ void compute(const In& in, const LossPrep&, const float out[1], float dl[1], float st[5]) const {
    float g = 0.f;
#pragma unroll
    for (int a = 0; a < kMaxAgents; ++a)
      if (a < per_row) g += term(out[0], in.ret[a], in.v_old[a], &st[1]);
    dl[0] = g * lc.vf_coef * lc.inv_B;
  }
  __device__ __forceinline__ void operator()(int64_t s, const float out[1], float dl[1], float st[5]) const {
    compute(load(s), prepare(), out, dl, st);
  }
};

// Output layer + loss + gradient of the output layer.  Persistent over tiles of 64 samples so that the
// W3 / b3 gradient and the loss statistics leave each workgroup once.
template <int NOUT, class LossFn, typename HT>
__global__ void __launch_bounds__(256) loss_head_kernel(const HT* __restrict__ H2, int64_t S, int H,
                                                        const float* __restrict__ W3, const float* __restrict__ b3,
                                                        LossFn fn, float* __restrict__ dl_out,
                                                        float* __restrict__ gW3, float* __restrict__ gb3,
                                                        Scalars* sc, float b3_bias_unused) {
  __shared__ HeadLds L;
  __shared__ float dls[kHeadTile * NOUT];
  const int tid = threadIdx.x;
  const int nchunks = (H + kHeadChunk - 1) / kHeadChunk;  // <= 4
  float gw[4][NOUT];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int k = 0; k < NOUT; ++k) gw[c][k] = 0.f;
  float gb[NOUT];
#pragma unroll
  for (int k = 0; k < NOUT; ++k) gb[k] = 0.f;
  float st[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
  float bias[NOUT];
#pragma unroll
  for (int k = 0; k < NOUT; ++k) bias[k] = b3[k];

  const int64_t ntiles = (S + kHeadTile - 1) / kHeadTile;
  for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const int64_t s0 = tile * kHeadTile;
    float out[NOUT];
    head_tile<NOUT>(H2, s0, S, H, W3, L, out);
    if (tid < kHeadTile) {
      float dl[NOUT];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) dl[k] = 0.f;
      const int64_t s = s0 + tid;
      if (s < S) {
#pragma unroll
        for (int k = 0; k < NOUT; ++k) out[k] += bias[k];
        fn(s, out, dl, st);
#pragma unroll
        for (int k = 0; k < NOUT; ++k) {
          dl_out[s * NOUT + k] = dl[k];
          gb[k] += dl[k];
        }
      }
#pragma unroll
      for (int k = 0; k < NOUT; ++k) dls[tid * NOUT + k] = dl[k];
    }
    __syncthreads();
    // gW3[i][k] += sum_s H2[s][i] * dl[s][k]; thread -> hidden unit i = tid % 128 of each chunk, half of the samples
    const int i = tid & (kHeadChunk - 1), half = tid >> 7;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (c < nchunks) {
        const int h0 = c * kHeadChunk, hc = min(kHeadChunk, H - h0);
        if (nchunks > 1) {  // the tile in LDS holds the last chunk only: stage chunk c again
          __syncthreads();
          for (int r = tid >> 6; r < kHeadTile; r += 4) {
            const int64_t s = s0 + r;
            for (int cc = tid & 63; cc < hc; cc += 64) L.tile[r * (kHeadChunk + 1) + cc] = s < S ? load_act(H2, s * H + h0 + cc) : 0.f;
          }
          __syncthreads();
        }
        if (i < hc) {
          for (int s = half * 32; s < half * 32 + 32; ++s) {
            const float h = L.tile[s * (kHeadChunk + 1) + i];
#pragma unroll
            for (int k = 0; k < NOUT; ++k) gw[c][k] = fmaf(h, dls[s * NOUT + k], gw[c][k]);
          }
        }
      }
    }
  }
  // flush
  const int i = tid & (kHeadChunk - 1);
#pragma unroll
  for (int c = 0; c < 4; ++c)
    if (c < nchunks && c * kHeadChunk + i < H) {
#pragma unroll
      for (int k = 0; k < NOUT; ++k) atomicAdd(&gW3[(int64_t)(c * kHeadChunk + i) * NOUT + k], gw[c][k]);
    }
  if (tid < kHeadTile) {  // one wavefront: reduce across its lanes, lane 0 adds
#pragma unroll
    for (int k = 0; k < NOUT; ++k) {
      float v = gb[k];
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
      if (tid == 0) atomicAdd(&gb3[k], v);
    }
#pragma unroll
    for (int k = 0; k < 5; ++k) {
      float v = st[k];
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
      if (tid == 0 && v != 0.f) atomicAdd(&sc->acc[k], v);
    }
  }
}

// Squared gradient norm in two fixed-order stages (no atomics, so the clipping factor is the same bits in every run):
// workgroup b of at most kNormBlocks sums its grid-stride share in fp64 and stores it; adam_kernel (256 threads per
// workgroup = kNormBlocks) adds the shares.
__global__ void __launch_bounds__(256) grad_norm_kernel(const float* __restrict__ grad, int64_t P, Scalars* sc) {
  __shared__ double red[4];
  double part = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < P; i += (int64_t)gridDim.x * blockDim.x) {
    const double g = grad[i];
    part += g * g;
  }
  const double t = block_sum_f64(part, red);
  if (threadIdx.x == 0) sc->norm_part[blockIdx.x] = t;
}
inline unsigned grad_norm_blocks(int64_t P) { return (unsigned)std::min<int64_t>(kNormBlocks, (P + 255) / 256); }

struct AdamArgs {
  float lr, b1, b2, eps, bc1, bc2, max_norm, ent_coef, vf_coef;
  int norm_blocks;        // workgroups grad_norm_kernel ran with
  const int64_t* k_base;  // nullable: device-resident count of optimiser steps taken before this call; then the bias
  int k_local;            // corrections are computed on the device for step *k_base + k_local instead of bc1 / bc2
};

// sc_next (nullable): the gradient and that set of scalars are zeroed for the next optimiser step, which accumulates
// into them (two sets of scalars alternate, so nobody reads the one being zeroed).
__global__ void __launch_bounds__(256) adam_kernel(float* __restrict__ params, float* __restrict__ m,
                                                   float* __restrict__ v, float* __restrict__ grad, int64_t P,
                                                   AdamArgs a, const Scalars* sc, float* __restrict__ stats_row,
                                                   float* __restrict__ grad_dump, Scalars* sc_next) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  // the workgroups' shares of |grad|^2, added by a fixed tree (the same in every workgroup and every run)
  __shared__ double nparts[kNormBlocks];
  nparts[threadIdx.x] = (int)threadIdx.x < a.norm_blocks ? sc->norm_part[threadIdx.x] : 0.0;
  __syncthreads();
  for (int o = kNormBlocks / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) nparts[threadIdx.x] += nparts[threadIdx.x + o];
    __syncthreads();
  }
  const float norm = sqrtf((float)nparts[0]);
  const float scale = a.max_norm > 0.f ? a.max_norm / fmaxf(norm, a.max_norm) : 1.0f;
  if (a.k_base != nullptr) {
    const double k = (double)(*a.k_base + a.k_local);
    a.bc1 = (float)(1.0 - pow((double)a.b1, k));
    a.bc2 = (float)(1.0 - pow((double)a.b2, k));
  }
  if (i < P) {
    const float g = grad[i] * scale;
    const float mi = a.b1 * m[i] + (1.0f - a.b1) * g;
    const float vi = a.b2 * v[i] + (1.0f - a.b2) * g * g;
    m[i] = mi;
    v[i] = vi;
    params[i] -= a.lr * (mi / a.bc1) / (sqrtf(vi / a.bc2) + a.eps);
    if (grad_dump) grad_dump[i] = g;
    if (sc_next != nullptr) grad[i] = 0.f;
  }
  if (i == 0 && sc_next != nullptr) {
    sc_next->adv_sum = 0.0;
    sc_next->adv_sq = 0.0;
    for (int k = 0; k < 8; ++k) sc_next->acc[k] = 0.f;
  }
  if (i == 0) {
    const float total = sc->acc[0] - a.ent_coef * sc->acc[2] + a.vf_coef * sc->acc[1];
    stats_row[0] = sc->acc[0];
    stats_row[1] = sc->acc[1];
    stats_row[2] = sc->acc[2];
    stats_row[3] = sc->acc[3];
    stats_row[4] = sc->acc[4];
    stats_row[5] = norm;
    stats_row[6] = total;
    stats_row[7] = (isfinite(total) && isfinite(norm)) ? 0.f : 1.f;
  }
}

}  // namespace
}  // namespace marl
