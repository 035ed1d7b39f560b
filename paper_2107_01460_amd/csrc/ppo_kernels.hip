// Clipped-PPO minibatch update: forward over the gathered minibatch, loss and its gradient with
// respect to logits / values on the ALUs, backward through the two hidden layers as MFMA GEMMs,
// gradient accumulation with fp32 atomics, global-norm clipping and Adam.
#include <algorithm>
#include <cmath>

#include "bf16_path.h"
#include "fused_forward.h"
#include "fused_train.h"
#include "gemm.h"
#include "wreg_gemm.h"
#include "heads.h"
#include "ppo_common.h"

namespace marl {

// implemented in policy_kernels.hip
void mlp_hidden_forward(const RowSrc& X, int64_t S, int Din, int H, const float* W1, const float* b1, const float* W2,
                        const float* b2, float* h1, float* h2, bool bf16, hipStream_t s);
const float* effective_params(const marl_config& c, const float* params, float* scratch, hipStream_t s);
int64_t effective_param_floats(const marl_config& c);
Bf16NetWeights effective_bf16_weights(const marl_config& c, const float* eff, int net);

namespace {

// Output layer + loss + W3 / b3 gradient + dz2 for bf16 activations of up to HMAX hidden units.  The whole 64-sample
// tile of h2 sits in LDS as bf16 (one pass over HBM, 16-byte loads) and serves the output layer, the W3 gradient
// and dz2 = (dL/dout W3^T) * (1 - h2^2), which overwrites h2 in place (row-major, the A operand of dz1) and goes to
// the sample-blocked transposed copy dz2T (zeros for the samples S .. 64 * tiles; the B operand of the W2 gradient).
// Persistent over tiles so that the gradients and statistics leave a workgroup once.
template <int NOUT, class LossFn, int HMAX, int NT>
__global__ void __launch_bounds__(NT) loss_head_bf16_kernel(bf16_t* __restrict__ H2, int64_t S, int H,
                                                             const float* __restrict__ W3, const float* __restrict__ b3,
                                                             LossFn fn, bf16_t* __restrict__ dz2T, float* __restrict__ gW3,
                                                             float* __restrict__ gb3, Scalars* sc, float* __restrict__ partial) {
  // partial (nullable): this workgroup's W3 / b3 gradient goes to partial + blockIdx.x * (H * NOUT + NOUT) with plain
  // stores and is added to gW3 (with gb3 directly behind it) by the reduction kernel afterwards
  constexpr int PITCH = HMAX + 8;  // elements; an odd number of 16-byte units, so row-per-lane 16-byte reads spread over the banks
  __shared__ __attribute__((aligned(16))) bf16_t T[kHeadTile * PITCH];
  __shared__ __attribute__((aligned(16))) float W3s[HMAX * NOUT];
  constexpr int NG = NT / 64;  // wavefronts: eight (two per SIMD cover each other's LDS latencies) where there is enough work per tile, else four
  __shared__ float red[NG * NOUT * kHeadTile];
  __shared__ __attribute__((aligned(16))) float dls[kHeadTile * 8];
  const int tid = threadIdx.x, lane = tid & 63, grp = tid >> 6;
  for (int e = tid; e < H * NOUT; e += NT) W3s[e] = W3[e];
  const auto prep = fn.prepare();
  // dz2: thread -> the eight hidden units 8 (tid % CPR) .. + 7 of the rows tid / CPR + (NT / CPR) q; their W3 rows
  float w8[8][NOUT];
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int k = 0; k < NOUT; ++k) {
      const int i = 8 * (tid % (HMAX / 8)) + e;
      w8[e][k] = i < H ? W3[(int64_t)i * NOUT + k] : 0.f;
    }
  constexpr int UMAX = 2;  // W3 gradient: thread -> the pair of hidden units 2 (tid % 256), + 1 and one share of the tile's samples
  constexpr int SHARES = NT / 256;
  static_assert(HMAX == 512 && (NT == 256 || NT == 512), "256 pairs of hidden units x 1 or 2 shares of the samples");
  float gw[UMAX][NOUT], gb[NOUT], st[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < NOUT; ++k) {
    gb[k] = 0.f;
#pragma unroll
    for (int u = 0; u < UMAX; ++u) gw[u][k] = 0.f;
  }
  const int vec_per_row = H / 8, per_grp = H / NG;
  const int64_t ntiles = (S + kHeadTile - 1) / kHeadTile;
  // A tile travels global -> registers -> LDS: all of a thread's 16-byte pieces are requested at once, and the next
  // tile's are requested before this tile's arithmetic, so that no load is waited for on its own.
  constexpr int NV = kHeadTile * (HMAX / 8) / NT;  // pieces per thread at the full width
  constexpr int CPR = HMAX / 8;                     // 16-byte pieces of a row at the full width
  static_assert(NT % CPR == 0 && NV * (NT / CPR) == kHeadTile, "a thread's pieces are one column of the tile");
  uint4 tv[NV];
  auto fetch_tile = [&](int64_t tile) {
    const int64_t s0 = tile * kHeadTile;
#pragma unroll
    for (int q = 0; q < NV; ++q) {  // thread -> rows tid / CPR + (NT / CPR) q, 16-byte piece tid % CPR of the row
      const int r = tid / CPR + (NT / CPR) * q, c8 = tid % CPR;
      tv[q] = make_uint4(0u, 0u, 0u, 0u);
      if (c8 < vec_per_row && s0 + r < S) tv[q] = *reinterpret_cast<const uint4*>(&H2[(s0 + r) * H + 8 * c8]);
    }
  };
  // The loss inputs of a sample sit behind a dependent pair of loads (row order entry, then the row): the first
  // wavefront requests the entries of the next tile at the top of a tile and the rows after the output layer, so
  // that neither is waited for in front of the loss.
  typename LossFn::In lin_next{};
  int32_t lentry = 0;
  if ((int64_t)blockIdx.x < ntiles) {
    fetch_tile(blockIdx.x);
    const int64_t s = (int64_t)blockIdx.x * kHeadTile + tid;
    if (tid < kHeadTile && s < S) lin_next = fn.load(s);
  }
  for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const int64_t s0 = tile * kHeadTile;
    const int64_t s_next = (tile + gridDim.x) * kHeadTile + tid;  // this thread's sample of the next tile
    const bool next_live = tid < kHeadTile && tile + gridDim.x < ntiles && s_next < S;
    const typename LossFn::In lin = lin_next;
    if (next_live) lentry = fn.row_entry(s_next);
    __syncthreads();  // the previous tile has been consumed (and W3s is in place)
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      const int r = tid / CPR + (NT / CPR) * q, c8 = tid % CPR;
      if (c8 < vec_per_row) *reinterpret_cast<uint4*>(&T[r * PITCH + 8 * c8]) = tv[q];
    }
    __syncthreads();
    if (tile + gridDim.x < ntiles) fetch_tile(tile + gridDim.x);
    {  // output layer: thread -> sample `lane`, share `grp` (one of NG) of the hidden units
      float part[NOUT];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) part[k] = 0.f;
#pragma unroll 4
      for (int i = grp * per_grp; i < (grp + 1) * per_grp; i += 8) {
        const uint4 hv = *reinterpret_cast<const uint4*>(&T[lane * PITCH + i]);
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
          const float4 t = *reinterpret_cast<const float4*>(&W3s[i * NOUT + 4 * q]);
          wv[4 * q] = t.x; wv[4 * q + 1] = t.y; wv[4 * q + 2] = t.z; wv[4 * q + 3] = t.w;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
          for (int k = 0; k < NOUT; ++k) part[k] = fmaf(hh[j], wv[j * NOUT + k], part[k]);
      }
#pragma unroll
      for (int k = 0; k < NOUT; ++k) red[(grp * NOUT + k) * kHeadTile + lane] = part[k];
    }
    if (next_live) lin_next = fn.load_with(s_next, lentry);
    __syncthreads();
    if (tid < kHeadTile) {
      float out[NOUT], dl[NOUT];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) {
        float v = 0.f;
#pragma unroll
        for (int gq = 0; gq < NG; ++gq) v += red[(gq * NOUT + k) * kHeadTile + tid];
        out[k] = b3[k] + v;
        dl[k] = 0.f;
      }
      const int64_t s = s0 + tid;
      if (s < S) {
        fn.compute(lin, prep, out, dl, st);
#pragma unroll
        for (int k = 0; k < NOUT; ++k) gb[k] += dl[k];
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) dls[tid * 8 + k] = k < NOUT ? dl[k < NOUT ? k : 0] : 0.f;
    }
    __syncthreads();
    // gW3[i][k] += sum_s h2[s][i] dl[s][k]: thread -> hidden units 2 (tid % 256), + 1 (one 4-byte LDS read per sample),
    // samples (64 / SHARES) (tid / 256) .. 
    const int pr = tid & 255, s_lo = (tid >> 8) * (kHeadTile / SHARES);
#pragma unroll 8
    for (int s = s_lo; s < s_lo + kHeadTile / SHARES; ++s) {
      const float4 d0 = *reinterpret_cast<const float4*>(&dls[s * 8]);
      float dv[8] = {d0.x, d0.y, d0.z, d0.w, 0.f, 0.f, 0.f, 0.f};
      if (NOUT > 4) {
        const float4 d1 = *reinterpret_cast<const float4*>(&dls[s * 8 + 4]);
        dv[4] = d1.x; dv[5] = d1.y; dv[6] = d1.z; dv[7] = d1.w;
      }
      const uint32_t hw = 2 * pr < H ? *reinterpret_cast<const uint32_t*>(&T[s * PITCH + 2 * pr]) : 0u;
      const float hp[2] = {__uint_as_float(hw << 16), __uint_as_float(hw & 0xffff0000u)};
#pragma unroll
      for (int u = 0; u < UMAX; ++u)
#pragma unroll
        for (int k = 0; k < NOUT; ++k) gw[u][k] = fmaf(hp[u], dv[k], gw[u][k]);
    }
    __syncthreads();  // every thread has read the h2 it needs; the tile is overwritten with dz2
#pragma unroll 4
    for (int q = 0; q < NV; ++q) {
      const int r = tid / CPR + (NT / CPR) * q, c8 = tid % CPR;
      if (c8 < vec_per_row) {
        const uint4 hv = *reinterpret_cast<const uint4*>(&T[r * PITCH + 8 * c8]);
        const float4 d0 = *reinterpret_cast<const float4*>(&dls[r * 8]);
        float dv[8] = {d0.x, d0.y, d0.z, d0.w, 0.f, 0.f, 0.f, 0.f};
        if (NOUT > 4) {
          const float4 d1 = *reinterpret_cast<const float4*>(&dls[r * 8 + 4]);
          dv[4] = d1.x; dv[5] = d1.y; dv[6] = d1.z; dv[7] = d1.w;
        }
        const uint32_t hw[4] = {hv.x, hv.y, hv.z, hv.w};
        uint32_t ow[4];
#pragma unroll
        for (int p2 = 0; p2 < 4; ++p2) {
          float o2[2];
#pragma unroll
          for (int z = 0; z < 2; ++z) {
            const float h = __uint_as_float(z == 0 ? hw[p2] << 16 : hw[p2] & 0xffff0000u);
            float g = 0.f;
#pragma unroll
            for (int k = 0; k < NOUT; ++k) g = fmaf(dv[k], w8[2 * p2 + z][k], g);
            o2[z] = g * (1.0f - h * h);  // rows past the end carry dl = 0
          }
          ow[p2] = pack2_bf16(o2[0], o2[1]);
        }
        const uint4 ov = make_uint4(ow[0], ow[1], ow[2], ow[3]);
        if (s0 + r < S) *reinterpret_cast<uint4*>(&H2[(s0 + r) * H + 8 * c8]) = ov;
        *reinterpret_cast<uint4*>(&T[r * PITCH + 8 * c8]) = ov;
      }
    }
    __syncthreads();
    // transposed copy: thread -> hidden unit tid / 8 + (NT / 8) q, samples 8 (tid % 8) .. + 7 (a wavefront writes 1 KB in one piece)
    for (int q = 0; (NT / 8) * q < H; ++q) {
      const int dd = (tid >> 3) + (NT / 8) * q, ss = 8 * (tid & 7);
      uint32_t ow[4];
#pragma unroll
      for (int p2 = 0; p2 < 4; ++p2)
        ow[p2] = (uint32_t)T[(ss + 2 * p2) * PITCH + dd] | ((uint32_t)T[(ss + 2 * p2 + 1) * PITCH + dd] << 16);
      *reinterpret_cast<uint4*>(&dz2T[((s0 >> 6) * H + dd) * 64 + ss]) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
    }
  }
  // two shares of the samples meet in LDS (the tile buffer is free after the last barrier of the loop)
  float* const comb = reinterpret_cast<float*>(T);
  if (SHARES == 2) {
    __syncthreads();
    if (tid >= 256) {
#pragma unroll
      for (int u = 0; u < UMAX; ++u)
#pragma unroll
        for (int k = 0; k < NOUT; ++k) comb[(u * NOUT + k) * 256 + (tid & 255)] = gw[u][k];
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < UMAX; ++u) {
    const int i = 2 * tid + u;
    if (tid < 256 && i < H) {
#pragma unroll
      for (int k = 0; k < NOUT; ++k)
        if (SHARES == 2) gw[u][k] += comb[(u * NOUT + k) * 256 + tid];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) {
        if (partial != nullptr) partial[(int64_t)blockIdx.x * (H * NOUT + NOUT) + (int64_t)i * NOUT + k] = gw[u][k];
        else atomicAdd(&gW3[(int64_t)i * NOUT + k], gw[u][k]);
      }
    }
  }
  if (tid < kHeadTile) {  // one wavefront
#pragma unroll
    for (int k = 0; k < NOUT; ++k) {
      float v = gb[k];
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
      if (tid == 0) {
        if (partial != nullptr) partial[(int64_t)blockIdx.x * (H * NOUT + NOUT) + (int64_t)H * NOUT + k] = v;
        else atomicAdd(&gb3[k], v);
      }
    }
#pragma unroll
    for (int k = 0; k < 5; ++k) {
      float v = st[k];
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
      if (tid == 0 && v != 0.f) atomicAdd(&sc->acc[k], v);
    }
  }
}

// In place: H2[s][j] <- (sum_k dl[s][k] W3[j][k]) * (1 - H2[s][j]^2); column sums -> gb2.
template <int NOUT>
__global__ void __launch_bounds__(256) dz2_kernel(float* __restrict__ H2, const float* __restrict__ dl,
                                                  const float* __restrict__ W3, float* __restrict__ gb2, int64_t S,
                                                  int H, int cb, int rows_per_block, int round_bf16) {
  __shared__ float red[256];
  const int tid = threadIdx.x;
  const int rg_count = 256 / cb;
  const int rg = tid / cb, jl = tid - rg * cb;
  const int j = blockIdx.y * cb + jl;
  const bool on = rg < rg_count && j < H;
  float w[NOUT];
#pragma unroll
  for (int k = 0; k < NOUT; ++k) w[k] = on ? W3[(int64_t)j * NOUT + k] : 0.f;
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
  const int64_t r1 = min(S, r0 + rows_per_block);
  float csum = 0.f;
  if (on) {
    for (int64_t r = r0 + rg; r < r1; r += rg_count) {
      float g = 0.f;
#pragma unroll
      for (int k = 0; k < NOUT; ++k) g = fmaf(dl[r * NOUT + k], w[k], g);
      const float h = H2[r * H + j];
      float v = g * (1.0f - h * h);
      if (round_bf16) v = round_to_bf16(v);
      H2[r * H + j] = v;
      csum += v;
    }
  }
  red[tid] = on ? csum : 0.f;
  __syncthreads();
  if (gb2 != nullptr && tid < cb && j < H) {
    float t = 0.f;
    for (int g2 = 0; g2 < rg_count; ++g2) t += red[g2 * cb + tid];
    atomicAdd(&gb2[j], t);
  }
}

struct UpdateWsView {
  float *eff_params, *grad;
  Scalars* sc;        // two sets: optimiser step k accumulates into set k % 2 while its Adam kernel zeroes the other
  double* adv_stats;  // [n_epochs * n_minibatches][2]: sum and sum of squares of every minibatch's advantages
  int32_t* ident;
  float *h1a, *h2a, *dz1a, *dla;
  float *h1c, *h2c, *dz1c, *dlc;
  float* partial;  // per-workgroup copies of one network's gradient (two-stage reduction of the fused training kernel)
  float* partial_w1;
  float* partial_head;  // per-workgroup W3 / b3 gradients of the output-layer kernels (bf16 configuration; register-resident fp32 critic)
  float* split_ws;      // fp32 layer-by-layer networks: the k splits of a weight-gradient product, added in a fixed order
  int64_t split_floats;
  // bf16 configuration: one set of activation buffers, used by the actor and then by the critic
  bf16_t *xb, *xbT, *bh1, *bh1T, *bh2, *dz2T, *dz1T;
};

int64_t align256(int64_t x) { return (x + 255) & ~(int64_t)255; }

int64_t split_want(int64_t tiles_mn) { return std::max<int64_t>(1, 1024 / std::max<int64_t>(1, tiles_mn)); }
// floats of workspace for the k splits of dW2 (H x H + H) and dW1 (Din x H + H) of one layer-by-layer network
int64_t split_ws_floats(int H, int Din) {
  const int64_t t2 = ((H + 127) / 128) * ((H + 127) / 128), t1 = ((Din + 127) / 128) * ((H + 127) / 128);
  return std::max(split_want(t2) * ((int64_t)H * H + H), split_want(t1) * ((int64_t)Din * H + H));
}

UpdateWsView carve_update_ws(const marl_config& c, void* ws, int64_t* total) {
  const Dims d = dims_of(c);
  const int64_t R = (int64_t)d.T * d.N, rows_mb = R / c.n_minibatches;
  const int64_t Sa = rows_mb * d.A, Sc = d.central ? rows_mb : Sa;
  char* p = static_cast<char*>(ws);
  int64_t off = 0;
  auto take = [&](int64_t bytes) {
    char* r = p + off;
    off += align256(bytes);
    return r;
  };
  UpdateWsView v{};
  v.eff_params = (float*)take(effective_param_floats(c) * 4);
  v.grad = (float*)take(d.P * 4);
  v.sc = (Scalars*)take(2 * sizeof(Scalars));
  v.adv_stats = (double*)take((int64_t)c.n_epochs * c.n_minibatches * 2 * sizeof(double));
  v.ident = (int32_t*)take(R * 4);
  if (!d.bf16) {
    // activations: rows rounded up to the 64-row tiles of the register-resident kernels, which store whole tiles
    const int64_t Sap = round_up64(Sa), Scp = round_up64(Sc);
    v.h1a = (float*)take(Sap * d.Ha * 4);
    v.h2a = (float*)take(Sap * d.Ha * 4);
    v.dz1a = (float*)take(Sap * d.Ha * 4);
    v.dla = (float*)take(Sa * kActions * 4);
    v.h1c = (float*)take(Scp * d.Hc * 4);
    v.h2c = (float*)take(Scp * d.Hc * 4);
    v.dz1c = (float*)take(Scp * d.Hc * 4);
    v.dlc = (float*)take(Sc * 4);
    int64_t pmax = 0;
    if (fused_train_supported(d.Ha, d.D)) pmax = std::max<int64_t>(pmax, d.Pa);
    if (fused_train_supported(d.Hc, d.Dc)) pmax = std::max<int64_t>(pmax, d.P - d.Pa);
    v.partial = pmax > 0 ? (float*)take((int64_t)kFusedTrainMaxGrid * pmax * 4) : nullptr;
    // ... and of the first-layer gradient of the 256-wide critic (accumulator-resident transposed product)
    v.partial_w1 = (d.Hc == kWregN && d.Dc == 300) ? (float*)take((int64_t)kWaccMaxGrid * (300 + 1) * kWregN * 4) : nullptr;
    // the k splits of the layer-by-layer weight gradients (at most `want` splits of pick_k_split per product)
    v.split_floats = 0;
    if (!fused_train_supported(d.Ha, d.D)) v.split_floats = std::max(v.split_floats, split_ws_floats(d.Ha, d.D));
    if (!fused_train_supported(d.Hc, d.Dc)) v.split_floats = std::max(v.split_floats, split_ws_floats(d.Hc, d.Dc));
    v.split_ws = v.split_floats > 0 ? (float*)take(v.split_floats * 4) : nullptr;
    v.partial_head = (d.Hc == kWregN || d.Ha == kWregN) ? (float*)take((int64_t)kFusedFwdTrainGrid * (kWregN * kActions + kActions) * 4) : nullptr;
  } else {
    const int64_t Sp = round_up64(std::max(Sa, Sc));
    const int64_t Dp = round_up64(std::max(d.D, d.Dc)), H = std::max(d.Ha, d.Hc);
    v.dla = (float*)take(Sa * kActions * 4);
    v.dlc = (float*)take(Sc * 4);
    v.xb = (bf16_t*)take(Sp * Dp * 2);
    v.xbT = (bf16_t*)take(Sp * Dp * 2);
    v.bh1 = (bf16_t*)take(Sp * H * 2);
    v.bh1T = (bf16_t*)take(Sp * H * 2);
    v.bh2 = (bf16_t*)take(Sp * H * 2);
    v.dz2T = (bf16_t*)take(Sp * H * 2);
    v.dz1T = (bf16_t*)take(Sp * H * 2);
    v.partial_head = (float*)take((int64_t)512 * (H * kActions + kActions) * 4);
  }
  if (total) *total = off;
  return v;
}

int64_t pick_k_split(int64_t K, int64_t tiles_mn) {
  // enough workgroups for ~4 per CU, each with a k range that is a multiple of the k tile
  int64_t want = split_want(tiles_mn);
  int64_t per = (K + want - 1) / want;
  per = std::max<int64_t>(256, ((per + kGemmBK - 1) / kGemmBK) * kGemmBK);
  return per;
}

// Forward and loss of one 256-wide fp32 network with each layer's weights resident in registers: h1 goes to HBM,
// the second hidden activation never does, `dz2` gets dL/d(pre-activation of layer 2), the output layer's gradient
// and the loss statistics are accumulated.
// The register-resident kernels pay for loading a whole weight matrix per workgroup (and for one round of atomics per
// workgroup in the transposed product): they win from about four 64-row tiles per workgroup on, i.e. 65 536 rows on
// 256 compute units (measured at the shape of workload 3: 16 384 rows 28.1 against 24.7 ms per step with the LDS-tiled
// kernels, 65 536 rows equal, 262 144 rows 134 against 152 ms).
inline bool wreg_worthwhile(int64_t S) { return S >= 256 * kWregBM * 4; }
inline bool wreg_forward_supported(const RowSrc& X, int64_t S, int Din, int H) {
  return H == kWregN && wreg_worthwhile(S) && wreg_gemm_supported<WREG_BIAS_TANH>(X, Din, H);
}
template <int NOUT, class LossFn>
int32_t train_forward_wreg(const RowSrc& X, int64_t S, int Din, const float* W1, const float* b1, const float* W2,
                           const float* b2, const float* W3, const float* b3, float* h1, float* dz2, float* gW3,
                           float* gb3, float* stats, const LossFn& fn, float* partial3, hipStream_t s) {
  {
    WregArgs g{};
    g.A = X; g.S = S; g.Kin = Din; g.B = W1; g.ldb = kWregN; g.b_kcont = 0; g.C = h1; g.bias = b1;
    TimedLaunch timed(KC_GEMM_NN, 2.0 * (double)S * Din * kWregN, s);
    const int32_t rc = launch_wreg_gemm<WREG_BIAS_TANH>(g, s);
    if (rc != MARL_OK) return rc;
  }
  WregArgs g{};
  g.A = RowSrc{h1, kWregN, nullptr, 1, S}; g.S = S; g.Kin = kWregN; g.B = W2; g.ldb = kWregN; g.b_kcont = 0; g.C = dz2;
  g.bias = b2; g.W3 = W3; g.b3 = b3; g.gW3 = gW3; g.gb3 = gb3; g.stats = stats;
  g.partial3 = partial3;  // (nullable) per-workgroup copies of the W3 / b3 gradient, added in a fixed order below
  int32_t rc;
  {
    TimedLaunch timed(KC_GEMM_NN, 2.0 * (double)S * kWregN * kWregN, s);
    rc = launch_wreg_loss<NOUT>(g, fn, s);
  }
  if (rc == MARL_OK && partial3 != nullptr) {
    const int64_t tiles = (S + kWregBM - 1) / kWregBM;
    launch_reduce_partials(partial3, (int)std::min<int64_t>(tiles, 256), (int64_t)kWregN * NOUT + NOUT, gW3, s);
  }
  return rc;
}

// Backward through one network given dL/d(output layer) in dl; h2 is overwritten by dz2.
template <int NOUT>
void mlp_backward(const RowSrc& X, int64_t S, int Din, int H, const float* W2, const float* W3, float* h1, float* h2,
                  float* dz1, const float* dl, float* gW1, float* gb1, float* gW2, float* gb2, bool bf16,
                  bool dz2_ready, float* wacc_partial, float* split_ws, int64_t split_floats, hipStream_t s) {
  // a weight-gradient product writes its k splits to split_ws and has them added in a fixed order, where the workspace
  // has room and the bias gradient directly follows the weight gradient (its column sums ride along)
  auto split_launch = [&](GemmArgs& g, float* gW, float* gb, int64_t rows) {
    const int64_t count = rows * H + H, nz = (g.K + g.k_per_split - 1) / g.k_per_split;
    if (split_ws != nullptr && gb == gW + rows * H && nz * count <= split_floats) {
      g.split_out = split_ws;
      g.split_count = count;
    }
    if (launch_gemm<GEMM_TN, EPI_ATOMIC_ADD>(g, s)) launch_reduce_partials(split_ws, (int)nz, count, gW, s);
  };
  if (!dz2_ready) {
    const int cb = std::min(H, 256), rpb = 256;
    dim3 grid((unsigned)((S + rpb - 1) / rpb), (unsigned)((H + cb - 1) / cb));
    hipLaunchKernelGGL(dz2_kernel<NOUT>, grid, dim3(256), 0, s, h2, dl, W3, (float*)nullptr, S, H, cb, rpb, (int)bf16);
  }
  {  // gW2 += h1^T dz2, gb2 += column sums
    GemmArgs g{};
    g.A = RowSrc{h1, H, nullptr, 1, S}; g.B = h2; g.ldb = H; g.C = gW2; g.ldc = H;
    g.M = H; g.N = H; g.K = S; g.colsum = gb2;
    g.k_per_split = pick_k_split(S, ((H + 127) / 128) * ((H + 127) / 128));
    split_launch(g, gW2, gb2, H);
  }
  const RowSrc dz2_rows{h2, H, nullptr, 1, S};
  if (!bf16 && wreg_worthwhile(S) && wreg_gemm_supported<WREG_DTANH>(dz2_rows, H, H)) {
    // dz1 = (dz2 W2^T) * (1 - h1^2) with W2 resident in registers
    WregArgs g{};
    g.A = dz2_rows; g.S = S; g.Kin = H; g.B = W2; g.ldb = H; g.b_kcont = 1; g.C = dz1; g.aux = h1;
    TimedLaunch timed(KC_GEMM_NT, 2.0 * (double)S * H * H, s);
    launch_wreg_gemm<WREG_DTANH>(g, s);
  } else {  // dz1 = (dz2 W2^T) * (1 - h1^2), gb1 += column sums
    GemmArgs g{};
    g.A = RowSrc{h2, H, nullptr, 1, S}; g.B = W2; g.ldb = H; g.C = dz1; g.ldc = H;
    g.aux_mat = h1; g.ldaux = H; g.colsum = nullptr;
    g.M = S; g.N = H; g.K = H; g.round_bf16 = bf16;
    launch_gemm<GEMM_NT, EPI_DTANH>(g, s);
  }
  if (!bf16 && wreg_worthwhile(S) && wacc_gemm_supported(X, Din, H)) {  // gW1 += X^T dz1, gb1 += column sums, the gradient resident in registers
    WaccArgs g{};
    g.A = X; g.S = S; g.B = dz1; g.C = gW1; g.colsum = gb1;
    g.partial = (gb1 == gW1 + (int64_t)Din * H) ? wacc_partial : nullptr;  // the bias gradient directly follows the weight gradient
    TimedLaunch timed(KC_GEMM_TN, 2.0 * (double)S * Din * H, s);
    launch_wacc_gemm(g, Din, s);
  } else {  // gW1 += X^T dz1
    GemmArgs g{};
    g.A = X; g.B = dz1; g.ldb = H; g.C = gW1; g.ldc = H;
    g.M = Din; g.N = H; g.K = S; g.colsum = gb1;
    g.k_per_split = pick_k_split(S, ((Din + 127) / 128) * ((H + 127) / 128));
    split_launch(g, gW1, gb1, Din);
  }
}

// Forward, loss and backward of one network in the bf16 configuration: every product runs on the bf16 matrix
// cores; the output layer, the loss and dz2 stay on the ALUs in fp32.
template <int NOUT, class LossFn>
void train_net_bf16(const RowSrc& X, int64_t S, int Din, int H, const Bf16NetWeights& bw, const float* eff,
                    const NetOffsets& o, float* grad, const NetOffsets& go, const LossFn& fn, float* dl,
                    const UpdateWsView& w, bool packed, hipStream_t s) {
  const int64_t Sp = round_up64(S);
  if (!packed) pack_obs_bf16(X, S, Din, bw.Dp, Sp, w.xb, w.xbT, s);  // packed: the previous network left these very rows there
  mlp_hidden_forward_bf16(w.xb, S, Sp, H, bw, eff + o.b1, eff + o.b2, w.bh1, w.bh1T, w.bh2, s);
  const unsigned nb = (unsigned)std::min<int64_t>(512, (S + kHeadTile - 1) / kHeadTile);
  float* const hp = (go.b3 == go.W3 + (int64_t)H * NOUT) ? w.partial_head : nullptr;  // b3's gradient directly follows W3's
  // output layer, loss and dz2 in one pass over h2 (the tiles cover the samples up to Sp: dz2T is zero-padded)
  constexpr int HEAD_NT = NOUT > 1 ? 512 : 256;  // the one-output head has too little work per tile for eight wavefronts
  hipLaunchKernelGGL((loss_head_bf16_kernel<NOUT, LossFn, 512, HEAD_NT>), dim3(nb), dim3(HEAD_NT), 0, s, w.bh2, S, H, eff + o.W3,
                     eff + o.b3, fn, w.dz2T, grad + go.W3, grad + go.b3, w.sc, hp);
  if (hp != nullptr) launch_reduce_partials(hp, (int)nb, (int64_t)H * NOUT + NOUT, grad + go.W3, s);
  auto k_split = [&](int64_t tiles_mn) {  // ~4 workgroups per CU, k ranges in multiples of the k tile
    const int64_t want = std::max<int64_t>(1, 1024 / std::max<int64_t>(1, tiles_mn));
    return std::max<int64_t>(512, round_up64((Sp + want - 1) / want));
  };
  {  // gW2 += h1^T dz2, gb2 += column sums of dz2
    GemmBf16Args g{};
    g.A = w.bh1T; g.a_rows = H; g.B = w.dz2T; g.b_rows = H;
    g.M = H; g.N = H; g.K = Sp; g.Cf = grad + go.W2; g.ldcf = H; g.rowsum_b = grad + go.b2;
    g.k_per_split = k_split(((H + 127) / 128) * ((H + 127) / 128));
    launch_gemm_bf16<BEPI_ATOMIC>(g, s);
  }
  {  // dz1 = (dz2 W2^T) * (1 - h1^2), transposed copy only
    GemmBf16Args g{};
    g.A = w.bh2; g.lda = H; g.a_rows = S; g.B = bw.W2; g.ldb = H; g.b_rows = H;
    g.M = S; g.N = H; g.K = H; g.CT = w.dz1T; g.ct_cols = Sp; g.aux = w.bh1; g.ldaux = H;
    launch_gemm_bf16<BEPI_DTANH_T>(g, s);
  }
  {  // gW1 += X^T dz1, gb1 += column sums of dz1
    GemmBf16Args g{};
    g.A = w.xbT; g.a_rows = bw.Dp; g.B = w.dz1T; g.b_rows = H;
    g.M = Din; g.N = H; g.K = Sp; g.Cf = grad + go.W1; g.ldcf = H; g.rowsum_b = grad + go.b1;
    g.k_per_split = k_split(((Din + 127) / 128) * ((H + 127) / 128));
    launch_gemm_bf16<BEPI_ATOMIC>(g, s);
  }
}

}  // namespace

int64_t update_workspace_bytes(const marl_config& c) {
  int64_t total = 0;
  carve_update_ws(c, nullptr, &total);
  return total;
}

namespace {
__global__ void advance_counters_kernel(marl_counters* counters, uint64_t steps, int64_t adam_steps) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    counters->step += steps;
    counters->adam_step += adam_steps;
  }
}
}  // namespace

int32_t launch_advance_counters(marl_counters* counters, uint64_t steps, int64_t adam_steps, hipStream_t s) {
  hipLaunchKernelGGL(advance_counters_kernel, dim3(1), dim3(64), 0, s, counters, steps, adam_steps);
  return launch_status();
}

int32_t launch_ppo_update(const marl_config& c, marl_traj tr, float* params, float* adam_m, float* adam_v,
                          int64_t adam_step0, const int32_t* perm, float* stats, float* grad_dump, void* workspace,
                          hipStream_t s, const int64_t* adam_step_base) {
  const Dims d = dims_of(c);
  const UpdateWsView w = carve_update_ws(c, workspace, nullptr);
  const int64_t R = (int64_t)d.T * d.N, rows_mb = R / c.n_minibatches;
  const int64_t Sa = rows_mb * d.A, Sc = d.central ? rows_mb : Sa;
  if (perm == nullptr)
    hipLaunchKernelGGL(iota_kernel, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, s, w.ident, R);
  // ga/gc: blocks of the gradient (parameter-vector layout); oa/oc: blocks of the aligned working copy of the weights
  const NetOffsets ga = net_offsets(0, d.D, d.Ha, kActions), gc = net_offsets(d.Pa, d.Dc, d.Hc, 1);
  const ParamMap pm = param_map(d);
  const NetOffsets oa = padded_offsets(pm, 0), oc = padded_offsets(pm, 1);
  int64_t k = adam_step0;
  // Once per update: the gradient, both sets of scalars and the advantage statistics start at zero (afterwards every
  // Adam kernel zeroes the gradient and the scalars of the next step), and the advantage statistics of ALL minibatches
  // of all epochs are summed in one launch -- the row orders are known up front.
  const int n_steps = c.n_epochs * c.n_minibatches;
  hipLaunchKernelGGL(zero_step_kernel, dim3((unsigned)((d.P + 255) / 256)), dim3(256), 0, s, w.grad, d.P, w.sc, 2,
                     w.adv_stats, 2 * n_steps);
  if (c.normalize_adv) {
    const unsigned nb = (unsigned)std::min<int64_t>(std::max(1, 256 / c.n_minibatches), (Sa + 255) / 256);  // every workgroup ends with two atomics on its minibatch's two doubles
    hipLaunchKernelGGL(adv_stats_all_kernel, dim3(nb, (unsigned)n_steps), dim3(256), 0, s, tr.adv, perm ? perm : w.ident,
                       perm ? R : (int64_t)0, c.n_minibatches, rows_mb, d.A, w.adv_stats);
  }
  for (int e = 0; e < c.n_epochs; ++e) {
    for (int mb = 0; mb < c.n_minibatches; ++mb) {
      const int step = e * c.n_minibatches + mb;
      Scalars* const sck = w.sc + (step & 1);
      UpdateWsView wk = w;  // the view the helpers get: this step's scalars
      wk.sc = sck;
      const int32_t* rows = (perm ? perm + (int64_t)e * R : w.ident) + (int64_t)mb * rows_mb;
      const float* eff = effective_params(c, params, w.eff_params, s);
      LossCommon lc{};
      lc.rows = rows; lc.A = d.A; lc.ad = make_small_div(d.A); lc.rows_mb = rows_mb; lc.inv_B = (float)(1.0 / (double)(rows_mb * d.A));
      lc.sc = sck; lc.adv_stats = w.adv_stats + 2 * step; lc.normalize = c.normalize_adv; lc.clip_eps = c.clip_eps;
      lc.ent_coef = c.ent_coef; lc.vf_coef = c.vf_coef; lc.clip_value = c.clip_value;
      const RowSrc Xa{tr.obs, d.D, rows, d.A, Sa, make_small_div(d.A)};
      const RowSrc Xc{tr.obs, d.Dc, rows, d.central ? 1 : d.A, Sc, make_small_div(d.central ? 1 : d.A)};
      // ---- both networks in one launch (same shape, few tiles)
      const bool pair = !d.bf16 && Sa < ((int64_t)1 << 31) && fused_train_pair_supported(d.Ha, d.D, Sa, d.Hc, d.Dc, Sc);
      if (pair) {
        ActorLoss fa{lc, tr.action, tr.logp, tr.adv};
        CriticLoss fc{lc, tr.ret, tr.value, d.central ? d.A : 1};
        FusedTrainArgs ta{}, tc{};
        ta.X = Xa; ta.S = Sa; ta.Din = d.D; ta.px = fused_train_px(d.D);
        ta.W1 = eff + oa.W1; ta.b1 = eff + oa.b1; ta.W2 = eff + oa.W2; ta.b2 = eff + oa.b2; ta.W3 = eff + oa.W3;
        ta.W1s = eff + pm.sw_w1[0]; ta.W2s = eff + pm.sw_w2[0]; ta.W2Ts = eff + pm.sw_w2t[0];
        ta.b3 = eff + oa.b3; ta.gW1 = w.grad + ga.W1; ta.gb1 = w.grad + ga.b1; ta.gW2 = w.grad + ga.W2;
        ta.gb2 = w.grad + ga.b2; ta.gW3 = w.grad + ga.W3; ta.gb3 = w.grad + ga.b3; ta.stats = sck->acc;
        ta.partial = w.partial; ta.gcount = d.Pa;
        tc.X = Xc; tc.S = Sc; tc.Din = d.Dc; tc.px = fused_train_px(d.Dc);
        tc.W1 = eff + oc.W1; tc.b1 = eff + oc.b1; tc.W2 = eff + oc.W2; tc.b2 = eff + oc.b2; tc.W3 = eff + oc.W3;
        tc.W1s = eff + pm.sw_w1[1]; tc.W2s = eff + pm.sw_w2[1]; tc.W2Ts = eff + pm.sw_w2t[1];
        tc.b3 = eff + oc.b3; tc.gW1 = w.grad + gc.W1; tc.gb1 = w.grad + gc.b1; tc.gW2 = w.grad + gc.W2;
        tc.gb2 = w.grad + gc.b2; tc.gW3 = w.grad + gc.W3; tc.gb3 = w.grad + gc.b3; tc.stats = sck->acc;
        tc.gcount = d.P - d.Pa;
        const int32_t rc = (launch_fused_train_pair<kActions, 1>(d.Ha, ta, fa, tc, fc, s));
        if (rc != MARL_OK) return rc;
      }
      // ---- actor
      const bool fused_a = fused_forward_supported(d.Ha, d.D);
      if (!pair) {
        ActorLoss fn{lc, tr.action, tr.logp, tr.adv};
        if (d.bf16) {
          train_net_bf16<kActions>(Xa, Sa, d.D, d.Ha, effective_bf16_weights(c, eff, 0), eff, oa, w.grad, ga, fn, w.dla, wk, false, s);
        } else if (fused_train_supported(d.Ha, d.D) && Sa < ((int64_t)1 << 31)) {
          FusedTrainArgs ta{};
          ta.X = Xa; ta.S = Sa; ta.Din = d.D; ta.px = fused_train_px(d.D);
          ta.W1 = eff + oa.W1; ta.b1 = eff + oa.b1; ta.W2 = eff + oa.W2; ta.b2 = eff + oa.b2; ta.W3 = eff + oa.W3;
          ta.W1s = eff + pm.sw_w1[0]; ta.W2s = eff + pm.sw_w2[0]; ta.W2Ts = eff + pm.sw_w2t[0];
          ta.b3 = eff + oa.b3; ta.gW1 = w.grad + ga.W1; ta.gb1 = w.grad + ga.b1; ta.gW2 = w.grad + ga.W2;
          ta.gb2 = w.grad + ga.b2; ta.gW3 = w.grad + ga.W3; ta.gb3 = w.grad + ga.b3; ta.stats = sck->acc;
          ta.partial = w.partial; ta.gcount = d.Pa;
          const int32_t rc = launch_fused_train<kActions>(d.Ha, ta, fn, s);
          if (rc != MARL_OK) return rc;
        } else {
          if (fused_a) {
            FusedFwdArgs fa{};
            fa.X = Xa; fa.S = Sa; fa.Din = d.D; fa.xvec = aligned16(Xa.base) && Xa.ld % 4 == 0 && d.D % 4 == 0;
            fa.W1 = eff + oa.W1; fa.b1 = eff + oa.b1; fa.W2 = eff + oa.W2; fa.b2 = eff + oa.b2; fa.W3 = eff + oa.W3;
            fa.b3 = eff + oa.b3; fa.h1_out = w.h1a; fa.dz2_out = w.h2a; fa.gW3 = w.grad + ga.W3; fa.gb3 = w.grad + ga.b3;
            fa.stats = sck->acc;
            fa.partial3 = ga.b3 == ga.W3 + (int64_t)d.Ha * kActions ? w.partial_head : nullptr;
            fa.W1s = eff + pm.sw_w1[0]; fa.W2s = eff + pm.sw_w2[0]; fa.kpad1 = pm.kpad1[0]; fa.px = fused_forward_px(d.D);
            const int32_t rc = launch_fused_forward<kActions, true>(d.Ha, fa, fn, s);
            if (rc != MARL_OK) return rc;
          } else {
            mlp_hidden_forward(Xa, Sa, d.D, d.Ha, eff + oa.W1, eff + oa.b1, eff + oa.W2, eff + oa.b2, w.h1a, w.h2a, d.bf16, s);
            const unsigned nb = (unsigned)std::min<int64_t>(2048, (Sa + kHeadTile - 1) / kHeadTile);
            hipLaunchKernelGGL((loss_head_kernel<kActions, ActorLoss, float>), dim3(nb), dim3(256), 0, s, w.h2a, Sa, d.Ha,
                               eff + oa.W3, eff + oa.b3, fn, w.dla, w.grad + ga.W3, w.grad + ga.b3, sck, 0.f);
          }
          mlp_backward<kActions>(Xa, Sa, d.D, d.Ha, eff + oa.W2, eff + oa.W3, w.h1a, w.h2a, w.dz1a, w.dla, w.grad + ga.W1,
                                 w.grad + ga.b1, w.grad + ga.W2, w.grad + ga.b2, d.bf16, fused_a, nullptr, w.split_ws, w.split_floats, s);
        }
      }
      // ---- critic
      const bool fused_c = fused_forward_supported(d.Hc, d.Dc);
      if (!pair) {
        CriticLoss fn{lc, tr.ret, tr.value, d.central ? d.A : 1};
        if (d.bf16) {
          // IPPO: the critic reads the rows the actor has just packed (same rows, same width)
          train_net_bf16<1>(Xc, Sc, d.Dc, d.Hc, effective_bf16_weights(c, eff, 1), eff, oc, w.grad, gc, fn, w.dlc, wk, !d.central, s);
        } else if (fused_train_supported(d.Hc, d.Dc) && Sc < ((int64_t)1 << 31)) {
          FusedTrainArgs ta{};
          ta.X = Xc; ta.S = Sc; ta.Din = d.Dc; ta.px = fused_train_px(d.Dc);
          ta.W1 = eff + oc.W1; ta.b1 = eff + oc.b1; ta.W2 = eff + oc.W2; ta.b2 = eff + oc.b2; ta.W3 = eff + oc.W3;
          ta.W1s = eff + pm.sw_w1[1]; ta.W2s = eff + pm.sw_w2[1]; ta.W2Ts = eff + pm.sw_w2t[1];
          ta.b3 = eff + oc.b3; ta.gW1 = w.grad + gc.W1; ta.gb1 = w.grad + gc.b1; ta.gW2 = w.grad + gc.W2;
          ta.gb2 = w.grad + gc.b2; ta.gW3 = w.grad + gc.W3; ta.gb3 = w.grad + gc.b3; ta.stats = sck->acc;
          ta.partial = w.partial; ta.gcount = d.P - d.Pa;
          const int32_t rc = launch_fused_train<1>(d.Hc, ta, fn, s);
          if (rc != MARL_OK) return rc;
        } else {
          if (wreg_forward_supported(Xc, Sc, d.Dc, d.Hc)) {
            const int32_t rc = train_forward_wreg<1>(Xc, Sc, d.Dc, eff + oc.W1, eff + oc.b1, eff + oc.W2, eff + oc.b2,
                                                     eff + oc.W3, eff + oc.b3, w.h1c, w.h2c, w.grad + gc.W3,
                                                     w.grad + gc.b3, sck->acc, fn,
                                                     gc.b3 == gc.W3 + (int64_t)kWregN ? w.partial_head : nullptr, s);
            if (rc != MARL_OK) return rc;
          } else if (fused_c) {
            FusedFwdArgs fa{};
            fa.X = Xc; fa.S = Sc; fa.Din = d.Dc; fa.xvec = aligned16(Xc.base) && Xc.ld % 4 == 0 && d.Dc % 4 == 0;
            fa.W1 = eff + oc.W1; fa.b1 = eff + oc.b1; fa.W2 = eff + oc.W2; fa.b2 = eff + oc.b2; fa.W3 = eff + oc.W3;
            fa.b3 = eff + oc.b3; fa.h1_out = w.h1c; fa.dz2_out = w.h2c; fa.gW3 = w.grad + gc.W3; fa.gb3 = w.grad + gc.b3;
            fa.stats = sck->acc;
            fa.partial3 = gc.b3 == gc.W3 + (int64_t)d.Hc ? w.partial_head : nullptr;
            fa.W1s = eff + pm.sw_w1[1]; fa.W2s = eff + pm.sw_w2[1]; fa.kpad1 = pm.kpad1[1]; fa.px = fused_forward_px(d.Dc);
            const int32_t rc = launch_fused_forward<1, true>(d.Hc, fa, fn, s);
            if (rc != MARL_OK) return rc;
          } else {
            mlp_hidden_forward(Xc, Sc, d.Dc, d.Hc, eff + oc.W1, eff + oc.b1, eff + oc.W2, eff + oc.b2, w.h1c, w.h2c, d.bf16, s);
            const unsigned nb = (unsigned)std::min<int64_t>(2048, (Sc + kHeadTile - 1) / kHeadTile);
            hipLaunchKernelGGL((loss_head_kernel<1, CriticLoss, float>), dim3(nb), dim3(256), 0, s, w.h2c, Sc, d.Hc, eff + oc.W3,
                               eff + oc.b3, fn, w.dlc, w.grad + gc.W3, w.grad + gc.b3, sck, 0.f);
          }
          mlp_backward<1>(Xc, Sc, d.Dc, d.Hc, eff + oc.W2, eff + oc.W3, w.h1c, w.h2c, w.dz1c, w.dlc, w.grad + gc.W1,
                          w.grad + gc.b1, w.grad + gc.W2, w.grad + gc.b2, d.bf16, fused_c, w.partial_w1, w.split_ws, w.split_floats, s);
        }
      }
      // ---- clip + Adam
      hipLaunchKernelGGL(grad_norm_kernel, dim3(grad_norm_blocks(d.P)), dim3(256), 0, s,
                         w.grad, d.P, sck);
      ++k;
      AdamArgs a{};
      a.norm_blocks = (int)grad_norm_blocks(d.P);
      a.k_base = adam_step_base;
      a.k_local = (int)k;
      a.lr = c.lr; a.b1 = c.beta1; a.b2 = c.beta2; a.eps = c.adam_eps;
      a.bc1 = (float)(1.0 - std::pow((double)c.beta1, (double)k));
      a.bc2 = (float)(1.0 - std::pow((double)c.beta2, (double)k));
      a.max_norm = c.max_grad_norm; a.ent_coef = c.ent_coef; a.vf_coef = c.vf_coef;
      const bool last = (e == c.n_epochs - 1 && mb == c.n_minibatches - 1);
      hipLaunchKernelGGL(adam_kernel, dim3((unsigned)((d.P + 255) / 256)), dim3(256), 0, s, params, adam_m, adam_v,
                         w.grad, d.P, a, sck, stats + (int64_t)(e * c.n_minibatches + mb) * MARL_N_STATS,
                         (last ? grad_dump : nullptr), w.sc + ((step + 1) & 1));
      const int32_t rc = launch_status();
      if (rc != MARL_OK) return rc;
    }
  }
  return MARL_OK;
}

}  // namespace marl

#ifdef MARL_PHASE_TIMERS
// Development aid (not part of the built library): cycles per phase of the fused training kernel, workgroup 0.
extern "C" int32_t marl_debug_phase_cycles(long long* out16, int32_t reset) {
  if (hipDeviceSynchronize() != hipSuccess) return -1;
  if (out16 && hipMemcpyFromSymbol(out16, HIP_SYMBOL(marl::g_phase_cycles), 16 * sizeof(long long)) != hipSuccess) return -1;
  if (reset) {
    long long z[16] = {0};
    if (hipMemcpyToSymbol(HIP_SYMBOL(marl::g_phase_cycles), z, sizeof(z)) != hipSuccess) return -1;
  }
  return 0;
}
#endif
