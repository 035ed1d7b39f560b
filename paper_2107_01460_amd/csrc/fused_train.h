// Whole-network training pass for the small networks (hidden width 64 or 128, input width <= 96):
// forward, PPO loss, and the complete backward pass of one network in ONE kernel.  Nothing but the
// observations and a few scalars per sample is read from HBM and nothing but the parameter gradient is
// written: h1, h2, dz2, dz1 live in LDS / registers for the lifetime of a row tile, and the weight
// gradients are accumulated in registers over all row tiles a workgroup owns.
//
// Workgroup = NW wavefronts, persistent.  Row tile = BM samples with (BM/32)(H/32) = NW, so that a layer
// output is exactly NW 32x32 MFMA tiles, one per wavefront.  With NW = 4 (BM 32 for H = 128, 64 for H = 64)
// two workgroups share a CU: their phases drift apart, so the ALU phases of one (tanh epilogues, output
// layer, loss) run in the shadow of the other's MFMA phases.  Per tile:
//   X -> LDS | L1 (W1 streamed in 32-row chunks) -> h1 (LDS) | L2 -> h2 (registers + LDS) |
//   output layer on the ALUs -> loss -> dL/dout | W3 gradient | dz2 = (dL/dout W3^T)(1-h2^2) -> LDS |
//   dW2 += h1^T dz2 | dz1 = (dz2 W2^T)(1-h1^2) -> LDS (W2 streamed as k-contiguous chunks) | dW1 += X^T dz1
// The observations and loss inputs of the NEXT tile are fetched into registers at the start of the
// current one, so their HBM latency is hidden behind a whole tile of arithmetic.
#pragma once
#include "gemm.h"

namespace marl {

#ifdef MARL_PHASE_TIMERS
__device__ long long g_phase_cycles[16];
#define PHASE_MARK(i)                                                    \
  do {                                                                   \
    if (tid == 0 && blockIdx.x == 0) {                                   \
      const long long now_ = (long long)__builtin_amdgcn_s_memtime();    \
      g_phase_cycles[i] += now_ - phase_t0_;                             \
      phase_t0_ = now_;                                                  \
    }                                                                    \
  } while (0)
#else
#define PHASE_MARK(i)
#endif

struct FusedTrainArgs {
  RowSrc X;  // S rows of Din floats (gathered)
  int64_t S;
  int Din;
  int px;  // pitch of the X tile in LDS: multiple of 4, px/4 odd, >= 32*ceil(Din/32)
  const float *W1, *b1, *W2, *b2, *W3, *b3;  // aligned working copy, W[in][H]
  float *gW1, *gb1, *gW2, *gb2, *gW3, *gb3;  // gradient blocks, accumulated with atomics
  float* stats;                              // 5 floats, atomics
  int round_bf16;
};

template <int H, int BM, int NOUT, int DMAX, int NW, class LossFn>
__global__ void __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) fused_train_kernel(FusedTrainArgs a, LossFn fn) {
  constexpr int NT = 64 * NW;
  constexpr int NTN = H / 32, MTF = BM / 32, PH = H + 4, GROUPS = NT / BM, PW = 36;
  static_assert(NTN * MTF == NW, "one forward tile per wavefront");
  constexpr int TPR = NT / BM;           // threads staging one row of X
  constexpr int XP = DMAX / TPR;         // X elements per thread
  constexpr int WV = 8 * H / NT;         // 16-byte vectors of a weight chunk per thread
  constexpr int DW2_TPW = NTN * NTN >= NW ? NTN * NTN / NW : 1;  // dW2 tiles per wavefront (one row of tiles at most)
  constexpr int DW2_KS = NTN * NTN >= NW ? 1 : NW / (NTN * NTN);  // split of the sample range when there are fewer tiles than wavefronts
  static_assert(DW2_TPW <= NTN && NTN % DW2_TPW == 0, "a wavefront's dW2 tiles share their row of tiles");
  constexpr int Q1 = ((DMAX / 32) * NTN + NW - 1) / NW;  // dW1 work items per wavefront
  constexpr int HPARTS = NT / H, SPP = BM / HPARTS;

  extern __shared__ __attribute__((aligned(16))) float lds[];
  float* Xs = lds;                         // [BM][px]
  float* H1 = Xs + BM * a.px;              // [BM][PH]  h1, later dz1
  float* H2 = H1 + BM * PH;                // [BM][PH]  h2, later dz2
  float* Ws = H2 + BM * PH;                // [32][H] or [H][36]
  float* red = Ws + H * PW;                // [GROUPS][BM][NOUT]
  float* dls = red + NT * NOUT;           // [BM][8]
  float* W3s = dls + BM * 8;               // [H][NOUT]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = lane & 31, hi = lane >> 5;
  const int mt = wave / NTN, nt = wave % NTN;  // forward / dz tile of this wavefront
  const int px = a.px;
  const int MT1 = (a.Din + 31) / 32;           // 32-row tiles of dW1
  const int tiles1 = MT1 * NTN;
  const int KS1 = tiles1 * 4 <= Q1 * NW ? 4 : (tiles1 * 2 <= Q1 * NW ? 2 : 1);
  const int items1 = tiles1 * KS1;

  for (int i = tid; i < BM * px; i += NT) Xs[i] = 0.f;  // the padding columns stay zero for good
  for (int i = tid; i < H * NOUT; i += NT) W3s[i] = a.W3[i];
  __syncthreads();

  floatx16 acc1[Q1], acc2[DW2_TPW];  // dW1 / dW2 tiles of this wavefront, persistent
#pragma unroll
  for (int q = 0; q < Q1; ++q)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc1[q][r] = 0.f;
#pragma unroll
  for (int q = 0; q < DW2_TPW; ++q)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc2[q][r] = 0.f;
  float gw[NOUT], gb[NOUT], st[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < NOUT; ++k) gw[k] = gb[k] = 0.f;
  float gb1r = 0.f, gb2r = 0.f;  // bias gradients of column nt*32+lo (lanes hi == 0)

  // ---- staging helpers
  float xr[XP];
  typename LossFn::In lin_next{};
  const int xrow_l = tid / TPR, xcol0 = tid % TPR;
  auto fetch_tile_inputs = [&](int64_t s0) {
    const float* row = a.X.ptr(min(s0 + xrow_l, a.S - 1));
#pragma unroll
    for (int p = 0; p < XP; ++p) {
      const int c = xcol0 + TPR * p;
      xr[p] = c < a.Din ? row[c] : 0.f;
    }
    if (tid < BM && s0 + tid < a.S) lin_next = fn.load(s0 + tid);
  };
  float4 wr[WV];
  auto fetch_w = [&](const float* W, int k0, int K) {  // rows k0..k0+31 of W[K][H]
#pragma unroll
    for (int p = 0; p < WV; ++p) {
      const int f = tid + NT * p, row = f / (H / 4), c4 = f % (H / 4);
      wr[p] = (k0 + row < K) ? *reinterpret_cast<const float4*>(W + (int64_t)(k0 + row) * H + 4 * c4)
                             : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  auto stage_w = [&]() {
#pragma unroll
    for (int p = 0; p < WV; ++p) {
      const int f = tid + NT * p;
      *reinterpret_cast<float4*>(&Ws[(f / (H / 4)) * H + 4 * (f % (H / 4))]) = wr[p];
    }
  };
  auto fetch_wt = [&](int j0) {  // columns j0..j0+31 of W2, all H rows (k-contiguous chunk for the transposed product)
#pragma unroll
    for (int p = 0; p < WV; ++p) {
      const int f = tid + NT * p, i = f >> 3, c4 = f & 7;
      wr[p] = *reinterpret_cast<const float4*>(a.W2 + (int64_t)i * H + j0 + 4 * c4);
    }
  };
  auto stage_wt = [&]() {
#pragma unroll
    for (int p = 0; p < WV; ++p) {
      const int f = tid + NT * p;
      *reinterpret_cast<float4*>(&Ws[(f >> 3) * PW + 4 * (f & 7)]) = wr[p];
    }
  };

  const int nk1 = MT1;
  const int64_t ntiles = (a.S + BM - 1) / BM;
  int64_t tile = blockIdx.x;
  if (tile < ntiles) fetch_tile_inputs(tile * BM);
#ifdef MARL_PHASE_TIMERS
  long long phase_t0_ = (long long)__builtin_amdgcn_s_memtime();
#endif
  for (; tile < ntiles; tile += gridDim.x) {
    const int64_t s0 = tile * BM;
    // ---- this tile's observations to LDS; next tile's on their way
#pragma unroll
    for (int p = 0; p < XP; ++p) {
      const int c = xcol0 + TPR * p;
      if (c < a.Din) Xs[xrow_l * px + c] = xr[p];
    }
    const typename LossFn::In lin = lin_next;
    fetch_w(a.W1, 0, a.Din);
    __syncthreads();
    if (tile + gridDim.x < ntiles) fetch_tile_inputs((tile + gridDim.x) * BM);

    PHASE_MARK(0);
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    // ---- layer 1
#pragma unroll 1
    for (int c = 0; c < nk1; ++c) {
      stage_w();
      __syncthreads();
      if (c + 1 < nk1) fetch_w(a.W1, 32 * (c + 1), a.Din);
      else fetch_w(a.W2, 0, H);
#pragma unroll
      for (int kb = 0; kb < 32; kb += 8) {
        const float4 av = *reinterpret_cast<const float4*>(&Xs[(mt * 32 + lo) * px + 32 * c + kb + 4 * hi]);
        const float af[4] = {av.x, av.y, av.z, av.w};
        float bf[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) bf[j] = Ws[(kb + 4 * hi + j) * H + nt * 32 + lo];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[j], acc, 0, 0, 0);
      }
      __syncthreads();
    }
    PHASE_MARK(1);
    {
      const int n = nt * 32 + lo;
      const float bias = a.b1[n];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        float v = tanh_f32(acc[r] + bias);
        if (a.round_bf16) v = round_to_bf16(v);
        H1[m * PH + n] = v;
        acc[r] = 0.f;
        if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);
      }
    }
    PHASE_MARK(2);
    // ---- layer 2
#pragma unroll 1
    for (int c = 0; c < H / 32; ++c) {
      stage_w();
      __syncthreads();  // also orders the h1 tile before its first use
      if (c + 1 < H / 32) fetch_w(a.W2, 32 * (c + 1), H);
      else fetch_wt(0);
#pragma unroll
      for (int kb = 0; kb < 32; kb += 8) {
        const float4 av = *reinterpret_cast<const float4*>(&H1[(mt * 32 + lo) * PH + 32 * c + kb + 4 * hi]);
        const float af[4] = {av.x, av.y, av.z, av.w};
        float bf[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) bf[j] = Ws[(kb + 4 * hi + j) * H + nt * 32 + lo];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[j], acc, 0, 0, 0);
      }
      __syncthreads();
    }
    PHASE_MARK(3);
    floatx16 h2r;  // h2 of this wavefront's tile
    {
      const int n = nt * 32 + lo;
      const float bias = a.b2[n];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        float v = tanh_f32(acc[r] + bias);
        if (a.round_bf16) v = round_to_bf16(v);
        h2r[r] = v;
        H2[m * PH + n] = v;
        if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();
    PHASE_MARK(4);
    // ---- output layer on the ALUs: thread -> (sample tid % BM, slice tid / BM of the hidden units)
    {
      const int s = tid % BM, grp = tid / BM;
      constexpr int PER = H / GROUPS;
      float part[NOUT];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) part[k] = 0.f;
#pragma unroll 4
      for (int i = grp * PER; i < (grp + 1) * PER; ++i) {
        const float h = H2[s * PH + i];
#pragma unroll
        for (int k = 0; k < NOUT; ++k) part[k] = fmaf(h, W3s[i * NOUT + k], part[k]);
      }
#pragma unroll
      for (int k = 0; k < NOUT; ++k) red[(grp * BM + s) * NOUT + k] = part[k];
    }
    __syncthreads();
    PHASE_MARK(5);
    if (tid < BM) {
      float out[NOUT], dl[NOUT];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) {
        float v = a.b3[k];
#pragma unroll
        for (int gq = 0; gq < GROUPS; ++gq) v += red[(gq * BM + tid) * NOUT + k];
        out[k] = v;
        dl[k] = 0.f;
      }
      if (s0 + tid < a.S) fn.compute(lin, out, dl, st);
#pragma unroll
      for (int k = 0; k < 8; ++k) dls[tid * 8 + k] = k < NOUT ? dl[k < NOUT ? k : 0] : 0.f;
#pragma unroll
      for (int k = 0; k < NOUT; ++k) gb[k] += dl[k];
    }
    __syncthreads();
    PHASE_MARK(6);
    // ---- W3 gradient: gW3[i][k] += sum_s h2[s][i] dl[s][k]   (thread -> hidden unit tid % H, a share of the samples)
    {
      const int i = tid % H, part = tid / H;
#pragma unroll 4
      for (int s = part * SPP; s < (part + 1) * SPP; ++s) {
        const float h = H2[s * PH + i];
#pragma unroll
        for (int k = 0; k < NOUT; ++k) gw[k] = fmaf(h, dls[s * 8 + k], gw[k]);
      }
    }
    __syncthreads();
    PHASE_MARK(7);
    // ---- dz2 = (dl W3^T) * (1 - h2^2) -> LDS over h2; the rank-NOUT product runs on the matrix cores (k padded to 8)
    {
      const int n = nt * 32 + lo;
      const float4 av = *reinterpret_cast<const float4*>(&dls[(mt * 32 + lo) * 8 + 4 * hi]);
      const float af[4] = {av.x, av.y, av.z, av.w};
      float bf[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) bf[j] = (4 * hi + j < NOUT) ? W3s[n * NOUT + (4 * hi + j < NOUT ? 4 * hi + j : 0)] : 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[j], acc, 0, 0, 0);
      float csum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        float v = acc[r] * (1.0f - h2r[r] * h2r[r]);
        if (a.round_bf16) v = round_to_bf16(v);
        H2[m * PH + n] = v;
        csum += v;
      }
      csum += __shfl_xor(csum, 32);
      gb2r += csum;
    }
    __syncthreads();
    PHASE_MARK(8);
    // ---- dW2 += h1^T dz2   (k runs over the samples of the tile)
    {
      const int t0 = (wave * DW2_TPW) % (NTN * NTN);
      const int it = t0 / NTN, jt = t0 % NTN;
      const int ks = (wave * DW2_TPW) / (NTN * NTN);
      constexpr int KLEN = BM / DW2_KS;
#pragma unroll 1
      for (int kb = ks * KLEN; kb < (ks + 1) * KLEN; kb += 8) {
        float af[4], bf[DW2_TPW][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          af[j] = H1[(kb + 4 * hi + j) * PH + it * 32 + lo];
#pragma unroll
          for (int q = 0; q < DW2_TPW; ++q) bf[q][j] = H2[(kb + 4 * hi + j) * PH + (jt + q) * 32 + lo];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int q = 0; q < DW2_TPW; ++q) acc2[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[q][j], acc2[q], 0, 0, 0);
      }
    }
    PHASE_MARK(9);
    // ---- dz1 = (dz2 W2^T) * (1 - h1^2), in place over h1
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll 1
    for (int c = 0; c < H / 32; ++c) {
      stage_wt();
      __syncthreads();
      if (c + 1 < H / 32) fetch_wt(32 * (c + 1));
#pragma unroll
      for (int kb = 0; kb < 32; kb += 8) {
        const float4 av = *reinterpret_cast<const float4*>(&H2[(mt * 32 + lo) * PH + 32 * c + kb + 4 * hi]);
        const float4 bv = *reinterpret_cast<const float4*>(&Ws[(nt * 32 + lo) * PW + kb + 4 * hi]);
        const float af[4] = {av.x, av.y, av.z, av.w}, bf[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[j], acc, 0, 0, 0);
      }
      __syncthreads();
    }
    PHASE_MARK(10);
    {
      const int n = nt * 32 + lo;
      float csum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        const float h = H1[m * PH + n];
        float v = acc[r] * (1.0f - h * h);
        if (a.round_bf16) v = round_to_bf16(v);
        H1[m * PH + n] = v;  // only this wavefront touches its tile of h1 from here on until the barrier
        csum += v;
      }
      csum += __shfl_xor(csum, 32);
      gb1r += csum;
    }
    __syncthreads();
    PHASE_MARK(11);
    // ---- dW1 += X^T dz1
#pragma unroll
    for (int q = 0; q < Q1; ++q) {
      const int item = wave + NW * q;
      if (item < items1) {
        const int t = item / KS1, ks = item - t * KS1;
        const int dt = t / NTN, jt = t % NTN;
        const int klen = BM / KS1;
#pragma unroll 1
        for (int kb = ks * klen; kb < (ks + 1) * klen; kb += 8) {
          float af[4], bf[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            af[j] = Xs[(kb + 4 * hi + j) * px + dt * 32 + lo];
            bf[j] = H1[(kb + 4 * hi + j) * PH + jt * 32 + lo];
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) acc1[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[j], acc1[q], 0, 0, 0);
        }
      }
    }
    PHASE_MARK(12);
    __syncthreads();  // the tile buffers are reused by the next row tile
    PHASE_MARK(13);
  }

  // ---- flush the register-resident gradients
  {
    const int t0 = (wave * DW2_TPW) % (NTN * NTN);
    const int it = t0 / NTN, jt = t0 % NTN;
#pragma unroll
    for (int q = 0; q < DW2_TPW; ++q)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = it * 32 + 8 * (r / 4) + 4 * hi + (r % 4), j = (jt + q) * 32 + lo;
        atomicAdd(&a.gW2[i * H + j], acc2[q][r]);
      }
  }
#pragma unroll
  for (int q = 0; q < Q1; ++q) {
    const int item = wave + NW * q;
    if (item < items1) {
      const int t = item / KS1, dt = t / NTN, jt = t % NTN;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int d = dt * 32 + 8 * (r / 4) + 4 * hi + (r % 4), j = jt * 32 + lo;
        if (d < a.Din) atomicAdd(&a.gW1[d * H + j], acc1[q][r]);
      }
    }
  }
  if (hi == 0) {
    atomicAdd(&a.gb1[nt * 32 + lo], gb1r);
    atomicAdd(&a.gb2[nt * 32 + lo], gb2r);
  }
  {
    const int i = tid % H;
#pragma unroll
    for (int k = 0; k < NOUT; ++k) atomicAdd(&a.gW3[i * NOUT + k], gw[k]);
  }
  if (tid < (BM < 64 ? 64 : BM)) {  // whole wavefronts; lanes past BM hold zeros
#pragma unroll
    for (int k = 0; k < NOUT; ++k) {
      float v = gb[k];
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
      if (lane == 0) atomicAdd(&a.gb3[k], v);
    }
#pragma unroll
    for (int k = 0; k < 5; ++k) {
      float v = st[k];
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
      if (lane == 0 && v != 0.f) atomicAdd(&a.stats[k], v);
    }
  }
}

inline bool fused_train_supported(int H, int Din) { return (H == 64 || H == 128) && Din <= 96; }

inline int fused_train_px(int Din) {
  int px = 32 * ((Din + 31) / 32);
  while (px % 4 != 0 || (px / 4) % 2 == 0) px += 4;
  return px;
}

template <int H, int BM, int NOUT, int DMAX, int NW, class LossFn>
inline int32_t launch_fused_train_inst(const FusedTrainArgs& a, const LossFn& fn, hipStream_t s) {
  auto kern = fused_train_kernel<H, BM, NOUT, DMAX, NW, LossFn>;
  const size_t floats = (size_t)BM * a.px + 2 * (size_t)BM * (H + 4) + (size_t)H * 36 + 64 * NW * NOUT + BM * 8 + H * NOUT;
  const size_t bytes = floats * 4;
  static bool configured = false;  // per instantiation
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
      return MARL_E_LAUNCH;
    configured = true;
  }
  const int64_t tiles = (a.S + BM - 1) / BM;
  const unsigned grid = (unsigned)std::min<int64_t>(tiles, NW == 4 ? 512 : 256);  // resident workgroups: two per CU with four wavefronts
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * NW), bytes, s, a, fn);
  return launch_status();
}

template <int NOUT, class LossFn>
inline int32_t launch_fused_train(int H, const FusedTrainArgs& a, const LossFn& fn, hipStream_t s) {
  // algorithmic flops: forward 2S(DH + HH), backward 2S(HH + HH + DH)
  TimedLaunch timed(KC_FUSED_TRAIN, 2.0 * (double)a.S * (2.0 * a.Din * H + 3.0 * H * H), s);
  if (H == 128) {
    if (a.Din <= 32) return launch_fused_train_inst<128, 64, NOUT, 32, 8, LossFn>(a, fn, s);
    return launch_fused_train_inst<128, 64, NOUT, 96, 8, LossFn>(a, fn, s);
  }
  if (a.Din <= 32) return launch_fused_train_inst<64, 128, NOUT, 32, 8, LossFn>(a, fn, s);
  return launch_fused_train_inst<64, 128, NOUT, 96, 8, LossFn>(a, fn, s);
}

}  // namespace marl
