// Fused network forward pass: both hidden layers, the output layer and whatever consumes the outputs
// (sampling during the rollout, the PPO loss during the update) in one kernel, with the first hidden
// activation kept in LDS between the two MFMA GEMMs.  In training mode the kernel also produces what the
// backward pass needs: h1 and dz2 = dL/d(pre-activation of layer 2) go to HBM once, h2 never does, and the
// output-layer gradient (W3, b3) is accumulated in registers across the row tiles a workgroup owns.
//
// Workgroup = 4 wavefronts on a tile of BM samples x H hidden units: (BM/32) x (H/32) MFMA tiles of
// 32x32, one or two per wavefront; several small workgroups per CU overlap each other's phases.  Weights stream from L2 through a 32-row LDS buffer; the next chunk
// travels global -> registers while the current one is multiplied.
#pragma once
#include "gemm.h"
#include "heads.h"

namespace marl {

struct FusedFwdArgs {
  RowSrc X;   // S rows of Din floats (optionally gathered)
  int64_t S;
  int Din;
  int xvec;   // rows are 16-byte aligned and Din % 4 == 0: 16-byte loads of X
  const float *W1, *b1, *W2, *b2, *W3, *b3;  // aligned working copy, W[in][H]
  float* h1_out;   // training: [S][H]
  float* dz2_out;  // training: [S][H]
  float* gW3;      // training: [H][NOUT] accumulated with atomics
  float* gb3;      // training: [NOUT]
  float* stats;    // training: 5 floats accumulated with atomics (policy loss, value loss, entropy, KL, clip fraction)
};

template <int H, int BM, int NOUT>
struct FusedFwdLds {
  static constexpr int PX = 36;     // pitch of the X chunk (k-contiguous, 16-byte reads)
  static constexpr int PH = H + 4;  // pitch of the activation tile
  static constexpr int GROUPS = 256 / BM;
  float Xc[BM * PX];
  float Ws[32 * H];
  float Hs[BM * PH];
  float red[GROUPS * BM * NOUT];
  float dls[BM * 8];  // dL/d(outputs) of the tile, rows padded to 8 with zeros (MFMA operand)
  float W3s[H * NOUT];
};

template <int H, int BM, int NOUT, bool TRAIN, class Finish>
__global__ void __launch_bounds__(256, 2) fused_forward_kernel(FusedFwdArgs a, Finish fin) {
  using Lds = FusedFwdLds<H, BM, NOUT>;
  constexpr int PX = Lds::PX, PH = Lds::PH, GROUPS = Lds::GROUPS;
  constexpr int NTN = H / 32, MT = BM / 32, TILES = MT * NTN, TPW = TILES / 4;
  static_assert(TILES % 4 == 0 && (TPW == 1 || TPW == 2), "4 wavefronts share the tile evenly");
  static_assert(TPW == 1 || NTN % 2 == 0, "two tiles of a wavefront share their rows");
  constexpr int NTH = 256;
  constexpr int WV = H / 32;   // 16-byte vectors of a weight chunk per thread
  constexpr int XS = BM / 8;   // scalars of an X chunk per thread
  constexpr int XV = BM / 32;  // 16-byte vectors of an X chunk per thread
  __shared__ __attribute__((aligned(16))) Lds L;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = lane & 31, hi = lane >> 5;
  const int mt = (wave * TPW) / NTN, nt0 = (wave * TPW) % NTN;  // this wavefront's tiles: (mt, nt0 .. nt0+TPW-1)

  // output-layer gradient, persistent over the tiles of this workgroup: thread -> hidden unit tid % H
  constexpr int HPARTS = (256 / H) > 0 ? (256 / H) : 1;  // threads per hidden unit
  constexpr int SPP = BM / HPARTS;        // samples each of them sums per tile
  float gw[NOUT], gb[NOUT], st[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < NOUT; ++k) gw[k] = gb[k] = 0.f;

  for (int i = tid; i < H * NOUT; i += NTH) L.W3s[i] = a.W3[i];  // ordered before its first use by the barriers of layer 1
  const int nk1 = (a.Din + 31) / 32;
  const int64_t ntiles = (a.S + BM - 1) / BM;
  for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const int64_t s0 = tile * BM;
    const int rows_left = (int)min((int64_t)BM, a.S - s0);
    float* const h1_tile = TRAIN ? a.h1_out + s0 * H : nullptr;    // uniform bases: lanes add 32-bit offsets
    float* const dz2_tile = TRAIN ? a.dz2_out + s0 * H : nullptr;
    // rows of X this thread stages
    const float* xrow[XS];
    if (a.xvec) {
#pragma unroll
      for (int p = 0; p < XV; ++p) xrow[p] = a.X.ptr(min(s0 + ((tid + NTH * p) >> 3), a.S - 1));
    } else {
#pragma unroll
      for (int p = 0; p < XS; ++p) xrow[p] = a.X.ptr(min(s0 + ((tid + NTH * p) >> 5), a.S - 1));
    }
    float xr[XS];
    float4 wr[WV];
    auto fetch_x = [&](int k0) {
      if (a.xvec) {
        const int k = k0 + 4 * (tid & 7);
#pragma unroll
        for (int p = 0; p < XV; ++p) {
          float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
          if (k < a.Din) v = *reinterpret_cast<const float4*>(xrow[p] + k);
          xr[4 * p] = v.x; xr[4 * p + 1] = v.y; xr[4 * p + 2] = v.z; xr[4 * p + 3] = v.w;
        }
      } else {
        const int k = k0 + (tid & 31);
#pragma unroll
        for (int p = 0; p < XS; ++p) xr[p] = k < a.Din ? xrow[p][k] : 0.f;
      }
    };
    auto stage_x = [&]() {
      if (a.xvec) {
#pragma unroll
        for (int p = 0; p < XV; ++p)
          *reinterpret_cast<float4*>(&L.Xc[((tid + NTH * p) >> 3) * PX + 4 * (tid & 7)]) =
              make_float4(xr[4 * p], xr[4 * p + 1], xr[4 * p + 2], xr[4 * p + 3]);
      } else {
#pragma unroll
        for (int p = 0; p < XS; ++p) L.Xc[((tid + NTH * p) >> 5) * PX + (tid & 31)] = xr[p];
      }
    };
    auto fetch_w = [&](const float* W, int k0, int K) {
#pragma unroll
      for (int p = 0; p < WV; ++p) {
        const int f = tid + NTH * p, row = f / (H / 4), c4 = f % (H / 4);
        wr[p] = (k0 + row < K) ? *reinterpret_cast<const float4*>(W + (int64_t)(k0 + row) * H + 4 * c4)
                               : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    };
    auto stage_w = [&]() {
#pragma unroll
      for (int p = 0; p < WV; ++p) {
        const int f = tid + NTH * p;
        *reinterpret_cast<float4*>(&L.Ws[(f / (H / 4)) * H + 4 * (f % (H / 4))]) = wr[p];
      }
    };
    floatx16 acc[TPW];
    auto zero_acc = [&]() {
#pragma unroll
      for (int q = 0; q < TPW; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;
    };
    // acc += A[32 rows of mt][32 k] * Ws[32 k][32 cols of each tile]; A is k-contiguous in LDS
    auto mma_chunk = [&](const float* A, int pitch, int koff) {
#pragma unroll
      for (int kb = 0; kb < 32; kb += 8) {
        const float4 av = *reinterpret_cast<const float4*>(&A[(mt * 32 + lo) * pitch + koff + kb + 4 * hi]);
        const float af[4] = {av.x, av.y, av.z, av.w};
        float bf[TPW][4];
#pragma unroll
        for (int q = 0; q < TPW; ++q)
#pragma unroll
          for (int j = 0; j < 4; ++j) bf[q][j] = L.Ws[(kb + 4 * hi + j) * H + (nt0 + q) * 32 + lo];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int q = 0; q < TPW; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[q][j], acc[q], 0, 0, 0);
      }
    };

    // ---- layer 1: h1 = tanh(X W1 + b1) -> LDS (and HBM when training)
    zero_acc();
    fetch_x(0);
    fetch_w(a.W1, 0, a.Din);
#pragma unroll 1
    for (int c = 0; c < nk1; ++c) {
      stage_x();
      stage_w();
      __syncthreads();
      if (c + 1 < nk1) {
        fetch_x(32 * (c + 1));
        fetch_w(a.W1, 32 * (c + 1), a.Din);
      } else {
        fetch_w(a.W2, 0, H);
      }
      mma_chunk(L.Xc, PX, 0);
      __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
      const int n = (nt0 + q) * 32 + lo;
      const float bias = a.b1[n];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        float v = tanh_f32(acc[q][r] + bias);
        L.Hs[m * PH + n] = v;
        if (TRAIN && m < rows_left) h1_tile[m * H + n] = v;
        if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);  // four elements in flight at a time keeps registers bounded
      }
    }
    // ---- layer 2: h2 = tanh(h1 W2 + b2), kept in registers
    zero_acc();
#pragma unroll 1
    for (int c = 0; c < H / 32; ++c) {
      stage_w();
      __syncthreads();  // also orders the h1 tile before its first use
      if (c + 1 < H / 32) fetch_w(a.W2, 32 * (c + 1), H);
      mma_chunk(L.Hs, PH, 32 * c);
      __syncthreads();
    }
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
      const int n = (nt0 + q) * 32 + lo;
      const float bias = a.b2[n];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        float v = tanh_f32(acc[q][r] + bias);
        acc[q][r] = v;
        L.Hs[m * PH + n] = v;  // every wavefront is past its last read of h1 (barrier above)
        if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);
      }
    }
    // W3 rows of this thread's columns, for the head (ALU) and for dz2
    __syncthreads();
    // ---- output layer on the ALUs: thread -> (sample tid % BM, slice tid / BM of the hidden units)
    {
      const int s = tid % BM, grp = tid / BM;
      constexpr int PER = H / GROUPS;
      float part[NOUT];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) part[k] = 0.f;
#pragma unroll 4
      for (int i = grp * PER; i < (grp + 1) * PER; ++i) {
        const float h = L.Hs[s * PH + i];
#pragma unroll
        for (int k = 0; k < NOUT; ++k) part[k] = fmaf(h, L.W3s[i * NOUT + k], part[k]);
      }
#pragma unroll
      for (int k = 0; k < NOUT; ++k) L.red[(grp * BM + s) * NOUT + k] = part[k];
    }
    __syncthreads();
    if (tid < BM) {
      float out[NOUT], dl[NOUT];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) {
        float v = a.b3[k];
#pragma unroll
        for (int gq = 0; gq < GROUPS; ++gq) v += L.red[(gq * BM + tid) * NOUT + k];
        out[k] = v;
        dl[k] = 0.f;
      }
      if (s0 + tid < a.S) fin(s0 + tid, out, dl, st);
      if (TRAIN) {
#pragma unroll
        for (int k = 0; k < 8; ++k) L.dls[tid * 8 + k] = k < NOUT ? dl[k < NOUT ? k : 0] : 0.f;
#pragma unroll
        for (int k = 0; k < NOUT; ++k) gb[k] += dl[k];
      }
    }
    if (TRAIN) {
      __syncthreads();
      // ---- dz2 = (dl W3^T) * (1 - h2^2): the rank-NOUT product runs on the matrix cores (k padded to 8) and
      // lands in the same lane layout as the register-resident h2
      const float4 av = *reinterpret_cast<const float4*>(&L.dls[(mt * 32 + lo) * 8 + 4 * hi]);
      const float af[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
      for (int q = 0; q < TPW; ++q) {
        const int n = (nt0 + q) * 32 + lo;
        float bf[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) bf[j] = (4 * hi + j < NOUT) ? L.W3s[n * NOUT + (4 * hi + j < NOUT ? 4 * hi + j : 0)] : 0.f;
        floatx16 gacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) gacc[r] = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) gacc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[j], gacc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
          const float h = acc[q][r];
          float v = gacc[r] * (1.0f - h * h);
          if (m < rows_left) dz2_tile[m * H + n] = v;
          if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }
      }
      // ---- gW3[i][k] += sum_s h2[s][i] dl[s][k]
      {
        const int i = tid % H, part = tid / H;
#pragma unroll 4
        for (int s = part * SPP; s < (part + 1) * SPP; ++s) {
          const float h = L.Hs[s * PH + i];
#pragma unroll
          for (int k = 0; k < NOUT; ++k) gw[k] = fmaf(h, L.dls[s * 8 + k], gw[k]);
        }
      }
    }
    __syncthreads();  // the tile buffers are reused by the next row tile
  }
  if (TRAIN) {
    const int i = tid % H;
#pragma unroll
    for (int k = 0; k < NOUT; ++k) atomicAdd(&a.gW3[i * NOUT + k], gw[k]);
    if (wave == 0) {  // samples live in threads tid < BM <= 64
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
}

// Which (H, BM) pairs exist: H = 64 -> BM 64; H = 128 or 256 -> BM 32.
inline bool fused_forward_supported(int H) { return H == 64 || H == 128 || H == 256; }

template <int NOUT, bool TRAIN, class Finish>
inline void launch_fused_forward(int H, const FusedFwdArgs& a, const Finish& fin, hipStream_t s) {
  // algorithmic flops of the two hidden layers
  TimedLaunch timed(KC_GEMM_NN, 2.0 * (double)a.S * ((double)a.Din * H + (double)H * H), s);
  const int64_t bm = H == 64 ? 64 : 32;
  const int64_t tiles = (a.S + bm - 1) / bm;
  const unsigned grid = (unsigned)std::min<int64_t>(tiles, TRAIN ? 1024 : 2048);  // persistent when training (register-resident W3 gradient)
  if (H == 64) hipLaunchKernelGGL((fused_forward_kernel<64, 64, NOUT, TRAIN, Finish>), dim3(grid), dim3(256), 0, s, a, fin);
  else if (H == 128) hipLaunchKernelGGL((fused_forward_kernel<128, 32, NOUT, TRAIN, Finish>), dim3(grid), dim3(256), 0, s, a, fin);
  else hipLaunchKernelGGL((fused_forward_kernel<256, 32, NOUT, TRAIN, Finish>), dim3(grid), dim3(256), 0, s, a, fin);
}

}  // namespace marl
