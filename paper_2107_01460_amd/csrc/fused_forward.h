// Fused network forward pass: both hidden layers, the output layer and whatever consumes the outputs
// (sampling during the rollout, the PPO loss during the update) in one kernel, with the first hidden
// activation kept in LDS between the two MFMA GEMMs.  In training mode the kernel also produces what the
// backward pass needs: h1 and dz2 = dL/d(pre-activation of layer 2) go to HBM once, h2 never does, and the
// output-layer gradient (W3, b3) is accumulated in registers across the row tiles a workgroup owns.
//
// Workgroup = 4 wavefronts on a tile of BM samples x H hidden units: (BM/32) x (H/32) MFMA tiles of
// 32x32, one or two per wavefront; several small workgroups per CU overlap each other's phases.  The row tile of
// the input sits in LDS at its whole width; the weights go straight from the operand-order copies in global memory
// (L2-resident) into registers with 16-byte loads (gemm_phase_regs), so a layer has no staging buffer and no barrier
// of its own.
#pragma once
#include "gemm.h"
#include "heads.h"

namespace marl {

struct FusedFwdArgs {
  RowSrc X;   // S rows of Din floats (optionally gathered)
  int64_t S;
  int Din;
  int xvec;   // 1: rows are 16-byte aligned and Din % 4 == 0: 16-byte loads of X.  2: rows start at any 4-byte boundary of a
              // buffer whose two ends are 16-byte aligned: a row is fetched as the aligned 16-byte chunks that cover it
  const float *W1, *b1, *W2, *b2, *W3, *b3;  // aligned working copy, W[in][H]
  const float *W1s, *W2s;  // operand-order copies: (k, n) at ((k / 4) * H + n) * 4 + k % 4; W1s zero-padded to kpad1 rows
  int kpad1;               // Din rounded up to a multiple of 16
  int px;                  // pitch of the X tile in LDS: a multiple of 4 with px / 4 odd, >= kpad1
  float* h1_out;   // training: [S][H]
  float* dz2_out;  // training: [S][H]
  float* gW3;      // training: [H][NOUT] accumulated with atomics
  float* gb3;      // training: [NOUT]
  float* stats;    // training: 5 floats accumulated with atomics (policy loss, value loss, entropy, KL, clip fraction)
  // training, H = 256 (one thread per hidden unit), nullable: workgroup b stores its share of the W3 gradient and, behind
  // it, of the b3 gradient at partial3 + b * (H * NOUT + NOUT) with plain stores; the launcher then adds the copies to
  // gW3 (which gb3 must directly follow) in a fixed order.  Room for kFusedFwdTrainGrid copies.
  float* partial3;
};
constexpr int kFusedFwdTrainGrid = 1024;  // workgroups of a training launch (persistent: register-resident W3 gradient)

inline int fused_forward_px(int Din) {
  int px = (Din + 15) / 16 * 16;
  while ((px / 4) % 2 == 0) px += 4;
  return px;
}

template <int H, int BM, int NOUT, bool TRAIN, class Finish>
__global__ void __launch_bounds__(256, 2) fused_forward_kernel(FusedFwdArgs a, Finish fin) {
  constexpr int PH = H + 4, GROUPS = 256 / BM;
  constexpr int NTN = H / 32, MT = BM / 32, TILES = MT * NTN, TPW = TILES / 4;
  static_assert(TILES % 4 == 0 && (TPW == 1 || TPW == 2), "4 wavefronts share the tile evenly");
  static_assert(TPW == 1 || NTN % 2 == 0, "two tiles of a wavefront share their rows");
  constexpr int NTH = 256;
  constexpr int TPR = NTH / BM;  // threads staging one row of X
  extern __shared__ __attribute__((aligned(16))) float lds[];
  struct {
    float *Xs, *Hs, *red, *dls, *W3s;
  } L;
  const int px = a.px;
  L.Xs = lds;                          // [BM][px]   input rows, k-contiguous; columns Din .. px stay zero
  L.Hs = L.Xs + BM * px;               // [BM][PH]   h1, then h2
  L.red = L.Hs + BM * PH;              // [GROUPS][BM][NOUT]
  L.dls = L.red + GROUPS * BM * NOUT;  // [BM][8]    dL/d(outputs), rows padded to 8 with zeros (MFMA operand)
  L.W3s = L.dls + BM * 8;              // [H][NOUT]

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
  for (int i = tid; i < BM * px; i += NTH) L.Xs[i] = 0.f;        // the padding columns stay zero for good
  __syncthreads();
  const int64_t ntiles = (a.S + BM - 1) / BM;
  for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const int64_t s0 = tile * BM;
    const int rows_left = (int)min((int64_t)BM, a.S - s0);
    float* const h1_tile = TRAIN ? a.h1_out + s0 * H : nullptr;    // uniform bases: lanes add 32-bit offsets
    float* const dz2_tile = TRAIN ? a.dz2_out + s0 * H : nullptr;
    // ---- this tile's rows to LDS: thread -> row tid / TPR, every TPR-th 16-byte (or 4-byte) piece of it, four
    // (twelve) loads in flight at a time.  Rows past the end re-read the last row (their results are never stored).
    {
      const int xr_row = tid / TPR, c0 = tid % TPR;
      const float* xrow = a.X.ptr(min(s0 + xr_row, a.S - 1));
      float* xdst = L.Xs + xr_row * px;
      if (a.xvec == 2) {
        // element j of chunk q is column 4 q + j - xo of the row; the chunks never leave the buffer (its ends are aligned)
        // (pointer arithmetic, not an integer round trip, so that the loads stay global loads)
        const int xo = (int)((reinterpret_cast<uintptr_t>(xrow) >> 2) & 3), last = ((xo + a.Din + 3) >> 2) - 1;
        const float4* const chunk = reinterpret_cast<const float4*>(xrow - xo);
        constexpr int XC = 3;  // chunks in flight per thread: a 75-wide row is one batch
        for (int q = c0; q <= last; q += XC * TPR) {
          float4 v[XC];
#pragma unroll
          for (int u = 0; u < XC; ++u) v[u] = chunk[min(q + u * TPR, last)];
#pragma unroll
          for (int u = 0; u < XC; ++u) {
            const float e[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int c = 4 * (q + u * TPR) + j - xo;
              if (c >= 0 && c < a.Din && q + u * TPR <= last) xdst[c] = e[j];
            }
          }
        }
      } else if (a.xvec) {
        const int nv = a.Din / 4;
        for (int c = c0; c < nv; c += 4 * TPR) {
          float4 v[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int cu = min(c + u * TPR, nv - 1);
            v[u] = *reinterpret_cast<const float4*>(xrow + 4 * cu);
          }
#pragma unroll
          for (int u = 0; u < 4; ++u)
            if (c + u * TPR < nv) *reinterpret_cast<float4*>(xdst + 4 * (c + u * TPR)) = v[u];
        }
      } else {
        constexpr int XB = 12;  // loads in flight per thread: a 75- or 27-wide row is one batch
        for (int c = c0; c < a.Din; c += XB * TPR) {
          float v[XB];
#pragma unroll
          for (int u = 0; u < XB; ++u) v[u] = xrow[min(c + u * TPR, a.Din - 1)];
#pragma unroll
          for (int u = 0; u < XB; ++u)
            if (c + u * TPR < a.Din) xdst[c + u * TPR] = v[u];
        }
      }
    }
    __syncthreads();
    floatx16 acc[TPW];
    auto zero_acc = [&]() {
#pragma unroll
      for (int q = 0; q < TPW; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;
    };
    // ---- layer 1: h1 = tanh(X W1 + b1) -> LDS (and HBM when training)
    zero_acc();
#pragma unroll
    for (int q = 0; q < TPW; ++q)
      gemm_phase_regs<H>(L.Xs + (mt * 32 + lo) * px + 4 * hi, a.W1s + (hi * H + (nt0 + q) * 32 + lo) * 4, a.kpad1 / 16, acc[q]);
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
    __syncthreads();  // the h1 tile is complete
    // ---- layer 2: h2 = tanh(h1 W2 + b2), kept in registers
    zero_acc();
#pragma unroll
    for (int q = 0; q < TPW; ++q)
      gemm_phase_regs<H>(L.Hs + (mt * 32 + lo) * PH + 4 * hi, a.W2s + (hi * H + (nt0 + q) * 32 + lo) * 4, H / 16, acc[q]);
    __syncthreads();  // every wavefront is past its last read of h1
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
      const int n = (nt0 + q) * 32 + lo;
      const float bias = a.b2[n];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        float v = tanh_f32(acc[q][r] + bias);
        acc[q][r] = v;
        L.Hs[m * PH + n] = v;
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
      static_assert(PER % 4 == 0, "hidden units are read four at a time");
#pragma unroll 2
      for (int i = grp * PER; i < (grp + 1) * PER; i += 4) {
        const float4 hv = *reinterpret_cast<const float4*>(&L.Hs[s * PH + i]);
        const float hh[4] = {hv.x, hv.y, hv.z, hv.w};
        float wv[4 * NOUT];  // W3 rows i..i+3: 4 * NOUT consecutive floats, the same for every lane of the wavefront
#pragma unroll
        for (int q = 0; q < NOUT; ++q) {
          const float4 t = *reinterpret_cast<const float4*>(&L.W3s[i * NOUT + 4 * q]);
          wv[4 * q] = t.x; wv[4 * q + 1] = t.y; wv[4 * q + 2] = t.z; wv[4 * q + 3] = t.w;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int k = 0; k < NOUT; ++k) part[k] = fmaf(hh[j], wv[j * NOUT + k], part[k]);
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
    float* const own = (H == 256 && a.partial3 != nullptr) ? a.partial3 + (int64_t)blockIdx.x * (H * NOUT + NOUT) : nullptr;
#pragma unroll
    for (int k = 0; k < NOUT; ++k) {
      if (own != nullptr) own[i * NOUT + k] = gw[k];
      else atomicAdd(&a.gW3[i * NOUT + k], gw[k]);
    }
    if (wave == 0) {  // samples live in threads tid < BM <= 64
#pragma unroll
      for (int k = 0; k < NOUT; ++k) {
        float v = gb[k];
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if (lane == 0) {
          if (own != nullptr) own[H * NOUT + k] = v;
          else atomicAdd(&a.gb3[k], v);
        }
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
inline size_t fused_forward_lds_bytes(int H, int Din, int nout) {
  const size_t bm = H == 64 ? 64 : 32;
  return (bm * fused_forward_px(Din) + bm * (H + 4) + 256 * (size_t)nout + bm * 8 + (size_t)H * nout) * sizeof(float);
}
// The row tile of the input sits in LDS at its whole width, which bounds the input width (two workgroups per CU up
// to about 320 inputs at H = 256, one up to about 950); wider networks take the layer-by-layer kernels.
inline bool fused_forward_supported(int H, int Din) {
  return (H == 64 || H == 128 || H == 256) && fused_forward_lds_bytes(H, Din, 6) <= 160 * 1024;
}

template <int H, int BM, int NOUT, bool TRAIN, class Finish>
inline int32_t launch_fused_forward_inst(const FusedFwdArgs& a, const Finish& fin, hipStream_t s) {
  auto kern = fused_forward_kernel<H, BM, NOUT, TRAIN, Finish>;
  const size_t bytes = fused_forward_lds_bytes(H, a.Din, NOUT);
  static bool configured = false;  // per instantiation
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return MARL_E_LAUNCH;
    configured = true;
  }
  const int64_t tiles = (a.S + BM - 1) / BM;
  const unsigned grid = (unsigned)std::min<int64_t>(tiles, TRAIN ? kFusedFwdTrainGrid : 2048);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), bytes, s, a, fin);
  const int32_t rc = launch_status();
  if (TRAIN && H == 256 && a.partial3 != nullptr && rc == MARL_OK)
    launch_reduce_partials(a.partial3, (int)grid, (int64_t)H * NOUT + NOUT, a.gW3, s);
  return rc;
}

template <int NOUT, bool TRAIN, class Finish>
inline int32_t launch_fused_forward(int H, const FusedFwdArgs& a, const Finish& fin, hipStream_t s) {
  // algorithmic flops of the two hidden layers
  TimedLaunch timed(KC_GEMM_NN, 2.0 * (double)a.S * ((double)a.Din * H + (double)H * H), s);
  if (H == 64) return launch_fused_forward_inst<64, 64, NOUT, TRAIN, Finish>(a, fin, s);
  if (H == 128) return launch_fused_forward_inst<128, 32, NOUT, TRAIN, Finish>(a, fin, s);
  return launch_fused_forward_inst<256, 32, NOUT, TRAIN, Finish>(a, fin, s);
}

}  // namespace marl
