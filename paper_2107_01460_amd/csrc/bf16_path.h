// Helpers of the bf16 configuration: bf16 copies of the weights in the orientations the MFMA kernel wants,
// the observation pack (gather + convert + transposed copy), and dz2 with its transposed copy.
#pragma once
#include "gemm_bf16.h"

namespace marl {

inline int64_t round_up64(int64_t x) { return (x + 63) / 64 * 64; }

// bf16 weights of one network: W1t [H][Dp] (= W1 transposed, k-contiguous, zero-padded to Dp), W2t [H][H]
// (= W2 transposed) for the forward products, W2 [H][H] as stored for dz1 = dz2 W2^T.
struct Bf16NetWeights {
  bf16_t *W1t, *W2t, *W2;
  int Dp;
};
inline int64_t bf16_net_weight_elems(int Din, int H) { return (int64_t)H * round_up64(Din) + 2 * (int64_t)H * H; }
inline Bf16NetWeights bf16_net_weights(bf16_t* base, int Din, int H) {
  Bf16NetWeights w;
  w.Dp = (int)round_up64(Din);
  w.W1t = base;
  w.W2t = w.W1t + (int64_t)H * w.Dp;
  w.W2 = w.W2t + (int64_t)H * H;
  return w;
}

namespace bf16_detail {

static __global__ void stage_weights_bf16_kernel(const float* __restrict__ W1, const float* __restrict__ W2, int Din, int Dp,
                                                 int H, bf16_t* __restrict__ W1t, bf16_t* __restrict__ W2t,
                                                 bf16_t* __restrict__ W2b) {
  const int64_t n1 = (int64_t)H * Dp, n2 = (int64_t)H * H;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < max(n1, n2); i += (int64_t)gridDim.x * blockDim.x) {
    if (i < n1) {
      const int h = (int)(i / Dp), dd = (int)(i % Dp);
      W1t[i] = dd < Din ? to_bf16(W1[(int64_t)dd * H + h]) : (bf16_t)0;
    }
    if (i < n2) {
      const int r = (int)(i / H), c = (int)(i % H);
      const bf16_t v = to_bf16(W2[i]);
      W2b[i] = v;
      W2t[(int64_t)c * H + r] = v;
    }
  }
}

// Xb [S][Dp] = bf16(X), zero-padded columns; XbT its transpose ([Dp][Sp], stored sample-blocked: see gemm_bf16.h) with
// zero-padded samples (nullable).
static __global__ void __launch_bounds__(256) pack_obs_bf16_kernel(RowSrc X, int64_t S, int Din, int Dp, int64_t Sp,
                                                                   bf16_t* __restrict__ Xb, bf16_t* __restrict__ XbT) {
  __shared__ float tile[64][65];
  const int tid = threadIdx.x;
  const int64_t s0 = (int64_t)blockIdx.x * 64;
  const float* rows[16];  // thread stages rows tid/64 + 4q, column tid%64
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int64_t s = s0 + (tid >> 6) + 4 * q;
    rows[q] = s < S ? X.ptr(s) : nullptr;
  }
  for (int d0 = 0; d0 < Dp; d0 += 64) {
    const int cc = tid & 63;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int r = (tid >> 6) + 4 * q;
      tile[r][cc] = (rows[q] != nullptr && d0 + cc < Din) ? rows[q][d0 + cc] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int r = (tid >> 6) + 4 * q;
      if (s0 + r < S && d0 + cc < Dp) Xb[(s0 + r) * Dp + d0 + cc] = to_bf16(tile[r][cc]);
    }
    if (XbT != nullptr) {
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int dd = (tid >> 6) + 4 * q, ss = tid & 63;
        if (d0 + dd < Dp && s0 + ss < Sp) XbT[((s0 >> 6) * Dp + d0 + dd) * 64 + ss] = to_bf16(tile[ss][dd]);
      }
    }
    __syncthreads();
  }
}

// In place: H2[s][j] <- (sum_k dl[s][k] W3[j][k]) * (1 - H2[s][j]^2); dz2T [H][Sp] (sample-blocked) gets the transposed copy (zeros past S).
// One workgroup per tile of 64 samples x 64 hidden units; a thread owns eight consecutive hidden units of two rows
// (16-byte loads and stores, no branches: rows past the end are clamped for the loads and produce zeros), and eight
// consecutive samples of two hidden units for the transposed copy, which goes through an LDS tile.
template <int NOUT>
static __global__ void __launch_bounds__(256) dz2_bf16_kernel(bf16_t* __restrict__ H2, bf16_t* __restrict__ dz2T,
                                                              const float* __restrict__ dl, const float* __restrict__ W3,
                                                              int64_t S, int64_t Sp, int H) {
  constexpr int PT = 72;  // pitch of the tile in elements: 16-byte aligned rows, 36 dwords (4 * odd)
  __shared__ __attribute__((aligned(16))) bf16_t tile[64 * PT];
  const int tid = threadIdx.x;
  const int64_t s0 = (int64_t)blockIdx.x * 64;
  const int j0 = blockIdx.y * 64;
  const int c8 = tid & 7, j = j0 + 8 * c8;  // H is a multiple of 64
  float w[8][NOUT];
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int k = 0; k < NOUT; ++k) w[e][k] = W3[(int64_t)(j + e) * NOUT + k];
  uint4 hv[2];
  float dlv[2][NOUT];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int64_t s = min(s0 + (tid >> 3) + 32 * q, S - 1);
    hv[q] = *reinterpret_cast<const uint4*>(&H2[s * H + j]);
#pragma unroll
    for (int k = 0; k < NOUT; ++k) dlv[q][k] = dl[s * NOUT + k];
  }
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int r = (tid >> 3) + 32 * q;
    const bool live = s0 + r < S;
    const uint32_t hw[4] = {hv[q].x, hv[q].y, hv[q].z, hv[q].w};
    uint32_t ow[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      float o2[2];
#pragma unroll
      for (int z = 0; z < 2; ++z) {
        const float h = __uint_as_float(z == 0 ? hw[p] << 16 : hw[p] & 0xffff0000u);
        float g = 0.f;
#pragma unroll
        for (int k = 0; k < NOUT; ++k) g = fmaf(dlv[q][k], w[2 * p + z][k], g);
        o2[z] = live ? g * (1.0f - h * h) : 0.f;
      }
      ow[p] = pack2_bf16(o2[0], o2[1]);
    }
    const uint4 ov = make_uint4(ow[0], ow[1], ow[2], ow[3]);
    if (live) *reinterpret_cast<uint4*>(&H2[(s0 + r) * H + j]) = ov;
    *reinterpret_cast<uint4*>(&tile[r * PT + 8 * c8]) = ov;
  }
  __syncthreads();
  // transposed copy: thread -> hidden unit dd = tid / 8 + 32 q, samples 8 (tid % 8) .. + 7
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int dd = (tid >> 3) + 32 * q, ss = 8 * (tid & 7);
    uint32_t ow[4];
#pragma unroll
    for (int p = 0; p < 4; ++p)
      ow[p] = (uint32_t)tile[(ss + 2 * p) * PT + dd] | ((uint32_t)tile[(ss + 2 * p + 1) * PT + dd] << 16);
    if (s0 + ss < Sp) *reinterpret_cast<uint4*>(&dz2T[((s0 >> 6) * H + j0 + dd) * 64 + ss]) = make_uint4(ow[0], ow[1], ow[2], ow[3]);
  }
}

}  // namespace bf16_detail

inline void stage_weights_bf16(const float* W1, const float* W2, int Din, int H, const Bf16NetWeights& w, hipStream_t s) {
  const int64_t n = std::max<int64_t>((int64_t)H * w.Dp, (int64_t)H * H);
  hipLaunchKernelGGL(bf16_detail::stage_weights_bf16_kernel, dim3((unsigned)std::min<int64_t>(1024, (n + 255) / 256)), dim3(256),
                     0, s, W1, W2, Din, w.Dp, H, w.W1t, w.W2t, w.W2);
}

inline void pack_obs_bf16(const RowSrc& X, int64_t S, int Din, int Dp, int64_t Sp, bf16_t* Xb, bf16_t* XbT, hipStream_t s) {
  const int64_t cover = XbT ? Sp : S;
  hipLaunchKernelGGL(bf16_detail::pack_obs_bf16_kernel, dim3((unsigned)((cover + 63) / 64)), dim3(256), 0, s, X, S, Din, Dp, Sp,
                     Xb, XbT);
}

// Two hidden layers in bf16: h1 (and optionally h1T), h2.
inline void mlp_hidden_forward_bf16(const bf16_t* Xb, int64_t S, int64_t Sp, int H, const Bf16NetWeights& w, const float* b1,
                                    const float* b2, bf16_t* h1, bf16_t* h1T, bf16_t* h2, hipStream_t s) {
  GemmBf16Args g{};
  g.A = Xb; g.lda = w.Dp; g.a_rows = S; g.B = w.W1t; g.ldb = w.Dp; g.b_rows = H;
  g.M = S; g.N = H; g.K = w.Dp; g.C = h1; g.ldc = H; g.CT = h1T; g.ct_cols = Sp; g.bias = b1;
  launch_gemm_bf16<BEPI_TANH>(g, s);
  GemmBf16Args g2{};
  g2.A = h1; g2.lda = H; g2.a_rows = S; g2.B = w.W2t; g2.ldb = H; g2.b_rows = H;
  g2.M = S; g2.N = H; g2.K = H; g2.C = h2; g2.ldc = H; g2.bias = b2;
  launch_gemm_bf16<BEPI_TANH>(g2, s);
}

}  // namespace marl
