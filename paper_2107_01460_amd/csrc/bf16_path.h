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
  const float* rows[16];  // thread stages rows tid/64 + 4q, column tid%64; rows past the end: the last row, zeroed below
#pragma unroll
  for (int q = 0; q < 16; ++q) rows[q] = X.ptr(min(s0 + (tid >> 6) + 4 * q, S - 1));
  for (int d0 = 0; d0 < Dp; d0 += 64) {
    const int cc = tid & 63, csrc = min(d0 + cc, Din - 1);
    float v[16];  // all loads of the chunk before the first store (no branch around a load)
#pragma unroll
    for (int q = 0; q < 16; ++q) v[q] = rows[q][csrc];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int r = (tid >> 6) + 4 * q;
      tile[r][cc] = (s0 + r < S && d0 + cc < Din) ? v[q] : 0.f;
    }
    __syncthreads();
    // both copies leave with 16-byte stores: eight columns of a row, eight samples of a column (Dp is a multiple of 64)
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int r = (tid >> 3) + 32 * q, c0 = 8 * (tid & 7);
      uint32_t w[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = pack2_bf16(tile[r][c0 + 2 * j], tile[r][c0 + 2 * j + 1]);
      if (s0 + r < S) *reinterpret_cast<uint4*>(&Xb[(s0 + r) * Dp + d0 + c0]) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    if (XbT != nullptr) {
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int dd = (tid >> 3) + 32 * q, ss = 8 * (tid & 7);
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = pack2_bf16(tile[ss + 2 * j][dd], tile[ss + 2 * j + 1][dd]);
        if (s0 + ss < Sp) *reinterpret_cast<uint4*>(&XbT[((s0 >> 6) * Dp + d0 + dd) * 64 + ss]) = make_uint4(w[0], w[1], w[2], w[3]);
      }
    }
    __syncthreads();
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
