// LDS-tiled fp32 MFMA GEMM for gfx950 (v_mfma_f32_32x32x2_f32), shared by the rollout forward
// pass and the PPO backward pass.  Three operand arrangements:
//   NN  C[m][n] = sum_k A[m][k] * B[k][n]     activations x weights
//   NT  C[m][n] = sum_k A[m][k] * B[n][k]     gradient x weights^T
//   TN  C[m][n] = sum_k A[k][m] * B[k][n]     activations^T x gradient (split over k across workgroups)
// "A" is always given by rows (optionally gathered through an index list), so a minibatch is read
// in place from the trajectory.  Tiles are staged in LDS in their source orientation; the operand
// fetch indexes them so that the 32 lanes of a half-wavefront hit 32 different banks.
#pragma once
#include "common.h"

namespace marl {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Rows of a matrix: row r = base + (src(r/per) * per + r%per) * ld, src = gather ? gather[.] : identity.
struct RowSrc {
  const float* base;
  int64_t ld;
  const int32_t* gather;
  int per;
  int64_t nrows;
  __device__ __forceinline__ const float* ptr(int64_t r) const {
    if (r >= nrows) return nullptr;
    if (gather == nullptr) return base + r * ld;
    const int64_t g = r / per;
    const int a = (int)(r - g * per);
    return base + ((int64_t)gather[g] * per + a) * ld;
  }
};

enum GemmMode { GEMM_NN = 0, GEMM_NT = 1, GEMM_TN = 2 };
enum GemmEpi {
  EPI_BIAS_TANH = 0,  // C = tanh(acc + aux_vec[n])
  EPI_DTANH = 1,      // C = acc * (1 - aux_mat[m][n]^2);  column sums of C are added to colsum[n]
  EPI_ATOMIC_ADD = 2  // C += acc (fp32 atomics; split-k partial results)
};

struct GemmArgs {
  RowSrc A;          // NN/NT: M rows of K;  TN: K rows of M
  const float* B;    // NN/TN: [K][ldb];  NT: [N][ldb]
  int64_t ldb;
  float* C;          // [M][ldc]
  int64_t ldc;
  const float* aux_vec;  // EPI_BIAS_TANH: bias [N]
  const float* aux_mat;  // EPI_DTANH: previous activation [M][ldaux]
  int64_t ldaux;
  float* colsum;         // EPI_DTANH: [N] (atomic), nullable
  int64_t M, N, K;
  int64_t k_per_split;   // TN: k range of one blockIdx.z
  int round_bf16;        // round stored results to bf16 precision (kept in fp32 storage)
};

__device__ __forceinline__ float round_to_bf16(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7f800000u) == 0x7f800000u) return x;
  u += 0x7fffu + ((u >> 16) & 1u);
  return __uint_as_float(u & 0xffff0000u);
}

// tanh with relative error ~1e-7: odd polynomial near zero, 1 - 2/(e^{2|x|}+1) elsewhere.
__device__ __forceinline__ float tanh_f32(float x) {
  const float ax = fabsf(x);
  const float x2 = x * x;
  const float poly = x * (1.0f + x2 * (-0.33333333333f + x2 * (0.13333333333f + x2 * (-0.05396825397f + x2 * 0.02186948854f))));
  const float e = __expf(2.0f * ax);
  const float big = copysignf(1.0f - __fdividef(2.0f, e + 1.0f), x);
  return ax < 0.25f ? poly : big;
}

constexpr int kGemmBK = 16;

template <int MODE, int EPI, int BM, int BN, int WGM, int WGN>
__global__ void __launch_bounds__(64 * WGM * WGN) gemm_f32_kernel(GemmArgs g) {
  constexpr int NT = 64 * WGM * WGN;
  constexpr int BK = kGemmBK;
  constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile");
  // LDS tiles in source orientation
  constexpr bool A_ROWS_ARE_M = (MODE != GEMM_TN);  // A strip: [BM][BK] (rows m) or [BK][BM] (rows k)
  constexpr bool B_ROWS_ARE_K = (MODE != GEMM_NT);  // B strip: [BK][BN] (rows k) or [BN][BK] (rows n)
  constexpr int A_ROWS = A_ROWS_ARE_M ? BM : BK, A_COLS = A_ROWS_ARE_M ? BK : BM;
  constexpr int B_ROWS = B_ROWS_ARE_K ? BK : BN, B_COLS = B_ROWS_ARE_K ? BN : BK;
  constexpr int A_LD = A_ROWS_ARE_M ? BK + 1 : BM;
  constexpr int B_LD = B_ROWS_ARE_K ? BN : BK + 1;
  constexpr int A_PER = A_ROWS * A_COLS / NT, B_PER = B_ROWS * B_COLS / NT;
  static_assert(A_ROWS * A_COLS % NT == 0 && B_ROWS * B_COLS % NT == 0, "strip size");
  static_assert(NT % A_COLS == 0 || A_COLS % NT == 0, "A strip mapping");
  __shared__ float As[A_ROWS * A_LD];
  __shared__ float Bs[B_ROWS * B_LD];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int lo = lane & 31, hi = lane >> 5;
  const int64_t m0 = (int64_t)blockIdx.x * BM, n0 = (int64_t)blockIdx.y * BN;
  int64_t k_begin = 0, k_end = g.K;
  if (MODE == GEMM_TN) {
    k_begin = (int64_t)blockIdx.z * g.k_per_split;
    k_end = min(g.K, k_begin + g.k_per_split);
  }

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  float ra[A_PER], rb[B_PER];
  // When A's strip rows are m, the row pointers do not change along k: look them up once.
  const float* arow[A_PER];
  if (A_ROWS_ARE_M) {
#pragma unroll
    for (int j = 0; j < A_PER; ++j) arow[j] = g.A.ptr(m0 + (tid + j * NT) / A_COLS);
  }

  auto fetch = [&](int64_t k0) {
#pragma unroll
    for (int j = 0; j < A_PER; ++j) {
      const int e = tid + j * NT, r = e / A_COLS, c = e % A_COLS;
      float v = 0.f;
      if (A_ROWS_ARE_M) {
        const int64_t k = k0 + c;
        if (arow[j] != nullptr && k < k_end) v = arow[j][k];
      } else {
        const int64_t k = k0 + r, m = m0 + c;
        if (k < k_end && m < g.M) {
          const float* p = g.A.ptr(k);
          v = p[m];
        }
      }
      ra[j] = v;
    }
#pragma unroll
    for (int j = 0; j < B_PER; ++j) {
      const int e = tid + j * NT, r = e / B_COLS, c = e % B_COLS;
      float v = 0.f;
      if (B_ROWS_ARE_K) {
        const int64_t k = k0 + r, n = n0 + c;
        if (k < k_end && n < g.N) v = g.B[k * g.ldb + n];
      } else {
        const int64_t n = n0 + r, k = k0 + c;
        if (k < k_end && n < g.N) v = g.B[n * g.ldb + k];
      }
      rb[j] = v;
    }
  };

  if (k_begin < k_end) fetch(k_begin);
  for (int64_t k0 = k_begin; k0 < k_end; k0 += BK) {
#pragma unroll
    for (int j = 0; j < A_PER; ++j) {
      const int e = tid + j * NT;
      As[(e / A_COLS) * A_LD + (e % A_COLS)] = ra[j];
    }
#pragma unroll
    for (int j = 0; j < B_PER; ++j) {
      const int e = tid + j * NT;
      Bs[(e / B_COLS) * B_LD + (e % B_COLS)] = rb[j];
    }
    __syncthreads();
    if (k0 + BK < k_end) fetch(k0 + BK);
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      const int k = kk + hi;
      float a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int m = wm * (BM / WGM) + i * 32 + lo;
        a[i] = A_ROWS_ARE_M ? As[m * A_LD + k] : As[k * A_LD + m];
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = wn * (BN / WGN) + j * 32 + lo;
        b[j] = B_ROWS_ARE_K ? Bs[k * B_LD + n] : Bs[n * B_LD + k];
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // Epilogue.  Accumulator register r of a lane holds C[8*(r/4) + 4*hi + r%4][lo] of its 32x32 tile.
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int64_t n = n0 + wn * (BN / WGN) + j * 32 + lo;
    const bool n_ok = n < g.N;
    float csum = 0.f;
    float bias = 0.f;
    if (EPI == EPI_BIAS_TANH && n_ok) bias = g.aux_vec[n];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t m = m0 + wm * (BM / WGM) + i * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        if (m < g.M && n_ok) {
          float v = acc[i][j][r];
          if (EPI == EPI_BIAS_TANH) {
            v = tanh_f32(v + bias);
            if (g.round_bf16) v = round_to_bf16(v);
            g.C[m * g.ldc + n] = v;
          } else if (EPI == EPI_DTANH) {
            const float h = g.aux_mat[m * g.ldaux + n];
            v = v * (1.0f - h * h);
            if (g.round_bf16) v = round_to_bf16(v);
            g.C[m * g.ldc + n] = v;
            csum += v;
          } else {
            atomicAdd(&g.C[m * g.ldc + n], v);
          }
        }
      }
    }
    if (EPI == EPI_DTANH && g.colsum != nullptr) {
      csum += __shfl_xor(csum, 32);
      if (hi == 0 && n_ok) atomicAdd(&g.colsum[n], csum);
    }
  }
}

// Host-side dispatch over the tile shapes used by the library.
template <int MODE, int EPI>
inline void launch_gemm(const GemmArgs& g, hipStream_t s) {
  const int64_t M = g.M, N = g.N;
  TimedLaunch timed(MODE == GEMM_NN ? KC_GEMM_NN : (MODE == GEMM_NT ? KC_GEMM_NT : KC_GEMM_TN),
                    2.0 * (double)g.M * (double)g.N * (double)g.K, s);
  unsigned gz = 1;
  if (MODE == GEMM_TN) gz = (unsigned)((g.K + g.k_per_split - 1) / g.k_per_split);
  if (MODE == GEMM_TN && M <= 32) {
    // very thin output (first-layer gradient of the small networks)
    dim3 grid(1, (unsigned)((N + 63) / 64), gz);
    hipLaunchKernelGGL((gemm_f32_kernel<MODE, EPI, 32, 64, 1, 2>), grid, dim3(128), 0, s, g);
  } else if (N % 128 == 0) {
    dim3 grid((unsigned)((M + 127) / 128), (unsigned)(N / 128), gz);
    hipLaunchKernelGGL((gemm_f32_kernel<MODE, EPI, 128, 128, 2, 2>), grid, dim3(256), 0, s, g);
  } else {
    dim3 grid((unsigned)((M + 127) / 128), (unsigned)((N + 63) / 64), gz);
    hipLaunchKernelGGL((gemm_f32_kernel<MODE, EPI, 128, 64, 2, 2>), grid, dim3(256), 0, s, g);
  }
}

}  // namespace marl
