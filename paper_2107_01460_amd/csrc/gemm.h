// LDS-tiled fp32 MFMA GEMM for gfx950 (v_mfma_f32_32x32x2_f32), shared by the rollout forward
// pass and the PPO backward pass.  Three operand arrangements:
//   NN  C[m][n] = sum_k A[m][k] * B[k][n]     activations x weights
//   NT  C[m][n] = sum_k A[m][k] * B[n][k]     gradient x weights^T
//   TN  C[m][n] = sum_k A[k][m] * B[k][n]     activations^T x gradient (split over k across workgroups)
// "A" is always given by rows (optionally gathered through an index list), so a minibatch is read
// in place from the trajectory.  Tiles are staged in LDS in their source orientation; the operand
// fetch indexes them so that the 32 lanes of a half-wavefront hit 32 different banks.
#pragma once
#include <algorithm>

#include "common.h"

namespace marl {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Division of a sample index by a small run-time divisor (agents per row) without the 64-bit division sequence,
// which is about 180 vector instructions and sat on the critical path of every row tile: for s < 2^31 and
// d <= 64, s / d = (s * magic) >> shift exactly, with magic = floor(2^shift / d) + 1 and
// shift = 31 + ceil(log2 d) (the error term s * (magic * d - 2^shift) stays below 2^shift; d = 1 gives
// magic 2^31 + 1, shift 31).  div<true> is that product and nothing else -- the caller has checked on the host that
// the divisor has a magic number and that every index is below 2^31 (small_div_ok); div<false> is the plain division.
// (One function that chooses at run time keeps the long sequence in the instruction stream and was slower.)
struct SmallDiv {
  uint32_t magic = 0;
  int shift = 0;
  template <bool FAST>
  __device__ __forceinline__ int64_t div(int64_t s, int d) const {
    if (FAST) return (int64_t)(((uint64_t)(uint32_t)s * magic) >> shift);
    return s / d;
  }
};
inline SmallDiv make_small_div(int d) {
  SmallDiv v;
  if (d < 1 || d > 64) return v;
  int lg = 0;
  while ((1 << lg) < d) ++lg;
  v.shift = 31 + lg;
  v.magic = (uint32_t)(((uint64_t)1 << v.shift) / (uint64_t)d + 1);
  return v;
}

// Rows of a matrix: row r = base + (src(r/per) * per + r%per) * ld, src = gather ? gather[.] : identity.
struct RowSrc {
  const float* base;
  int64_t ld;
  const int32_t* gather;
  int per;
  int64_t nrows;
  SmallDiv pd{};  // make_small_div(per), or default
  __device__ __forceinline__ const float* ptr(int64_t r) const {
    if (r >= nrows) return nullptr;
    if (gather == nullptr) return base + r * ld;
    const int64_t g = per == 1 ? r : r / per;  // (a 64-bit division is about 180 instructions; one row per entry needs none)
    const int a = (int)(r - g * per);
    return base + ((int64_t)gather[g] * per + a) * ld;
  }
  // The same address in two steps, so that the gather entry can be fetched long before the row is.
  template <bool FAST = false>
  __device__ __forceinline__ int32_t gather_entry(int64_t r) const {
    return gather == nullptr ? 0 : gather[pd.div<FAST>(r, per)];
  }
  template <bool FAST = false>
  __device__ __forceinline__ const float* ptr_with(int64_t r, int32_t entry) const {
    if (gather == nullptr) return base + r * ld;
    const int a = (int)(r - pd.div<FAST>(r, per) * per);
    return base + ((int64_t)entry * per + a) * ld;
  }
};
// div<true> may be used for indices below `count` with this divisor
inline bool small_div_ok(const SmallDiv& v, int64_t count) { return v.magic != 0 && count < ((int64_t)1 << 31); }

enum GemmMode { GEMM_NN = 0, GEMM_NT = 1, GEMM_TN = 2 };
enum GemmEpi {
  EPI_BIAS_TANH = 0,  // C = tanh(acc + aux_vec[n])
  EPI_DTANH = 1,      // C = acc * (1 - aux_mat[m][n]^2);  column sums of C are added to colsum[n]
  EPI_ATOMIC_ADD = 2, // C += acc (fp32 atomics; split-k partial results)
  EPI_STORE = 3       // C = acc + aux_vec[n] (aux_vec nullable)
};

struct GemmArgs {
  RowSrc A;          // NN/NT: M rows of K;  TN: K rows of M
  const float* B;    // NN/TN: [K][ldb];  NT: [N][ldb]
  int64_t ldb;
  float* C;          // [M][ldc]
  int64_t ldc;
  const float* aux_vec;  // EPI_BIAS_TANH: bias [N]; EPI_STORE: nullable bias [N]
  const float* aux_mat;  // EPI_DTANH: previous activation [M][ldaux]
  int64_t ldaux;
  float* colsum;         // TN: column sums of B are added here ([N], atomic), nullable; EPI_DTANH: column sums of C
  int64_t M, N, K;
  int64_t k_per_split;   // TN: k range of one blockIdx.z
  int round_bf16;        // round stored results to bf16 precision (kept in fp32 storage)
  // TN with EPI_ATOMIC_ADD, nullable: k split z stores its products at split_out + z * split_count + m * ldc + n and its
  // column sums of B behind them (at + M * ldc + n) with plain stores instead of adding to C / colsum with atomics; the
  // caller then adds the splits in a fixed order (reduce_partials_kernel), which makes the result the same in every run.
  // Only the large-tile kernel honours it: launch_gemm says whether it did.
  float* split_out;
  int64_t split_count;
};

// The kernels that finish with one partial result per workgroup (the fused training kernel, the accumulator-resident
// transposed product) store those with plain stores and add them up here: a few hundred workgroups adding to the same
// cache lines with atomics at the same moment queue up at the L2 (60-180 us per launch).  The split-k tile kernel below
// does the same with one slab per k split when the caller passes split_out; without it, it adds with atomics.

// out[i] += sum_b partial[b * count + i], the copies added in a fixed order, so that the result does not depend on the
// run.  A workgroup takes 32 consecutive elements; its 8 thread groups sum the copies b = g, g + 8, g + 16, ... of an
// element (four interleaved running sums each, so that four loads are in flight), and one thread per element adds the
// eight group sums through LDS, again in a fixed order.
static __global__ void __launch_bounds__(256) reduce_partials_kernel(const float* __restrict__ partial, int nblocks, int64_t count,
                                                                     float* __restrict__ out) {
  __shared__ float part[8][32];
  const int e = threadIdx.x & 31, g = threadIdx.x >> 5;
  const int64_t i = (int64_t)blockIdx.x * 32 + e;
  float s[4] = {0.f, 0.f, 0.f, 0.f};
  if (i < count) {
    int b = g;
    for (; b + 24 < nblocks; b += 32) {
#pragma unroll
      for (int u = 0; u < 4; ++u) s[u] += partial[(int64_t)(b + 8 * u) * count + i];
    }
    for (; b < nblocks; b += 8) s[0] += partial[(int64_t)b * count + i];
  }
  part[g][e] = (s[0] + s[1]) + (s[2] + s[3]);
  __syncthreads();
  if (g == 0 && i < count) {
    float v = part[0][e];
#pragma unroll
    for (int q = 1; q < 8; ++q) v += part[q][e];
    out[i] += v;
  }
}
inline void launch_reduce_partials(const float* partial, int nblocks, int64_t count, float* out, hipStream_t s) {
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((count + 31) / 32)), dim3(256), 0, s, partial, nblocks, count, out);
}

// tanh(x) = 1 - 2 / (e^{2x} + 1) with the hardware exp2 and reciprocal: absolute error ~1e-7 (the values feed
// sums of O(1) activations, so an absolute bound is what the 1e-4 tolerance on the outputs needs); saturates
// cleanly to +-1 when e^{2x} overflows or underflows.
__device__ __forceinline__ float tanh_f32(float x) {
  const float e = __builtin_amdgcn_exp2f(x * 2.885390081777927f);  // e^{2x}
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(e + 1.0f);
}

// acc += A B for this wavefront's 32x32 tile: A rows in LDS (As points at this lane's row, + 4 * hi), B in global
// memory in operand order (element (k, n) of the [K][LDB] matrix at ((k / 4) * LDB + n) * 4 + k % 4; Bg points at
// this lane's 16 bytes of k quad `hi`), `kgroups` groups of 16 along k.  B goes straight from the cache hierarchy
// into registers with 16-byte loads that are contiguous across the wavefront, one group ahead of its use, so a
// layer needs no staging buffer and no barrier of its own.  Both operands must be readable (zero-padded) up to
// 16 * kgroups along k.
// B of the first two groups may come in already loaded (b00 b01: group 0, b10 b11: group 1; see gemm_phase_prefetch):
// a phase that follows a barrier or an element-wise epilogue then starts on operands requested before it, instead of
// waiting an L2 round trip for them.
struct PhaseB {
  float4 b00, b01, b10, b11;
};
template <int LDB>
__device__ __forceinline__ PhaseB gemm_phase_prefetch(const float* __restrict__ Bg, int kgroups) {
  const int g1 = kgroups > 1 ? 1 : 0;
  PhaseB p;
  p.b00 = *reinterpret_cast<const float4*>(Bg);
  p.b01 = *reinterpret_cast<const float4*>(Bg + (int64_t)8 * LDB);
  p.b10 = *reinterpret_cast<const float4*>(Bg + ((int64_t)16 * g1) * LDB);
  p.b11 = *reinterpret_cast<const float4*>(Bg + ((int64_t)16 * g1 + 8) * LDB);
  return p;
}

template <int LDB, bool PRE = false>
__device__ __forceinline__ void gemm_phase_regs(const float* __restrict__ As, const float* __restrict__ Bg, int kgroups,
                                                floatx16& acc, PhaseB pre = PhaseB()) {
  constexpr int kDepth = 3;  // groups in flight: the one in use and two on their way
  float4 av[kDepth][2], bv[kDepth][2];
  auto load = [&](int g, float4 (&a2)[2], float4 (&b2)[2]) {
    const int gc = g < kgroups ? g : kgroups - 1;  // past the end: re-read the last group
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      a2[u] = *reinterpret_cast<const float4*>(As + 16 * gc + 8 * u);
      b2[u] = *reinterpret_cast<const float4*>(Bg + ((int64_t)16 * gc + 8 * u) * LDB);
    }
  };
#pragma unroll
  for (int d = 0; d < kDepth - 1; ++d) load(d, av[d], bv[d]);
  if (PRE) {
    bv[0][0] = pre.b00; bv[0][1] = pre.b01; bv[1][0] = pre.b10; bv[1][1] = pre.b11;
  }
#pragma unroll 1
  for (int g0 = 0; g0 < kgroups; g0 += kDepth) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      const int g = g0 + d;
      if (g < kgroups) {  // uniform
        load(g + kDepth - 1, av[(d + kDepth - 1) % kDepth], bv[(d + kDepth - 1) % kDepth]);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const float af[4] = {av[d][u].x, av[d][u].y, av[d][u].z, av[d][u].w};
          const float bf[4] = {bv[d][u].x, bv[d][u].y, bv[d][u].z, bv[d][u].w};
#pragma unroll
          for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[j], acc, 0, 0, 0);
        }
      }
    }
  }
}

// All B fragments of one product against weights, for this lane: KG groups of 16 along k, two 16-byte loads each
// (operand-order copy: element (k, n) at ((k / 4) * LDB + n) * 4 + k % 4; lane_off is this lane's offset
// (hi * LDB + n) * 4 in floats).  The loads are buffer loads -- a resource descriptor in scalar registers, ONE vector
// register with the lane's byte offset for all of them, the group's offset as a scalar: as global loads each of them
// got a 64-bit address register pair of its own, computed outside the tile loop and kept (or spilled) across it.  The whole set is requested one phase AHEAD of the product that uses it -- during the element-wise epilogue
// or the LDS-only product in front of it -- so that the product never waits for the L2: with two or three groups in
// flight (gemm_phase_regs) every workgroup of the chip asks the same few cache lines at the same moment and the
// answers take longer than the 16 matrix instructions that were meant to cover them.
template <int KG>
struct PhaseW {
  float4 w[KG][2];
};
typedef __amdgpu_buffer_rsrc_t WeightRsrc;
// descriptor of `floats` floats at p (raw buffer, no swizzle; reads past the end return zero)
__device__ __forceinline__ WeightRsrc weight_rsrc(const float* p, int floats) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p), (short)0, floats * 4, 0x00020000);
}
template <int LDB, int KG, int G0 = 0, int G1 = KG>  // groups G0 .. G1 - 1
__device__ __forceinline__ void phase_w_request(PhaseW<KG>& pw, WeightRsrc B, int lane_off, int kgroups) {
#pragma unroll
  for (int g = G0; g < G1; ++g) {
    const int gc = g < kgroups ? g : kgroups - 1;  // past the end: the last group again (never used)
#pragma unroll
    for (int u = 0; u < 2; ++u)
      pw.w[g][u] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(B, lane_off * 4, (16 * gc + 8 * u) * LDB * 4, 0));
  }
}
// acc += A B for this wavefront's 32x32 tile: A rows in LDS (As points at this lane's row, + 4 * hi; the fragments of
// the next group are read before the matrix instructions of the current one), B from pw.
template <int KG>
__device__ __forceinline__ void gemm_phase_w(const float* __restrict__ As, int kgroups, floatx16& acc, const PhaseW<KG>& pw) {
  float4 av[2][2];
  av[0][0] = *reinterpret_cast<const float4*>(As);
  av[0][1] = *reinterpret_cast<const float4*>(As + 8);
#pragma unroll
  for (int g = 0; g < KG; ++g) {
    if (g < kgroups) {  // uniform
      const int gn = g + 1 < kgroups ? g + 1 : g;
      av[(g + 1) & 1][0] = *reinterpret_cast<const float4*>(As + 16 * gn);
      av[(g + 1) & 1][1] = *reinterpret_cast<const float4*>(As + 16 * gn + 8);
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const float af[4] = {av[g & 1][u].x, av[g & 1][u].y, av[g & 1][u].z, av[g & 1][u].w};
        const float bf[4] = {pw.w[g][u].x, pw.w[g][u].y, pw.w[g][u].z, pw.w[g][u].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[j], acc, 0, 0, 0);
      }
    }
  }
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

  // TN: column sums of B (the bias gradient).  B_COLS divides NT here, so a thread always stages the same column.
  float bsum = 0.f;
  const bool want_bsum = MODE == GEMM_TN && g.colsum != nullptr && blockIdx.x == 0;

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
      if (MODE == GEMM_TN && want_bsum) bsum += rb[j];
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

  if (MODE == GEMM_TN && want_bsum) {
    static_assert(MODE != GEMM_TN || NT % B_COLS == 0, "a thread must stage one column");
    const int64_t n = n0 + tid % B_COLS;
    if (n < g.N) atomicAdd(&g.colsum[n], bsum);
  }

  // Epilogue.  Accumulator register r of a lane holds C[8*(r/4) + 4*hi + r%4][lo] of its 32x32 tile.
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int64_t n = n0 + wn * (BN / WGN) + j * 32 + lo;
    const bool n_ok = n < g.N;
    float csum = 0.f;
    float bias = 0.f;
    if (EPI == EPI_BIAS_TANH && n_ok) bias = g.aux_vec[n];
    if (EPI == EPI_STORE && n_ok && g.aux_vec != nullptr) bias = g.aux_vec[n];
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
          } else if (EPI == EPI_STORE) {
            g.C[m * g.ldc + n] = v + bias;
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

// ---------------------------------------------------------------------------------------------
// Second-generation kernel for the large shapes: 128 x BN tile (BN = 64 or 128), k-tile 32, four
// wavefronts as 2 x 2, 16-byte global loads and LDS stores where the source rows are 16-byte
// aligned (AVEC), operands fetched from LDS with one 16-byte read per four k-steps on k-contiguous
// tiles.  Within a group of eight k values the lower half-wavefront supplies k = 0..3 and the
// upper half k = 4..7 of both operands, so that each lane's four values are one aligned LDS read.
// One LDS buffer; the next k-tile travels global -> registers while the current one is multiplied.
// ---------------------------------------------------------------------------------------------
constexpr int kG2BK = 32;
constexpr int kG2PitchK = kG2BK + 4;  // k-contiguous tiles: pitch 36 floats keeps 16-byte alignment and spreads banks

template <int MODE, int EPI, int BN, bool AVEC>
__global__ void __launch_bounds__(256, 2) gemm2_f32_kernel(GemmArgs g) {
  constexpr int BM = 128, BK = kG2BK, PK = kG2PitchK;
  constexpr int TM = 2, TN = BN / 64;
  constexpr bool A_KCONT = (MODE != GEMM_TN);  // A tile stored [m][k] (pitch PK) else [k][m] (pitch BM)
  constexpr bool B_KCONT = (MODE == GEMM_NT);  // B tile stored [n][k] (pitch PK) else [k][n] (pitch BN)
  constexpr int A_FLOATS = A_KCONT ? BM * PK : BK * BM;
  constexpr int B_FLOATS = B_KCONT ? BN * PK : BK * BN;
  __shared__ __attribute__((aligned(16))) float As[A_FLOATS];
  __shared__ __attribute__((aligned(16))) float Bs[B_FLOATS];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int lo = lane & 31, hi = lane >> 5;
  // TN: the tiles of one k slab are made neighbours on one XCD (workgroups are dealt round-robin to the eight XCDs in
  // the order x, y, z), so that a slab of A / B is fetched from HBM once and found in that XCD's L2 by the other tiles
  // that contract over it; with the plain (x, y, z) order every tile of a slab ran on another XCD and the operands
  // were read twice (1074 MB per launch at 256 x 256 outputs where 537 are algorithmic).
  unsigned bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
  if (MODE == GEMM_TN) {
    const unsigned lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const unsigned lg = xcd_remap(lin, gridDim.x * gridDim.y * gridDim.z);
    bx = lg % gridDim.x;
    by = (lg / gridDim.x) % gridDim.y;
    bz = lg / (gridDim.x * gridDim.y);
  }
  const int64_t n0 = (int64_t)by * BN;
  // NN / NT: the workgroup is persistent over row tiles (tile, tile + gridDim.x, ...) and the first k-tile of
  // the next row tile is already in flight while the current one finishes, so that neither the first load
  // latency nor the epilogue of a row tile leaves the memory pipe idle.  TN: one output tile, k split over z.
  const int64_t num_mt = (g.M + BM - 1) / BM;
  int64_t k_begin = 0, k_end = g.K;
  if (MODE == GEMM_TN) {
    k_begin = (int64_t)bz * g.k_per_split;
    k_end = min(g.K, k_begin + g.k_per_split);
  }

  floatx16 acc[TM][TN];

  // ---- global -> register staging
  // A, k-contiguous (NN/NT): vector: thread -> (row = tid/8 + 32p, 4 floats at k = 4*(tid%8)), p < 4
  //                          scalar: thread -> (row = tid/32 + 8p, k = tid%32), p < 16
  // A, m-contiguous (TN):    vector: thread -> (k = tid/32 + 8p, 4 floats at m = 4*(tid%32)), p < 4
  //                          scalar: thread -> (k = tid/128 + 2p, m = tid%128), p < 16
  constexpr int A_REGS = 16;
  float ra[A_REGS];
  const float* arow[AVEC ? 4 : 16];
  int64_t m0_fetch = (int64_t)bx * BM;  // row tile the staging registers belong to
  auto set_rows = [&](int64_t m0) {
    m0_fetch = m0;
    if (A_KCONT) {
#pragma unroll
      for (int p = 0; p < (AVEC ? 4 : 16); ++p) {
        int64_t row = m0 + (AVEC ? (tid >> 3) + 32 * p : (tid >> 5) + 8 * p);
        row = min(row, g.M - 1);  // rows past the end re-read the last row; their results are never stored
        arow[p] = g.A.ptr(row);
      }
    }
  };
  // B, n-contiguous (NN/TN): thread -> (k = tid/(BN/4) + (1024/BN) p, 4 floats at n = 4*(tid % (BN/4)))
  // B, k-contiguous (NT):    thread -> (n = tid/8 + 32p, 4 floats at k = 4*(tid%8)), p < BN/32
  constexpr int B_VECS = BK * BN / 4 / 256;
  float4 rb[B_VECS];

  auto fetch = [&](int64_t k0) {
    if (A_KCONT) {
      if (AVEC) {
        const int64_t k = k0 + 4 * (tid & 7);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
          if (k < k_end) v = *reinterpret_cast<const float4*>(arow[p] + k);
          ra[4 * p + 0] = v.x; ra[4 * p + 1] = v.y; ra[4 * p + 2] = v.z; ra[4 * p + 3] = v.w;
        }
      } else {
        const int64_t k = k0 + (tid & 31);
#pragma unroll
        for (int p = 0; p < 16; ++p) ra[p] = k < k_end ? arow[p][k] : 0.f;
      }
    } else {
      if (AVEC) {
        const int64_t m = m0_fetch + 4 * (tid & 31);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const int64_t k = k0 + (tid >> 5) + 8 * p;
          float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
          if (k < k_end && m < g.M) v = *reinterpret_cast<const float4*>(g.A.ptr(k) + m);
          ra[4 * p + 0] = v.x; ra[4 * p + 1] = v.y; ra[4 * p + 2] = v.z; ra[4 * p + 3] = v.w;
        }
      } else {
        const int64_t m = m0_fetch + (tid & 127);
#pragma unroll
        for (int p = 0; p < 16; ++p) {
          const int64_t k = k0 + (tid >> 7) + 2 * p;
          ra[p] = (k < k_end && m < g.M) ? g.A.ptr(k)[m] : 0.f;
        }
      }
    }
    if (B_KCONT) {
      const int64_t k = k0 + 4 * (tid & 7);
#pragma unroll
      for (int p = 0; p < B_VECS; ++p) {
        const int64_t n = n0 + (tid >> 3) + 32 * p;
        rb[p] = k < k_end ? *reinterpret_cast<const float4*>(g.B + n * g.ldb + k) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    } else {
      const int64_t n = n0 + 4 * (tid % (BN / 4));
#pragma unroll
      for (int p = 0; p < B_VECS; ++p) {
        const int64_t k = k0 + tid / (BN / 4) + (1024 / BN) * p;
        rb[p] = k < k_end ? *reinterpret_cast<const float4*>(g.B + k * g.ldb + n) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  };

  auto stage = [&]() {
    if (A_KCONT) {
      if (AVEC) {
#pragma unroll
        for (int p = 0; p < 4; ++p)
          *reinterpret_cast<float4*>(&As[((tid >> 3) + 32 * p) * PK + 4 * (tid & 7)]) =
              make_float4(ra[4 * p], ra[4 * p + 1], ra[4 * p + 2], ra[4 * p + 3]);
      } else {
#pragma unroll
        for (int p = 0; p < 16; ++p) As[((tid >> 5) + 8 * p) * PK + (tid & 31)] = ra[p];
      }
    } else {
      if (AVEC) {
#pragma unroll
        for (int p = 0; p < 4; ++p)
          *reinterpret_cast<float4*>(&As[((tid >> 5) + 8 * p) * BM + 4 * (tid & 31)]) =
              make_float4(ra[4 * p], ra[4 * p + 1], ra[4 * p + 2], ra[4 * p + 3]);
      } else {
#pragma unroll
        for (int p = 0; p < 16; ++p) As[((tid >> 7) + 2 * p) * BM + (tid & 127)] = ra[p];
      }
    }
    if (B_KCONT) {
#pragma unroll
      for (int p = 0; p < B_VECS; ++p) *reinterpret_cast<float4*>(&Bs[((tid >> 3) + 32 * p) * PK + 4 * (tid & 7)]) = rb[p];
    } else {
#pragma unroll
      for (int p = 0; p < B_VECS; ++p)
        *reinterpret_cast<float4*>(&Bs[(tid / (BN / 4) + (1024 / BN) * p) * BN + 4 * (tid % (BN / 4))]) = rb[p];
    }
  };

  // TN: column sums of B (the bias gradient) ride along: each thread adds up the values it stages
  float4 bsum = make_float4(0.f, 0.f, 0.f, 0.f);
  const bool want_bsum = MODE == GEMM_TN && g.colsum != nullptr && bx == 0;

  int64_t tile = bx;
  if (tile < num_mt && k_begin < k_end) {
    set_rows(tile * BM);
    fetch(k_begin);
  }
  for (; tile < num_mt; tile += (MODE == GEMM_TN ? num_mt : (int64_t)gridDim.x)) {
    const int64_t m0 = tile * BM;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    for (int64_t k0 = k_begin; k0 < k_end; k0 += BK) {
      stage();
      if (MODE == GEMM_TN && want_bsum) {
#pragma unroll
        for (int p = 0; p < B_VECS; ++p) {
          bsum.x += rb[p].x; bsum.y += rb[p].y; bsum.z += rb[p].z; bsum.w += rb[p].w;
        }
      }
      __syncthreads();
      if (k0 + BK < k_end) {
        fetch(k0 + BK);
      } else if (MODE != GEMM_TN && tile + (int64_t)gridDim.x < num_mt) {
        set_rows((tile + (int64_t)gridDim.x) * BM);
        fetch(k_begin);
      }
#pragma unroll
      for (int kb = 0; kb < BK; kb += 8) {
        // lane (lo, hi) supplies k = kb + 4*hi + j in MFMA step j
        float a[TM][4], b[TN][4];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const int m = wm * 64 + i * 32 + lo;
          if (A_KCONT) {
            const float4 v = *reinterpret_cast<const float4*>(&As[m * PK + kb + 4 * hi]);
            a[i][0] = v.x; a[i][1] = v.y; a[i][2] = v.z; a[i][3] = v.w;
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) a[i][j] = As[(kb + 4 * hi + j) * BM + m];
          }
        }
#pragma unroll
        for (int jn = 0; jn < TN; ++jn) {
          const int n = wn * (BN / 2) + jn * 32 + lo;
          if (B_KCONT) {
            const float4 v = *reinterpret_cast<const float4*>(&Bs[n * PK + kb + 4 * hi]);
            b[jn][0] = v.x; b[jn][1] = v.y; b[jn][2] = v.z; b[jn][3] = v.w;
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) b[jn][j] = Bs[(kb + 4 * hi + j) * BN + n];
          }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int jn = 0; jn < TN; ++jn)
              acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][j], b[jn][j], acc[i][jn], 0, 0, 0);
      }
      __syncthreads();
    }

    if (MODE == GEMM_TN && want_bsum) {
      // threads with equal tid % (BN/4) hold partial sums of the same four columns: combine them through LDS
      float4* red = reinterpret_cast<float4*>(Bs);  // the tile is no longer needed (the loop ended with a barrier)
      red[tid] = bsum;
      __syncthreads();
      constexpr int GROUPS = 256 / (BN / 4);
      if (tid < BN / 4) {
        float4 t = red[tid];
#pragma unroll
        for (int q = 1; q < GROUPS; ++q) {
          const float4 o = red[tid + q * (BN / 4)];
          t.x += o.x; t.y += o.y; t.z += o.z; t.w += o.w;
        }
        if (g.split_out != nullptr) {  // this k split's column sums, directly behind its copy of C
          *reinterpret_cast<float4*>(g.split_out + (int64_t)bz * g.split_count + g.M * g.ldc + n0 + 4 * tid) = t;
        } else {
          float* dst = g.colsum + n0 + 4 * tid;
          atomicAdd(dst + 0, t.x); atomicAdd(dst + 1, t.y); atomicAdd(dst + 2, t.z); atomicAdd(dst + 3, t.w);
        }
      }
    }

    // Epilogue (accumulator register r of a lane holds C[8*(r/4) + 4*hi + r%4][lo] of its 32x32 tile).
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
      const int64_t n = n0 + wn * (BN / 2) + jn * 32 + lo;
      float csum = 0.f, bias = 0.f;
      if (EPI == EPI_BIAS_TANH) bias = g.aux_vec[n];
      if (EPI == EPI_STORE && g.aux_vec != nullptr) bias = g.aux_vec[n];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t m = m0 + wm * 64 + i * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
          if (m < g.M) {
            float v = acc[i][jn][r];
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
            } else if (EPI == EPI_STORE) {
              g.C[m * g.ldc + n] = v + bias;
            } else if (g.split_out != nullptr) {
              g.split_out[(int64_t)bz * g.split_count + m * g.ldc + n] = v;
            } else {
              atomicAdd(&g.C[m * g.ldc + n], v);
            }
          }
        }
      }
      if (EPI == EPI_DTANH && g.colsum != nullptr) {
        csum += __shfl_xor(csum, 32);
        if (hi == 0) atomicAdd(&g.colsum[n], csum);
      }
    }
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Host-side dispatch over the tile shapes used by the library.
// Returns true when the launch wrote its k splits to g.split_out (false: it added to C / colsum directly).
template <int MODE, int EPI>
inline bool launch_gemm(const GemmArgs& g_in, hipStream_t s) {
  GemmArgs g = g_in;
  const int64_t M = g.M, N = g.N;
  TimedLaunch timed(MODE == GEMM_NN ? KC_GEMM_NN : (MODE == GEMM_NT ? KC_GEMM_NT : KC_GEMM_TN),
                    2.0 * (double)g.M * (double)g.N * (double)g.K, s);
  unsigned gz = 1;
  if (MODE == GEMM_TN) gz = (unsigned)((g.K + g.k_per_split - 1) / g.k_per_split);
  // Large shapes: N a multiple of 64, weights 16-byte aligned with a row pitch that keeps them so.
  const bool b_ok = aligned16(g.B) && g.ldb % 4 == 0 && N % 64 == 0 && (MODE != GEMM_NT || g.K % 4 == 0);
  if (b_ok && !(MODE == GEMM_TN && M <= 32)) {
    const bool avec = aligned16(g.A.base) && g.A.ld % 4 == 0 && (MODE == GEMM_TN ? M % 4 == 0 : g.K % 4 == 0);
    const int bn = N % 128 == 0 ? 128 : 64;
    unsigned gx = (unsigned)((M + 127) / 128);
    // (The kernel can also run persistently over row tiles with a smaller grid; measured slower here: stores
    // share the load counter on this target, so the next tile's staged loads wait for the epilogue's stores.)
    dim3 grid(gx, (unsigned)(N / bn), gz);
    if (!(MODE == GEMM_TN && EPI == EPI_ATOMIC_ADD && g.ldc == N && N % 4 == 0)) g.split_out = nullptr;
    if (bn == 128) {
      if (avec) hipLaunchKernelGGL((gemm2_f32_kernel<MODE, EPI, 128, true>), grid, dim3(256), 0, s, g);
      else hipLaunchKernelGGL((gemm2_f32_kernel<MODE, EPI, 128, false>), grid, dim3(256), 0, s, g);
    } else {
      if (avec) hipLaunchKernelGGL((gemm2_f32_kernel<MODE, EPI, 64, true>), grid, dim3(256), 0, s, g);
      else hipLaunchKernelGGL((gemm2_f32_kernel<MODE, EPI, 64, false>), grid, dim3(256), 0, s, g);
    }
    return g.split_out != nullptr;
  }
  g.split_out = nullptr;
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
  return false;
}

}  // namespace marl
