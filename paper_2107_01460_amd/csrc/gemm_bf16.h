// bf16 MFMA GEMM for the bf16 configuration (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// One operand arrangement serves every product of the training step: C[m][n] = sum_k A[m][k] * B[n][k] with
// BOTH operands k-contiguous in memory, because the producers write each activation twice where it is needed
// twice: row-major [sample][feature] (the A operand of the next layer / of dz1 = dz2 W2^T) and transposed
// [feature][sample] (the operands of the weight gradients dW = act^T dz, whose contraction index is the
// sample).  So no kernel ever has to transpose 2-byte elements on its way into the matrix cores:
//   h1  = tanh(Xb  W1t^T + b1)      A = Xb  [S][Dp]   B = W1t [H][Dp]    -> h1 [S][H] and h1T [H][Sp]
//   h2  = tanh(h1  W2t^T + b2)      A = h1  [S][H]    B = W2t [H][H]     -> h2 [S][H]
//   dW2 = h1T dz2T^T                A = h1T [H][Sp]   B = dz2T [H][Sp]   -> fp32 atomics (k split over workgroups)
//   dz1 = (dz2 W2^T) (1 - h1^2)     A = dz2 [S][H]    B = W2  [H][H]     -> dz1T [H][Sp] only
//   dW1 = XbT dz1T^T                A = XbT [Dp][Sp]  B = dz1T [H][Sp]   -> fp32 atomics
// The transposed copies are stored SAMPLE-BLOCKED: element (row r, sample s) of an R-row copy sits at
// ((s / 64) R + r) 64 + s % 64, i.e. the R rows of 64 consecutive samples form one contiguous block of 128 R bytes.
// A 64-sample chunk of any range of rows is then one contiguous piece of memory for the weight-gradient kernels (with
// plain [R][Sp] rows of 512 KB pitch every row of a chunk lay in another page and on the same memory channel), and
// the producers write their 64-sample tiles as one contiguous piece too.
// Tile 128 x 128 x 64 per workgroup of four wavefronts (2 x 2, each 2 x 2 MFMA tiles of 32 x 32); operands are
// staged in LDS with a 144-byte row pitch so that the 16-byte operand reads of eight consecutive rows fall into
// eight different bank groups; results leave through an LDS-staged tile with 16-byte stores in both orientations.
#pragma once
#include <type_traits>
#include "gemm.h"

namespace marl {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // 16 bytes in flight between a load and an LDS store

enum Bf16Epi {
  BEPI_TANH = 0,     // v = tanh(acc + bias[n]) -> C [m][n] (nullable) and CT [n][m] (nullable)
  BEPI_DTANH_T = 1,  // v = acc * (1 - aux[m][n]^2) -> CT [n][m]
  BEPI_ATOMIC = 2    // Cf[m][n] += acc (fp32 atomics); optional row sums of B over k -> rowsum_b[n]
};

struct GemmBf16Args {
  const bf16_t* A;  // [a_rows][lda]; BEPI_ATOMIC: sample-blocked transposed copy of a_rows rows (lda unused)
  int64_t lda, a_rows;
  const bf16_t* B;  // [b_rows][ldb]; BEPI_ATOMIC: sample-blocked transposed copy of b_rows rows (ldb unused)
  int64_t ldb, b_rows;
  int64_t M, N, K;  // K a multiple of 64 (buffers are zero-padded along k)
  int64_t k_per_split;
  bf16_t* C;
  int64_t ldc;
  bf16_t* CT;
  int64_t ct_cols;  // CT is the sample-blocked transposed copy with N rows; samples m in [M, ct_cols) are written as zeros (ct_cols a multiple of 64)
  float* Cf;
  int64_t ldcf;
  const float* bias;
  const bf16_t* aux;
  int64_t ldaux;
  float* rowsum_b;
  unsigned tiles_m, tiles_n;  // filled by the launcher
};

template <int EPI>
__global__ void __launch_bounds__(256, 2) gemm_bf16_kernel(GemmBf16Args g) {
  constexpr int BM = 128, BN = 128, BK = 64, P = BK + 8;  // pitch in elements (144 bytes)
  constexpr bool KBLK = EPI == BEPI_ATOMIC;               // the operands are sample-blocked transposed copies
  constexpr int PT = 128 + 8;                             // pitch of the output staging tile (272 bytes)
  static_assert(2 * 2 * BM * P >= 128 * PT, "the output tile reuses the operand buffers");
  // two stages of operand tiles: while stage c is multiplied, stage c + 1 sits in LDS and stage c + 2 is on its way
  // from memory in registers -- the loop is bound by (bytes in flight per CU) / (memory latency), not by the MFMAs
  __shared__ __attribute__((aligned(16))) bf16_t smem[2 * 2 * BM * P];
  constexpr int STAGE = 2 * BM * P;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, lo = lane & 31, hi = lane >> 5;
  // 1-D grid: logical index = (split, m tile, n tile) with the n tile fastest, in XCD-aware order, so that the
  // workgroups that share an A panel (and, for the split products, a k slab) run on one XCD and meet in its L2
  const unsigned logical = xcd_remap(blockIdx.x, gridDim.x);
  const unsigned tn = logical % g.tiles_n, tmn = logical / g.tiles_n;
  const unsigned tm = tmn % g.tiles_m, split = tmn / g.tiles_m;
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
  int64_t k_begin = 0, k_end = g.K;
  if (EPI == BEPI_ATOMIC) {
    k_begin = (int64_t)split * g.k_per_split;
    k_end = min(g.K, k_begin + g.k_per_split);
  }

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // staging: thread -> rows tid/8 + 32p (p < 4), 16-byte segment tid%8 of the 128-byte k-chunk of each row
  const int seg = tid & 7, srow = tid >> 3;
  const bf16_t *arow[4], *brow[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    arow[p] = g.A + min(m0 + srow + 32 * p, g.a_rows - 1) * (KBLK ? 64 : g.lda) + 8 * seg;  // rows past the end re-read the last one
    brow[p] = g.B + min(n0 + srow + 32 * p, g.b_rows - 1) * (KBLK ? 64 : g.ldb) + 8 * seg;
  }
  // Register sets R0 / R1 hold the chunks in flight: chunk j travels in set j & 1, is written to LDS stage j & 1 one
  // iteration before it is multiplied, and was requested three iterations before -- two chunks of MFMA work hide
  // its latency, and one barrier per chunk is all the synchronisation.
  uint4 ra0[4], rb0[4], ra1[4], rb1[4];
  float bsum[4] = {0.f, 0.f, 0.f, 0.f};
  const bool want_bsum = EPI == BEPI_ATOMIC && g.rowsum_b != nullptr && tm == 0;
  // Chunks are visited in a rotated order that differs from workgroup to workgroup: with a power-of-two row pitch
  // every workgroup reading the same k offset at the same time would keep hitting the same few memory channels.
  const int nchunks = (int)((k_end - k_begin + BK - 1) / BK);
  // (not for the sample-blocked operands, whose chunks are contiguous: there the workgroups that share a panel walk in step)
  const int rot = (!KBLK && nchunks > 0) ? (int)((tm * 5u + tn * 3u + split) % (unsigned)nchunks) : 0;
  const int64_t astep = KBLK ? g.a_rows * 64 : BK, bstep = KBLK ? g.b_rows * 64 : BK;  // elements from one chunk to the next
  auto chunk_c = [&](int i) { return k_begin / BK + (int64_t)((i + rot) % nchunks); };
  // (the two register sets are named, never passed by reference: a set that is selected at run time, or handed to a
  // helper through a reference, ends up in scratch memory, and a load whose destination is memory is waited for at once)
  auto fetch = [&](int i, auto set) {
    // past the end: the last chunk once more (an L2 hit, never staged) -- a branch here would make every wait in the
    // loop a wait for all outstanding loads
    const int64_t c = chunk_c(i < nchunks ? i : nchunks - 1);
    const int64_t ka = c * astep, kb = c * bstep;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      if constexpr (decltype(set)::value == 0) {
        ra0[p] = *reinterpret_cast<const uint4*>(arow[p] + ka);
        rb0[p] = *reinterpret_cast<const uint4*>(brow[p] + kb);
      } else {
        ra1[p] = *reinterpret_cast<const uint4*>(arow[p] + ka);
        rb1[p] = *reinterpret_cast<const uint4*>(brow[p] + kb);
      }
    }
  };
  auto stage = [&](int buf, auto set) {
    bf16_t* As = smem + buf * STAGE;
    bf16_t* Bs = As + BM * P;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      uint4 va, vb;
      if constexpr (decltype(set)::value == 0) {
        va = ra0[p]; vb = rb0[p];
      } else {
        va = ra1[p]; vb = rb1[p];
      }
      *reinterpret_cast<uint4*>(&As[(srow + 32 * p) * P + 8 * seg]) = va;
      *reinterpret_cast<uint4*>(&Bs[(srow + 32 * p) * P + 8 * seg]) = vb;
      if (EPI == BEPI_ATOMIC && want_bsum) {
        const uint32_t w[4] = {vb.x, vb.y, vb.z, vb.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) bsum[p] += __uint_as_float(w[q] << 16) + __uint_as_float(w[q] & 0xffff0000u);
      }
    }
  };
  auto multiply = [&](int cur) {
    const bf16_t* As = smem + cur * STAGE;
    const bf16_t* Bs = As + BM * P;
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const bf16x8*>(&As[(wm * 64 + i * 32 + lo) * P + ks + 8 * hi]);
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const bf16x8*>(&Bs[(wn * 64 + j * 32 + lo) * P + ks + 8 * hi]);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };
  using Set0 = std::integral_constant<int, 0>;
  using Set1 = std::integral_constant<int, 1>;
  // one iteration: chunk i sits in LDS stage `cur`; chunk i + 1 goes from its register set into the other stage and
  // chunk i + 3 is requested into the same registers.  Chunk j travels in set j & 1.
  if (nchunks > 0) {
    fetch(0, Set0{});
    fetch(1, Set1{});
    stage(0, Set0{});
    fetch(2, Set0{});
  }
  for (int i = 0; i < nchunks; i += 2) {
    __syncthreads();  // stage 0 is complete; everybody is done reading stage 1
    if (i + 1 < nchunks) stage(1, Set1{});
    fetch(i + 3, Set1{});
    multiply(0);
    if (i + 1 < nchunks) {
      __syncthreads();
      if (i + 2 < nchunks) stage(0, Set0{});
      fetch(i + 4, Set0{});
      multiply(1);
    }
  }
  __syncthreads();  // the operand stages are free for the output tile

  if (EPI == BEPI_ATOMIC) {
    if (want_bsum) {
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        float v = bsum[p];
        v += __shfl_xor(v, 1);
        v += __shfl_xor(v, 2);
        v += __shfl_xor(v, 4);
        const int64_t n = n0 + srow + 32 * p;
        if (seg == 0 && n < g.N) atomicAdd(&g.rowsum_b[n], v);
      }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t m = m0 + wm * 64 + i * 32 + 8 * (r / 4) + 4 * hi + (r % 4), n = n0 + wn * 64 + j * 32 + lo;
          if (m < g.M && n < g.N) atomicAdd(&g.Cf[m * g.ldcf + n], acc[i][j][r]);
        }
    return;
  }

  bf16_t* T = smem;  // [128][PT]; the operand buffers are free (the k loop ended with a barrier)
  if (EPI == BEPI_DTANH_T) {  // the aux tile comes in through LDS with 16-byte loads (element-wise 2-byte loads crawl)
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int row = (tid >> 4) + 16 * q, sg = tid & 15;
      const int64_t m = m0 + row, n = n0 + 8 * sg;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (m < g.M && n < g.N) v = *reinterpret_cast<const uint4*>(&g.aux[m * g.ldaux + n]);
      *reinterpret_cast<uint4*>(&T[row * PT + 8 * sg]) = v;
    }
    __syncthreads();
  }
  // ---- element-wise epilogue in registers
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int nl = wn * 64 + j * 32 + lo;
    const int64_t n = n0 + nl;
    const int64_t nc = min(n, g.N - 1);
    const float bias = EPI == BEPI_TANH ? g.bias[nc] : 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int ml = wm * 64 + i * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        const int64_t m = m0 + ml;
        float v = acc[i][j][r];
        if (EPI == BEPI_TANH) {
          v = tanh_f32(v + bias);
        } else {
          const float h = from_bf16(T[ml * PT + nl]);
          v = v * (1.0f - h * h);
        }
        acc[i][j][r] = (m < g.M) ? v : 0.f;  // rows past the end leave as zeros (padding of the transposed copy)
      }
  }
  if (EPI == BEPI_DTANH_T) __syncthreads();  // the aux tile has been consumed; T is reused for the output
  // ---- row-major copy C [m][n]
  if (EPI == BEPI_TANH && g.C != nullptr) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          T[(wm * 64 + i * 32 + 8 * (r / 4) + 4 * hi + (r % 4)) * PT + wn * 64 + j * 32 + lo] = to_bf16(acc[i][j][r]);
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int row = (tid >> 4) + 16 * q, sg = tid & 15;
      const int64_t m = m0 + row, n = n0 + 8 * sg;
      if (m < g.M && n < g.N) *reinterpret_cast<uint4*>(&g.C[m * g.ldc + n]) = *reinterpret_cast<const uint4*>(&T[row * PT + 8 * sg]);
    }
    __syncthreads();
  }
  // ---- transposed copy CT [n][m]
  if (g.CT != nullptr) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const uint32_t w0 = pack2_bf16(acc[i][j][4 * gq + 0], acc[i][j][4 * gq + 1]);
          const uint32_t w1 = pack2_bf16(acc[i][j][4 * gq + 2], acc[i][j][4 * gq + 3]);
          *reinterpret_cast<uint2*>(&T[(wn * 64 + j * 32 + lo) * PT + wm * 64 + i * 32 + 8 * gq + 4 * hi]) = make_uint2(w0, w1);
        }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int row = (tid >> 4) + 16 * q, sg = tid & 15;
      const int64_t n = n0 + row, m = m0 + 8 * sg;
      if (n < g.N && m < g.ct_cols)
        *reinterpret_cast<uint4*>(&g.CT[((m >> 6) * g.N + n) * 64 + (m & 63)]) = *reinterpret_cast<const uint4*>(&T[row * PT + 8 * sg]);
    }
  }
}

// The weight gradients (k split over workgroups, fp32 atomics) on a 256 x 256 x 64 workgroup tile: eight wavefronts
// (2 x 4, each 128 x 64: 4 x 2 MFMA tiles, 128 accumulators).  An operand fragment read from LDS feeds more MFMAs
// than in the 128 x 128 kernel, two wavefronts per SIMD cover each other's LDS and barrier latencies, and two
// register sets of staged operands keep two 64 KB chunks per CU on their way.  (A four-wavefront form with 256
// accumulators per lane has room for one set only and measured 10 % slower; with an element-wise epilogue the big
// tile loses more than it gains, so the products with an epilogue do not use it.)  The operands are the sample-blocked
// transposed copies: a chunk of 256 rows is 32 KB of contiguous memory.
template <int EPI>
__global__ void __launch_bounds__(512, 1) gemm_bf16_big_kernel(GemmBf16Args g) {
  static_assert(EPI == BEPI_ATOMIC, "weight gradients only");
  constexpr int BM = 256, BN = 256, BK = 64, P = BK + 8;
  extern __shared__ __attribute__((aligned(16))) bf16_t big_lds[];  // two stages of [A 256 rows | B 256 rows] x P
  bf16_t* const smem = big_lds;
  constexpr int STAGE = 2 * BM * P;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3, lo = lane & 31, hi = lane >> 5;
  const unsigned logical = xcd_remap(blockIdx.x, gridDim.x);
  const unsigned tn = logical % g.tiles_n, tmn = logical / g.tiles_n;
  const unsigned tm = tmn % g.tiles_m, split = tmn / g.tiles_m;
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
  const int64_t k_begin = (int64_t)split * g.k_per_split, k_end = min(g.K, k_begin + g.k_per_split);

  floatx16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // staging: thread -> rows tid / 8 + 64 p (p < 4) of each operand, 16-byte segment tid % 8 of the row's chunk
  const int seg = tid & 7, srow = tid >> 3;
  uint32_t aoff[4], boff[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    aoff[p] = (uint32_t)min(m0 + srow + 64 * p, g.a_rows - 1) * 64u + 8u * seg;  // rows past the end re-read the last one
    boff[p] = (uint32_t)min(n0 + srow + 64 * p, g.b_rows - 1) * 64u + 8u * seg;
  }
  u32x4 ra0[4], rb0[4], ra1[4], rb1[4];
  float bsum[4] = {0.f, 0.f, 0.f, 0.f};
  const bool want_bsum = g.rowsum_b != nullptr && tm == 0;
  const int nchunks = (int)((k_end - k_begin + BK - 1) / BK);
  const int64_t astep = g.a_rows * 64, bstep = g.b_rows * 64;  // elements from one chunk to the next
  auto fetch = [&](int i, auto set) {
    const int64_t c = k_begin / BK + (i < nchunks ? i : nchunks - 1);  // past the end: the last chunk again, never staged
    const bf16_t* const pa = g.A + c * astep;
    const bf16_t* const pb = g.B + c * bstep;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      if constexpr (decltype(set)::value == 0) {
        ra0[p] = *reinterpret_cast<const u32x4*>(pa + aoff[p]);
        rb0[p] = *reinterpret_cast<const u32x4*>(pb + boff[p]);
      } else {
        ra1[p] = *reinterpret_cast<const u32x4*>(pa + aoff[p]);
        rb1[p] = *reinterpret_cast<const u32x4*>(pb + boff[p]);
      }
    }
  };
  auto stage = [&](int buf, auto set, bool live) {  // live: the chunk exists (one past the end is staged but never multiplied)
    bf16_t* As = smem + buf * STAGE;
    bf16_t* Bs = As + BM * P;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      u32x4 va, vb;
      if constexpr (decltype(set)::value == 0) {
        va = ra0[p]; vb = rb0[p];
      } else {
        va = ra1[p]; vb = rb1[p];
      }
      *reinterpret_cast<u32x4*>(&As[(srow + 64 * p) * P + 8 * seg]) = va;
      *reinterpret_cast<u32x4*>(&Bs[(srow + 64 * p) * P + 8 * seg]) = vb;
      if (want_bsum && live) {
        bsum[p] += (__uint_as_float(vb.x << 16) + __uint_as_float(vb.x & 0xffff0000u)) +
                   (__uint_as_float(vb.y << 16) + __uint_as_float(vb.y & 0xffff0000u)) +
                   (__uint_as_float(vb.z << 16) + __uint_as_float(vb.z & 0xffff0000u)) +
                   (__uint_as_float(vb.w << 16) + __uint_as_float(vb.w & 0xffff0000u));
      }
    }
  };
  auto multiply = [&](int cur) {
    const bf16_t* As = smem + cur * STAGE + (wm * 128 + lo) * P + 8 * hi;
    const bf16_t* Bs = smem + cur * STAGE + BM * P + (wn * 64 + lo) * P + 8 * hi;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 a[4], b[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = *reinterpret_cast<const bf16x8*>(As + i * 32 * P + 16 * ks);
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const bf16x8*>(Bs + j * 32 * P + 16 * ks);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };
  using Set0 = std::integral_constant<int, 0>;
  using Set1 = std::integral_constant<int, 1>;
  // chunk j travels in set j & 1, is written to LDS stage j & 1 one iteration before it is multiplied and was
  // requested three iterations before
  // requested three iterations before.  The loop body has no branch (a uniform branch around a stage or a request
  // makes every wait in the loop a wait for all outstanding loads): chunks are taken in pairs, a chunk past the end
  // is the last one read once more, and an odd last chunk is multiplied after the loop.
  if (nchunks > 0) {
    fetch(0, Set0{});
    fetch(1, Set1{});
    stage(0, Set0{}, true);
    fetch(2, Set0{});
  }
  for (int i = 0; i + 1 < nchunks; i += 2) {
    __syncthreads();  // stage 0 is complete; everybody is done reading stage 1
    stage(1, Set1{}, true);
    fetch(i + 3, Set1{});
    multiply(0);
    __syncthreads();
    stage(0, Set0{}, i + 2 < nchunks);
    fetch(i + 4, Set0{});
    multiply(1);
  }
  if (nchunks & 1) {
    __syncthreads();
    multiply(0);
  }
  if (want_bsum) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      float v = bsum[p];
      v += __shfl_xor(v, 1);
      v += __shfl_xor(v, 2);
      v += __shfl_xor(v, 4);
      const int64_t n = n0 + srow + 64 * p;
      if (seg == 0 && n < g.N) atomicAdd(&g.rowsum_b[n], v);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t m = m0 + wm * 128 + i * 32 + 8 * (r / 4) + 4 * hi + (r % 4), n = n0 + wn * 64 + j * 32 + lo;
        if (m < g.M && n < g.N) atomicAdd(&g.Cf[m * g.ldcf + n], acc[i][j][r]);
      }
}

// The products with an element-wise epilogue (forward layers, dz1) when the weight matrix is small enough to LIVE IN
// REGISTERS: a persistent workgroup of eight wavefronts owns a 256-column panel of the output, wavefront w holds the
// B rows n0 + 32 w .. + 31 for all of k as MFMA operand fragments (4 KG registers per lane), and 64-row tiles of A
// stream through LDS as one continuous sequence of 64 x BK chunks that runs across tile boundaries, so the loads of
// the next tile are in flight during the epilogue of the current one.  Against the 128 x 128 tile kernel above this
// halves twice what a workgroup pulls through the L2 per flop (no B traffic at all, and A is read by N / 256
// workgroups instead of N / 128), which is what bounded that kernel: per 64-row tile only 64 x K elements arrive.
// Chunk j travels in register set j % NS and LDS stage j % NS: it is requested NS + 1 iterations before it is
// multiplied and written to LDS one iteration before; one barrier per chunk.  NS divides the chunks per tile, so
// every set / stage / fragment index is a compile-time constant after unrolling.
// The forward products run the MFMA with the operands swapped (weights as the row operand), so that a lane ends up
// with four consecutive columns of one output row and the row-major tile is staged with 8-byte LDS stores; dz1, whose
// only output is the transposed copy, keeps the activations as the row operand for the same reason.
// Grid: a multiple of 8 * (N / 256) workgroups; consecutive slots of one XCD take the panels of the same row tiles,
// so an A chunk is fetched from HBM once and found in that XCD's L2 by the other panels.
// What bounds it: the bytes a CU keeps in flight.  128 of a lane's 256 registers hold weights, which leaves room for
// NS = 4 chunks of 8 KB on their way; a k-loop iteration therefore lasts a quarter of the loaded memory latency, not
// its 512 MFMA cycles (two stages of 128-wide chunks measure the same).  The staging registers are native vectors:
// an array of HIP's uint4 structs stays in scratch memory here, and every load is then waited for at once.
template <int KG, int BK, int NS, int EPI>
__global__ void __launch_bounds__(512, 1) gemm_bf16_wres_kernel(GemmBf16Args g) {
  static_assert(EPI == BEPI_TANH || EPI == BEPI_DTANH_T, "element-wise epilogues only");
  constexpr int BM = 64, BN = 256, P = BK + 8, KS = BK / 16, NCH = 16 * KG / BK, CPT = BK / 64;
  constexpr int PT = BN + 8, PT2 = BM + 8;  // pitches of the row-major and of the transposed output tile
  constexpr bool SWAP = EPI == BEPI_TANH;   // weights as the MFMA row operand
  static_assert(BK % 64 == 0 && (16 * KG) % BK == 0 && NS >= 2 && NS <= NCH && NCH % NS == 0, "chunks per tile are a multiple of the stages");
  static_assert(EPI == BEPI_TANH || NCH >= 3, "the aux tile is fetched during the k loop");
  extern __shared__ __attribute__((aligned(16))) bf16_t wres_lds[];
  bf16_t* const As = wres_lds;             // [NS][BM][P]
  bf16_t* const T = As + NS * BM * P;      // [BM][PT]   C tile (row-major) / aux tile
  bf16_t* const T2 = T + BM * PT;          // [BN][PT2]  C^T tile
  float* const biasS = reinterpret_cast<float*>(T2 + BN * PT2);  // [BN]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lo = lane & 31, hi = lane >> 5;
  const unsigned xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3;
  const unsigned panels = g.tiles_n, panel = slot % panels;
  const int64_t stream = (int64_t)(slot / panels) * 8 + xcd, nstreams = gridDim.x / panels;
  if (stream >= (int64_t)g.tiles_m) return;  // the whole workgroup
  const int nt = (int)(((int64_t)g.tiles_m - stream + nstreams - 1) / nstreams);  // row tiles of this workgroup
  const int64_t n0 = (int64_t)panel * BN;

  bf16x8 breg[KG];
  {
    const bf16_t* brow = g.B + min(n0 + 32 * wave + lo, g.b_rows - 1) * g.ldb + 8 * hi;
#pragma unroll
    for (int s = 0; s < KG; ++s) breg[s] = *reinterpret_cast<const bf16x8*>(brow + 16 * s);
  }
  if (EPI == BEPI_TANH && tid < BN) biasS[tid] = g.bias[n0 + tid];  // read after the barriers of the first k loop

  // staging: thread -> row tid / 8 of the tile, 16-byte segments tid % 8 + 8 u of the row's chunk
  const int srow = tid >> 3, seg = tid & 7;
  auto a_ptr = [&](int ti, int kc) -> const bf16_t* {  // tiles past the last one: the last one again (never multiplied)
    const int64_t tm = stream + (int64_t)min(ti, nt - 1) * nstreams;
    return g.A + min(tm * BM + srow, g.a_rows - 1) * g.lda + kc * BK + 8 * seg;
  };
  u32x4 R[NS][CPT];
  {
    const bf16_t* p0 = a_ptr(0, 0);
#pragma unroll
    for (int u = 0; u < CPT; ++u) R[0][u] = *reinterpret_cast<const u32x4*>(p0 + 64 * u);
#pragma unroll
    for (int u = 0; u < CPT; ++u) *reinterpret_cast<u32x4*>(&As[srow * P + 8 * seg + 64 * u]) = R[0][u];
  }
#pragma unroll
  for (int j = 1; j <= NS; ++j) {
    const bf16_t* pj = a_ptr(j / NCH, j % NCH);
#pragma unroll
    for (int u = 0; u < CPT; ++u) R[j % NS][u] = *reinterpret_cast<const u32x4*>(pj + 64 * u);
  }

  floatx16 acc[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  for (int t = 0; t < nt; ++t) {
    const int64_t m0 = (stream + (int64_t)t * nstreams) * BM;
    u32x4 xr[4];  // aux tile of this row tile (BEPI_DTANH_T): thread -> rows tid / 32 + 16 q, 16-byte segment tid % 32
    if (EPI == BEPI_DTANH_T) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int64_t m = min(m0 + (tid >> 5) + 16 * q, g.M - 1);  // rows past the end: any row (their results are zeroed)
        xr[q] = *reinterpret_cast<const u32x4*>(&g.aux[m * g.ldaux + n0 + 8 * (tid & 31)]);
      }
    }
#pragma unroll
    for (int kc = 0; kc < NCH; ++kc) {
      __syncthreads();  // stage kc % NS is complete; everybody is done reading the stage written next
      const int nset = (kc + 1) % NS;
#pragma unroll
      for (int u = 0; u < CPT; ++u) *reinterpret_cast<u32x4*>(&As[(nset * BM + srow) * P + 8 * seg + 64 * u]) = R[nset][u];
      {
        const bf16_t* pn = a_ptr(t + (kc + 1 + NS) / NCH, (kc + 1 + NS) % NCH);
#pragma unroll
        for (int u = 0; u < CPT; ++u) R[nset][u] = *reinterpret_cast<const u32x4*>(pn + 64 * u);
      }
      if (EPI == BEPI_DTANH_T && kc == NCH - 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<u32x4*>(&T[((tid >> 5) + 16 * q) * PT + 8 * (tid & 31)]) = xr[q];
      }
      const bf16_t* Ab = As + (kc % NS) * BM * P + lo * P + 8 * hi;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(Ab + 16 * ks);
        const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(Ab + 32 * P + 16 * ks);
        const bf16x8 b = breg[KS * kc + ks];
        if (SWAP) {
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a0, acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a1, acc[1], 0, 0, 0);
        } else {
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc[1], 0, 0, 0);
        }
      }
    }
    // ---- epilogue.  T, T2 (and biasS) were last touched before the barriers of this tile's k loop.
    if (SWAP) {
      // acc[i][4 gq + j] = element (row 32 i + lo, column 32 wave + 8 gq + 4 hi + j) of the tile
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const bool live = m0 + 32 * i + lo < g.M;  // rows past the end leave as zeros (padding of the transposed copy)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const int nc = 32 * wave + 8 * gq + 4 * hi;
          const float4 bq = *reinterpret_cast<const float4*>(&biasS[nc]);
          const float bb[4] = {bq.x, bq.y, bq.z, bq.w};
          float v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float x = tanh_f32(acc[i][4 * gq + j] + bb[j]);
            v[j] = live ? x : 0.f;
            acc[i][4 * gq + j] = 0.f;
          }
          if (g.C != nullptr)
            *reinterpret_cast<uint2*>(&T[(32 * i + lo) * PT + nc]) = make_uint2(pack2_bf16(v[0], v[1]), pack2_bf16(v[2], v[3]));
          if (g.CT != nullptr) {
#pragma unroll
            for (int j = 0; j < 4; ++j) T2[(nc + j) * PT2 + 32 * i + lo] = to_bf16(v[j]);
          }
        }
      }
    } else {
      // acc[i][r] = element (row 32 i + 8 (r / 4) + 4 hi + r % 4, column 32 wave + lo) of the tile
      const int nl = 32 * wave + lo;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          float v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int ml = 32 * i + 8 * gq + 4 * hi + j;
            const float h = from_bf16(T[ml * PT + nl]);
            const float x = acc[i][4 * gq + j] * (1.0f - h * h);
            v[j] = (m0 + ml < g.M) ? x : 0.f;
            acc[i][4 * gq + j] = 0.f;
          }
          *reinterpret_cast<uint2*>(&T2[nl * PT2 + 32 * i + 8 * gq + 4 * hi]) = make_uint2(pack2_bf16(v[0], v[1]), pack2_bf16(v[2], v[3]));
        }
    }
    __syncthreads();
    if (EPI == BEPI_TANH && g.C != nullptr) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int row = (tid >> 5) + 16 * q, sg = tid & 31;
        if (m0 + row < g.M)
          *reinterpret_cast<uint4*>(&g.C[(m0 + row) * g.ldc + n0 + 8 * sg]) = *reinterpret_cast<const uint4*>(&T[row * PT + 8 * sg]);
      }
    }
    if (g.CT != nullptr) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nrow = (tid >> 3) + 64 * q, sg = tid & 7;
        if (m0 + 8 * sg < g.ct_cols)
          *reinterpret_cast<uint4*>(&g.CT[((m0 >> 6) * g.N + n0 + nrow) * 64 + 8 * sg]) = *reinterpret_cast<const uint4*>(&T2[nrow * PT2 + 8 * sg]);
      }
    }
  }
}

// Workgroups of a gemm_bf16_wres_kernel launch: one per CU.
constexpr unsigned kWresGrid = 256;

template <int EPI>
inline bool gemm_bf16_wres_supported(const GemmBf16Args& g) {
  if (EPI == BEPI_ATOMIC) return false;
  const int64_t panels = g.N / 256;
  if (g.N % 256 != 0 || !(panels == 1 || panels == 2 || panels == 4) || g.b_rows < g.N) return false;
  if (EPI == BEPI_TANH) return g.K == 128 || g.K == 192 || g.K == 256 || g.K == 512;
  return g.K == 512;
}

template <int KG, int BK, int NS, int EPI>
inline void launch_gemm_bf16_wres_inst(const GemmBf16Args& g, hipStream_t s) {
  auto kern = gemm_bf16_wres_kernel<KG, BK, NS, EPI>;
  const size_t bytes = ((size_t)NS * 64 * (BK + 8) + 64 * 264 + 256 * 72) * sizeof(bf16_t) + 256 * sizeof(float);
  static bool configured = false;  // per instantiation
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return;
    configured = true;
  }
  hipLaunchKernelGGL(kern, dim3(kWresGrid), dim3(512), bytes, s, g);
}

template <int EPI>
inline void launch_gemm_bf16_wres(GemmBf16Args g, hipStream_t s) {
  const int64_t mcover = g.CT == nullptr ? g.M : std::max(g.M, g.ct_cols);
  g.tiles_m = (unsigned)((mcover + 63) / 64);
  g.tiles_n = (unsigned)(g.N / 256);
  if constexpr (EPI == BEPI_TANH) {
    if (g.K == 128) return launch_gemm_bf16_wres_inst<8, 64, 2, EPI>(g, s);
    if (g.K == 192) return launch_gemm_bf16_wres_inst<12, 64, 3, EPI>(g, s);
    if (g.K == 256) return launch_gemm_bf16_wres_inst<16, 64, 4, EPI>(g, s);
  }
  if constexpr (EPI != BEPI_ATOMIC) return launch_gemm_bf16_wres_inst<32, 64, 4, EPI>(g, s);
}

template <int EPI>
inline void launch_gemm_bf16(const GemmBf16Args& g0, hipStream_t s) {
  GemmBf16Args g = g0;
  TimedLaunch timed(EPI == BEPI_TANH ? KC_GEMM_NN : (EPI == BEPI_DTANH_T ? KC_GEMM_NT : KC_GEMM_TN),
                    2.0 * (double)g.M * (double)g.N * (double)g.K, s);
  unsigned gz = 1;
  if (EPI == BEPI_ATOMIC) gz = (unsigned)((g.K + g.k_per_split - 1) / g.k_per_split);
  if constexpr (EPI != BEPI_ATOMIC) {
    if (gemm_bf16_wres_supported<EPI>(g)) return launch_gemm_bf16_wres<EPI>(g, s);
  }
  const int64_t mcover = (EPI == BEPI_ATOMIC || g.CT == nullptr) ? g.M : std::max(g.M, g.ct_cols);
  if constexpr (EPI == BEPI_ATOMIC) if (mcover > 128 && g.N > 128) {
    // 256 x 256 tiles for the weight gradients.  (For the products with an element-wise epilogue the big tile
    // measured slower, 466 against 291 us for layer 2 and 725 against 298 us for dz1 at 262 144 rows: 256 tanh
    // evaluations per lane with one wavefront per SIMD are not hidden behind anything.)
    g.tiles_m = (unsigned)((mcover + 255) / 256);
    g.tiles_n = (unsigned)((g.N + 255) / 256);
    {
      auto kern = gemm_bf16_big_kernel<EPI>;
      static bool configured = false;
      if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return;
        configured = true;
      }
      hipLaunchKernelGGL(kern, dim3(g.tiles_m * g.tiles_n * gz), dim3(512), 2 * 2 * 256 * 72 * sizeof(bf16_t), s, g);
    }
    return;
  }
  g.tiles_m = (unsigned)((mcover + 127) / 128);
  g.tiles_n = (unsigned)((g.N + 127) / 128);
  hipLaunchKernelGGL(gemm_bf16_kernel<EPI>, dim3(g.tiles_m * g.tiles_n * gz), dim3(256), 0, s, g);
}

}  // namespace marl
