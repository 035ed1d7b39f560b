// Row-streaming fp32 MFMA products with the weight matrix resident in registers, for the 256-wide layers.
//
//   C[m][n] = epilogue( sum_k A[m][k] * B(k, n) ),   m < S (hundreds of thousands of rows), n < 256, k < K <= 304
//
// A 256 x 256 fp32 weight matrix is 256 KB: half of the register file of one compute unit.  A workgroup of four
// wavefronts (one per SIMD, up to 512 registers per lane) -- or of eight (two per SIMD, 256 registers each) -- therefore
// keeps the whole matrix in registers for its lifetime: wavefront w holds columns 64 w .. 64 w + 63 (32 w .. 32 w + 31
// with eight) in the lane layout the matrix cores read their second operand in.  The workgroup is persistent over tiles of 64 rows; a tile of A travels global -> registers -> LDS while the
// previous one is multiplied (two LDS stages), every wavefront reads the same A fragments from LDS and multiplies
// them into its own 64 columns (2 x 2 accumulator tiles of 32 x 32).  Nothing but A and C moves per tile: no weight
// traffic at all, one barrier per tile.
//
// Within a group of eight k values the lower half-wavefront supplies k = 0..3 and the upper half k = 4..7 to four
// consecutive v_mfma_f32_32x32x2_f32 steps, so that a lane's four A values are one 16-byte LDS read.
#pragma once
#include "gemm.h"

namespace marl {

enum WregEpi {
  WREG_BIAS_TANH = 0,  // C = tanh(acc + bias[n])
  WREG_DTANH = 1,      // C = acc * (1 - aux[m][n]^2)
  // The last hidden layer of a network in training: h = tanh(acc + bias[n]) stays in registers, the output layer
  // out = h W3 + b3 and the loss functor turn it into dL/d(out), and C = (dL/d(out) W3^T) * (1 - h^2), the gradient
  // with respect to this layer's pre-activation; the output layer's own gradient is accumulated on the way.
  WREG_TANH_LOSS = 2
};

struct WregArgs {
  RowSrc A;        // S rows of Kin floats (optionally gathered); rows must be 16-byte aligned, Kin % 4 == 0
  int64_t S;
  int Kin;         // columns of A actually present (<= K; the rest of the contraction is zero)
  const float* B;  // b_kcont ? [256][ldb] with B(k, n) = B[n * ldb + k] : [Kin][ldb] with B(k, n) = B[k * ldb + n]
  int ldb;
  int b_kcont;
  // C and aux have room for S rounded up to whole tiles of 64 rows: the kernel stores (and reads) whole tiles without
  // row checks, what lands in the rows past S is never used
  float* C;           // [S][256]
  const float* bias;  // WREG_BIAS_TANH, WREG_TANH_LOSS: [256]
  const float* aux;   // WREG_DTANH: [S][256]
  // WREG_TANH_LOSS: the output layer W3 [256][NOUT], b3 [NOUT]; its gradient and the loss statistics (5 floats),
  // accumulated with atomics
  const float *W3, *b3;
  float *gW3, *gb3, *stats;
  // (nullable) workgroup b writes its W3 / b3 gradient to partial3 + b * (256 * NOUT + NOUT) with plain stores instead;
  // the caller adds the copies to gW3 (with gb3 directly behind it) in a fixed order
  float* partial3;
};

// The loss functor of WREG_TANH_LOSS splits into load (the trajectory values of a sample, requested while the tile is
// still being multiplied) and compute (out -> dL/d(out), statistics); this one stands in for the other epilogues.
struct WregNoFinish {
  struct In {};
  struct Prep {};
  __device__ int32_t row_entry(int64_t) const { return 0; }
  __device__ In load_with(int64_t, int32_t) const { return In{}; }
  __device__ Prep prepare() const { return Prep{}; }
  __device__ void compute(const In&, const Prep&, const float*, float*, float*) const {}
};

constexpr int kWregBM = 64;   // rows per tile
constexpr int kWregN = 256;   // columns (4 wavefronts x 64)

template <int K>
struct WregShape {
  static constexpr int P = K + 4;                      // LDS row pitch: 4 * odd, conflict-free 16-byte row-per-lane reads
  static constexpr int VPR = K / 4;                    // 16-byte vectors per row
  static constexpr int NB = 8;                         // staging batches per tile
  static constexpr int GROUPS = K / 8;
  static constexpr size_t lds_bytes = sizeof(float) * 2 * kWregBM * P + sizeof(int64_t) * 2 * kWregBM;
  // WREG_TANH_LOSS adds: W3 [256][NOUT], partial outputs [4][BM][NOUT], dL/d(out) [BM][8]
  static constexpr size_t loss_lds_bytes(int nout, int nwv) {
    return sizeof(float) * (kWregN * nout + nwv * kWregBM * nout + kWregBM * 8 + kWregBM * (nout + 5));
  }
  static_assert(K % 16 == 0 && (P / 4) % 2 == 1, "K a multiple of 16 with an odd K/4 + 1");
};

// NWV wavefronts (4: one per SIMD, 64 columns each; 8: two per SIMD, 32 columns each, half the registers per lane)
template <int K, int EPI, int NOUT = 1, class Fin = WregNoFinish, int NWV = 4>
__global__ void __launch_bounds__(64 * NWV, 1) wreg_gemm_kernel(WregArgs a, Fin fin) {
  using Sh = WregShape<K>;
  constexpr int NT = 64 * NWV, CW = kWregN / NWV, JN = CW / 32, EPL = 32 * JN;  // threads, columns per wavefront, column tiles, outputs per lane
  constexpr int P = Sh::P, VPR = Sh::VPR, NB = Sh::NB, GROUPS = Sh::GROUPS, BM = kWregBM;
  constexpr int TOT = (BM * VPR + NT - 1) / NT, PER = (TOT + NB - 1) / NB;  // vectors a thread stages per tile, per batch
  constexpr bool RAGGED = (BM * VPR) % NT != 0;  // the last vector index of some threads lies past the tile
  extern __shared__ __attribute__((aligned(16))) unsigned char wreg_smem[];
  float* const As = reinterpret_cast<float*>(wreg_smem);                       // [2][BM][P]
  int64_t* const ent = reinterpret_cast<int64_t*>(As + 2 * BM * P);            // [2][BM] offsets (floats) of a tile's rows
  float* const W3s = reinterpret_cast<float*>(ent + 2 * BM);                    // WREG_TANH_LOSS only, as are the next two
  float* const red = W3s + kWregN * NOUT;                                       // [NWV][BM][NOUT]
  float* const dls = red + NWV * BM * NOUT;                                       // [BM][8]
  // per-sample-slot sums that only the first BM threads touch, once per tile (b3 gradient, loss statistics): in LDS rather
  // than in registers of every thread, which this kernel does not have to spare
  constexpr int AS = NOUT + 5;
  float* const accS = dls + BM * 8;                                             // [BM][AS]
  static_assert(EPI != WREG_TANH_LOSS || K == kWregN, "the activation tile reuses the stage of A it came from");
  // The two plain epilogues are deferred where the registers allow: a tile's accumulators move to a second register set and are finished two
  // elements per k group INSIDE the next tile's stream of matrix instructions, so that the single wavefront of a SIMD
  // keeps its matrix core busy while it applies tanh and stores (only a workgroup's last tile finishes on its own).
  constexpr bool DEFER = EPI != WREG_TANH_LOSS && K <= 256;
  constexpr int EPG = EPL / 32;  // deferred elements finished per k group  // a longer contraction leaves no room for the second set
  constexpr int LOOK = 8;  // WREG_DTANH: k groups between the request of an element's operand and its use

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = lane & 31, hi = lane >> 5;
  const int64_t ntiles = (a.S + BM - 1) / BM;

  // ---- the weights: breg[g][j][jn] = B(8 g + 4 hi + j, 64 wave + 32 jn + lo)
  float breg[GROUPS][4][JN];
#pragma unroll
  for (int g = 0; g < GROUPS; ++g)
#pragma unroll
    for (int jn = 0; jn < JN; ++jn) {
      const int n = CW * wave + 32 * jn + lo;
      const int k = 8 * g + 4 * hi;
      if (a.b_kcont) {
        const float4 v = (k < a.Kin) ? *reinterpret_cast<const float4*>(a.B + (int64_t)n * a.ldb + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        breg[g][0][jn] = v.x; breg[g][1][jn] = v.y; breg[g][2][jn] = v.z; breg[g][3][jn] = v.w;
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) breg[g][j][jn] = (k + j < a.Kin) ? a.B[(int64_t)(k + j) * a.ldb + n] : 0.f;
      }
    }

  // ---- staging of a tile of A: vector f = tid + 256 p of the tile is (row f / VPR, columns 4 (f % VPR) ..)
  auto row_of = [&](int p) { return (tid + NT * p) / VPR; };
  auto col_of = [&](int p) { return 4 * ((tid + NT * p) % VPR); };
  auto in_tile = [&](int p) { return !RAGGED || tid + NT * p < BM * VPR; };
  // A batch is requested SETS batch intervals before it is stored (one register set each), and the row offsets it needs
  // are read from LDS one k group before the request.
  constexpr int SETS = K <= 256 ? 2 : 1;  // the longer contraction has registers for one batch in flight only
  float4 stg[SETS][PER];
  int64_t eoff[PER];
  auto read_offsets = [&](int slot, int b) {
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int p = b * PER + q;
      if (p < TOT && in_tile(p)) eoff[q] = ent[slot * BM + row_of(p)];
    }
  };
  auto fetch_batch = [&](int b) {
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int p = b * PER + q;
      if (p < TOT && in_tile(p)) {
        const int c = col_of(p);
        stg[b % SETS][q] = (c < a.Kin) ? *reinterpret_cast<const float4*>(a.A.base + eoff[q] + c) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  };
  auto store_batch = [&](int stage, int b) {
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int p = b * PER + q;
      if (p < TOT && in_tile(p)) *reinterpret_cast<float4*>(&As[(stage * BM + row_of(p)) * P + col_of(p)]) = stg[b % SETS][q];
    }
  };
  // offset of row tid of a tile (threads tid < BM); rows past the end repeat the last row, whose results are never stored
  auto load_entries = [&](int64_t tile) -> int64_t {
    if (tid >= BM || tile >= ntiles) return 0;
    const int64_t row = min(tile * BM + tid, a.S - 1);
    return a.A.ptr(row) - a.A.base;
  };

  // ---- prologue: entries of the first two tiles, then the first tile itself
  int64_t tile = blockIdx.x;
  if (tile >= ntiles) return;  // uniform per workgroup
  // output-layer gradient of this lane's two columns (its half of the rows), the bias gradient and the loss statistics, summed over this workgroup's tiles
  float gw[JN][NOUT];
#pragma unroll
  for (int jn = 0; jn < JN; ++jn)
#pragma unroll
    for (int k = 0; k < NOUT; ++k) gw[jn][k] = 0.f;
  if (EPI == WREG_TANH_LOSS && tid < BM) {  // read and written by thread tid only
#pragma unroll
    for (int k = 0; k < AS; ++k) accS[tid * AS + k] = 0.f;
  }
  if (EPI == WREG_TANH_LOSS)
    for (int i = tid; i < kWregN * NOUT; i += NT) W3s[i] = a.W3[i];  // ordered before its first use by the barriers below
  const auto prep = fin.prepare();
  {
    const int64_t e0 = load_entries(tile), e1 = load_entries(tile + gridDim.x);
    if (tid < BM) {
      ent[0 * BM + tid] = e0;
      ent[1 * BM + tid] = e1;
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      read_offsets(0, b);
      fetch_batch(b);
      store_batch(0, b);
    }
    __syncthreads();
  }

  floatx16 prev[2][JN];     // DEFER: the previous tile's accumulators ...
  int64_t prev_off = 0;    // ... and where its outputs go.  Before the first tile: zeros, "finished" into the first
#pragma unroll
  for (int i = 0; i < 2; ++i)  // tile's own place, where the real values overwrite them one tile later (same lane, same
#pragma unroll
    for (int jn = 0; jn < JN; ++jn)  // addresses, program order)
#pragma unroll
      for (int r = 0; r < 16; ++r) prev[i][jn][r] = 0.f;
  float bias2[JN];
#pragma unroll
  for (int jn = 0; jn < JN; ++jn) bias2[jn] = EPI != WREG_DTANH ? a.bias[CW * wave + 32 * jn + lo] : 0.f;
  float b3r[NOUT];  // WREG_TANH_LOSS: the output layer's bias (used by the threads that own a sample)
#pragma unroll
  for (int k = 0; k < NOUT; ++k) b3r[k] = EPI == WREG_TANH_LOSS ? a.b3[k] : 0.f;
  // element e = 32 jn + 16 i + r of a lane's 64 outputs: offset from the lane's address, and its finish
  auto elem_off = [](int e) { return (32 * ((e >> 4) & 1) + 8 * ((e & 15) / 4) + (e & 3)) * kWregN + 32 * (e >> 5); };
  float auxr[EPL];
  auto finish_elem = [&](int e, int64_t off) {
    const int jn = e >> 5, i = (e >> 4) & 1, r = e & 15;
    float v = prev[i][jn][r];
    if (EPI == WREG_BIAS_TANH) {
      v = tanh_f32(v + bias2[jn]);
    } else {
      const float h = auxr[e];
      v = v * (1.0f - h * h);
    }
    a.C[off + elem_off(e)] = v;
  };

  int it = 0;
  for (; tile < ntiles; tile += gridDim.x, ++it) {
    const int stage = it & 1;
    const int64_t next = tile + gridDim.x;
    const int64_t e2 = load_entries(next + gridDim.x);  // consumed at the end of this tile
    const float* const At = As + stage * BM * P;
    const int64_t m0 = tile * BM;

    // A lane's 64 outputs sit at fixed offsets from one address: rows 32 i + 8 (r/4) + r%4 below row m0 + 4 hi,
    // columns 32 jn right of column 64 wave + lo.
    const int64_t lane_off = (m0 + 4 * hi) * kWregN + CW * wave + lo;
    if (it == 0) prev_off = lane_off;
    if (DEFER && EPI == WREG_DTANH) {  // operands of the first elements of the previous tile's finish
#pragma unroll
      for (int e = 0; e < EPG * LOOK; ++e) auxr[e] = a.aux[prev_off + elem_off(e)];
    }

    // the loss inputs of sample tid of this tile (threads tid < BM): the row entry now, the values half-way through
    const int64_t my_sample = min(m0 + tid, a.S - 1);
    const int32_t loss_entry = (EPI == WREG_TANH_LOSS && tid < BM) ? fin.row_entry(my_sample) : 0;
    typename Fin::In loss_in{};

    floatx16 acc[2][JN];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int jn = 0; jn < JN; ++jn)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][jn][r] = 0.f;

    // (after a workgroup's last tile the same requests run once more on the row offsets 0 that load_entries left for
    // tiles past the end: harmless reads into a stage nobody uses, and a loop body without branches)
#pragma unroll
    for (int b = 0; b < SETS; ++b) {
      read_offsets(stage ^ 1, b);
      fetch_batch(b);
    }
    // fragments of A: those of group g + 1 are read from LDS before the products of group g are issued (SETS == 2;
    // the longer contraction has no registers for the second pair and reads each group's fragments at its top)
    // (with two wavefronts per SIMD the other wavefront covers the LDS latency, and the registers are needed elsewhere)
    constexpr bool FPRE = SETS == 2 && NWV == 4;
    float4 fa[2][2];
    if (FPRE) {
      fa[0][0] = *reinterpret_cast<const float4*>(&At[lo * P + 4 * hi]);
      fa[0][1] = *reinterpret_cast<const float4*>(&At[(32 + lo) * P + 4 * hi]);
    }
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
      if (FPRE && g + 1 < GROUPS) {
        fa[(g + 1) & 1][0] = *reinterpret_cast<const float4*>(&At[lo * P + 8 * (g + 1) + 4 * hi]);
        fa[(g + 1) & 1][1] = *reinterpret_cast<const float4*>(&At[(32 + lo) * P + 8 * (g + 1) + 4 * hi]);
        __builtin_amdgcn_sched_barrier(0);  // keep these reads ahead of this group's matrix instructions
      }
      if (!FPRE) {
        fa[g & 1][0] = *reinterpret_cast<const float4*>(&At[lo * P + 8 * g + 4 * hi]);
        fa[g & 1][1] = *reinterpret_cast<const float4*>(&At[(32 + lo) * P + 8 * g + 4 * hi]);
      }
      const float4 a0 = fa[g & 1][0], a1 = fa[g & 1][1];
      const float af[2][4] = {{a0.x, a0.y, a0.z, a0.w}, {a1.x, a1.y, a1.z, a1.w}};
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int jn = 0; jn < JN; ++jn)
            acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][j], breg[g][j][jn], acc[i][jn], 0, 0, 0);
      if (EPI == WREG_TANH_LOSS && g == GROUPS / 2 && tid < BM) loss_in = fin.load_with(my_sample, loss_entry);
      if (DEFER && g < 32) {  // EPG elements of the previous tile per k group
        if (EPI == WREG_DTANH && g + LOOK < 32) {
#pragma unroll
          for (int q = 0; q < EPG; ++q) auxr[EPG * (g + LOOK) + q] = a.aux[prev_off + elem_off(EPG * (g + LOOK) + q)];
        }
#pragma unroll
        for (int q = 0; q < EPG; ++q) finish_elem(EPG * g + q, prev_off);
      }
      // the next tile moves in NB batches spread over the products: batch b leaves its registers for the other LDS
      // stage at the end of its interval and batch b + 2 is requested into them; its row offsets were read a group earlier
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        if (g == ((b + 1) * GROUPS) / NB - SETS && b + SETS < NB) read_offsets(stage ^ 1, b + SETS);
        if (g == ((b + 1) * GROUPS) / NB - 1) {
          store_batch(stage ^ 1, b);
          if (b + SETS < NB) fetch_batch(b + SETS);
        }
      }
    }

    // ---- epilogue (accumulator register r of a lane holds C[8 (r/4) + 4 hi + r%4][lo] of its 32 x 32 tile)
    float* const out = a.C + lane_off;
    if (DEFER) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jn = 0; jn < JN; ++jn) prev[i][jn] = acc[i][jn];
      prev_off = lane_off;
    } else if (EPI != WREG_TANH_LOSS) {
#pragma unroll
      for (int jn = 0; jn < JN; ++jn)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float v = acc[i][jn][r];
            if (EPI == WREG_BIAS_TANH) {
              v = tanh_f32(v + bias2[jn]);
            } else {
              const float h = a.aux[lane_off + elem_off(32 * jn + 16 * i + r)];
              v = v * (1.0f - h * h);
            }
            out[elem_off(32 * jn + 16 * i + r)] = v;
          }
    } else {
      // h = tanh(acc + bias) stays in the accumulators and goes to LDS, into the stage of A this tile came from
      float* const Hs = As + stage * BM * P;
      __syncthreads();  // every wavefront has read its last fragment of A
#pragma unroll
      for (int jn = 0; jn < JN; ++jn) {
        const int n = CW * wave + 32 * jn + lo;
        const float bias = bias2[jn];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int m = 32 * i + 8 * (r / 4) + 4 * hi + (r % 4);
            const float v = tanh_f32(acc[i][jn][r] + bias);
            acc[i][jn][r] = v;
            Hs[m * P + n] = v;
          }
      }
      __syncthreads();
      // output layer on the ALUs: thread -> (sample tid % 64, hidden units CW (tid / 64) ..)
      {
        const int smp = tid & 63, grp = tid >> 6;
        float part[NOUT];
#pragma unroll
        for (int k = 0; k < NOUT; ++k) part[k] = 0.f;
#pragma unroll 4
        for (int i = CW * grp; i < CW * grp + CW; i += 4) {  // 16-byte reads of the row (P is a multiple of 4)
          const float4 hv = *reinterpret_cast<const float4*>(&Hs[smp * P + i]);
          const float hh[4] = {hv.x, hv.y, hv.z, hv.w};
#pragma unroll
          for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int k = 0; k < NOUT; ++k) part[k] = fmaf(hh[j], W3s[(i + j) * NOUT + k], part[k]);
        }
#pragma unroll
        for (int k = 0; k < NOUT; ++k) red[(grp * BM + smp) * NOUT + k] = part[k];
      }
      __syncthreads();
      if (tid < BM) {
        float out[NOUT], dl[NOUT];
#pragma unroll
        for (int k = 0; k < NOUT; ++k) {
          float v = b3r[k];
#pragma unroll
          for (int gq = 0; gq < NWV; ++gq) v += red[(gq * BM + tid) * NOUT + k];
          out[k] = v;
          dl[k] = 0.f;
        }
        float st[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
        if (m0 + tid < a.S) fin.compute(loss_in, prep, out, dl, st);
#pragma unroll
        for (int k = 0; k < 5; ++k) accS[tid * AS + NOUT + k] += st[k];
#pragma unroll
        for (int k = 0; k < 8; ++k) dls[tid * 8 + k] = k < NOUT ? dl[k < NOUT ? k : 0] : 0.f;
#pragma unroll
        for (int k = 0; k < NOUT; ++k) accS[tid * AS + k] += dl[k];
      }
      __syncthreads();
      // C = (dl W3^T) * (1 - h^2): the rank-NOUT product runs on the matrix cores (k padded to 8) and lands in the
      // lane layout of the register-resident h
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const float4 av = *reinterpret_cast<const float4*>(&dls[(32 * i + lo) * 8 + 4 * hi]);
        const float af[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
        for (int jn = 0; jn < JN; ++jn) {
          const int n = CW * wave + 32 * jn + lo;
          float bf[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) bf[j] = (4 * hi + j < NOUT) ? W3s[n * NOUT + (4 * hi + j < NOUT ? 4 * hi + j : 0)] : 0.f;
          floatx16 gacc;
#pragma unroll
          for (int r = 0; r < 16; ++r) gacc[r] = 0.f;
#pragma unroll
          for (int j = 0; j < 4; ++j) gacc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[j], gacc, 0, 0, 0);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float h = acc[i][jn][r];
            out[(32 * i + 8 * (r / 4) + (r % 4)) * kWregN + 32 * jn] = gacc[r] * (1.0f - h * h);
          }
        }
      }
      // W3 gradient: sum_s h[s][n] dl[s][k] over the rows whose h this lane holds in registers (32 of the tile's 64 for
      // each of its two columns; the lane 32 further on holds the other half, and the two meet after the last tile).
      // Rows past the end carry dl = 0.
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = 32 * i + 8 * (r / 4) + 4 * hi + (r % 4);
          float dlv[NOUT];
#pragma unroll
          for (int k = 0; k < NOUT; ++k) dlv[k] = dls[m * 8 + k];
          if (r % 4 == 0) __builtin_amdgcn_sched_barrier(0);  // four rows' reads at a time: no more registers than that in flight
#pragma unroll
          for (int jn = 0; jn < JN; ++jn)
#pragma unroll
            for (int k = 0; k < NOUT; ++k) gw[jn][k] = fmaf(acc[i][jn][r], dlv[k], gw[jn][k]);
        }
    }
    if (tid < BM) ent[stage * BM + tid] = e2;  // this tile's entries were last read while the previous tile was multiplied
    __syncthreads();  // the other stage is complete; this one may be overwritten
  }
  if (DEFER) {  // the last tile of this workgroup
    if (EPI == WREG_DTANH) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) auxr[e] = a.aux[prev_off + elem_off(e)];
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) finish_elem(e, prev_off);
  }
  if (EPI == WREG_TANH_LOSS) {
    float* const own = a.partial3 != nullptr ? a.partial3 + (int64_t)blockIdx.x * (kWregN * NOUT + NOUT) : nullptr;
#pragma unroll
    for (int jn = 0; jn < JN; ++jn)
#pragma unroll
      for (int k = 0; k < NOUT; ++k) {
        const float v = gw[jn][k] + __shfl_xor(gw[jn][k], 32);  // the two halves of the rows
        const int n = CW * wave + 32 * jn + lo;
        if (hi == 0) {
          if (own != nullptr) own[n * NOUT + k] = v;
          else atomicAdd(&a.gW3[n * NOUT + k], v);
        }
      }
    if (wave == 0) {  // samples live in threads tid < 64
#pragma unroll
      for (int k = 0; k < NOUT; ++k) {
        float v = accS[tid * AS + k];
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if (lane == 0) {
          if (own != nullptr) own[kWregN * NOUT + k] = v;
          else atomicAdd(&a.gb3[k], v);
        }
      }
#pragma unroll
      for (int k = 0; k < 5; ++k) {
        float v = accS[tid * AS + NOUT + k];
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if (lane == 0 && v != 0.f) atomicAdd(&a.stats[k], v);
      }
    }
  }
}

template <int K, int EPI, int NOUT = 1, class Fin = WregNoFinish, int NWV = 4>
inline int32_t launch_wreg_gemm_inst(const WregArgs& a, hipStream_t s, const Fin& fin = Fin()) {
  auto kern = wreg_gemm_kernel<K, EPI, NOUT, Fin, NWV>;
  static bool configured = false;  // per instantiation
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
      return MARL_E_LAUNCH;
    configured = true;
  }
  const int64_t tiles = (a.S + kWregBM - 1) / kWregBM;
  const size_t lds = WregShape<K>::lds_bytes + (EPI == WREG_TANH_LOSS ? WregShape<K>::loss_lds_bytes(NOUT, NWV) : 0);
  hipLaunchKernelGGL(kern, dim3((unsigned)std::min<int64_t>(tiles, 256)), dim3(64 * NWV), lds, s, a, fin);
  return MARL_OK;
}

// Shapes this kernel serves: 256 output columns, 16-byte aligned rows, a contraction of at most 304 for
// WREG_BIAS_TANH and of at most 256 otherwise (WREG_DTANH keeps its prefetched operand in the registers the longer
// contraction would take; WREG_TANH_LOSS reuses the stage of A for the 256-wide activation tile).
template <int EPI>
inline bool wreg_gemm_supported(const RowSrc& A, int Kin, int N) {
  return N == kWregN && Kin <= (EPI == WREG_BIAS_TANH ? 304 : 256) && Kin % 4 == 0 && A.ld % 4 == 0 && aligned16(A.base);
}

template <int EPI>
inline int32_t launch_wreg_gemm(const WregArgs& a, hipStream_t s) {
  static_assert(EPI != WREG_TANH_LOSS, "launch_wreg_loss");
  // Wavefronts per workgroup, by measurement at 262 144 rows: the padded contraction (no registers for the deferred
  // epilogue either way) gains from two wavefronts per SIMD taking turns on the matrix core (368 -> 346 us); the
  // kernels that finish a tile inside the next tile's products are faster with one (299 against 343 us).
  if (EPI == WREG_DTANH || a.Kin <= 256) return launch_wreg_gemm_inst<256, EPI, 1, WregNoFinish, 4>(a, s);
  return launch_wreg_gemm_inst<EPI == WREG_DTANH ? 256 : 304, EPI, 1, WregNoFinish, 8>(a, s);
}

template <int NOUT, class Fin>
inline int32_t launch_wreg_loss(const WregArgs& a, const Fin& fin, hipStream_t s) {
  // eight wavefronts: the barrier-separated phases of its epilogue are latency chains that a second wavefront per SIMD
  // fills (371 -> 336 us at 262 144 rows)
  return launch_wreg_gemm_inst<256, WREG_TANH_LOSS, NOUT, Fin, 8>(a, s, fin);
}

// ---------------------------------------------------------------------------------------------------------------
// The transposed product of the backward pass with the OUTPUT resident in registers:
//
//   C[m][n] += sum_s A[s][m] * B[s][n],   m < MIN <= 320, n < 256, s < S (hundreds of thousands of rows)
//
// A weight gradient of 320 x 256 floats fits the accumulators of one workgroup (wavefront w owns columns
// 64 w .. 64 w + 63 of all rows: MT x 2 tiles of 32 x 32, 32 MT registers per lane).  The workgroup is persistent over
// tiles of 32 rows of A and B, which travel global -> registers -> LDS (two stages) while the previous tile is
// multiplied; at the end every workgroup adds its partial sum to C with fp32 atomics.  Column sums of B (the bias
// gradient) ride along in the staging registers.
// ---------------------------------------------------------------------------------------------------------------
struct WaccArgs {
  RowSrc A;       // S rows of MIN floats (optionally gathered); rows 16-byte aligned
  int64_t S;
  const float* B;  // [S][256]
  float* C;        // [MIN][256], accumulated
  float* colsum;   // nullable [256]: column sums of B, accumulated
  // Two-stage reduction (nullable): workgroup b stores its partial results -- MIN x 256 of C, then the 256 column sums --
  // at partial + b * (MIN + 1) * 256 with plain stores, and the caller adds the copies up afterwards
  // (reduce_partials_kernel); colsum must then directly follow C in memory.  Without it every workgroup adds to C with
  // atomics, and a few hundred workgroups doing that to the same cache lines at the same moment queue up at the L2.
  float* partial;
};

constexpr int kWaccMaxGrid = 256;  // workgroups of a launch (the copies a caller's `partial` has room for)

template <int MIN, int WM>
struct WaccShape {
  static constexpr int NT = 256 * WM;           // threads: WM x 4 wavefronts
  static constexpr int BS = 32;                 // rows (the contraction) per tile
  static constexpr int MT = (MIN + 31) / 32;    // 32-row tiles of the output
  static constexpr int MTW = MT / WM;           // ... of one wavefront
  static constexpr int PA = 32 * MT + 4;        // pitch of the A tile (covers the padded output rows)
  static constexpr int PB = kWregN + 4;
  static constexpr int VA = MIN / 4;            // 16-byte vectors per row of A
  static constexpr int TOT_A = (BS * VA + NT - 1) / NT;
  static constexpr int TOT_B = BS * (kWregN / 4) / NT;
  static constexpr size_t lds_bytes = sizeof(float) * 2 * BS * (PA + PB) + sizeof(int64_t) * 2 * BS;
  static_assert(MIN % 4 == 0 && MT % WM == 0 && MTW * 32 <= 256, "whole 16-byte vectors; the accumulators of a wavefront fit its registers");
};

// WM = 1: four wavefronts, each all MT row tiles of its 64 columns (up to 256 accumulator registers, one wavefront
// per SIMD).  WM = 2: eight wavefronts, each half of the row tiles (two wavefronts per SIMD, 256 registers each).
template <int MIN, int WM>
__global__ void __launch_bounds__(256 * WM, 1) wacc_gemm_kernel(WaccArgs a) {
  using Sh = WaccShape<MIN, WM>;
  constexpr int NT = Sh::NT, BS = Sh::BS, MTW = Sh::MTW, PA = Sh::PA, PB = Sh::PB, VA = Sh::VA, TOT_A = Sh::TOT_A, TOT_B = Sh::TOT_B;
  extern __shared__ __attribute__((aligned(16))) unsigned char wreg_smem[];
  float* const As = reinterpret_cast<float*>(wreg_smem);             // [2][BS][PA]
  float* const Bs = As + 2 * BS * PA;                                 // [2][BS][PB]
  int64_t* const ent = reinterpret_cast<int64_t*>(Bs + 2 * BS * PB);  // [2][BS] offsets (floats) of a tile's rows of A

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave & 3, wm = wave >> 2;
  const int lo = lane & 31, hi = lane >> 5;
  const int64_t ntiles = (a.S + BS - 1) / BS;

  // columns of the A tiles past MIN are never staged: they feed output rows that are never stored, zero all the same
  for (int i = tid; i < 2 * BS * PA; i += NT) As[i] = 0.f;

  // The next tile moves in two halves through one set of registers: its rows of A are requested when a tile's
  // products start and stored half-way, its rows of B are requested then and stored at the end.
  constexpr int TOT_MAX = TOT_A > TOT_B ? TOT_A : TOT_B;
  float4 stg[TOT_MAX];
  float4 bsum = make_float4(0.f, 0.f, 0.f, 0.f);
  auto fetch_a = [&](int64_t tile, int slot) {
#pragma unroll
    for (int q = 0; q < TOT_A; ++q) {
      const int f = tid + NT * q;
      if (f < BS * VA) {
        const int r = f / VA, c = 4 * (f % VA);
        // (unconditional: the entries of rows past the end point at the last row, and those rows of B are zero -- a
        // load under a branch of its own is waited for before the next one is issued, one memory latency per load)
        stg[q] = *reinterpret_cast<const float4*>(a.A.base + ent[slot * BS + r] + c);
      }
    }
  };
  auto store_a = [&](int stage) {
#pragma unroll
    for (int q = 0; q < TOT_A; ++q) {
      const int f = tid + NT * q;
      if (f < BS * VA) *reinterpret_cast<float4*>(&As[(stage * BS + f / VA) * PA + 4 * (f % VA)]) = stg[q];
    }
  };
  auto fetch_b = [&](int64_t tile) {
#pragma unroll
    for (int q = 0; q < TOT_B; ++q) {
      const int f = tid + NT * q;
      const int r = f / (kWregN / 4), c = 4 * (f % (kWregN / 4));
      const int64_t row = tile * BS + r;
      float4 v = *reinterpret_cast<const float4*>(a.B + min(row, a.S - 1) * kWregN + c);
      if (row >= a.S) v = make_float4(0.f, 0.f, 0.f, 0.f);
      stg[q] = v;
    }
  };
  auto store_b = [&](int stage) {
#pragma unroll
    for (int q = 0; q < TOT_B; ++q) {
      const int f = tid + NT * q;
      *reinterpret_cast<float4*>(&Bs[(stage * BS + f / (kWregN / 4)) * PB + 4 * (f % (kWregN / 4))]) = stg[q];
      bsum.x += stg[q].x; bsum.y += stg[q].y; bsum.z += stg[q].z; bsum.w += stg[q].w;  // this thread's columns: 4 (tid % 64) ..
    }
  };
  auto load_entries = [&](int64_t tile) -> int64_t {
    if (tid >= BS || tile >= ntiles) return 0;
    const int64_t row = min(tile * BS + tid, a.S - 1);
    return a.A.ptr(row) - a.A.base;
  };

  floatx16 acc[MTW][2];
#pragma unroll
  for (int mi = 0; mi < MTW; ++mi)
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][jn][r] = 0.f;

  int64_t tile = blockIdx.x;
  if (tile < ntiles) {
    const int64_t e0 = load_entries(tile), e1 = load_entries(tile + gridDim.x);
    if (tid < BS) {
      ent[0 * BS + tid] = e0;
      ent[1 * BS + tid] = e1;
    }
    __syncthreads();  // also orders the zero fill before the first staging stores
    fetch_a(tile, 0);
    store_a(0);
    fetch_b(tile);
    store_b(0);
    __syncthreads();
  }

  int it = 0;
  for (; tile < ntiles; tile += gridDim.x, ++it) {
    const int stage = it & 1;
    const int64_t next = tile + gridDim.x;
    const bool has_next = next < ntiles;  // uniform
    const int64_t e2 = load_entries(next + gridDim.x);
    const float* const At = As + stage * BS * PA + 32 * MTW * wm;
    const float* const Bt = Bs + stage * BS * PB + 64 * wn;
    if (has_next) fetch_a(next, stage ^ 1);
#pragma unroll
    for (int t = 0; t < BS / 2; ++t) {  // matrix-core step t contracts rows 2 t and 2 t + 1 of the tile
      float af[MTW], bf[2];
#pragma unroll
      for (int mi = 0; mi < MTW; ++mi) af[mi] = At[(2 * t + hi) * PA + 32 * mi + lo];
#pragma unroll
      for (int jn = 0; jn < 2; ++jn) bf[jn] = Bt[(2 * t + hi) * PB + 32 * jn + lo];
#pragma unroll
      for (int mi = 0; mi < MTW; ++mi)
#pragma unroll
        for (int jn = 0; jn < 2; ++jn) acc[mi][jn] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[mi], bf[jn], acc[mi][jn], 0, 0, 0);
      if (t == BS / 4 - 1 && has_next) {
        store_a(stage ^ 1);
        fetch_b(next);
      }
    }
    if (has_next) store_b(stage ^ 1);
    if (tid < BS) ent[stage * BS + tid] = e2;
    __syncthreads();
  }

  // ---- this workgroup's partial sums
#pragma unroll
  for (int mi = 0; mi < MTW; ++mi)
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = 32 * (MTW * wm + mi) + 8 * (r / 4) + 4 * hi + (r % 4);
        if (m < MIN) {
          if (a.partial != nullptr) a.partial[(int64_t)blockIdx.x * (MIN + 1) * kWregN + m * kWregN + 64 * wn + 32 * jn + lo] = acc[mi][jn][r];
          else atomicAdd(&a.C[m * kWregN + 64 * wn + 32 * jn + lo], acc[mi][jn][r]);
        }
      }
  if (a.colsum != nullptr) {
    float4* red = reinterpret_cast<float4*>(Bs);  // the loop ended with a barrier
    red[tid] = bsum;
    __syncthreads();
    if (tid < 64) {
      float4 v = red[tid];
#pragma unroll
      for (int q = 1; q < NT / 64; ++q) {
        const float4 o = red[tid + 64 * q];
        v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
      }
      if (a.partial != nullptr) {
        *reinterpret_cast<float4*>(a.partial + (int64_t)blockIdx.x * (MIN + 1) * kWregN + MIN * kWregN + 4 * tid) = v;
      } else {
        float* dst = a.colsum + 4 * tid;
        atomicAdd(dst + 0, v.x); atomicAdd(dst + 1, v.y); atomicAdd(dst + 2, v.z); atomicAdd(dst + 3, v.w);
      }
    }
  }
}

template <int MIN, int WM>
inline int32_t launch_wacc_gemm_inst(const WaccArgs& a, hipStream_t s) {
  using Sh = WaccShape<MIN, WM>;
  auto kern = wacc_gemm_kernel<MIN, WM>;
  static bool configured = false;  // per instantiation
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
      return MARL_E_LAUNCH;
    configured = true;
  }
  const int64_t tiles = (a.S + Sh::BS - 1) / Sh::BS;
  const unsigned grid = (unsigned)std::min<int64_t>(tiles, kWaccMaxGrid);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(Sh::NT), Sh::lds_bytes, s, a);
  if (a.partial != nullptr) launch_reduce_partials(a.partial, (int)grid, (int64_t)(MIN + 1) * kWregN, a.C, s);  // C and the column sums behind it
  return MARL_OK;
}

// The instantiated shape: 256 columns and the 300 output rows of the centralised critic's first layer (4 x 75 inputs),
// eight wavefronts.  (For 256 output rows the split-k tile kernel of gemm.h measured faster: 310 against 361 us per
// 262 144 rows, with either four or eight wavefronts here.)
inline bool wacc_gemm_supported(const RowSrc& A, int M, int N) {
  return N == kWregN && M == 300 && A.ld % 4 == 0 && aligned16(A.base);
}

inline int32_t launch_wacc_gemm(const WaccArgs& a, int M, hipStream_t s) {
  if (M != 300) return MARL_E_CONFIG;  // the only instantiated shape; callers ask wacc_gemm_supported first
  return launch_wacc_gemm_inst<300, 2>(a, s);
}

}  // namespace marl
