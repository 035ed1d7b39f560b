// Whole-network training pass for the small networks (hidden width 64 or 128, input width <= 93):
// forward, PPO loss, and the complete backward pass of one network in ONE kernel.  Nothing but the
// observations and a few scalars per sample is read from HBM and nothing but the parameter gradient is
// written: h1, h2, dz2, dz1 live in LDS / registers for the lifetime of a row tile, and the weight
// gradients are accumulated in registers over all row tiles a workgroup owns.
//
// Workgroup = 8 wavefronts, persistent, one per CU.  Row tile = BM samples (64 at H = 128, 128 at H = 64), so
// that a layer output is 8 MFMA tiles of 32x32, one per wavefront.  The three products against weights (layer 1,
// layer 2, dz1) take their A operand from the tile in LDS and their B operand from registers: the weights of a whole
// product are requested one phase ahead (buffer loads from the operand-order copies, L2-resident; see PhaseW in
// gemm.h), so there is no weight staging buffer, no barrier inside a layer and no wait for the L2 inside a product.
// Per tile:
//   layer 1 -> h1 (LDS) | layer 2 -> h2 (registers + LDS) |
//   output layer on the ALUs -> loss -> dL/dout | W3 gradient | dz2 = (dL/dout W3^T)(1-h2^2) -> LDS |
//   dW2 += h1^T dz2 | dz1 = (dz2 W2^T)(1-h1^2) -> LDS, next tile's X -> LDS | dW1 += X^T dz1
// (two X tiles where LDS allows; otherwise a tile starts with its own X -> LDS phase).  The inputs of later tiles are
// requested for every tile slot, without conditions, far ahead of their use: the loss inputs of the next tile and the
// gather entries of the tile after it right after the loss, the next tile's observation rows (as the aligned 16-byte
// chunks that cover each row) after layer 2 -- no load is waited for where it is issued, and none sits in front of a
// load that is.  At the end a workgroup stores its partial gradient into a copy of its own, every sum in a fixed
// order; reduce_partials_kernel adds the copies.
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
  const float *W1s, *W2s, *W2Ts;             // operand-order copies: (k, n) at ((k / 4) * H + n) * 4 + k % 4; W1s zero-padded to 16-row groups
  float *gW1, *gb1, *gW2, *gb2, *gW3, *gb3;  // gradient blocks, accumulated with atomics
  float* stats;                              // 5 floats, atomics
  // Two-stage reduction of the gradient (nullable): the six blocks above are one contiguous range of `gcount` floats
  // starting at gW1; workgroup b writes its sums into its own copy of that range at partial + b * gcount
  // and reduce_partials_kernel adds the copies to the gradient afterwards.  Several hundred workgroups adding
  // to the same few hundred cache lines at the same moment is what the direct atomics cost: 60-180 us per launch.
  float* partial;
  int64_t gcount;
  int64_t pstride;  // distance between the copies of consecutive workgroups (0: gcount)
};

// Floats of LDS the kernel lays out for a tile of BM samples at X pitch px with `xtiles` X tiles.
constexpr size_t fused_train_lds_floats(int H, int BM, int NOUT, int NW, int px, int xtiles) {
  return (size_t)xtiles * BM * px + 2 * (size_t)BM * (H + 4) + 64 * (size_t)NW * NOUT + BM * 8 + H * NOUT + 4 + 8 +
         (size_t)(BM < 64 ? 64 : BM) * (NOUT + 5);
}

// acc[q] += A^T B_q over the samples kb0 .. kb0 + klen of a row tile held in LDS: A column block at Ap (pitch pa),
// B column blocks at Bp + 32 q (pitch pb).  The operands of the next k step are read before the MFMAs of the
// current one are issued, so the LDS latency hides behind the matrix pipe even with one wavefront per SIMD.
template <int NB>
__device__ __forceinline__ void outer_product_accumulate(const float* __restrict__ Ap, int pa, const float* __restrict__ Bp,
                                                         int pb, int kb0, int klen, int hi, floatx16* acc) {
  float af[4], bf[NB][4];
  auto read = [&](int kb, float (&x)[4], float (&y)[NB][4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      x[j] = Ap[(kb + 4 * hi + j) * pa];
#pragma unroll
      for (int q = 0; q < NB; ++q) y[q][j] = Bp[(kb + 4 * hi + j) * pb + 32 * q];
    }
  };
  read(kb0, af, bf);
#pragma unroll 2
  for (int kb = kb0; kb < kb0 + klen; kb += 8) {
    float an[4], bn[NB][4];
    const int kn = kb + 8 < kb0 + klen ? kb + 8 : kb;  // the last step re-reads its own operands
    read(kn, an, bn);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int q = 0; q < NB; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[q][j], acc[q], 0, 0, 0);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      af[j] = an[j];
#pragma unroll
      for (int q = 0; q < NB; ++q) bf[q][j] = bn[q][j];
    }
  }
}

// acc[q] += A_q^T B over the samples kb0 .. kb0 + klen: the NA row blocks A_q at Ap + 32 q (pitch pa) share the
// column block B at Bp (pitch pb).  NA independent accumulation chains keep the matrix pipe fed from one wavefront.
template <int NA>
__device__ __forceinline__ void outer_product_accumulate_rows(const float* __restrict__ Ap, int pa, const float* __restrict__ Bp,
                                                              int pb, int kb0, int klen, int hi, floatx16* acc) {
  float af[NA][4], bf[4];
  auto read = [&](int kb, float (&x)[NA][4], float (&y)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      y[j] = Bp[(kb + 4 * hi + j) * pb];
#pragma unroll
      for (int q = 0; q < NA; ++q) x[q][j] = Ap[(kb + 4 * hi + j) * pa + 32 * q];
    }
  };
  read(kb0, af, bf);
#pragma unroll 2
  for (int kb = kb0; kb < kb0 + klen; kb += 8) {
    float an[NA][4], bn[4];
    const int kn = kb + 8 < kb0 + klen ? kb + 8 : kb;  // the last step re-reads its own operands
    read(kn, an, bn);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int q = 0; q < NA; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[q][j], bf[j], acc[q], 0, 0, 0);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf[j] = bn[j];
#pragma unroll
      for (int q = 0; q < NA; ++q) af[q][j] = an[q][j];
    }
  }
}

// The kernel's body: workgroup `bid` of `nblk` that share the tiles of one network's minibatch.
template <int H, int BM, int NOUT, int DMAX, int NW, class LossFn>
__device__ __forceinline__ void fused_train_body(const FusedTrainArgs& a, const LossFn& fn, const unsigned bid, const unsigned nblk) {
  constexpr int NT = 64 * NW;
  constexpr int NTN = H / 32, MTF = BM / 32, PH = H + 4, GROUPS = NT / BM;
  static_assert(NTN * MTF == NW, "one forward tile per wavefront");
  constexpr int TPR = NT / BM;           // threads staging one row of X
  constexpr int XV = DMAX / TPR / 4;     // 16-byte chunks of an X row per thread
  static_assert(DMAX % (4 * TPR) == 0, "whole chunks per thread");
  constexpr int DW2_TPW = NTN * NTN >= NW ? NTN * NTN / NW : 1;  // dW2 tiles per wavefront (one row of tiles at most)
  constexpr int DW2_KS = NTN * NTN >= NW ? 1 : NW / (NTN * NTN);  // split of the sample range when there are fewer tiles than wavefronts
  static_assert(DW2_TPW <= NTN && NTN % DW2_TPW == 0, "a wavefront's dW2 tiles share their row of tiles");
  // dW1: wavefront -> (column tile wave % NTN of the gradient, share wave / NTN of the tile's samples); it holds all
  // Q1 row tiles of that column (they share the dz1 operand), Q1 independent accumulation chains
  constexpr int Q1 = DMAX / 32, KS1 = NW / NTN, KLEN1 = BM / KS1;
  static_assert(NW % NTN == 0 && BM % KS1 == 0 && KLEN1 % 8 == 0, "dW1 sample shares");
  constexpr int HPARTS = NT / H, SPP = BM / HPARTS;
  constexpr int KG1 = DMAX / 16, KG2 = H / 16;  // k groups of layer 1 (at most) and of the H-deep products

  // Two X tiles when they fit: the next tile's rows then go to LDS inside the dz1 epilogue of the current one (the
  // loads were requested after layer 2), and a tile starts with layer 1 instead of a staging phase and its barrier.
  constexpr bool XDB = fused_train_lds_floats(H, BM, NOUT, NW, DMAX + 4, 2) * 4 <= 160 * 1024;
  extern __shared__ __attribute__((aligned(16))) float lds[];
  float* const Xs0 = lds;                  // [XDB ? 2 : 1][BM][px]
  float* H1 = Xs0 + (XDB ? 2 : 1) * BM * a.px;  // [BM][PH]  h1, later dz1
  float* H2 = H1 + BM * PH;                // [BM][PH]  h2, later dz2
  float* red = H2 + BM * PH;               // [GROUPS][NOUT][BM]
  float* dls = red + NT * NOUT;           // [BM][8]
  float* W3s = dls + BM * 8;               // [H][NOUT]
  float* const xdump = W3s + H * NOUT;     // one float: where the staged values that are not part of a row go
  float* const b3s = xdump + 4;            // [8] the output layer's bias
  // per-sample-slot sums that only the first BM threads touch, once per tile (b3 gradient, loss statistics): in LDS
  // rather than in 11 registers of every thread, which this kernel does not have to spare
  constexpr int AS = NOUT + 5;
  float* const accS = b3s + 8;             // [max(BM, 64)][AS]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = lane & 31, hi = lane >> 5;
  const int mt = wave / NTN, nt = wave % NTN;  // forward / dz tile of this wavefront
  // where this workgroup's gradient goes: the gradient itself, or its own copy of the range
  float* const gout = a.partial != nullptr ? a.partial + (int64_t)bid * (a.pstride != 0 ? a.pstride : a.gcount) : a.gW1;
  // (a copy needs no zeroing: the flush at the end writes every one of its elements exactly once)
  float* const gW1 = gout;
  float* const gb1 = gout + (a.gb1 - a.gW1);
  float* const gW2 = gout + (a.gW2 - a.gW1);
  float* const gb2 = gout + (a.gb2 - a.gW1);
  float* const gW3 = gout + (a.gW3 - a.gW1);
  float* const gb3 = gout + (a.gb3 - a.gW1);
  const int px = a.px;
  for (int i = tid; i < (XDB ? 2 : 1) * BM * px; i += NT) Xs0[i] = 0.f;  // the padding columns stay zero for good
  for (int i = tid; i < H * NOUT; i += NT) W3s[i] = a.W3[i];
  if (tid < NOUT) b3s[tid] = a.b3[tid];
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
  float gw[NOUT];
#pragma unroll
  for (int k = 0; k < NOUT; ++k) gw[k] = 0.f;
  for (int i = tid; i < (BM < 64 ? 64 : BM) * AS; i += NT) accS[i] = 0.f;  // ordered before its first use by the barriers below
  float gb1r = 0.f, gb2r = 0.f;  // bias gradients of column nt*32+lo (lanes hi == 0)
  // the biases of this lane's column, once: a load inside the tile loop would be waited for on the spot, and with it
  // (loads return in order) the next tile's rows requested just before
  const float bias1 = a.b1[nt * 32 + lo], bias2 = a.b2[nt * 32 + lo];
  const int kpad1 = 16 * ((a.Din + 15) / 16);  // layer 1 contracts over the input width rounded up to a k group (W1 is zero-padded to it)
  const int wlane = (hi * H + nt * 32 + lo) * 4;  // this lane's 16 bytes of k quad `hi` in an operand-order weight copy
  const WeightRsrc rsW1 = weight_rsrc(a.W1s, kpad1 * H), rsW2 = weight_rsrc(a.W2s, H * H), rsW2T = weight_rsrc(a.W2Ts, H * H);

  // ---- staging helpers.  The inputs of the next tile come in two steps: the gather entries at the top of a
  // tile, the rows themselves half a tile later, so that neither dependent load is ever waited for.
  // A row of X starts at any 4-byte boundary (its width need not be a multiple of four), so it is fetched as the
  // aligned 16-byte chunks that cover it -- a few wide loads per thread instead of one 4-byte load per element,
  // which the address path serves no faster -- and sorted out on the way into LDS: element j of chunk q is column
  // 4 q + j - xoff of the row, xoff being where the row starts inside its first chunk.  (The base of X is 16-byte
  // aligned and rows before / after a row exist, so the chunks never leave the buffer.)
  float4 xr[XV];
  int xoff = 0;
  typename LossFn::In lin_next{};
  int32_t xentry = 0, lentry = 0;
  const int xrow_l = tid / TPR, xcol0 = tid % TPR;
  const auto prep = fn.prepare();
  // These requests are issued for every tile slot, also past a workgroup's last tile (row indices are clamped to the
  // last sample and the values never used): with the same loads in every iteration the compiler can count the loads
  // in flight and wait for exactly the ones it needs, where a conditional request makes every wait a wait for all.
  auto fetch_tile_entries = [&](int64_t s0) {
    xentry = a.X.template gather_entry<true>(min(s0 + xrow_l, a.S - 1));
    if (tid < BM) lentry = fn.template row_entry<true>(min(s0 + tid, a.S - 1));
  };
  auto fetch_tile_inputs = [&](int64_t s0) {
    const float* const row = a.X.template ptr_with<true>(min(s0 + xrow_l, a.S - 1), xentry);
    xoff = (int)((reinterpret_cast<uintptr_t>(row) >> 2) & 3);
    // (pointer arithmetic, not an integer round trip: the loads stay global loads -- a flat load also counts as an
    // LDS operation, and every barrier would wait for these rows)
    const float4* const chunk = reinterpret_cast<const float4*>(row - xoff);
    const int last = ((xoff + a.Din + 3) >> 2) - 1;  // chunks past the row: the last one again (none of its elements is stored)
#pragma unroll
    for (int p = 0; p < XV; ++p) xr[p] = chunk[min(xcol0 + TPR * p, last)];
  };
  // (the loss inputs of the next tile are requested right after the loss of the current one, into the same registers)
  auto fetch_tile_loss_inputs = [&](int64_t s0) {
    if (tid < BM) lin_next = fn.template load_with<true>(min(s0 + tid, a.S - 1), lentry);
  };
  auto store_tile_inputs = [&](float* Xdst) {
    float* const xdst = Xdst + xrow_l * px - xoff;
#pragma unroll
    for (int p = 0; p < XV; ++p) {
      const float v[4] = {xr[p].x, xr[p].y, xr[p].z, xr[p].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = 4 * (xcol0 + TPR * p) + j - xoff;
        float* const dst = (c >= 0 && c < a.Din) ? xdst + 4 * (xcol0 + TPR * p) + j : xdump;
        *dst = v[j];
      }
    }
  };
  const int64_t ntiles = (a.S + BM - 1) / BM;
  int64_t tile = bid;
  if (tile < ntiles) {
    fetch_tile_entries(tile * BM);
    fetch_tile_inputs(tile * BM);
    fetch_tile_loss_inputs(tile * BM);
    fetch_tile_entries((tile + nblk) * BM);
  }
#ifdef MARL_PHASE_TIMERS
  long long phase_t0_ = (long long)__builtin_amdgcn_s_memtime();
#endif
  if (XDB && tile < ntiles) {
    store_tile_inputs(Xs0);
    __syncthreads();
  }
  PhaseW<KG1> pw1;  // layer 1's weights: the first half requested before dW1 of the tile before (here for the first tile)
  phase_w_request<H, KG1, 0, KG1 / 2>(pw1, rsW1, wlane, kpad1 / 16);
  for (int it = 0; tile < ntiles; tile += nblk, ++it) {
    const int64_t s0 = tile * BM;
    const bool have_next = tile + nblk < ntiles;
    float* const Xs = XDB ? Xs0 + (it & 1) * BM * px : Xs0;
    if (!XDB) {  // ---- this tile's observations to LDS
      store_tile_inputs(Xs);
    }
    if (!XDB) __syncthreads();

    PHASE_MARK(0);
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    // ---- layer 1
    phase_w_request<H, KG1, KG1 / 2, KG1>(pw1, rsW1, wlane, kpad1 / 16);
    gemm_phase_w<KG1>(Xs + (mt * 32 + lo) * px + 4 * hi, kpad1 / 16, acc, pw1);
    PhaseW<KG2> pw2;  // layer 2's weights arrive during the tanh epilogue of layer 1
    phase_w_request<H, KG2>(pw2, rsW2, wlane, KG2);
    PHASE_MARK(1);
    {
      const int n = nt * 32 + lo;
      const float bias = bias1;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        float v = tanh_f32(acc[r] + bias);
        H1[m * PH + n] = v;
        acc[r] = 0.f;
        if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);
      }
    }
    PHASE_MARK(2);
    // ---- layer 2
    __syncthreads();  // the h1 tile is complete
    gemm_phase_w<KG2>(H1 + (mt * 32 + lo) * PH + 4 * hi, KG2, acc, pw2);
    PHASE_MARK(3);
    fetch_tile_inputs((tile + nblk) * BM);  // lands during the ALU phases and dW2
    floatx16 h2r;  // h2 of this wavefront's tile
    {
      const int n = nt * 32 + lo;
      const float bias = bias2;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        float v = tanh_f32(acc[r] + bias);
        h2r[r] = v;
        H2[m * PH + n] = v;
        if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();
    PHASE_MARK(4);
    // ---- output layer on the ALUs: thread -> (sample tid % BM, slice tid / BM of the hidden units); 16-byte LDS reads
    {
      const int s = tid % BM, grp = tid / BM;
      constexpr int PER = H / GROUPS;
      static_assert(PER % 4 == 0, "hidden units are read four at a time");
      float part[NOUT];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) part[k] = 0.f;
#pragma unroll 2
      for (int i = grp * PER; i < (grp + 1) * PER; i += 4) {
        const float4 hv = *reinterpret_cast<const float4*>(&H2[s * PH + i]);
        const float hh[4] = {hv.x, hv.y, hv.z, hv.w};
        float wv[4 * NOUT];  // W3 rows i..i+3: 4 * NOUT consecutive floats, the same for every lane of the wavefront
#pragma unroll
        for (int q = 0; q < NOUT; ++q) {
          const float4 t = *reinterpret_cast<const float4*>(&W3s[i * NOUT + 4 * q]);
          wv[4 * q] = t.x; wv[4 * q + 1] = t.y; wv[4 * q + 2] = t.z; wv[4 * q + 3] = t.w;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int k = 0; k < NOUT; ++k) part[k] = fmaf(hh[j], wv[j * NOUT + k], part[k]);
      }
#pragma unroll
      for (int k = 0; k < NOUT; ++k) red[(grp * NOUT + k) * BM + s] = part[k];
    }
    __syncthreads();
    PHASE_MARK(5);
    if (tid < BM) {
      float out[NOUT], dl[NOUT];
#pragma unroll
      for (int k = 0; k < NOUT; ++k) {
        float v = b3s[k];
#pragma unroll
        for (int gq = 0; gq < GROUPS; ++gq) v += red[(gq * NOUT + k) * BM + tid];
        out[k] = v;
        dl[k] = 0.f;
      }
      float st[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
      if (s0 + tid < a.S) fn.compute(lin_next, prep, out, dl, st);
      float d8[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) d8[k] = k < NOUT ? dl[k < NOUT ? k : 0] : 0.f;
      *reinterpret_cast<float4*>(&dls[tid * 8]) = make_float4(d8[0], d8[1], d8[2], d8[3]);
      *reinterpret_cast<float4*>(&dls[tid * 8 + 4]) = make_float4(d8[4], d8[5], d8[6], d8[7]);
#pragma unroll
      for (int k = 0; k < NOUT; ++k) accS[tid * AS + k] += dl[k];
#pragma unroll
      for (int k = 0; k < 5; ++k) accS[tid * AS + NOUT + k] += st[k];
    }
    fetch_tile_loss_inputs((tile + nblk) * BM);
    // the gather entries of the tile after the next: requested here, where the next wait on a global load (the weights
    // of the dz1 product) is a whole dW2 phase away, and not in front of layer 1, whose first in-loop weight group
    // would wait for them (loads return in order)
    fetch_tile_entries((tile + 2 * (int64_t)nblk) * BM);
    __syncthreads();
    PHASE_MARK(6);
    // ---- W3 gradient: gW3[i][k] += sum_s h2[s][i] dl[s][k]   (thread -> hidden unit tid % H, a share of the samples)
    {
      const int i = tid % H, part = tid / H;
#pragma unroll 4
      for (int s = part * SPP; s < (part + 1) * SPP; ++s) {
        const float h = H2[s * PH + i];
        const float4 d0 = *reinterpret_cast<const float4*>(&dls[s * 8]);
        float dv[8] = {d0.x, d0.y, d0.z, d0.w, 0.f, 0.f, 0.f, 0.f};
        if (NOUT > 4) {
          const float4 d1 = *reinterpret_cast<const float4*>(&dls[s * 8 + 4]);
          dv[4] = d1.x; dv[5] = d1.y; dv[6] = d1.z; dv[7] = d1.w;
        }
#pragma unroll
        for (int k = 0; k < NOUT; ++k) gw[k] = fmaf(h, dv[k], gw[k]);
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
        H2[m * PH + n] = v;
        csum += v;
      }
      csum += __shfl_xor(csum, 32);
      gb2r += csum;
    }
    __syncthreads();
    PHASE_MARK(8);
    PhaseW<KG2> pwz;  // the weights of the dz1 product arrive during dW2, whose operands are all in LDS
    phase_w_request<H, KG2>(pwz, rsW2T, wlane, KG2);
    // ---- dW2 += h1^T dz2   (k runs over the samples of the tile)
    {
      const int t0 = (wave * DW2_TPW) % (NTN * NTN);
      const int it = t0 / NTN, jt = t0 % NTN;
      const int ks = (wave * DW2_TPW) / (NTN * NTN);
      constexpr int KLEN = BM / DW2_KS;
      outer_product_accumulate<DW2_TPW>(H1 + it * 32 + lo, PH, H2 + jt * 32 + lo, PH, ks * KLEN, KLEN, hi, acc2);
    }
    PHASE_MARK(9);
    // ---- dz1 = (dz2 W2^T) * (1 - h1^2), in place over h1
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    gemm_phase_w<KG2>(H2 + (mt * 32 + lo) * PH + 4 * hi, KG2, acc, pwz);
    __syncthreads();  // every wavefront is done reading h1 (dW2) before its tiles are overwritten
    PHASE_MARK(10);
    {
      const int n = nt * 32 + lo;
      float csum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mt * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        const float h = H1[m * PH + n];
        float v = acc[r] * (1.0f - h * h);
        H1[m * PH + n] = v;  // only this wavefront touches its tile of h1 from here on until the barrier
        csum += v;
      }
      csum += __shfl_xor(csum, 32);
      gb1r += csum;
    }
    if (XDB && have_next) store_tile_inputs(Xs0 + ((it & 1) ^ 1) * BM * px);  // the next tile's observations
    __syncthreads();
    PHASE_MARK(11);
    // ---- dW1 += X^T dz1   (the next tile's layer-1 weights arrive meanwhile)
    phase_w_request<H, KG1, 0, KG1 / 2>(pw1, rsW1, wlane, kpad1 / 16);
    outer_product_accumulate_rows<Q1>(Xs + lo, px, H1 + (wave % NTN) * 32 + lo, PH, (wave / NTN) * KLEN1, KLEN1, hi, acc1);
    PHASE_MARK(12);
    __syncthreads();  // the tile buffers are reused by the next row tile
    PHASE_MARK(13);
  }

  // ---- flush the register-resident gradients.  Into the workgroup's own copy (a.partial): where several wavefronts
  // (or threads) hold parts of one sum, the parts of all but the first contributor go through LDS (the tile buffers
  // are free now) and the first contributor adds them in a FIXED order before one plain store, so that the copy --
  // and, with the fixed-order reduction of the copies, the gradient -- comes out the same bits in every run.  Without
  // a copy the parts meet in atomics on the gradient itself.
  const bool own = a.partial != nullptr;
  float* const L = lds;  // staging: at most NW tiles of 32 x 32 (the last barrier of the tile loop has passed)
  static_assert(NW * 1024 <= BM * (2 * (H + 4)), "the staging tiles fit into the h1 / h2 tile buffers");
  {  // dW2
    const int t0 = (wave * DW2_TPW) % (NTN * NTN);
    const int it = t0 / NTN, jt = t0 % NTN;
    const int rank = (wave * DW2_TPW) / (NTN * NTN);  // 0 unless the sample range of a tile is split over wavefronts
    if (own && DW2_KS > 1) {
      if (rank > 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) L[wave * 1024 + r * 64 + lane] = acc2[0][r];
      }
      __syncthreads();
      if (rank == 0) {
#pragma unroll 1
        for (int k = 1; k < DW2_KS; ++k) {
          const int pw = wave + k * (NTN * NTN / DW2_TPW);
#pragma unroll
          for (int r = 0; r < 16; ++r) acc2[0][r] += L[pw * 1024 + r * 64 + lane];
        }
      }
      __syncthreads();
    }
    if (!own || rank == 0) {
#pragma unroll
      for (int q = 0; q < DW2_TPW; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = it * 32 + 8 * (r / 4) + 4 * hi + (r % 4), j = (jt + q) * 32 + lo;
          if (own) gW2[i * H + j] = acc2[q][r];
          else atomicAdd(&gW2[i * H + j], acc2[q][r]);
        }
    }
  }
#pragma unroll
  for (int q = 0; q < Q1; ++q) {  // dW1: the wavefronts wave % NTN + NTN k hold the shares of a tile
    const int rank = wave / NTN, jt = wave % NTN;
    if (own && KS1 > 1) {
      if (rank > 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) L[wave * 1024 + r * 64 + lane] = acc1[q][r];
      }
      __syncthreads();
      if (rank == 0) {
#pragma unroll 1
        for (int k = 1; k < KS1; ++k) {
#pragma unroll
          for (int r = 0; r < 16; ++r) acc1[q][r] += L[(wave + k * NTN) * 1024 + r * 64 + lane];
        }
      }
      __syncthreads();
    }
    if (!own || rank == 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int d = q * 32 + 8 * (r / 4) + 4 * hi + (r % 4), j = jt * 32 + lo;
        if (d < a.Din) {
          if (own) gW1[d * H + j] = acc1[q][r];
          else atomicAdd(&gW1[d * H + j], acc1[q][r]);
        }
      }
    }
  }
  if (!own) {
    if (hi == 0) {
      atomicAdd(&gb1[nt * 32 + lo], gb1r);
      atomicAdd(&gb2[nt * 32 + lo], gb2r);
    }
    const int i = tid % H;
#pragma unroll
    for (int k = 0; k < NOUT; ++k) atomicAdd(&gW3[i * NOUT + k], gw[k]);
    if (tid < (BM < 64 ? 64 : BM)) {
#pragma unroll
      for (int k = 0; k < NOUT; ++k) {
        float v = accS[tid * AS + k];
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if (lane == 0) atomicAdd(&gb3[k], v);
      }
    }
  } else {  // bias and output-layer gradients: every contributor's part to LDS, then one thread per element adds them in order
    float* const Lb = L;                        // [MTF][2][H]
    float* const Lw = Lb + MTF * 2 * H;         // [HPARTS][H * NOUT]
    float* const L3 = Lw + HPARTS * H * NOUT;   // [2][NOUT]
    static_assert(MTF * 2 * H + HPARTS * H * NOUT + 2 * NOUT <= BM * (2 * (H + 4)), "the parts fit into the tile buffers");
    if (hi == 0) {
      Lb[(mt * 2 + 0) * H + nt * 32 + lo] = gb1r;
      Lb[(mt * 2 + 1) * H + nt * 32 + lo] = gb2r;
    }
#pragma unroll
    for (int k = 0; k < NOUT; ++k) Lw[(tid / H) * H * NOUT + (tid % H) * NOUT + k] = gw[k];
    if (tid < (BM < 64 ? 64 : BM)) {  // whole wavefronts; lanes past BM hold zeros
#pragma unroll
      for (int k = 0; k < NOUT; ++k) {
        float v = accS[tid * AS + k];
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if (lane == 0) L3[wave * NOUT + k] = v;
      }
    }
    __syncthreads();
    for (int e = tid; e < 2 * H; e += NT) {
      const int which = e / H, col = e - which * H;
      float v = Lb[which * H + col];
      for (int m = 1; m < MTF; ++m) v += Lb[(m * 2 + which) * H + col];
      (which == 0 ? gb1 : gb2)[col] = v;
    }
    for (int e = tid; e < H * NOUT; e += NT) {
      float v = Lw[e];
      for (int part = 1; part < HPARTS; ++part) v += Lw[part * H * NOUT + e];
      gW3[e] = v;
    }
    if (tid < NOUT) gb3[tid] = (BM > 64) ? L3[tid] + L3[NOUT + tid] : L3[tid];
  }
  if (tid < (BM < 64 ? 64 : BM)) {  // loss statistics: reported only, summed over the workgroups with atomics
#pragma unroll
    for (int k = 0; k < 5; ++k) {
      float v = accS[tid * AS + NOUT + k];
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
      if (lane == 0 && v != 0.f) atomicAdd(&a.stats[k], v);
    }
  }
}

template <int H, int BM, int NOUT, int DMAX, int NW, class LossFn>
__global__ void __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) fused_train_kernel(FusedTrainArgs a, LossFn fn) {
  fused_train_body<H, BM, NOUT, DMAX, NW, LossFn>(a, fn, blockIdx.x, gridDim.x);
}

// Two networks of the same shape on the same number of samples in ONE launch: workgroups 0 .. grid_a - 1 train the
// first, the others the second.  For minibatches so small that neither launch fills the compute units (a few tiles
// each) the update is a chain of dependent launches, and this takes two links (a kernel and its reduction) out of it.
template <int H, int BM, int NOUT_A, int NOUT_B, int DMAX, int NW, class LossA, class LossB>
__global__ void __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) fused_train_pair_kernel(FusedTrainArgs a, LossA fa, FusedTrainArgs b,
                                                                                   LossB fb, unsigned grid_a) {
  if (blockIdx.x < grid_a) fused_train_body<H, BM, NOUT_A, DMAX, NW, LossA>(a, fa, blockIdx.x, grid_a);
  else fused_train_body<H, BM, NOUT_B, DMAX, NW, LossB>(b, fb, blockIdx.x - grid_a, gridDim.x - grid_a);
}

// (an input row is staged as the aligned 16-byte chunks that cover it: up to three values more than its width)
inline bool fused_train_supported(int H, int Din) { return (H == 64 || H == 128) && Din <= 93; }

inline int fused_train_px(int Din) {
  int px = 32 * ((Din + 31) / 32);
  while (px % 4 != 0 || (px / 4) % 2 == 0) px += 4;
  return px;
}

template <int H, int BM, int NOUT, int DMAX, int NW, class LossFn>
inline int32_t launch_fused_train_inst(const FusedTrainArgs& a, const LossFn& fn, hipStream_t s) {
  auto kern = fused_train_kernel<H, BM, NOUT, DMAX, NW, LossFn>;
  constexpr bool XDB = fused_train_lds_floats(H, BM, NOUT, NW, DMAX + 4, 2) * 4 <= 160 * 1024;  // as in the kernel
  const size_t bytes = fused_train_lds_floats(H, BM, NOUT, NW, a.px, XDB ? 2 : 1) * 4;
  static bool configured = false;  // per instantiation
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
      return MARL_E_LAUNCH;
    configured = true;
  }
  const int64_t tiles = (a.S + BM - 1) / BM;
  const unsigned grid = (unsigned)std::min<int64_t>(tiles, NW == 4 ? 512 : 256);  // resident workgroups: two per CU with four wavefronts
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * NW), bytes, s, a, fn);
  if (a.partial != nullptr) launch_reduce_partials(a.partial, (int)grid, a.gcount, a.gW1, s);
  return launch_status();
}

template <int H, int BM, int NOUT_A, int NOUT_B, int DMAX, int NW, class LossA, class LossB>
inline int32_t launch_fused_train_pair_inst(const FusedTrainArgs& a, const LossA& fa, const FusedTrainArgs& b, const LossB& fb,
                                            hipStream_t s) {
  auto kern = fused_train_pair_kernel<H, BM, NOUT_A, NOUT_B, DMAX, NW, LossA, LossB>;
  constexpr int NMAX = NOUT_A > NOUT_B ? NOUT_A : NOUT_B;
  constexpr bool XDB_A = fused_train_lds_floats(H, BM, NOUT_A, NW, DMAX + 4, 2) * 4 <= 160 * 1024;  // as in the kernel
  constexpr bool XDB_B = fused_train_lds_floats(H, BM, NOUT_B, NW, DMAX + 4, 2) * 4 <= 160 * 1024;
  const size_t bytes = std::max(fused_train_lds_floats(H, BM, NOUT_A, NW, a.px, XDB_A ? 2 : 1),
                                fused_train_lds_floats(H, BM, NOUT_B, NW, b.px, XDB_B ? 2 : 1)) * 4;
  static_assert(fused_train_lds_floats(H, BM, NMAX, NW, DMAX + 4, 1) * 4 <= 160 * 1024, "fits");
  static bool configured = false;  // per instantiation
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
      return MARL_E_LAUNCH;
    configured = true;
  }
  const unsigned grid_a = (unsigned)((a.S + BM - 1) / BM);  // == the second network's (the caller checks the sizes)
  hipLaunchKernelGGL(kern, dim3(2 * grid_a), dim3(64 * NW), bytes, s, a, fa, b, fb, grid_a);
  // copy k of the first network's range is directly followed by copy k of the second's: one reduction for both
  launch_reduce_partials(a.partial, (int)grid_a, a.gcount + b.gcount, a.gW1, s);
  return launch_status();
}

// Workgroups a launch can have (the copies of the gradient range the caller provides room for).
constexpr int kFusedTrainMaxGrid = 512;

template <int NOUT, class LossFn>
inline int32_t launch_fused_train(int H, const FusedTrainArgs& a, const LossFn& fn, hipStream_t s) {
  // the kernel divides sample indices by the rows' and the loss's agent counts with SmallDiv's product
  if (!small_div_ok(a.X.pd, a.S) || !small_div_ok(fn.lc.ad, a.S)) return MARL_E_SIZE;
  // algorithmic flops: forward 2S(DH + HH), backward 2S(HH + HH + DH)
  TimedLaunch timed(KC_FUSED_TRAIN, 2.0 * (double)a.S * (2.0 * a.Din * H + 3.0 * H * H), s);
  if (H == 128) {
    if (a.Din <= 29) return launch_fused_train_inst<128, 64, NOUT, 32, 8, LossFn>(a, fn, s);
    return launch_fused_train_inst<128, 64, NOUT, 96, 8, LossFn>(a, fn, s);
  }
  if (a.Din <= 29) return launch_fused_train_inst<64, 128, NOUT, 32, 8, LossFn>(a, fn, s);
  return launch_fused_train_inst<64, 128, NOUT, 96, 8, LossFn>(a, fn, s);
}

// Whether two networks can share a launch: the same shape on the same number of samples, so few tiles that both
// launches together have at most one workgroup per compute unit, and gradient ranges that follow one another (a's, then
// b's) so that the interleaved copies reduce in one pass.
inline bool fused_train_pair_supported(int Ha, int Da, int64_t Sa, int Hb, int Db, int64_t Sb) {
  if (Ha != Hb || Da != Db || Sa != Sb || !fused_train_supported(Ha, Da)) return false;
  const int BM = Ha == 128 ? 64 : 128;
  return 2 * ((Sa + BM - 1) / BM) <= 256;
}

// a.partial must have room for (a.gcount + b.gcount) floats per workgroup of ONE network; a.gW1 + a.gcount == b.gW1.
template <int NOUT_A, int NOUT_B, class LossA, class LossB>
inline int32_t launch_fused_train_pair(int H, FusedTrainArgs a, const LossA& fa, FusedTrainArgs b, const LossB& fb, hipStream_t s) {
  if (!small_div_ok(a.X.pd, a.S) || !small_div_ok(fa.lc.ad, a.S) || !small_div_ok(b.X.pd, b.S) || !small_div_ok(fb.lc.ad, b.S))
    return MARL_E_SIZE;
  if (a.partial == nullptr || b.gW1 != a.gW1 + a.gcount) return MARL_E_SIZE;
  a.pstride = b.pstride = a.gcount + b.gcount;
  b.partial = a.partial + a.gcount;
  TimedLaunch timed(KC_FUSED_TRAIN, 2.0 * (double)(a.S + b.S) * (2.0 * a.Din * H + 3.0 * H * H), s);
  if (H == 128) {
    if (a.Din <= 29) return launch_fused_train_pair_inst<128, 64, NOUT_A, NOUT_B, 32, 8, LossA, LossB>(a, fa, b, fb, s);
    return launch_fused_train_pair_inst<128, 64, NOUT_A, NOUT_B, 96, 8, LossA, LossB>(a, fa, b, fb, s);
  }
  if (a.Din <= 29) return launch_fused_train_pair_inst<64, 128, NOUT_A, NOUT_B, 32, 8, LossA, LossB>(a, fa, b, fb, s);
  return launch_fused_train_pair_inst<64, 128, NOUT_A, NOUT_B, 96, 8, LossA, LossB>(a, fa, b, fb, s);
}

}  // namespace marl
