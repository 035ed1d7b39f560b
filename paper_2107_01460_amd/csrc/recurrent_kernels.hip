// Recurrent IPPO / MAPPO: a GRU cell in place of the second hidden layer of both networks.
//
//   e = tanh(x We + be);  r = sigma(e Wi_r + bi_r + h Wh_r + bh_r);  z likewise;
//   n = tanh(e Wi_n + bi_n + r (h Wh_n + bh_n));  h' = (1 - z) n + z h;  out = h' W3 + b3
//
// Every product with a weight matrix is an MFMA GEMM (gemm.h); the gate arithmetic is element-wise.  The products
// that do not depend on the hidden state (the embedding e and its gate pre-activations e Wi) run once over all
// T steps of a minibatch of sequences; only h Wh and the gates are stepped through time, forward for t = 0..T-1
// and backward for t = T-1..0, where the weight gradients are again taken in one product over all steps.
#include <algorithm>
#include <cmath>

#include "gemm.h"
#include "heads.h"
#include "ppo_common.h"

namespace marl {

int32_t launch_env_step(const marl_config& c, marl_env_state st, const int32_t* actions, float* obs, float* reward,
                        uint8_t* done, bool do_step, hipStream_t s);

namespace {

// Offsets (in floats) of one recurrent network's blocks inside the flat parameter vector.
struct RecOffsets {
  int64_t We, be, Wi, bi, Wh, bh, W3, b3, end;
};
RecOffsets rec_offsets(int64_t base, int Din, int H, int Dout) {
  RecOffsets o;
  o.We = base;
  o.be = o.We + (int64_t)Din * H;
  o.Wi = o.be + H;
  o.bi = o.Wi + (int64_t)H * 3 * H;
  o.Wh = o.bi + 3 * H;
  o.bh = o.Wh + (int64_t)H * 3 * H;
  o.W3 = o.bh + 3 * H;
  o.b3 = o.W3 + (int64_t)H * Dout;
  o.end = o.b3 + Dout;
  return o;
}

// Working copy of the parameters with every block on a 64-float boundary (16-byte loads of weight rows).
struct RecParamMap {
  int64_t src[17], dst[17];  // 16 blocks (actor 8, critic 8) + end
  // per network, after the blocks: Wh and Wh transposed once more in the order a lane feeds them to the matrix cores
  // straight from memory: element (k, n) of a [K][N] matrix at ((k / 4) * N + n) * 4 + k % 4
  int64_t wh_op[2], wht_op[2];
  int hidden[2];
  int64_t total;
};
RecParamMap rec_param_map(const Dims& d) {
  RecParamMap m;
  const RecOffsets a = rec_offsets(0, d.D, d.Ha, kActions), c = rec_offsets(d.Pa, d.Dc, d.Hc, 1);
  const int64_t src[17] = {a.We, a.be, a.Wi, a.bi, a.Wh, a.bh, a.W3, a.b3, c.We, c.be, c.Wi, c.bi, c.Wh, c.bh, c.W3, c.b3, c.end};
  int64_t off = 0;
  for (int i = 0; i < 17; ++i) {
    m.src[i] = src[i];
    m.dst[i] = off;
    if (i < 16) off += ((src[i + 1] - src[i] + 63) / 64) * 64;
  }
  m.hidden[0] = d.Ha;
  m.hidden[1] = d.Hc;
  for (int n = 0; n < 2; ++n) {
    const int64_t sz = (((int64_t)m.hidden[n] * 3 * m.hidden[n] + 63) / 64) * 64;
    m.wh_op[n] = off;
    off += sz;
    m.wht_op[n] = off;
    off += sz;
  }
  m.total = off;
  return m;
}
RecOffsets rec_padded(const RecParamMap& m, int net) {
  const int64_t* o = m.dst + 8 * net;
  return RecOffsets{o[0], o[1], o[2], o[3], o[4], o[5], o[6], o[7], o[8]};
}

__global__ void rec_stage_params_kernel(const float* __restrict__ src, float* __restrict__ dst, RecParamMap pm) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pm.src[16]) return;
  int b = 0;
#pragma unroll
  for (int k = 1; k < 16; ++k) b += (i >= pm.src[k]) ? 1 : 0;
  const float v = src[i];
  const int64_t e = i - pm.src[b];
  dst[pm.dst[b] + e] = v;
  if (b == 4 || b == 12) {  // a Wh block [H][3H]: also its two operand-order copies
    const int net = b == 12, H = pm.hidden[net];
    const int64_t k = e / (3 * H), c = e - k * (3 * H);
    dst[pm.wh_op[net] + ((k / 4) * (3 * H) + c) * 4 + k % 4] = v;    // (k, c) of Wh
    dst[pm.wht_op[net] + ((c / 4) * H + k) * 4 + c % 4] = v;          // (c, k) of Wh^T
  }
}

__global__ void copy_f32_kernel(const float* __restrict__ src, float* __restrict__ dst, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

// h[s][j] = 0 where the previous step ended the episode of sample s's environment (per samples per environment).
__global__ void mask_hidden_kernel(float* __restrict__ h, const uint8_t* __restrict__ done, int64_t n_elems, int H, int per) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_elems) return;
  const int64_t s = i / H;
  if (done[s / per]) h[i] = 0.f;
}

__device__ __forceinline__ float sigmoid_f32(float x) { return __builtin_amdgcn_rcpf(1.0f + fast_exp(-x)); }

// Gate arithmetic of one step, one thread per (sample, hidden unit).  Gi / Gh are the products without their
// biases.  hout may alias hprev.  hnext (nullable) gets hout * keep[s / per]: the input of the next step.
__global__ void __launch_bounds__(256) gru_forward_kernel(const float* __restrict__ Gi, const float* __restrict__ Gh,
                                                          const float* __restrict__ bi, const float* __restrict__ bh,
                                                          const float* hprev, float* __restrict__ rzn,
                                                          float* __restrict__ ghn, float* hout, float* __restrict__ hnext,
                                                          const float* __restrict__ keep, int per, int64_t S, int H) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S * H) return;
  const int64_t s = i / H;
  const int j = (int)(i - s * H);
  const float* gi = Gi + s * 3 * H;
  const float* gh = Gh + s * 3 * H;
  const float r = sigmoid_f32((gi[j] + bi[j]) + (gh[j] + bh[j]));
  const float z = sigmoid_f32((gi[H + j] + bi[H + j]) + (gh[H + j] + bh[H + j]));
  const float hn = gh[2 * H + j] + bh[2 * H + j];
  const float n = tanh_f32((gi[2 * H + j] + bi[2 * H + j]) + r * hn);
  const float h = (1.0f - z) * n + z * hprev[i];
  if (rzn != nullptr) {
    rzn[s * 3 * H + j] = r;
    rzn[s * 3 * H + H + j] = z;
    rzn[s * 3 * H + 2 * H + j] = n;
  }
  if (ghn != nullptr) ghn[i] = hn;
  hout[i] = h;
  if (hnext != nullptr) hnext[i] = h * keep[s / per];
}

// Backward of the gate arithmetic of one step.  dh = gradient from the next step (dh_next * keep_next, absent at the
// last step) + the output layer's (dl W3^T).  Writes the gradients of the two gate products and dh * z, the direct
// part of the gradient with respect to the incoming hidden state (the product dgh Wh^T is added by a GEMM).
template <int NOUT>
__global__ void __launch_bounds__(256) gru_backward_kernel(const float* __restrict__ dh_next, const float* __restrict__ keep_next,
                                                           const float* __restrict__ dl, const float* __restrict__ W3,
                                                           const float* __restrict__ rzn, const float* __restrict__ ghn,
                                                           const float* __restrict__ hprev, float* __restrict__ dgi,
                                                           float* __restrict__ dgh, float* __restrict__ dhprev, int per,
                                                           int64_t S, int H) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S * H) return;
  const int64_t s = i / H;
  const int j = (int)(i - s * H);
  float dh = dh_next != nullptr ? dh_next[i] * keep_next[s / per] : 0.f;
#pragma unroll
  for (int k = 0; k < NOUT; ++k) dh = fmaf(dl[s * NOUT + k], W3[(int64_t)j * NOUT + k], dh);
  const float r = rzn[s * 3 * H + j], z = rzn[s * 3 * H + H + j], n = rzn[s * 3 * H + 2 * H + j];
  const float dn = dh * (1.0f - z);
  const float dz = dh * (hprev[i] - n);
  const float dpre_n = dn * (1.0f - n * n);
  const float dr = dpre_n * ghn[i];
  const float dpre_z = dz * z * (1.0f - z);
  const float dpre_r = dr * r * (1.0f - r);
  dgi[s * 3 * H + j] = dpre_r;
  dgi[s * 3 * H + H + j] = dpre_z;
  dgi[s * 3 * H + 2 * H + j] = dpre_n;
  dgh[s * 3 * H + j] = dpre_r;
  dgh[s * 3 * H + H + j] = dpre_z;
  dgh[s * 3 * H + 2 * H + j] = dpre_n * r;
  dhprev[i] = dh * z;
}

// Index arrays of a minibatch of sequences: row r = t * J + j is trajectory row t * N + envs[j];
// keep[r] = 0 where the step before t ended the episode of that environment (rows of t = 0 keep everything).
__global__ void seq_index_kernel(const int32_t* __restrict__ envs, const uint8_t* __restrict__ done, int J, int N, int T,
                                 int32_t* __restrict__ rows, float* __restrict__ keep) {
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= (int64_t)T * J) return;
  const int t = (int)(r / J), j = (int)(r - (int64_t)t * J);
  const int env = envs[j];
  rows[r] = t * N + env;
  keep[r] = (t > 0 && done[(int64_t)(t - 1) * N + env]) ? 0.f : 1.f;
}

// dst[(j * per + a)][u] = h0[(envs[j] * per + a)][u]
__global__ void gather_hidden_kernel(const float* __restrict__ h0, const int32_t* __restrict__ envs, int J, int per, int H,
                                     float* __restrict__ dst) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)J * per * H) return;
  const int64_t q = i / H;
  const int u = (int)(i - q * H);
  const int j = (int)(q / per), a = (int)(q - (int64_t)j * per);
  dst[i] = h0[((int64_t)envs[j] * per + a) * H + u];
}

// ---- fused steps ---------------------------------------------------------------------------------------------
// One time step of the cell in one kernel each way, for H <= 256: the product with the hidden-to-hidden weights runs
// on the matrix cores with its A operand in LDS and the weights read in operand order straight from memory, and the
// gate arithmetic is its epilogue (forward) or its prologue (backward).  A workgroup owns 32 samples and all H
// units: H / 32 wavefronts, wavefront u the units 32 u .. 32 u + 31.

constexpr int kStepRows = 32;
inline bool fused_step_supported(int H) { return H % 32 == 0 && H <= 256; }
inline size_t fused_fwd_lds(int H) { return sizeof(float) * kStepRows * (H + 4); }
inline size_t fused_bwd_lds(int H) { return sizeof(float) * kStepRows * (3 * H + 4); }

// Forward: gates of one step from Gi (input products, no bias) and hprev; see gru_forward_kernel for the outputs.
__global__ void __launch_bounds__(512) gru_step_fwd_kernel(const float* __restrict__ Gi, const float* __restrict__ Wh_op,
                                                           const float* __restrict__ bi, const float* __restrict__ bh,
                                                           const float* hprev, float* __restrict__ rzn,
                                                           float* __restrict__ ghn, float* hout, float* __restrict__ hnext,
                                                           const float* __restrict__ keep, int per, int64_t S, int H) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  const int PH = H + 4;
  float* Hs = lds;  // [32][PH]
  // blockIdx.y: which share of the units this workgroup computes (blockDim.x / 64 wavefronts of 32 units each).  With
  // few samples per step the units of a tile are split over several workgroups so that every CU has work; every one of
  // them stages the whole h tile, so hout / hnext must then not alias hprev.
  const int tid = threadIdx.x, lane = tid & 63, u = blockIdx.y * (blockDim.x >> 6) + (tid >> 6), lo = lane & 31, hi = lane >> 5;
  const int nthreads = blockDim.x;
  const int64_t s0 = (int64_t)blockIdx.x * kStepRows;
  for (int f = tid; f < kStepRows * (H / 4); f += nthreads) {
    const int r = f / (H / 4), c4 = f - r * (H / 4);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (s0 + r < S) v = *reinterpret_cast<const float4*>(hprev + (s0 + r) * H + 4 * c4);
    *reinterpret_cast<float4*>(&Hs[r * PH + 4 * c4]) = v;
  }
  const int n = u * 32 + lo;  // this lane's hidden unit
  // the input products of this lane's 16 (sample, unit) elements, requested before the matrix loop
  float gi[3][16];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int64_t s = min(s0 + 8 * (r / 4) + 4 * hi + (r % 4), S - 1);
#pragma unroll
    for (int g = 0; g < 3; ++g) gi[g][r] = Gi[s * 3 * H + g * H + n];
  }
  __syncthreads();
  floatx16 acc[3];
#pragma unroll
  for (int g = 0; g < 3; ++g)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[g][r] = 0.f;
  const float* As = Hs + lo * PH + 4 * hi;
  const float* Bg = Wh_op + ((int64_t)hi * 3 * H + n) * 4;  // quad `hi` of k group 0, column n of gate 0
  const int ksteps = H / 8;  // a multiple of 4
  // the weights of four k steps are in flight: a wavefront streams its own 3 x 32 columns of Wh from L2 and has
  // nothing else to hide that latency behind
  constexpr int kDepth = 4;
  float4 bq[kDepth][3];
  auto load_b = [&](int ks, float4 (&b3)[3]) {
    const int kc = ks < ksteps ? ks : ksteps - 1;
#pragma unroll
    for (int g = 0; g < 3; ++g) b3[g] = *reinterpret_cast<const float4*>(Bg + ((int64_t)2 * kc * 3 * H + g * H) * 4);
  };
#pragma unroll
  for (int d = 0; d < kDepth - 1; ++d) load_b(d, bq[d]);
#pragma unroll 1
  for (int k0 = 0; k0 < ksteps; k0 += kDepth) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      const int ks = k0 + d;
      load_b(ks + kDepth - 1, bq[(d + kDepth - 1) % kDepth]);
      const float4 av = *reinterpret_cast<const float4*>(As + 8 * ks);
      const float af[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g = 0; g < 3; ++g) {
          const float4 b = bq[d][g];
          acc[g] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], j == 0 ? b.x : j == 1 ? b.y : j == 2 ? b.z : b.w, acc[g], 0, 0, 0);
        }
    }
  }
  const float bir = bi[n], biz = bi[H + n], bin_ = bi[2 * H + n];
  const float bhr = bh[n], bhz = bh[H + n], bhn = bh[2 * H + n];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int m = 8 * (r / 4) + 4 * hi + (r % 4);
    const int64_t s = s0 + m;
    if (s < S) {
      const float rr = sigmoid_f32((gi[0][r] + bir) + (acc[0][r] + bhr));
      const float zz = sigmoid_f32((gi[1][r] + biz) + (acc[1][r] + bhz));
      const float hn = acc[2][r] + bhn;
      const float nn = tanh_f32((gi[2][r] + bin_) + rr * hn);
      const float h = (1.0f - zz) * nn + zz * Hs[m * PH + n];
      if (rzn != nullptr) {
        rzn[s * 3 * H + n] = rr;
        rzn[s * 3 * H + H + n] = zz;
        rzn[s * 3 * H + 2 * H + n] = nn;
      }
      if (ghn != nullptr) ghn[s * H + n] = hn;
      hout[s * H + n] = h;
      if (hnext != nullptr) hnext[s * H + n] = h * keep[s / per];
    }
  }
}

// Backward: the gate gradients of one step (see gru_backward_kernel) and, when want_dhprev, the whole gradient with
// respect to the incoming hidden state: dh * z + dgh Wh^T.
template <int NOUT>
__global__ void __launch_bounds__(512) gru_step_bwd_kernel(const float* __restrict__ dh_next, const float* __restrict__ keep_next,
                                                           const float* __restrict__ dl, const float* __restrict__ W3,
                                                           const float* __restrict__ rzn, const float* __restrict__ ghn,
                                                           const float* __restrict__ hprev, const float* __restrict__ WhT_op,
                                                           float* __restrict__ dgi, float* __restrict__ dgh,
                                                           float* dhprev, int want_dhprev, int per, int64_t S, int H) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  // The dgh tile, the A operand, is all that is kept in LDS ([32][PG]): the direct term dh * z travels through dhprev
  // itself (written here by the thread that computes it, read back after the barrier by the thread that finishes that
  // element), so that the 256-wide instantiation leaves room on a compute unit for a workgroup of the other network's
  // kernel, which runs beside it on a second stream.
  const int PG = 3 * H + 4;
  float* Gs = lds;
  const int tid = threadIdx.x, lane = tid & 63, u = tid >> 6, lo = lane & 31, hi = lane >> 5;
  const int64_t s0 = (int64_t)blockIdx.x * kStepRows;
  {  // gate arithmetic: thread -> unit j = tid % H, samples tid / H + 2 q
    const int j = tid % H, mq = tid / H;
    float w3[NOUT];
#pragma unroll
    for (int k = 0; k < NOUT; ++k) w3[k] = W3[(int64_t)j * NOUT + k];
#pragma unroll 4
    for (int q = 0; q < kStepRows / 2; ++q) {
      const int m = mq + 2 * q;
      const int64_t s = s0 + m;
      float g_r = 0.f, g_z = 0.f, g_n = 0.f, g_hn = 0.f, dz_direct = 0.f;
      if (s < S) {
        const int64_t i = s * H + j;
        float dh = dh_next != nullptr ? dh_next[i] * keep_next[s / per] : 0.f;
#pragma unroll
        for (int k = 0; k < NOUT; ++k) dh = fmaf(dl[s * NOUT + k], w3[k], dh);
        const float r = rzn[s * 3 * H + j], z = rzn[s * 3 * H + H + j], n = rzn[s * 3 * H + 2 * H + j];
        const float dn = dh * (1.0f - z);
        const float dz = dh * (hprev[i] - n);
        const float dpre_n = dn * (1.0f - n * n);
        const float dr = dpre_n * ghn[i];
        g_z = dz * z * (1.0f - z);
        g_r = dr * r * (1.0f - r);
        g_n = dpre_n;
        g_hn = dpre_n * r;
        dz_direct = dh * z;
        dgi[s * 3 * H + j] = g_r;
        dgi[s * 3 * H + H + j] = g_z;
        dgi[s * 3 * H + 2 * H + j] = g_n;
        dgh[s * 3 * H + j] = g_r;
        dgh[s * 3 * H + H + j] = g_z;
        dgh[s * 3 * H + 2 * H + j] = g_hn;
        if (want_dhprev) dhprev[i] = dz_direct;
      }
      Gs[m * PG + j] = g_r;
      Gs[m * PG + H + j] = g_z;
      Gs[m * PG + 2 * H + j] = g_hn;
    }
  }
  if (!want_dhprev) return;  // uniform
  __syncthreads();  // orders the tile in LDS and this workgroup's stores to dhprev before the reads below
  // dhprev tile = Ds + Gs WhT: wavefront u the 32 units 32 u .., contraction over the 3 H gate columns,
  // two accumulators over alternate k steps so that consecutive MFMAs do not wait for each other
  const int n = u * 32 + lo;
  floatx16 acc[2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
  float direct[16];  // dh * z of this lane's output elements, requested before the product
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int64_t s = s0 + 8 * (r / 4) + 4 * hi + (r % 4);
    direct[r] = s < S ? dhprev[s * H + n] : 0.f;
  }
  const float* As = Gs + lo * PG + 4 * hi;
  const float* Bg = WhT_op + ((int64_t)hi * H + n) * 4;
  const int ksteps = 3 * H / 8;  // a multiple of 12: H is a multiple of 32
  constexpr int kDepth = 6;      // k steps in flight
  float4 bq[kDepth];
  auto load_b = [&](int ks, float4& b) {
    const int kc = ks < ksteps ? ks : ksteps - 1;
    b = *reinterpret_cast<const float4*>(Bg + (int64_t)2 * kc * H * 4);
  };
#pragma unroll
  for (int d = 0; d < kDepth - 1; ++d) load_b(d, bq[d]);
#pragma unroll 1
  for (int k0 = 0; k0 < ksteps; k0 += kDepth) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      const int ks = k0 + d;
      load_b(ks + kDepth - 1, bq[(d + kDepth - 1) % kDepth]);
      const float4 av = *reinterpret_cast<const float4*>(As + 8 * ks);
      const float4 b = bq[d];
      acc[d & 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av.x, b.x, acc[d & 1], 0, 0, 0);
      acc[d & 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av.y, b.y, acc[d & 1], 0, 0, 0);
      acc[d & 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av.z, b.z, acc[d & 1], 0, 0, 0);
      acc[d & 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av.w, b.w, acc[d & 1], 0, 0, 0);
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int m = 8 * (r / 4) + 4 * hi + (r % 4);
    const int64_t s = s0 + m;
    if (s < S) dhprev[s * H + n] = (acc[0][r] + acc[1][r]) + direct[r];
  }
}

template <class K>
int32_t allow_big_lds(K kern) {
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
    return MARL_E_LAUNCH;
  return MARL_OK;
}

// One forward step: fused when the width allows it, else the GEMM + gate kernel pair.
int32_t launch_step_forward(const float* Gi, const float* hprev, int64_t S, int H, const float* eff, const RecOffsets& o,
                            const float* wh_op, float* GhT, float* rzn, float* ghn, float* hout, float* hnext,
                            const float* keep, int per, hipStream_t s);
template <int NOUT>
int32_t launch_step_backward(const float* dh_next, const float* keep_next, const float* dl, const float* rzn,
                             const float* ghn, const float* hprev, int64_t S, int H, const float* eff, const RecOffsets& o,
                             const float* wht_op, float* dgi, float* dgh, float* dhprev, bool want_dhprev, int per,
                             hipStream_t s);

int64_t align256(int64_t x) { return (x + 255) & ~(int64_t)255; }
unsigned blocks_for(int64_t n) { return (unsigned)((n + 255) / 256); }

int64_t k_split(int64_t K, int64_t tiles_mn) {  // about four workgroups per CU, k ranges in multiples of the k tile
  const int64_t want = std::max<int64_t>(1, 1024 / std::max<int64_t>(1, tiles_mn));
  const int64_t per = (K + want - 1) / want;
  return std::max<int64_t>(256, ((per + kGemmBK - 1) / kGemmBK) * kGemmBK);
}

const float* stage_params(const Dims& d, const float* params, float* scratch, hipStream_t s) {
  hipLaunchKernelGGL(rec_stage_params_kernel, dim3(blocks_for(d.P)), dim3(256), 0, s, params, scratch, rec_param_map(d));
  return scratch;
}

// e = tanh(X We + be) [S][H] and Gi = e Wi [S][3H] (bias added with the gates)
void embed_and_input_gates(const RowSrc& X, int64_t S, int Din, int H, const float* eff, const RecOffsets& o, float* E,
                           float* Gi, hipStream_t s) {
  GemmArgs g{};
  g.A = X; g.B = eff + o.We; g.ldb = H; g.C = E; g.ldc = H; g.aux_vec = eff + o.be;
  g.M = S; g.N = H; g.K = Din;
  launch_gemm<GEMM_NN, EPI_BIAS_TANH>(g, s);
  GemmArgs g2{};
  g2.A = RowSrc{E, H, nullptr, 1, S}; g2.B = eff + o.Wi; g2.ldb = 3 * H; g2.C = Gi; g2.ldc = 3 * H;
  g2.M = S; g2.N = 3 * H; g2.K = H;
  launch_gemm<GEMM_NN, EPI_STORE>(g2, s);
}

void hidden_gates(const float* hprev, int64_t S, int H, const float* eff, const RecOffsets& o, float* Gh, hipStream_t s) {
  GemmArgs g{};
  g.A = RowSrc{hprev, H, nullptr, 1, S}; g.B = eff + o.Wh; g.ldb = 3 * H; g.C = Gh; g.ldc = 3 * H;
  g.M = S; g.N = 3 * H; g.K = H;
  launch_gemm<GEMM_NN, EPI_STORE>(g, s);
}

int32_t launch_step_forward(const float* Gi, const float* hprev, int64_t S, int H, const float* eff, const RecOffsets& o,
                            const float* wh_op, float* GhT, float* rzn, float* ghn, float* hout, float* hnext,
                            const float* keep, int per, hipStream_t s) {
  if (fused_step_supported(H)) {
    TimedLaunch timed(KC_GEMM_NN, 2.0 * (double)S * H * 3.0 * H, s);
    const int64_t tiles = (S + kStepRows - 1) / kStepRows;
    int ysplit = 1;  // workgroups per tile: enough for one per CU where the state is not updated in place
    if (hprev != hout && hprev != hnext)
      while (tiles * ysplit < 256 && ysplit < H / 32) ysplit *= 2;
    while ((H / 32) % ysplit != 0) ysplit /= 2;
    hipLaunchKernelGGL(gru_step_fwd_kernel, dim3((unsigned)tiles, (unsigned)ysplit), dim3(2 * H / ysplit), fused_fwd_lds(H),
                       s, Gi, wh_op, eff + o.bi, eff + o.bh, hprev, rzn, ghn, hout, hnext, keep, per, S, H);
    return MARL_OK;
  }
  hidden_gates(hprev, S, H, eff, o, GhT, s);
  hipLaunchKernelGGL(gru_forward_kernel, dim3(blocks_for(S * H)), dim3(256), 0, s, Gi, GhT, eff + o.bi, eff + o.bh, hprev, rzn,
                     ghn, hout, hnext, keep, per, S, H);
  return MARL_OK;
}

template <int NOUT>
int32_t launch_step_backward(const float* dh_next, const float* keep_next, const float* dl, const float* rzn,
                             const float* ghn, const float* hprev, int64_t S, int H, const float* eff, const RecOffsets& o,
                             const float* wht_op, float* dgi, float* dgh, float* dhprev, bool want_dhprev, int per,
                             hipStream_t s) {
  if (fused_step_supported(H)) {
    static bool configured = false;  // per NOUT
    if (!configured) {
      const int32_t rc = allow_big_lds(gru_step_bwd_kernel<NOUT>);
      if (rc != MARL_OK) return rc;
      configured = true;
    }
    TimedLaunch timed(KC_GEMM_NT, want_dhprev ? 2.0 * (double)S * H * 3.0 * H : 0.0, s);
    hipLaunchKernelGGL(gru_step_bwd_kernel<NOUT>, dim3((unsigned)((S + kStepRows - 1) / kStepRows)), dim3(2 * H),
                       fused_bwd_lds(H), s, dh_next, keep_next, dl, eff + o.W3, rzn, ghn, hprev, wht_op, dgi, dgh, dhprev,
                       (int)want_dhprev, per, S, H);
    return MARL_OK;
  }
  hipLaunchKernelGGL(gru_backward_kernel<NOUT>, dim3(blocks_for(S * H)), dim3(256), 0, s, dh_next, keep_next, dl, eff + o.W3,
                     rzn, ghn, hprev, dgi, dgh, dhprev, per, S, H);
  if (want_dhprev) {  // dL/dhprev += dgh Wh^T (what flows into the step before)
    GemmArgs g{};
    g.A = RowSrc{dgh, 3 * H, nullptr, 1, S}; g.B = eff + o.Wh; g.ldb = 3 * H; g.C = dhprev; g.ldc = H;
    g.M = S; g.N = H; g.K = 3 * H;
    launch_gemm<GEMM_NT, EPI_ATOMIC_ADD>(g, s);
  }
  return MARL_OK;
}

// ---- rollout ---------------------------------------------------------------------------------------------

struct RecRolloutWs {
  float *eff, *ha, *hc, *hc_tmp, *E, *Gi, *Gh;
};
RecRolloutWs carve_rec_rollout(const marl_config& c, void* ws, int64_t* total) {
  const Dims d = dims_of(c);
  const int64_t Sc = d.central ? d.N : d.NA;
  const int64_t Hm = std::max(d.Ha, d.Hc), Sm = d.NA;
  char* p = static_cast<char*>(ws);
  int64_t off = 0;
  auto take = [&](int64_t bytes) {
    char* r = p + off;
    off += align256(bytes);
    return (float*)r;
  };
  RecRolloutWs w;
  w.eff = take(rec_param_map(d).total * 4);
  w.ha = take(d.NA * d.Ha * 4);
  w.hc = take(Sc * d.Hc * 4);
  w.hc_tmp = take(Sc * d.Hc * 4);
  w.E = take(Sm * Hm * 4);
  w.Gi = take(Sm * 3 * Hm * 4);
  w.Gh = take(Sm * 3 * Hm * 4);
  if (total) *total = off;
  return w;
}

// One step of one recurrent network on S samples: hidden state h_in -> h_out (may alias).
void rec_cell_step(const RowSrc& X, int64_t S, int Din, int H, const float* eff, const RecOffsets& o, const float* wh_op,
                   const float* h_in, float* h_out, const RecRolloutWs& w, hipStream_t s) {
  embed_and_input_gates(X, S, Din, H, eff, o, w.E, w.Gi, s);
  launch_step_forward(w.Gi, h_in, S, H, eff, o, wh_op, w.Gh, nullptr, nullptr, h_out, nullptr, nullptr, 1, s);
}

}  // namespace

int64_t rec_rollout_workspace_bytes(const marl_config& c) {
  int64_t total = 0;
  carve_rec_rollout(c, nullptr, &total);
  return total;
}

int32_t launch_rollout_recurrent(const marl_config& c, marl_env_state st, const float* params, marl_traj tr,
                                 marl_rec_state rec, uint64_t step_offset, const int32_t* forced_actions,
                                 const float* forced_uniforms, void* workspace, hipStream_t s) {
  const Dims d = dims_of(c);
  const RecRolloutWs w = carve_rec_rollout(c, workspace, nullptr);
  const float* eff = stage_params(d, params, w.eff, s);
  const RecParamMap pm = rec_param_map(d);
  const RecOffsets oa = rec_padded(pm, 0), oc = rec_padded(pm, 1);
  const int64_t NA = d.NA, slab = NA * d.D;
  const int64_t Sc = d.central ? d.N : NA;
  const int per_c = d.central ? 1 : d.A;
  hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks_for(NA * d.Ha)), dim3(256), 0, s, rec.ha0, w.ha, NA * d.Ha);
  hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks_for(Sc * d.Hc)), dim3(256), 0, s, rec.hc0, w.hc, Sc * d.Hc);
  int32_t rc = launch_env_step(c, st, nullptr, tr.obs, nullptr, nullptr, /*do_step=*/false, s);
  if (rc != MARL_OK) return rc;
  auto mask = [&](int t_done) {  // a new episode starts from the zero state
    const uint8_t* dn = tr.done + (int64_t)t_done * d.N;
    hipLaunchKernelGGL(mask_hidden_kernel, dim3(blocks_for(NA * d.Ha)), dim3(256), 0, s, w.ha, dn, NA * d.Ha, d.Ha, d.A);
    hipLaunchKernelGGL(mask_hidden_kernel, dim3(blocks_for(Sc * d.Hc)), dim3(256), 0, s, w.hc, dn, Sc * d.Hc, d.Hc, per_c);
  };
  for (int t = 0; t < d.T; ++t) {
    if (t > 0) mask(t - 1);
    const float* obs_t = tr.obs + (int64_t)t * slab;
    SampleArgs a{};
    a.uniforms = forced_uniforms ? forced_uniforms + (int64_t)t * NA * kActions : nullptr;
    a.forced = forced_actions ? forced_actions + (int64_t)t * NA : nullptr;
    a.action = tr.action + (int64_t)t * NA;
    a.sampled = tr.sampled ? tr.sampled + (int64_t)t * NA : nullptr;
    a.logp = tr.logp + (int64_t)t * NA;
    a.step = step_offset + (uint64_t)t;
    a.k0 = (uint32_t)(c.seed & 0xffffffffu);
    a.k1 = (uint32_t)(c.seed >> 32);
    rec_cell_step(RowSrc{obs_t, d.D, nullptr, 1, NA}, NA, d.D, d.Ha, eff, oa, eff + pm.wh_op[0], w.ha, w.ha, w, s);
    launch_actor_head_rollout(w.ha, NA, d.Ha, eff + oa.W3, eff + oa.b3,
                              tr.logits ? tr.logits + (int64_t)t * NA * kActions : (float*)nullptr, &a, s);
    rec_cell_step(RowSrc{obs_t, d.Dc, nullptr, 1, Sc}, Sc, d.Dc, d.Hc, eff, oc, eff + pm.wh_op[1], w.hc, w.hc, w, s);
    launch_critic_head_rollout(w.hc, Sc, d.Hc, eff + oc.W3, eff + oc.b3, tr.value + (int64_t)t * NA, d.central ? d.A : 1, s);
    rc = launch_env_step(c, st, a.action, tr.obs + (int64_t)(t + 1) * slab, tr.reward + (int64_t)t * NA,
                         tr.done + (int64_t)t * d.N, true, s);
    if (rc != MARL_OK) return rc;
  }
  mask(d.T - 1);
  hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks_for(NA * d.Ha)), dim3(256), 0, s, w.ha, rec.ha1, NA * d.Ha);
  hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks_for(Sc * d.Hc)), dim3(256), 0, s, w.hc, rec.hc1, Sc * d.Hc);
  // bootstrap value of the post-rollout observation; the hidden state of the next rollout stays as it is
  rec_cell_step(RowSrc{tr.obs + (int64_t)d.T * slab, d.Dc, nullptr, 1, Sc}, Sc, d.Dc, d.Hc, eff, oc, eff + pm.wh_op[1], w.hc, w.hc_tmp, w, s);
  launch_critic_head_rollout(w.hc_tmp, Sc, d.Hc, eff + oc.W3, eff + oc.b3, tr.last_value, d.central ? d.A : 1, s);
  return launch_status();
}

// ---- sequence PPO update ------------------------------------------------------------------------------------

namespace {

// buffers of one network's forward and backward pass over a minibatch
struct RecNetWs {
  float *dl, *E, *G, *RZN, *GHN, *Hout, *Hprev, *GhT, *dGh, *dHp;
};
struct RecUpdateWs {
  float *eff, *grad;
  Scalars* sc;
  int32_t *ident, *rows;
  float* keep;
  RecNetWs net[2];  // actor, critic: a set each, so that the two networks can run side by side
};

RecUpdateWs carve_rec_update(const marl_config& c, void* ws, int64_t* total) {
  const Dims d = dims_of(c);
  const int64_t J = d.N / c.n_minibatches, TJ = (int64_t)d.T * J;
  const int64_t Sa = TJ * d.A, Sc = d.central ? TJ : Sa;                // samples of a minibatch over all steps
  const int64_t S1a = J * d.A, S1c = d.central ? J : S1a;              // samples of one step
  char* p = static_cast<char*>(ws);
  int64_t off = 0;
  auto take = [&](int64_t bytes) {
    char* r = p + off;
    off += align256(bytes);
    return r;
  };
  RecUpdateWs w;
  w.eff = (float*)take(rec_param_map(d).total * 4);
  w.grad = (float*)take(d.P * 4);
  w.sc = (Scalars*)take(sizeof(Scalars));
  w.ident = (int32_t*)take((int64_t)d.N * 4);
  w.rows = (int32_t*)take(TJ * 4);
  w.keep = (float*)take(TJ * 4);
  for (int k = 0; k < 2; ++k) {
    const int64_t SH = k == 0 ? Sa * d.Ha : Sc * d.Hc, S1H = k == 0 ? S1a * d.Ha : S1c * d.Hc;
    RecNetWs& n = w.net[k];
    n.dl = (float*)take((k == 0 ? Sa * kActions : Sc) * 4);
    n.E = (float*)take(SH * 4);
    n.G = (float*)take(3 * SH * 4);
    n.RZN = (float*)take(3 * SH * 4);
    n.GHN = (float*)take(SH * 4);
    n.Hout = (float*)take(SH * 4);
    n.Hprev = (float*)take((SH + S1H) * 4);
    n.GhT = (float*)take(3 * S1H * 4);
    n.dGh = (float*)take(3 * SH * 4);
    n.dHp = (float*)take(2 * S1H * 4);
  }
  if (total) *total = off;
  return w;
}

// Forward over the T steps, loss, and back-propagation through time of one network on a minibatch of J sequences
// (`per` samples per environment row).  Samples are ordered [t][j][a].
template <int NOUT, class LossFn>
int32_t train_net_recurrent(const RowSrc& X, int T, int64_t J, int per, int Din, int H, const float* h0,
                            const int32_t* envs, const float* eff, const RecOffsets& o, const float* wh_op,
                            const float* wht_op, float* grad, const RecOffsets& go, const LossFn& fn, const RecNetWs& w,
                            const float* keep, Scalars* sc, hipStream_t s) {
  const int64_t S1 = J * per, S = (int64_t)T * S1;
  hipLaunchKernelGGL(gather_hidden_kernel, dim3(blocks_for(S1 * H)), dim3(256), 0, s, h0, envs, (int)J, per, H, w.Hprev);
  embed_and_input_gates(X, S, Din, H, eff, o, w.E, w.G, s);
  for (int t = 0; t < T; ++t) {
    const float* hprev = w.Hprev + (int64_t)t * S1 * H;
    const int32_t rc = launch_step_forward(w.G + (int64_t)t * S1 * 3 * H, hprev, S1, H, eff, o, wh_op, w.GhT,
                                           w.RZN + (int64_t)t * S1 * 3 * H, w.GHN + (int64_t)t * S1 * H,
                                           w.Hout + (int64_t)t * S1 * H,
                                           t + 1 < T ? w.Hprev + (int64_t)(t + 1) * S1 * H : (float*)nullptr,
                                           t + 1 < T ? keep + (int64_t)(t + 1) * J : (const float*)nullptr, per, s);
    if (rc != MARL_OK) return rc;
  }
  {  // output layer, loss, dL/dout, W3 / b3 gradient over all steps
    const unsigned nb = (unsigned)std::min<int64_t>(2048, (S + kHeadTile - 1) / kHeadTile);
    hipLaunchKernelGGL((loss_head_kernel<NOUT, LossFn, float>), dim3(nb), dim3(256), 0, s, w.Hout, S, H, eff + o.W3,
                       eff + o.b3, fn, w.dl, grad + go.W3, grad + go.b3, sc, 0.f);
  }
  for (int t = T - 1; t >= 0; --t) {
    float* dhp = w.dHp + (int64_t)(t & 1) * S1 * H;
    const float* dh_next = t + 1 < T ? w.dHp + (int64_t)((t + 1) & 1) * S1 * H : (const float*)nullptr;
    float* dgi = w.G + (int64_t)t * S1 * 3 * H;  // the input-gate products are no longer needed: their gradient takes their place
    float* dgh = w.dGh + (int64_t)t * S1 * 3 * H;
    const int32_t rc = launch_step_backward<NOUT>(dh_next, t + 1 < T ? keep + (int64_t)(t + 1) * J : (const float*)nullptr,
                                                  w.dl + (int64_t)t * S1 * NOUT, w.RZN + (int64_t)t * S1 * 3 * H,
                                                  w.GHN + (int64_t)t * S1 * H, w.Hprev + (int64_t)t * S1 * H, S1, H, eff, o,
                                                  wht_op, dgi, dgh, dhp, t > 0, per, s);
    if (rc != MARL_OK) return rc;
  }
  const int64_t tiles_h3 = ((H + 127) / 128) * ((3 * H + 127) / 128);
  {  // gWh += Hprev^T dGh, gbh += column sums
    GemmArgs g{};
    g.A = RowSrc{w.Hprev, H, nullptr, 1, S}; g.B = w.dGh; g.ldb = 3 * H; g.C = grad + go.Wh; g.ldc = 3 * H;
    g.M = H; g.N = 3 * H; g.K = S; g.colsum = grad + go.bh; g.k_per_split = k_split(S, tiles_h3);
    launch_gemm<GEMM_TN, EPI_ATOMIC_ADD>(g, s);
  }
  {  // gWi += E^T dGi, gbi += column sums
    GemmArgs g{};
    g.A = RowSrc{w.E, H, nullptr, 1, S}; g.B = w.G; g.ldb = 3 * H; g.C = grad + go.Wi; g.ldc = 3 * H;
    g.M = H; g.N = 3 * H; g.K = S; g.colsum = grad + go.bi; g.k_per_split = k_split(S, tiles_h3);
    launch_gemm<GEMM_TN, EPI_ATOMIC_ADD>(g, s);
  }
  {  // dE = (dGi Wi^T) * (1 - e^2), in place over e
    GemmArgs g{};
    g.A = RowSrc{w.G, 3 * H, nullptr, 1, S}; g.B = eff + o.Wi; g.ldb = 3 * H; g.C = w.E; g.ldc = H;
    g.aux_mat = w.E; g.ldaux = H; g.M = S; g.N = H; g.K = 3 * H;
    launch_gemm<GEMM_NT, EPI_DTANH>(g, s);
  }
  {  // gWe += X^T dE, gbe += column sums
    GemmArgs g{};
    g.A = X; g.B = w.E; g.ldb = H; g.C = grad + go.We; g.ldc = H;
    g.M = Din; g.N = H; g.K = S; g.colsum = grad + go.be;
    g.k_per_split = k_split(S, ((Din + 127) / 128) * ((H + 127) / 128));
    launch_gemm<GEMM_TN, EPI_ATOMIC_ADD>(g, s);
  }
  return MARL_OK;
}

}  // namespace

int64_t rec_update_workspace_bytes(const marl_config& c) {
  int64_t total = 0;
  carve_rec_update(c, nullptr, &total);
  return total;
}

int32_t launch_ppo_update_recurrent(const marl_config& c, marl_traj tr, marl_rec_state rec, float* params, float* adam_m,
                                    float* adam_v, int64_t adam_step0, const int32_t* perm, float* stats,
                                    float* grad_dump, void* workspace, hipStream_t s) {
  const Dims d = dims_of(c);
  const RecUpdateWs w = carve_rec_update(c, workspace, nullptr);
  const int64_t J = d.N / c.n_minibatches, TJ = (int64_t)d.T * J;
  if (perm == nullptr) hipLaunchKernelGGL(iota_kernel, dim3(blocks_for(d.N)), dim3(256), 0, s, w.ident, (int64_t)d.N);
  const RecOffsets ga = rec_offsets(0, d.D, d.Ha, kActions), gc = rec_offsets(d.Pa, d.Dc, d.Hc, 1);
  const RecParamMap pm = rec_param_map(d);
  const RecOffsets oa = rec_padded(pm, 0), oc = rec_padded(pm, 1);
  const SideStream* const side = side_stream();
  int64_t k = adam_step0;
  for (int e = 0; e < c.n_epochs; ++e) {
    for (int mb = 0; mb < c.n_minibatches; ++mb) {
      const int32_t* envs = (perm ? perm + (int64_t)e * d.N : w.ident) + (int64_t)mb * J;
      const float* eff = stage_params(d, params, w.eff, s);
      hipLaunchKernelGGL(zero_step_kernel, dim3(blocks_for(d.P)), dim3(256), 0, s, w.grad, d.P, w.sc, 1, (double*)nullptr, 0);
      hipLaunchKernelGGL(seq_index_kernel, dim3(blocks_for(TJ)), dim3(256), 0, s, envs, tr.done, (int)J, d.N, d.T, w.rows, w.keep);
      LossCommon lc{};
      lc.rows = w.rows; lc.A = d.A; lc.ad = make_small_div(d.A); lc.rows_mb = TJ; lc.inv_B = (float)(1.0 / (double)(TJ * d.A));
      lc.sc = w.sc; lc.adv_stats = &w.sc->adv_sum; lc.normalize = c.normalize_adv; lc.clip_eps = c.clip_eps; lc.ent_coef = c.ent_coef;
      lc.vf_coef = c.vf_coef; lc.clip_value = c.clip_value;
      if (c.normalize_adv) {
        const unsigned nb = (unsigned)std::min<int64_t>(256, (TJ * d.A + 255) / 256);
        hipLaunchKernelGGL(adv_stats_kernel, dim3(nb), dim3(256), 0, s, tr.adv, lc, w.sc);
      }
      // The two networks share nothing but their inputs and write disjoint parts of the gradient: the critic runs on the
      // second stream beside the actor.  A time step of either is a short chain of dependent matrix instructions on a
      // few hundred workgroups, so the two chains interleave on the compute units instead of following one another.
      hipStream_t s2 = s;
      if (side != nullptr && hipEventRecord(side->fork, s) == hipSuccess && hipStreamWaitEvent(side->stream, side->fork, 0) == hipSuccess)
        s2 = side->stream;
      int32_t rc_a, rc_c;
      {
        ActorLoss fn{lc, tr.action, tr.logp, tr.adv};
        rc_a = train_net_recurrent<kActions>(RowSrc{tr.obs, d.D, w.rows, d.A, TJ * d.A}, d.T, J, d.A, d.D, d.Ha, rec.ha0, envs,
                                             eff, oa, eff + pm.wh_op[0], eff + pm.wht_op[0], w.grad, ga, fn, w.net[0], w.keep,
                                             w.sc, s);
      }
      {
        CriticLoss fn{lc, tr.ret, tr.value, d.central ? d.A : 1};
        const int per = d.central ? 1 : d.A;
        rc_c = train_net_recurrent<1>(RowSrc{tr.obs, d.Dc, w.rows, per, TJ * per}, d.T, J, per, d.Dc, d.Hc, rec.hc0, envs, eff,
                                      oc, eff + pm.wh_op[1], eff + pm.wht_op[1], w.grad, gc, fn, w.net[1], w.keep, w.sc, s2);
      }
      if (s2 != s) {  // join also after an error, so that the caller's stream never runs ahead of work still queued beside it
        if (hipEventRecord(side->join, s2) != hipSuccess || hipStreamWaitEvent(s, side->join, 0) != hipSuccess) {
          (void)hipStreamSynchronize(s2);
          return MARL_E_LAUNCH;
        }
      }
      if (rc_a != MARL_OK) return rc_a;
      if (rc_c != MARL_OK) return rc_c;
      hipLaunchKernelGGL(grad_norm_kernel, dim3(grad_norm_blocks(d.P)), dim3(256), 0, s,
                         w.grad, d.P, w.sc);
      ++k;
      AdamArgs a{};
      a.norm_blocks = (int)grad_norm_blocks(d.P);
      a.lr = c.lr; a.b1 = c.beta1; a.b2 = c.beta2; a.eps = c.adam_eps;
      a.bc1 = (float)(1.0 - std::pow((double)c.beta1, (double)k));
      a.bc2 = (float)(1.0 - std::pow((double)c.beta2, (double)k));
      a.max_norm = c.max_grad_norm; a.ent_coef = c.ent_coef; a.vf_coef = c.vf_coef;
      const bool last = (e == c.n_epochs - 1 && mb == c.n_minibatches - 1);
      hipLaunchKernelGGL(adam_kernel, dim3(blocks_for(d.P)), dim3(256), 0, s, params, adam_m, adam_v, w.grad, d.P, a, w.sc,
                         stats + (int64_t)(e * c.n_minibatches + mb) * MARL_N_STATS, (last ? grad_dump : (float*)nullptr),
                         (Scalars*)nullptr);
      const int32_t rc = launch_status();
      if (rc != MARL_OK) return rc;
    }
  }
  return MARL_OK;
}

}  // namespace marl
