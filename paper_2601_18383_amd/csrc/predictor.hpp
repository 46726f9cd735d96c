// Importance Predictor head (Sec. 4.1; App. A "Predictor Overhead"; App. C: 3584->7168->1792->1 and
// 4096->8192->2048->1): a three-layer MLP on the final hidden state of the current token of every
// sequence, s = w3 . act(W2 act(W1 h + b1) + b2) + b3, one score per token.  At decode batch sizes
// this is a skinny GEMM whose cost is reading the weights once (3 d^2 bf16 values, ~100 MB): HBM-bound.
//
// One GEMM kernel serves layers 1 and 2:  P[split][b][o] = sum_{k in split} W[o][k] * x[b][k].
//   * Weights are the MFMA A operand (16 output features per wave), loaded straight from HBM into
//     operand registers, a whole chunk of k-steps ahead.  Eight waves of a workgroup take eight
//     neighbouring feature tiles and share the activations.
//   * Activations are the B operand (batch as columns).  A chunk of them is fetched with coalesced
//     loads into one of two padded LDS buffers and read back in operand layout by all eight waves.
//     Layer 2 takes its input as two bf16 arrays (hi + lo of the fp32 activation), two MFMAs per
//     weight fragment, so nothing is rounded to bf16 between the layers.
//   * K is split across workgroups (grid.y) so that a few hundred workgroups exist; the fp32
//     partials go to scratch and a small second kernel adds them, applies bias and activation and
//     writes the next layer's input (layer 1) or finishes with the dot product against w3 (layer 2).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attend.hpp"

namespace dynts {

constexpr int kMlpWaves = 8;
constexpr int kMlpThreads = kMlpWaves * 64;
constexpr int kMlpFeaturesPerWg = 16 * kMlpWaves;
constexpr int kMlpStageLoads = 2;  // 16-byte loads per thread and chunk of activations

struct MlpGemmParams {
  const uint16_t *W;    // [m][K] bf16
  const uint16_t *x0;   // [Nb][K] bf16 (hi part)
  const uint16_t *x1;   // [Nb][K] bf16 lo part, or null
  float *P;             // [nsplit][Nb][m] partial sums
  int Nb, m, K;
  int steps_per_split;  // k-steps (32 elements) per grid.y slice
};

__device__ __forceinline__ float mlp_act(float x, int act) {
  if (act == 1) return x > 0.f ? x : 0.f;
  if (act == 2) return x / (1.f + __expf(-x));
  return x;
}

// round-to-nearest-even bf16 of a finite float
__device__ __forceinline__ uint16_t f32_to_bf16(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// BT = batch tiles of 16 (batch padded to 16 BT), PARTS = 1 (bf16 input) or 2 (hi + lo).
// grid (ceil(m / 128), nsplit), 512 threads.
template <int BT, int PARTS>
__global__ __launch_bounds__(kMlpThreads) void mlp_gemm_kernel(const MlpGemmParams p) {
  constexpr int NBP = 16 * BT;                                   // padded batch
  constexpr int KCS = (256 / (PARTS * NBP)) > 0 ? 256 / (PARTS * NBP) : 1;  // k-steps per chunk
  constexpr int KC = 32 * KCS;                                   // elements per chunk
  constexpr int LROW = KC * 2 + 16;                              // padded LDS pitch of one batch row
  constexpr int PIECES = KC / 8;                                 // 16-byte pieces per row and chunk
  constexpr int NLD = (PARTS * NBP * PIECES + kMlpThreads - 1) / kMlpThreads;
  __shared__ __attribute__((aligned(16))) char lds[2][PARTS * NBP * LROW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kg = lane >> 4;
  const int f0 = blockIdx.x * kMlpFeaturesPerWg + wave * 16;
  const bool has_rows = f0 < p.m;
  const int n_steps_all = p.K / 32;
  const int s0 = blockIdx.y * p.steps_per_split;
  int s1 = s0 + p.steps_per_split;
  s1 = s1 < n_steps_all ? s1 : n_steps_all;
  if (s0 >= s1) return;  // uniform
  const int n_chunks = (s1 - s0 + KCS - 1) / KCS;

  // this lane's weight row (rows past the last repeat it; their results are not written)
  int frow = f0 + r16;
  frow = frow < p.m ? frow : p.m - 1;
  const char *Wrow = reinterpret_cast<const char *>(p.W + (size_t)frow * p.K) + 16 * kg;
  const int last_step = s1 - 1;

  // staging of the activations: piece q of the chunk = (part, batch row, 16-byte piece)
  u32x4 stage[NLD];
#define DYNTS_MLP_FETCH(chunk_)                                                                        \
  _Pragma("unroll") for (int k = 0; k < NLD; ++k) {                                                    \
    const int q = tid + kMlpThreads * k;                                                               \
    if (q < PARTS * NBP * PIECES) {                                                                    \
      const int part = q / (NBP * PIECES), rem = q - part * (NBP * PIECES);                            \
      int row = rem / PIECES;                                                                          \
      const int piece = rem - row * PIECES;                                                            \
      row = row < p.Nb ? row : p.Nb - 1;                                                               \
      int e = (s0 + (chunk_) * KCS) * 32 + 8 * piece;  /* element index along K */                     \
      e = e < s1 * 32 ? e : s1 * 32 - 8;               /* past the slice: repeat its last piece */    \
      const uint16_t *src = (PARTS == 2 && part == 1) ? p.x1 : p.x0;                                   \
      stage[k] = *reinterpret_cast<const u32x4 *>(src + (size_t)row * p.K + e);                        \
    }                                                                                                  \
  }
#define DYNTS_MLP_PARK(buf_)                                                                           \
  _Pragma("unroll") for (int k = 0; k < NLD; ++k) {                                                    \
    const int q = tid + kMlpThreads * k;                                                               \
    if (q < PARTS * NBP * PIECES) {                                                                    \
      const int part = q / (NBP * PIECES), rem = q - part * (NBP * PIECES);                            \
      const int row = rem / PIECES, piece = rem - row * PIECES;                                        \
      *reinterpret_cast<u32x4 *>((buf_) + (part * NBP + row) * LROW + 16 * piece) = stage[k];          \
    }                                                                                                  \
  }
  // weight fragments of one chunk (steps past the slice repeat the last step; they are skipped below)
#define DYNTS_MLP_WLOAD(wf_, chunk_)                                                                   \
  _Pragma("unroll") for (int ks = 0; ks < KCS; ++ks) {                                                 \
    int st = s0 + (chunk_) * KCS + ks;                                                                 \
    st = st < last_step ? st : last_step;                                                              \
    wf_[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(Wrow + (size_t)st * 64));    \
  }
#define DYNTS_MLP_COMPUTE(wf_, buf_, chunk_)                                                           \
  if (has_rows) {                                                                                      \
    _Pragma("unroll") for (int ks = 0; ks < KCS; ++ks) {                                               \
      if (s0 + (chunk_) * KCS + ks < s1) { /* uniform */                                               \
        _Pragma("unroll") for (int bt = 0; bt < BT; ++bt) {                                            \
          _Pragma("unroll") for (int part = 0; part < PARTS; ++part) {                                 \
            const bf16x8 xf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(             \
                (buf_) + (part * NBP + 16 * bt + r16) * LROW + 64 * ks + 16 * kg));                    \
            acc[bt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf_[ks], xf, acc[bt], 0, 0, 0);          \
          }                                                                                            \
        }                                                                                              \
      }                                                                                                \
    }                                                                                                  \
  }

  f32x4 acc[BT];
#pragma unroll
  for (int bt = 0; bt < BT; ++bt) acc[bt] = f32x4{0.f, 0.f, 0.f, 0.f};
  bf16x8 wa[KCS], wb[KCS];

  DYNTS_MLP_FETCH(0)
  DYNTS_MLP_WLOAD(wa, 0)
  DYNTS_MLP_PARK(lds[0])
  if (n_chunks > 1) { DYNTS_MLP_FETCH(1) }
  __syncthreads();
  for (int ch = 0; ch < n_chunks; ch += 2) {
    // even chunk: weights in wa, activations in lds[0]
    if (ch + 1 < n_chunks) { DYNTS_MLP_WLOAD(wb, ch + 1) }
    DYNTS_MLP_COMPUTE(wa, lds[0], ch)
    if (ch + 1 < n_chunks) { DYNTS_MLP_PARK(lds[1]) }
    if (ch + 2 < n_chunks) { DYNTS_MLP_FETCH(ch + 2) }
    __syncthreads();
    if (ch + 1 >= n_chunks) break;
    // odd chunk: weights in wb, activations in lds[1]
    if (ch + 2 < n_chunks) { DYNTS_MLP_WLOAD(wa, ch + 2) }
    DYNTS_MLP_COMPUTE(wb, lds[1], ch + 1)
    if (ch + 2 < n_chunks) { DYNTS_MLP_PARK(lds[0]) }
    if (ch + 3 < n_chunks) { DYNTS_MLP_FETCH(ch + 3) }
    __syncthreads();
  }
#undef DYNTS_MLP_FETCH
#undef DYNTS_MLP_PARK
#undef DYNTS_MLP_WLOAD
#undef DYNTS_MLP_COMPUTE

  // acc[bt][i]: feature f0 + 4 kg + i, batch 16 bt + r16
  if (!has_rows) return;
  const int f = f0 + 4 * kg;
#pragma unroll
  for (int bt = 0; bt < BT; ++bt) {
    const int b = 16 * bt + r16;
    if (b < p.Nb && f < p.m) {  // m is a multiple of 16, so the four features are all valid
      float *dst = p.P + ((size_t)blockIdx.y * p.Nb + b) * p.m + f;
      *reinterpret_cast<f32x4 *>(dst) = acc[bt];
    }
  }
}

// y = act(sum over splits of P + bias), written as bf16 hi and lo parts for the next layer.
// grid (ceil(Nb * m / 4 / 256)), 256 threads, 4 features per thread.
__global__ __launch_bounds__(256) void mlp_reduce_act_kernel(const float *P, const float *bias, int nsplit, int Nb,
                                                             int m, int act, uint16_t *y_hi, uint16_t *y_lo) {
  const size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (idx >= (size_t)Nb * m) return;
  const int o = (int)(idx % m);
  f32x4 v = *reinterpret_cast<const f32x4 *>(P + idx);
  for (int s = 1; s < nsplit; ++s) v += *reinterpret_cast<const f32x4 *>(P + (size_t)s * Nb * m + idx);
  uint16_t hi[4], lo[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float y = mlp_act(v[i] + (bias ? bias[o + i] : 0.f), act);
    hi[i] = f32_to_bf16(y);
    lo[i] = f32_to_bf16(y - bf16_to_f32(hi[i]));
  }
  *reinterpret_cast<uint2 *>(y_hi + idx) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
  *reinterpret_cast<uint2 *>(y_lo + idx) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
}

// s[b] = w3 . act(sum over splits of P[.][b][:] + bias) + b3, written n_rep times.  grid (Nb), 256 threads.
__global__ __launch_bounds__(256) void mlp_reduce_dot_kernel(const float *P, const float *bias, int nsplit, int Nb,
                                                             int m, int act, const uint16_t *w3, const float *b3,
                                                             float *s_out, int n_rep) {
  __shared__ float red[4];
  const int b = blockIdx.x, tid = threadIdx.x;
  float acc = 0.f;
  for (int o = tid; o < m; o += 256) {
    float v = 0.f;
    for (int s = 0; s < nsplit; ++s) v += P[((size_t)s * Nb + b) * m + o];
    acc += bf16_to_f32(w3[o]) * mlp_act(v + (bias ? bias[o] : 0.f), act);
  }
#pragma unroll
  for (int sh = 32; sh >= 1; sh >>= 1) acc += __shfl_xor(acc, sh);
  if ((tid & 63) == 0) red[tid >> 6] = acc;
  __syncthreads();
  if (tid < n_rep) s_out[(size_t)b * n_rep + tid] = red[0] + red[1] + red[2] + red[3] + (b3 ? b3[0] : 0.f);
}

}  // namespace dynts
