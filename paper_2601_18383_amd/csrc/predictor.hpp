// Importance Predictor head (Sec. 4.1; App. A "Predictor Overhead"; App. C: 3584->7168->1792->1 and
// 4096->8192->2048->1): a three-layer MLP on the final hidden state of the current token of every
// sequence, s = w3 . act(W2 act(W1 h + b1) + b2) + b3, one score per token.  At decode batch sizes
// this is a skinny GEMM whose cost is reading the weights once (3 d^2 bf16 values, ~100 MB): HBM-bound.
//
// One GEMM kernel serves layers 1 and 2:  P[split][b][o] = sum_{k in split} W[o][k] * x[b][k].
//   * Weights are the MFMA A operand (16 output features per wave), loaded straight from HBM into
//     operand registers, 16 k-steps ahead.  The eight waves of a workgroup take eight neighbouring
//     feature tiles and share the activations.
//   * Activations are the B operand (batch as columns).  The workgroup's whole K slice of them is
//     fetched once with coalesced loads into padded LDS and read back in operand layout by all eight
//     waves.
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

struct MlpGemmParams {
  const uint16_t *W;    // [m][K] bf16
  const uint16_t *x0;   // [Nb][K] bf16 (hi part)
  const uint16_t *x1;   // [Nb][K] bf16 lo part, or null
  float *P;             // [nsplit][Nb][m] partial sums
  int Nb, m, K;
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

// k-steps (32 elements of K) one workgroup covers: its whole slice of the activations sits in 64 KB of LDS
// (128 KB for batches above 32, where the partial sums would otherwise outweigh the weights)
constexpr int mlp_slice_steps(int bt, int parts) { return (bt >= 4 ? 128 : 64) / (parts * bt); }

// BT = batch tiles of 16 (batch padded to 16 BT), PARTS = 1 (bf16 input) or 2 (hi + lo).
// grid (ceil(m / 128), ceil(K / 32 / S)), 512 threads, S = mlp_slice_steps(BT, PARTS).
// A workgroup fetches its slice of the activations once (all loads in flight together), parks it in
// LDS, meets at ONE barrier, and then only streams weights: a ring of DEPTH weight fragments per lane
// is kept in flight, so HBM latency is paid once per workgroup, not once per chunk.
template <int BT, int PARTS, bool PACKED>
__global__ __launch_bounds__(kMlpThreads) void mlp_gemm_kernel(const MlpGemmParams p) {
  constexpr int NBP = 16 * BT;                       // padded batch
  constexpr int S = mlp_slice_steps(BT, PARTS);      // k-steps per workgroup
  constexpr int DEPTH = S < 16 ? S : 16;             // weight fragments in flight per lane
  constexpr int LROW = S * 64 + 16;                  // padded LDS pitch of one batch row, bytes
  constexpr int PIECES = S * 4;                      // 16-byte pieces per batch row
  constexpr int NLD = PARTS * NBP * PIECES / kMlpThreads;  // = 8 staging loads per thread
  static_assert(PARTS * NBP * PIECES % kMlpThreads == 0, "staging must divide evenly");
  __shared__ __attribute__((aligned(16))) char lds[PARTS * NBP * LROW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kg = lane >> 4;
  const int f0 = blockIdx.x * kMlpFeaturesPerWg + wave * 16;
  const bool has_rows = f0 < p.m;
  const int n_steps_all = p.K / 32;
  const int s0 = blockIdx.y * S;
  int s1 = s0 + S;
  s1 = s1 < n_steps_all ? s1 : n_steps_all;
  if (s0 >= s1) return;  // uniform
  const int n_steps = s1 - s0;

  // this lane's weight fragments.  Row-major weights: 16 bytes of row f0 + r16 per k-step, i.e. 16 rows a
  // whole weight row apart per load instruction.  Packed weights ([m/16][K/32][16][32], see
  // mlp_pack_kernel): the 1 KB a load instruction needs is contiguous, and so is the whole slice.
  // (Rows past the last repeat it; their results are not written.)
  int frow = f0 + r16;
  frow = frow < p.m ? frow : p.m - 1;
  const char *Wrow =
      PACKED ? reinterpret_cast<const char *>(p.W + ((size_t)(frow >> 4) * n_steps_all + s0) * 512 + (frow & 15) * 32) + 16 * kg
             : reinterpret_cast<const char *>(p.W + (size_t)frow * p.K + (size_t)s0 * 32) + 16 * kg;
  constexpr size_t kStepBytes = PACKED ? 1024 : 64;
  // first weight fragments on their way before anything else (steps past the slice repeat its last)
  bf16x8 wf[DEPTH];
#pragma unroll
  for (int j = 0; j < DEPTH; ++j) {
    const int st = j < n_steps ? j : n_steps - 1;
    wf[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(Wrow + (size_t)st * kStepBytes));
  }

  // the slice of the activations: piece q = (part, batch row, 16-byte piece), coalesced along K
  {
    u32x4 stage[NLD];
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
      const int q = tid + kMlpThreads * k;
      const int part = q / (NBP * PIECES), rem = q - part * (NBP * PIECES);
      int row = rem / PIECES;
      const int piece = rem - row * PIECES;
      row = row < p.Nb ? row : p.Nb - 1;
      int e = s0 * 32 + 8 * piece;
      e = e < s1 * 32 ? e : s1 * 32 - 8;  // past the slice: repeat its last piece (never multiplied)
      const uint16_t *src = (PARTS == 2 && part == 1) ? p.x1 : p.x0;
      stage[k] = *reinterpret_cast<const u32x4 *>(src + (size_t)row * p.K + e);
    }
#pragma unroll
    for (int k = 0; k < NLD; ++k) {
      const int q = tid + kMlpThreads * k;
      const int part = q / (NBP * PIECES), rem = q - part * (NBP * PIECES);
      const int row = rem / PIECES, piece = rem - row * PIECES;
      *reinterpret_cast<u32x4 *>(lds + (part * NBP + row) * LROW + 16 * piece) = stage[k];
    }
  }
  __syncthreads();
  if (!has_rows) return;

  f32x4 acc[BT];
#pragma unroll
  for (int bt = 0; bt < BT; ++bt) acc[bt] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int sb = 0; sb < n_steps; sb += DEPTH) {
#pragma unroll
    for (int j = 0; j < DEPTH; ++j) {
      const int st = sb + j;
      if (st < n_steps) {  // uniform
#pragma unroll
        for (int bt = 0; bt < BT; ++bt) {
#pragma unroll
          for (int part = 0; part < PARTS; ++part) {
            const bf16x8 xf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(
                lds + (part * NBP + 16 * bt + r16) * LROW + 64 * st + 16 * kg));
            acc[bt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j], xf, acc[bt], 0, 0, 0);
          }
        }
      }
      if (S > DEPTH) {  // refill this ring slot with the fragment DEPTH steps ahead
        int nx = st + DEPTH;
        nx = nx < n_steps ? nx : n_steps - 1;
        wf[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(Wrow + (size_t)nx * kStepBytes));
      }
    }
  }

  // acc[bt][i]: feature f0 + 4 kg + i, batch 16 bt + r16
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

// Row-major bf16 weights [m][K] -> tiles of 16 rows x 32 columns stored contiguously, [m/16][K/32][16][32]:
// what one MFMA A-operand load of a wave reads becomes one contiguous kilobyte.  One-off, at load time.
// grid (ceil(m * K / 8 / 256)), 256 threads, 16 bytes per thread.
__global__ __launch_bounds__(256) void mlp_pack_kernel(const uint16_t *W, int m, int K, uint16_t *Wp) {
  const size_t piece = (size_t)blockIdx.x * 256 + threadIdx.x;  // 16-byte piece of the packed array
  if (piece >= (size_t)m * K / 8) return;
  const size_t e = piece * 8;                  // element index in the packed array
  const int c = (int)(e % 32), r = (int)((e / 32) % 16);
  const size_t ts = e / 512;                   // tile * n_steps + step
  const int n_steps = K / 32;
  const size_t tile = ts / n_steps, step = ts % n_steps;
  *reinterpret_cast<u32x4 *>(Wp + e) =
      *reinterpret_cast<const u32x4 *>(W + (tile * 16 + r) * (size_t)K + step * 32 + c);
}

// y = act(sum over splits of P + bias), written as bf16 hi and lo parts for the next layer.
// grid (ceil(Nb * m / 4 / 256)), 256 threads, 4 features per thread.
__global__ __launch_bounds__(256) void mlp_reduce_act_kernel(const float *P, const float *bias, int nsplit, int Nb,
                                                             int m, int act, uint16_t *y_hi, uint16_t *y_lo,
                                                             uint32_t *row_cnt) {
  // (the arrival counters of the final kernel of this call start from zero: stream order puts this first)
  if (blockIdx.x == 0 && (int)threadIdx.x < Nb) row_cnt[threadIdx.x] = 0;
  const size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (idx >= (size_t)Nb * m) return;
  const int o = (int)(idx % m);
  f32x4 v = *reinterpret_cast<const f32x4 *>(P + idx);
#pragma unroll 4
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

// s[b] = w3 . act(sum over splits of P[.][b][:] + bias) + b3, written n_rep times.
// grid (ceil(m / 256), Nb), 256 threads: a workgroup takes 256 features of one sequence and leaves its part of
// the dot product in part[b][blockIdx.x] as a tagged word (value + this call's serial number in one 64-bit
// atomic store, as the attention kernel's split partials); the workgroup that draws the last ticket of a
// sequence adds the parts in index order, re-reading a word until it carries this call's tag, so the result
// does not depend on the arrival order and no store has to be waited for.
__global__ __launch_bounds__(256) void mlp_reduce_dot_kernel(const float *P, const float *bias, int nsplit, int Nb,
                                                             int m, int act, const uint16_t *w3, const float *b3,
                                                             uint64_t *part, uint32_t tag, uint32_t *row_cnt,
                                                             float *s_out, int n_rep) {
  __shared__ float red[4];
  __shared__ int is_last;
  const int b = blockIdx.y, tid = threadIdx.x, o = blockIdx.x * 256 + tid;
  float t = 0.f;
  if (o < m) {
    float v = 0.f;
#pragma unroll 8
    for (int s = 0; s < nsplit; ++s) v += P[((size_t)s * Nb + b) * m + o];
    t = bf16_to_f32(w3[o]) * mlp_act(v + (bias ? bias[o] : 0.f), act);
  }
#pragma unroll
  for (int sh = 32; sh >= 1; sh >>= 1) t += __shfl_xor(t, sh);
  if ((tid & 63) == 0) red[tid >> 6] = t;
  __syncthreads();
  if (tid == 0) {
    tagged_store(part + (size_t)b * gridDim.x + blockIdx.x, (red[0] + red[1]) + (red[2] + red[3]), tag);
    is_last = atomicAdd(row_cnt + b, 1u) == gridDim.x - 1;
  }
  __syncthreads();
  if (!is_last) return;
  if (tid < n_rep) {
    float tot = 0.f;
    for (unsigned k = 0; k < gridDim.x; ++k) {
      uint64_t w;
      do w = tagged_load(part + (size_t)b * gridDim.x + k);
      while (!tag_is(w, tag));
      tot += tagged_value(w);
    }
    s_out[(size_t)b * n_rep + tid] = tot + (b3 ? b3[0] : 0.f);
  }
}

}  // namespace dynts
