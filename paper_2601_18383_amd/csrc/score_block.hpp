// Importance score from a block of T queries at once (Eq. importance-score with the sum over the
// answer tokens written out; App. B.1: the answer-by-thinking sub-matrix of the attention weights,
// summed over heads and over the answer dimension).  A dense [T*G x n] contraction per
// (sequence, KV head), done on the matrix cores in two passes over Q.K^T:
//   pass 1 (stats):  for every query row the log2 of its softmax denominator over the cached slots
//                    and, causally, the block's own keys  ->  L[row]  (one float per row);
//   pass 2 (colsum): logits again, p = 2^(logit - L[row]), summed over the rows for every cached
//                    slot  ->  dst[slot].
// Recomputing the logits costs a second pass of MFMAs; keeping them would cost 4 bytes per
// (row, slot) of HBM traffic each way, which at these shapes is several times slower.
//
// Both passes have the same shape.  A wave keeps 64 rows of one operand in registers (pass 1: query
// rows, pass 2: cached keys) and streams the other operand through in 16-row tiles straight from
// global memory into MFMA operand registers (lane (r, kg) holds elements 32*ks + 8*kg .. +7 of row
// r, the layout v_mfma_f32_16x16x32_bf16 wants for A and for B alike), next tile's loads in flight
// while the current one is multiplied.  The product is always  keys (A, rows)  x  queries (B,
// columns): a lane ends up with 4 keys of ONE query column, so
//   * pass 1 keeps a private running (max, sum) per lane and query column and merges the four lane
//     groups once, at the end;
//   * pass 2 keeps private partial column sums per lane and key and merges the 16 lanes of a group
//     once, at the end.
// The four waves of a workgroup hold different stationary rows and stream the same tiles, which
// therefore come from L1/L2 after the first wave has touched them.  No LDS, no barrier.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attend.hpp"

namespace dynts {

constexpr int kSbWaves = 4;        // waves per workgroup
constexpr int kSbTiles = 4;        // stationary 16-row tiles per wave
constexpr int kSbRowsPerWave = 16 * kSbTiles;
constexpr int kSbRowsPerWg = kSbRowsPerWave * kSbWaves;

struct ScoreBlockParams {
  const uint16_t *K;        // layer base, [Nb][Hkv][cap][D]
  const uint16_t *q_blk;    // [Nb][T][Hq][D]
  const uint16_t *k_blk;    // [Nb][T][Hkv][D] or null
  const int32_t *seq_len;   // [Nb]
  const int32_t *n_prompt;  // [Nb]
  const uint8_t *active;    // [Nb] or null
  float *stats;             // [Nb][Hkv][Rpad]  log2 of the softmax denominator per query row
  float *dst;               // [Nb][Hkv][cap]
  int Nb, T, Hq, Hkv, G, cap, Rpad;
  int skip_prompt;          // 1: slots below n_prompt[b] are left alone (dst is the score array)
  int accumulate;           // 1: dst += sums, 0: dst = sums
  float scale_log2;         // softmax scale * log2(e)
};

// MFMA operand fragments of one row: 16 bytes per k-step at the lane's column group.
template <int D>
__device__ __forceinline__ void load_row_frags(bf16x8 (&f)[D / 32], const char *row, int kg) {
  const char *base = row + 16 * kg;
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks)
    f[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(base + 64 * ks));
}

// Workgroup -> (unit, block).  Consecutive workgroup ids go to the 8 XCDs in turn; this mapping
// keeps all blocks of one (sequence, KV head) unit on one XCD, so the operand they all stream is
// fetched into one L2 instead of eight.  Returns false for the padding of the last group of units.
__device__ __forceinline__ bool sb_map(int n_blk, int n_units, int &unit, int &blk) {
  const int id = blockIdx.x, xcd = id & 7, slot = id >> 3;
  unit = (slot / n_blk) * 8 + xcd;
  blk = slot % n_blk;
  return unit < n_units;
}

// A lane's walk over the query rows r = i * G + g of a KV head's group, 16 rows at a time.
struct QueryWalk {
  int r, i, g;
  uint32_t off;         // byte offset of row (i, g) from the (sequence, head-group) base
  int step_i, step_g;   // 16 = step_i * G + step_g
  uint32_t stride_i, stride_g;
  __device__ __forceinline__ void init(int r0, int G, int Hq, int D) {
    r = r0;
    i = r0 / G;
    g = r0 - i * G;
    step_i = 16 / G;
    step_g = 16 - step_i * G;
    stride_i = (uint32_t)Hq * D * 2;
    stride_g = (uint32_t)D * 2;
    off = (uint32_t)i * stride_i + (uint32_t)g * stride_g;
  }
  __device__ __forceinline__ void advance(int G) {
    r += 16;
    i += step_i;
    g += step_g;
    off += (uint32_t)step_i * stride_i + (uint32_t)step_g * stride_g;
    if (g >= G) {
      g -= G;
      i += 1;
      off += stride_i - (uint32_t)G * stride_g;
    }
  }
};

// ---- pass 1: log2 of the softmax denominator of every query row ---------------------------------
// 1-D grid of ceil(R / 256) * round_up(units, 8) workgroups, 256 threads.
template <int D>
__global__ __launch_bounds__(kSbWaves * 64) void score_block_stats_kernel(const ScoreBlockParams p) {
  constexpr int KS = D / 32;
  const int R = p.T * p.G;
  int unit, blk;
  if (!sb_map((R + kSbRowsPerWg - 1) / kSbRowsPerWg, p.Nb * p.Hkv, unit, blk)) return;
  const int b = unit / p.Hkv, h = unit - b * p.Hkv;
  if (p.active && !p.active[b]) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane & 15, kg = lane >> 4;
  const int row0 = blk * kSbRowsPerWg + wave * kSbRowsPerWave;
  if (row0 >= R) return;
  int n = p.seq_len[b];
  n = n < 0 ? 0 : (n > p.cap ? p.cap : n);
  const char *Kb = reinterpret_cast<const char *>(p.K + (size_t)unit * (size_t)p.cap * D);
  const char *Qb = reinterpret_cast<const char *>(p.q_blk + ((size_t)b * p.T * p.Hq + (size_t)h * p.G) * D);
  const float c = p.scale_log2;

  // stationary: this wave's query rows (B operand: column r16 of tile qt is row row0 + 16 qt + r16)
  bf16x8 qf[kSbTiles][KS];
  int vis_blk[kSbTiles];  // block keys [0, vis_blk) are visible to this lane's query column
#pragma unroll
  for (int qt = 0; qt < kSbTiles; ++qt) {
    int r = row0 + 16 * qt + r16;
    r = r < R ? r : R - 1;
    const int i = r / p.G, g = r - i * p.G;
    vis_blk[qt] = i + 1;
    load_row_frags<D>(qf[qt], Qb + ((size_t)i * p.Hq + g) * (size_t)(2 * D), kg);
  }

  // running max (in raw dot-product units) and sum of 2^(c * (dot - max)), private to the lane
  float m[kSbTiles], l[kSbTiles];
#pragma unroll
  for (int qt = 0; qt < kSbTiles; ++qt) {
    m[qt] = -1e30f;
    l[qt] = 0.f;
  }

  // one streamed tile: keys (4 kg + i) x query column r16, folded into (m, l).  MASKED: keys whose
  // index key0 + 4 kg + i is not below lim[qt] do not exist for this query column.
#define DYNTS_SB_FOLD(kf_, MASKED, key0_, lim_)                                                        \
  _Pragma("unroll") for (int qt = 0; qt < kSbTiles; ++qt) {                                            \
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};                                                                  \
    _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                                  \
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf_[ks], qf[qt][ks], acc, 0, 0, 0);              \
    if (MASKED) {                                                                                      \
      _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                    \
          if ((key0_) + 4 * kg + i >= lim_[qt]) acc[i] = -INFINITY;                                    \
    }                                                                                                  \
    const float mn = fmaxf(fmaxf(fmaxf(acc[0], acc[1]), fmaxf(acc[2], acc[3])), m[qt]);                \
    const float nm = -mn * c;                                                                          \
    float sum = l[qt] * fast_exp2((m[qt] - mn) * c); /* exactly 2^0 while nothing has been seen */     \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) sum += fast_exp2(fmaf(acc[i], c, nm));               \
    m[qt] = mn;                                                                                        \
    l[qt] = sum;                                                                                       \
  }

  // cached slots: pairs of full tiles from two register buffers in turn, then the ragged rest
  {
    int lim[kSbTiles];
#pragma unroll
    for (int qt = 0; qt < kSbTiles; ++qt) lim[qt] = n;
    bf16x8 ka[KS], kb[KS];
    const int n_pairs = n & ~31;
    const uint32_t last_off = (uint32_t)(n > 0 ? n - 1 : 0) * (uint32_t)(2 * D);
    uint32_t off = (uint32_t)r16 * (uint32_t)(2 * D);
    if (n > 0) load_row_frags<D>(ka, Kb + (off < last_off ? off : last_off), kg);
    for (int j0 = 0; j0 < n_pairs; j0 += 32) {
      load_row_frags<D>(kb, Kb + off + 16 * 2 * D, kg);  // tile j0 + 16 is full: j0 + 32 <= n
      DYNTS_SB_FOLD(ka, false, 0, lim)
      off += 32 * 2 * D;
      load_row_frags<D>(ka, Kb + (off < last_off ? off : last_off), kg);
      DYNTS_SB_FOLD(kb, false, 0, lim)
    }
    if (n_pairs < n) {
      DYNTS_SB_FOLD(ka, true, n_pairs, lim)
      if (n_pairs + 16 < n) {
        const uint32_t o2 = off + 16 * 2 * D;
        load_row_frags<D>(kb, Kb + (o2 < last_off ? o2 : last_off), kg);
        DYNTS_SB_FOLD(kb, true, n_pairs + 16, lim)
      }
    }
  }

  // the block's own keys, causally: key i' is visible to query row (i, g) iff i' <= i
  if (p.k_blk) {
    int last = row0 + kSbRowsPerWave - 1;
    last = last < R ? last : R - 1;
    const int i_hi = last / p.G + 1;  // keys [0, i_hi) are visible to some row of this wave
    const char *kb0 = reinterpret_cast<const char *>(p.k_blk + ((size_t)b * p.T * p.Hkv + h) * D);
    const size_t kstride = (size_t)p.Hkv * D * 2;
    bf16x8 kf[KS], kn[KS];
    load_row_frags<D>(kf, kb0 + (size_t)(r16 < p.T ? r16 : p.T - 1) * kstride, kg);
    for (int i0 = 0; i0 < i_hi; i0 += 16) {
      int row = i0 + 16 + r16;
      row = row < p.T ? row : p.T - 1;
      load_row_frags<D>(kn, kb0 + (size_t)row * kstride, kg);
      DYNTS_SB_FOLD(kf, true, i0, vis_blk)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kf[ks] = kn[ks];
    }
  }
#undef DYNTS_SB_FOLD

  // merge the four lane groups of every query column, write L = c * m + log2(l)
#pragma unroll
  for (int qt = 0; qt < kSbTiles; ++qt) {
#pragma unroll
    for (int sh = 16; sh <= 32; sh <<= 1) {
      const float mo = __shfl_xor(m[qt], sh), lo = __shfl_xor(l[qt], sh);
      const float mn = fmaxf(m[qt], mo);
      l[qt] = l[qt] * fast_exp2((m[qt] - mn) * c) + lo * fast_exp2((mo - mn) * c);
      m[qt] = mn;
    }
    const int r = row0 + 16 * qt + r16;
    if (kg == 0 && r < R) p.stats[(size_t)unit * (size_t)p.Rpad + r] = m[qt] * c + __builtin_amdgcn_logf(l[qt]);
  }
}

// ---- pass 2: attention received by every cached slot, summed over the block's query rows ----------
// 1-D grid of ceil(cap / 256) * round_up(units, 8) workgroups, 256 threads.
template <int D>
__global__ __launch_bounds__(kSbWaves * 64) void score_block_colsum_kernel(const ScoreBlockParams p) {
  constexpr int KS = D / 32;
  int unit, blk;
  if (!sb_map((p.cap + kSbRowsPerWg - 1) / kSbRowsPerWg, p.Nb * p.Hkv, unit, blk)) return;
  const int b = unit / p.Hkv, h = unit - b * p.Hkv;
  if (p.active && !p.active[b]) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane & 15, kg = lane >> 4;
  const int R = p.T * p.G;
  int n = p.seq_len[b];
  n = n < 0 ? 0 : (n > p.cap ? p.cap : n);
  int first = 0;
  if (p.skip_prompt) {
    first = p.n_prompt[b];
    first = first < 0 ? 0 : first;
  }
  const int key0 = blk * kSbRowsPerWg + wave * kSbRowsPerWave;
  if (key0 >= n || key0 + kSbRowsPerWave <= first) return;
  const char *Kb = reinterpret_cast<const char *>(p.K + (size_t)unit * (size_t)p.cap * D);
  const char *Qb = reinterpret_cast<const char *>(p.q_blk + ((size_t)b * p.T * p.Hq + (size_t)h * p.G) * D);
  const float *Lb = p.stats + (size_t)unit * (size_t)p.Rpad;
  const float c = p.scale_log2;

  // stationary: this wave's cached keys (A operand: row r16 of tile kt is slot key0 + 16 kt + r16)
  bf16x8 kf[kSbTiles][KS];
#pragma unroll
  for (int kt = 0; kt < kSbTiles; ++kt) {
    int row = key0 + 16 * kt + r16;
    row = row < n ? row : n - 1;
    load_row_frags<D>(kf[kt], Kb + (size_t)row * (size_t)(2 * D), kg);
  }
  f32x4 sum[kSbTiles];
#pragma unroll
  for (int kt = 0; kt < kSbTiles; ++kt) sum[kt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // streamed: 16 query rows at a time from two register buffers in turn.  A row beyond the last
  // repeats the last row's data with L = +inf, so it contributes 2^(-inf) = 0.
  QueryWalk w;
  w.init(r16, p.G, p.Hq, D);
  const uint32_t last_off = (uint32_t)(p.T - 1) * w.stride_i + (uint32_t)(p.G - 1) * w.stride_g;
#define DYNTS_SB_LOAD(qf_, L_)                                           \
  load_row_frags<D>(qf_, Qb + (w.r < R ? w.off : last_off), kg);        \
  L_ = w.r < R ? Lb[w.r] : INFINITY;                                     \
  w.advance(p.G);
#define DYNTS_SB_ADD(qf_, L_)                                                                          \
  _Pragma("unroll") for (int kt = 0; kt < kSbTiles; ++kt) {                                            \
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};                                                                  \
    _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                                  \
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kt][ks], qf_[ks], acc, 0, 0, 0);              \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) sum[kt][i] += fast_exp2(fmaf(acc[i], c, -L_));       \
  }
  bf16x8 qa[KS], qb[KS];
  float La, Lq;
  DYNTS_SB_LOAD(qa, La)
  for (int r0 = 0; r0 < R; r0 += 32) {
    DYNTS_SB_LOAD(qb, Lq)
    DYNTS_SB_ADD(qa, La)
    DYNTS_SB_LOAD(qa, La)
    DYNTS_SB_ADD(qb, Lq)
  }
#undef DYNTS_SB_LOAD
#undef DYNTS_SB_ADD

  // sum[kt][i] holds slot key0 + 16 kt + 4 kg + i for query columns == r16 (mod 16): add the 16 lanes
#pragma unroll
  for (int kt = 0; kt < kSbTiles; ++kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float v = sum[kt][i];
      v += __shfl_xor(v, 1);
      v += __shfl_xor(v, 2);
      v += __shfl_xor(v, 4);
      v += __shfl_xor(v, 8);
      sum[kt][i] = v;
    }
  }
  // lane (r16 = 4 kt' + i', kg) writes slot key0 + 16 kt' + 4 kg + i'
  const int kt_w = r16 >> 2, i_w = r16 & 3;
  float v = 0.f;
#pragma unroll
  for (int kt = 0; kt < kSbTiles; ++kt)
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (kt == kt_w && i == i_w) v = sum[kt][i];
  const int slot = key0 + 16 * kt_w + 4 * kg + i_w;
  if (slot < n && slot >= first) {
    float *d = p.dst + (size_t)unit * (size_t)p.cap + slot;
    *d = p.accumulate ? *d + v : v;
  }
}

}  // namespace dynts
