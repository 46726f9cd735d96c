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
  int T, Hq, Hkv, G, cap, Rpad;
  int skip_prompt;          // 1: slots below n_prompt[b] are left alone (dst is the score array)
  int accumulate;           // 1: dst += sums, 0: dst = sums
  float scale_log2;         // softmax scale * log2(e)
};

// MFMA operand fragments of one row: 16 bytes per k-step at the lane's column group.
template <int D>
__device__ __forceinline__ void load_row_frags(bf16x8 (&f)[D / 32], const uint16_t *row, int kg) {
  const char *base = reinterpret_cast<const char *>(row) + 16 * kg;
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks)
    f[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(base + 64 * ks));
}

// Address of query row r = i * G + g of the group of KV head h (rows beyond the last repeat it).
template <int D>
__device__ __forceinline__ const uint16_t *query_row(const ScoreBlockParams &p, int b, int h, int r, int R) {
  r = r < R ? r : R - 1;
  const int i = r / p.G, g = r - i * p.G;
  return p.q_blk + (((size_t)b * p.T + i) * p.Hq + (size_t)h * p.G + g) * D;
}

// ---- pass 1: log2 of the softmax denominator of every query row ---------------------------------
// grid (ceil(R / 256), Hkv, Nb), 256 threads.
template <int D>
__global__ __launch_bounds__(kSbWaves * 64) void score_block_stats_kernel(const ScoreBlockParams p) {
  constexpr int KS = D / 32;
  const int b = blockIdx.z, h = blockIdx.y;
  if (p.active && !p.active[b]) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane & 15, kg = lane >> 4;
  const int R = p.T * p.G;
  const int row0 = blockIdx.x * kSbRowsPerWg + wave * kSbRowsPerWave;
  if (row0 >= R) return;
  int n = p.seq_len[b];
  n = n < 0 ? 0 : (n > p.cap ? p.cap : n);
  const size_t unit = (size_t)b * p.Hkv + h;
  const uint16_t *Kb = p.K + unit * (size_t)p.cap * D;

  // stationary: this wave's query rows (B operand: column r16 of tile qt is row row0 + 16 qt + r16)
  bf16x8 qf[kSbTiles][KS];
#pragma unroll
  for (int qt = 0; qt < kSbTiles; ++qt) load_row_frags<D>(qf[qt], query_row<D>(p, b, h, row0 + 16 * qt + r16, R), kg);

  float m[kSbTiles], l[kSbTiles];
#pragma unroll
  for (int qt = 0; qt < kSbTiles; ++qt) {
    m[qt] = -1e30f;
    l[qt] = 0.f;
  }

  // one streamed tile: logits of keys (4 kg + i) x query column r16, folded into (m, l);
  // `vis[qt]`: keys with index below it are visible to this lane's query column of tile qt
  auto fold = [&](const bf16x8 (&kf)[KS], int key0, const int (&vis)[kSbTiles], bool masked) {
#pragma unroll
    for (int qt = 0; qt < kSbTiles; ++qt) {
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks], qf[qt][ks], acc, 0, 0, 0);
      float x[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        x[i] = acc[i] * p.scale_log2;
        if (masked && key0 + 4 * kg + i >= vis[qt]) x[i] = -INFINITY;
      }
      const float mx = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
      const float mn = fmaxf(m[qt], mx);
      float s = l[qt] * fast_exp2(m[qt] - mn);
#pragma unroll
      for (int i = 0; i < 4; ++i) s += fast_exp2(x[i] - mn);
      m[qt] = mn;
      l[qt] = s;
    }
  };

  // cached slots: full tiles unmasked, then the ragged tail
  {
    int vis[kSbTiles];
#pragma unroll
    for (int qt = 0; qt < kSbTiles; ++qt) vis[qt] = n;
    bf16x8 kf[KS], kn[KS];
    const int n_full = n & ~15;
    if (n > 0) {
      int row = r16 < n ? r16 : n - 1;
      load_row_frags<D>(kf, Kb + (size_t)row * D, kg);
    }
    for (int j0 = 0; j0 < n_full; j0 += 16) {
      int row = j0 + 16 + r16;
      row = row < n ? row : n - 1;
      load_row_frags<D>(kn, Kb + (size_t)row * D, kg);
      fold(kf, j0, vis, false);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kf[ks] = kn[ks];
    }
    if (n_full < n) fold(kf, n_full, vis, true);
  }

  // the block's own keys, causally: key i' is visible to query row r iff i' <= r / G
  if (p.k_blk) {
    int vis[kSbTiles];
    int last = row0 + kSbRowsPerWave - 1;
    last = last < R ? last : R - 1;
    const int i_hi = last / p.G + 1;  // keys [0, i_hi) are visible to some row of this wave
#pragma unroll
    for (int qt = 0; qt < kSbTiles; ++qt) {
      int r = row0 + 16 * qt + r16;
      r = r < R ? r : R - 1;
      vis[qt] = r / p.G + 1;
    }
    const uint16_t *kb0 = p.k_blk + ((size_t)b * p.T * p.Hkv + h) * D;
    const size_t kstride = (size_t)p.Hkv * D;
    for (int i0 = 0; i0 < i_hi; i0 += 16) {
      bf16x8 kf[KS];
      int row = i0 + r16;
      row = row < p.T ? row : p.T - 1;
      load_row_frags<D>(kf, kb0 + (size_t)row * kstride, kg);
      fold(kf, i0, vis, true);
    }
  }

  // merge the four lane groups of every query column, write L = m + log2(l)
#pragma unroll
  for (int qt = 0; qt < kSbTiles; ++qt) {
#pragma unroll
    for (int sh = 16; sh <= 32; sh <<= 1) {
      const float mo = __shfl_xor(m[qt], sh), lo = __shfl_xor(l[qt], sh);
      const float mn = fmaxf(m[qt], mo);
      l[qt] = l[qt] * fast_exp2(m[qt] - mn) + lo * fast_exp2(mo - mn);
      m[qt] = mn;
    }
    const int r = row0 + 16 * qt + r16;
    if (kg == 0 && r < R) p.stats[unit * (size_t)p.Rpad + r] = m[qt] + __builtin_amdgcn_logf(l[qt]);
  }
}

// ---- pass 2: attention received by every cached slot, summed over the block's query rows ----------
// grid (ceil(cap / 256), Hkv, Nb), 256 threads.
template <int D>
__global__ __launch_bounds__(kSbWaves * 64) void score_block_colsum_kernel(const ScoreBlockParams p) {
  constexpr int KS = D / 32;
  const int b = blockIdx.z, h = blockIdx.y;
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
  const int key0 = blockIdx.x * kSbRowsPerWg + wave * kSbRowsPerWave;
  if (key0 >= n || key0 + kSbRowsPerWave <= first) return;
  const size_t unit = (size_t)b * p.Hkv + h;
  const uint16_t *Kb = p.K + unit * (size_t)p.cap * D;
  const float *Lb = p.stats + unit * (size_t)p.Rpad;

  // stationary: this wave's cached keys (A operand: row r16 of tile kt is slot key0 + 16 kt + r16)
  bf16x8 kf[kSbTiles][KS];
#pragma unroll
  for (int kt = 0; kt < kSbTiles; ++kt) {
    int row = key0 + 16 * kt + r16;
    row = row < n ? row : n - 1;
    load_row_frags<D>(kf[kt], Kb + (size_t)row * D, kg);
  }
  f32x4 sum[kSbTiles];
#pragma unroll
  for (int kt = 0; kt < kSbTiles; ++kt) sum[kt] = f32x4{0.f, 0.f, 0.f, 0.f};

  bf16x8 qf[KS], qn[KS];
  float L, Ln;
  load_row_frags<D>(qf, query_row<D>(p, b, h, r16, R), kg);
  L = r16 < R ? Lb[r16] : INFINITY;
  for (int r0 = 0; r0 < R; r0 += 16) {
    const int rn = r0 + 16 + r16;
    load_row_frags<D>(qn, query_row<D>(p, b, h, rn, R), kg);
    Ln = rn < R ? Lb[rn] : INFINITY;   // a row beyond the last contributes 2^(-inf) = 0
#pragma unroll
    for (int kt = 0; kt < kSbTiles; ++kt) {
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kt][ks], qf[ks], acc, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) sum[kt][i] += fast_exp2(acc[i] * p.scale_log2 - L);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = qn[ks];
    L = Ln;
  }

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
    float *d = p.dst + unit * (size_t)p.cap + slot;
    *d = p.accumulate ? *d + v : v;
  }
}

}  // namespace dynts
