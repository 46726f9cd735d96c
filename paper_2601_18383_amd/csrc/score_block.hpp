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
// rows, pass 2: cached keys) as MFMA operand fragments (lane (r, kg) holds elements
// 32*ks + 8*kg .. +7 of row r, the layout v_mfma_f32_16x16x32_bf16 wants for A and for B alike).
// The other operand is streamed: the workgroup's 256 threads fetch 32 rows at a time with whole-row
// coalesced 16-byte loads (a strided fetch straight into operand layout touches 16 cache lines per
// instruction and makes the L1 tag rate the limit), park them in one of two padded LDS buffers, and
// every wave reads its operand fragments back from there (row pitch +16 bytes: the 16 rows a
// ds_read_b128 touches fall into different banks).  Loads for chunk c+2 are in flight while chunk
// c is multiplied; one barrier per chunk.
// The product is always  keys (A, rows)  x  queries (B, columns): a lane ends up with 4 keys of ONE
// query column, so
//   * pass 1 keeps a private running (max, sum) per lane and query column and merges the four lane
//     groups once, at the end;
//   * pass 2 keeps private partial column sums per lane and key and merges the 16 lanes of a group
//     once, at the end.
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
  // paged layout: K is the page pool, slot j of a unit is row j % 64 of page block_table[unit][j / 64]
  const int32_t *block_table;  // layer base [Nb][Hkv][max_pages], or null (dense layout)
  int max_pages, n_pages;
};

// byte address of cached key row `row` of a unit (dense rows, or through the block table)
template <int D>
__device__ __forceinline__ const char *sb_key_row(const ScoreBlockParams &p, size_t unit, int row) {
  if (p.block_table) {
    int pi = row / kPageSlots;
    pi = pi < p.max_pages ? pi : p.max_pages - 1;
    int pg = p.block_table[unit * (size_t)p.max_pages + pi];
    pg = pg < 0 ? 0 : (pg >= p.n_pages ? p.n_pages - 1 : pg);
    return reinterpret_cast<const char *>(p.K + ((size_t)pg * kPageSlots + row % kPageSlots) * D);
  }
  return reinterpret_cast<const char *>(p.K + (unit * (size_t)p.cap + row) * D);
}

// MFMA operand fragments of one row in global memory: 16 bytes per k-step at the lane's column group.
template <int D>
__device__ __forceinline__ void load_row_frags(bf16x8 (&f)[D / 32], const char *row, int kg) {
  const char *base = row + 16 * kg;
#pragma unroll
  for (int ks = 0; ks < D / 32; ++ks)
    f[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(base + 64 * ks));
}

// Staging of the streamed operand: a chunk is 32 rows; thread t of the 256 fetches 16 bytes of row
// t / PIECES (+ RPP per further load) at piece t % PIECES, so 16 (8) neighbouring lanes read one
// whole row.
template <int D>
struct SbStage {
  static constexpr int kChunk = 32;              // rows per chunk
  static constexpr int PIECES = D / 8;           // 16-byte pieces per row
  static constexpr int RPP = 256 / PIECES;       // rows one load instruction of the workgroup covers
  static constexpr int NL = kChunk / RPP;        // load instructions per chunk and thread
#ifndef SB_PITCH_EXTRA
#define SB_PITCH_EXTRA 16
#endif
  static constexpr int LROW = 2 * D + SB_PITCH_EXTRA;        // padded row pitch in LDS, bytes
  static constexpr int kBufBytes = kChunk * LROW;
};

// operand fragments of row `row` (0..31) of a staged chunk
template <int D>
__device__ __forceinline__ void lds_row_frags(bf16x8 (&f)[D / 32], const char *buf, int row, int kg) {
  const char *base = buf + row * SbStage<D>::LROW + 16 * kg;
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

// A thread's walk over the query rows r = i * G + g of a KV head's group, `step` rows at a time.
struct QueryWalk {
  int r, i, g, step;
  uint32_t off;         // byte offset of row (i, g) from the (sequence, head-group) base
  int step_i, step_g;   // step = step_i * G + step_g
  uint32_t stride_i, stride_g;
  __device__ __forceinline__ void init(int r0, int step_, int G, int Hq, int D) {
    r = r0;
    step = step_;
    i = r0 / G;
    g = r0 - i * G;
    step_i = step / G;
    step_g = step - step_i * G;
    stride_i = (uint32_t)Hq * D * 2;
    stride_g = (uint32_t)D * 2;
    off = (uint32_t)i * stride_i + (uint32_t)g * stride_g;
  }
  __device__ __forceinline__ void advance(int G) {
    r += step;
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
  using St = SbStage<D>;
  __shared__ __attribute__((aligned(16))) char lds[2][St::kBufBytes];
  const int R = p.T * p.G;
  int unit, blk;
  if (!sb_map((R + kSbRowsPerWg - 1) / kSbRowsPerWg, p.Nb * p.Hkv, unit, blk)) return;
  const int b = unit / p.Hkv, h = unit - b * p.Hkv;
  if (p.active && !p.active[b]) return;
  if (blk * kSbRowsPerWg >= R) return;  // (cannot happen with the grid above; uniform over the workgroup)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kg = lane >> 4;
  const int row0 = blk * kSbRowsPerWg + wave * kSbRowsPerWave;
  // (the same in every lane of a wave, and told so to the compiler; a wave without rows still helps staging and
  // meets the barriers)
  const bool has_rows = __builtin_amdgcn_readfirstlane((int)(row0 < R)) != 0;
  int n = p.seq_len[b];
  n = n < 0 ? 0 : (n > p.cap ? p.cap : n);
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
  float m[kSbTiles], nm[kSbTiles], l[kSbTiles];  // nm = -c * m, the exponent's addend
#pragma unroll
  for (int qt = 0; qt < kSbTiles; ++qt) {
    m[qt] = -1e30f;
    nm[qt] = 1e30f * c;
    l[qt] = 0.f;
  }

  // One streamed tile in two parts, so that the loop below can put the MFMAs of the NEXT tile (four independent
  // accumulators, issued back to back) beside the vector work of the current one:
  //   MM:   logits of keys (4 kg + i) x query column r16 for the wave's four query tiles;
  //   FOLD: fold them into (m, l).  MASKED: keys whose index key0 + 4 kg + i is not below lim[qt] do not exist
  //         for this query column.
#define DYNTS_SB_MM(acc_, buf_, tt_)                                                                   \
  {                                                                                                    \
    bf16x8 kf[KS];                                                                                     \
    lds_row_frags<D>(kf, buf_, 16 * (tt_) + r16, kg);                                                  \
    _Pragma("unroll") for (int qt = 0; qt < kSbTiles; ++qt) acc_[qt] = f32x4{0.f, 0.f, 0.f, 0.f};      \
    _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                                  \
      _Pragma("unroll") for (int qt = 0; qt < kSbTiles; ++qt)                                          \
          acc_[qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks], qf[qt][ks], acc_[qt], 0, 0, 0);   \
  }
#define DYNTS_SB_FOLD(acc_, MASKED, key0_, lim_)                                                       \
  _Pragma("unroll") for (int qt = 0; qt < kSbTiles; ++qt) {                                            \
    f32x4 acc = acc_[qt];                                                                              \
    if (MASKED) {                                                                                      \
      _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                    \
          if ((key0_) + 4 * kg + i >= lim_[qt]) acc[i] = -INFINITY;                                    \
    }                                                                                                  \
    const float mx = fmaxf(fmaxf(acc[0], acc[1]), fmaxf(acc[2], acc[3]));                              \
    if (__any(mx > m[qt])) { /* some lane's maximum rises (rare after the first tiles): rescale */     \
      const float mn = fmaxf(mx, m[qt]);                                                               \
      l[qt] *= fast_exp2((m[qt] - mn) * c); /* exactly 2^0 where nothing changes */                    \
      m[qt] = mn;                                                                                      \
      nm[qt] = -mn * c;                                                                                \
    }                                                                                                  \
    float sum = l[qt];                                                                                 \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) sum += fast_exp2(fmaf(acc[i], c, nm[qt]));           \
    l[qt] = sum;                                                                                       \
  }

  // Streaming of `rows` rows that start at `src` with pitch `pitch` bytes (src null: the unit's cached key
  // rows), 32 per chunk; row indices beyond the last repeat it (the fold masks them).  Every thread of the workgroup runs this.
  const int st_row = tid / St::PIECES, st_piece = tid % St::PIECES;
  u32x4 stage[St::NL];
#define DYNTS_SB_FETCH(src_, pitch_, rows_, chunk_)                                                    \
  _Pragma("unroll") for (int k = 0; k < St::NL; ++k) {                                                 \
    int row = (chunk_) * St::kChunk + st_row + St::RPP * k;                                            \
    row = row < (rows_) ? row : (rows_) - 1;                                                           \
    const char *rp = (src_) ? (src_) + (size_t)row * (pitch_) : sb_key_row<D>(p, (size_t)unit, row);   \
    stage[k] = *reinterpret_cast<const u32x4 *>(rp + 16 * st_piece);                                   \
  }
#define DYNTS_SB_PARK(buf_)                                                                            \
  _Pragma("unroll") for (int k = 0; k < St::NL; ++k)                                                   \
      *reinterpret_cast<u32x4 *>((buf_) + (st_row + St::RPP * k) * St::LROW + 16 * st_piece) = stage[k];
#define DYNTS_SB_STREAM(src_, pitch_, rows_, lim_, CAUSAL_)                                            \
  {                                                                                                    \
    const int n_chunks = ((rows_) + St::kChunk - 1) / St::kChunk;                                      \
    if (n_chunks > 0) {                                                                                \
      DYNTS_SB_FETCH(src_, pitch_, rows_, 0)                                                           \
      DYNTS_SB_PARK(lds[0])                                                                            \
      if (n_chunks > 1) { DYNTS_SB_FETCH(src_, pitch_, rows_, 1) }                                     \
      __syncthreads();                                                                                 \
      f32x4 acc_a[kSbTiles], acc_b[kSbTiles];                                                          \
      if (has_rows) DYNTS_SB_MM(acc_a, lds[0], 0)                                                      \
      for (int ch = 0; ch + 1 < n_chunks; ++ch) { /* whole chunks: no key is masked unless CAUSAL_ */  \
        const int nb = (ch + 1) & 1;                                                                   \
        if (has_rows) {                                                                                \
          DYNTS_SB_MM(acc_b, lds[ch & 1], 1)                                                           \
          DYNTS_SB_FOLD(acc_a, CAUSAL_, ch * St::kChunk, lim_)                                         \
        }                                                                                              \
        DYNTS_SB_PARK(lds[nb])                                                                         \
        if (ch + 2 < n_chunks) { DYNTS_SB_FETCH(src_, pitch_, rows_, ch + 2) }                         \
        __syncthreads();                                                                               \
        if (has_rows) {                                                                                \
          DYNTS_SB_MM(acc_a, lds[nb], 0)                                                               \
          DYNTS_SB_FOLD(acc_b, CAUSAL_, ch * St::kChunk + 16, lim_)                                    \
        }                                                                                              \
      }                                                                                                \
      if (has_rows) { /* the last chunk may be partial: masked */                                      \
        const int lc = n_chunks - 1;                                                                   \
        DYNTS_SB_MM(acc_b, lds[lc & 1], 1)                                                             \
        DYNTS_SB_FOLD(acc_a, true, lc * St::kChunk, lim_)                                              \
        DYNTS_SB_FOLD(acc_b, true, lc * St::kChunk + 16, lim_)                                         \
      }                                                                                                \
      __syncthreads(); /* the buffers are filled again by the next stream */                           \
    }                                                                                                  \
  }

  // cached slots: every query column sees all n of them
  {
    int lim[kSbTiles];
#pragma unroll
    for (int qt = 0; qt < kSbTiles; ++qt) lim[qt] = n;
    const char *const cached = nullptr;  // (null source: cached key rows, found by sb_key_row)
    DYNTS_SB_STREAM(cached, (size_t)0, n, lim, false)
  }
  // the block's own keys, causally: key i' is visible to query row (i, g) iff i' <= i.  Keys
  // [0, i_hi) are visible to some row of this workgroup.
  if (p.k_blk) {
    int last = blk * kSbRowsPerWg + kSbRowsPerWg - 1;
    last = last < R ? last : R - 1;
    const int i_hi = last / p.G + 1;
    const char *kb0 = reinterpret_cast<const char *>(p.k_blk + ((size_t)b * p.T * p.Hkv + h) * D);
    DYNTS_SB_STREAM(kb0, (size_t)p.Hkv * D * 2, i_hi, vis_blk, true)
  }
#undef DYNTS_SB_STREAM
#undef DYNTS_SB_PARK
#undef DYNTS_SB_FETCH
#undef DYNTS_SB_FOLD
#undef DYNTS_SB_MM
  if (!has_rows) return;

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
  using St = SbStage<D>;
  __shared__ __attribute__((aligned(16))) char lds[2][St::kBufBytes];
  int unit, blk;
  if (!sb_map((p.cap + kSbRowsPerWg - 1) / kSbRowsPerWg, p.Nb * p.Hkv, unit, blk)) return;
  const int b = unit / p.Hkv, h = unit - b * p.Hkv;
  if (p.active && !p.active[b]) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kg = lane >> 4;
  const int R = p.T * p.G;
  int n = p.seq_len[b];
  n = n < 0 ? 0 : (n > p.cap ? p.cap : n);
  int first = 0;
  if (p.skip_prompt) {
    first = p.n_prompt[b];
    first = first < 0 ? 0 : first;
  }
  // uniform over the workgroup: nothing of this block is wanted
  if (blk * kSbRowsPerWg >= n || (blk + 1) * kSbRowsPerWg <= first) return;
  const int key0 = blk * kSbRowsPerWg + wave * kSbRowsPerWave;
  // (the same in every lane of a wave, and told so to the compiler: a plain branch instead of lane masks)
  const bool has_keys = __builtin_amdgcn_readfirstlane((int)(key0 < n && key0 + kSbRowsPerWave > first)) != 0;  // else: staging and barriers only
  const char *Qb = reinterpret_cast<const char *>(p.q_blk + ((size_t)b * p.T * p.Hq + (size_t)h * p.G) * D);
  const float *Lb = p.stats + (size_t)unit * (size_t)p.Rpad;
  const float c = p.scale_log2;

  // stationary: this wave's cached keys (A operand: row r16 of tile kt is slot key0 + 16 kt + r16)
  bf16x8 kf[kSbTiles][KS];
#pragma unroll
  for (int kt = 0; kt < kSbTiles; ++kt) {
    int row = key0 + 16 * kt + r16;
    row = row < n ? row : n - 1;
    load_row_frags<D>(kf[kt], sb_key_row<D>(p, (size_t)unit, row), kg);
  }
  f32x4 sum[kSbTiles];
#pragma unroll
  for (int kt = 0; kt < kSbTiles; ++kt) sum[kt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // streamed: the R query rows, 32 per chunk through LDS, and with them their log2 denominators (one float
  // per row, fetched by the first 32 threads and parked behind the rows: a load of its own inside the
  // multiply loop would make every chunk wait for all outstanding loads).  A row beyond the last repeats the
  // last row's data and gets L = +inf, so it contributes 2^(-inf) = 0.
  __shared__ float ldsL[2][St::kChunk];
  const int st_piece = tid % St::PIECES;
  QueryWalk w[St::NL];
#pragma unroll
  for (int k = 0; k < St::NL; ++k) w[k].init(tid / St::PIECES + St::RPP * k, St::kChunk, p.G, p.Hq, D);
  const uint32_t last_off = (uint32_t)(p.T - 1) * w[0].stride_i + (uint32_t)(p.G - 1) * w[0].stride_g;
  u32x4 stage[St::NL];
  float stageL = INFINITY;
  bool stageL_valid = false;
  int l_row = tid & (St::kChunk - 1);  // the row whose L this thread fetches next (threads 0..31 park it)
#define DYNTS_SB_FETCH()                                                                               \
  _Pragma("unroll") for (int k = 0; k < St::NL; ++k) {                                                 \
    stage[k] = *reinterpret_cast<const u32x4 *>(Qb + (w[k].r < R ? w[k].off : last_off) + 16 * st_piece); \
    w[k].advance(p.G);                                                                                 \
  }                                                                                                    \
  stageL = Lb[l_row < R ? l_row : R - 1];                                                              \
  stageL_valid = l_row < R;                                                                            \
  l_row += St::kChunk;
#define DYNTS_SB_PARK(b_)                                                                              \
  _Pragma("unroll") for (int k = 0; k < St::NL; ++k)                                                   \
      *reinterpret_cast<u32x4 *>(lds[b_] + (tid / St::PIECES + St::RPP * k) * St::LROW + 16 * st_piece) = stage[k]; \
  if (tid < St::kChunk) ldsL[b_][tid] = stageL_valid ? stageL : INFINITY;

  // The tiles are software-pipelined: the MFMAs of tile t+1 (independent accumulators, so they issue
  // back to back) stand next to the exponentials and sums of tile t, so that the scheduler has
  // independent work for the matrix pipe and the vector ALU at the same time.
#define DYNTS_SB_MM(acc_, buf_, tt_)                                                                   \
  {                                                                                                    \
    bf16x8 qf[KS];                                                                                     \
    lds_row_frags<D>(qf, buf_, 16 * (tt_) + r16, kg);                                                  \
    _Pragma("unroll") for (int kt = 0; kt < kSbTiles; ++kt) acc_[kt] = f32x4{0.f, 0.f, 0.f, 0.f};      \
    _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                                  \
      _Pragma("unroll") for (int kt = 0; kt < kSbTiles; ++kt)                                          \
          acc_[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kt][ks], qf[ks], acc_[kt], 0, 0, 0);   \
  }
#define DYNTS_SB_SUM(acc_, L_)                                                                         \
  _Pragma("unroll") for (int kt = 0; kt < kSbTiles; ++kt)                                              \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) sum[kt][i] += fast_exp2(fmaf(acc_[kt][i], c, -(L_)));

  const int n_chunks = (R + St::kChunk - 1) / St::kChunk;
  DYNTS_SB_FETCH()
  DYNTS_SB_PARK(0)
  if (n_chunks > 1) { DYNTS_SB_FETCH() }
  f32x4 acc_a[kSbTiles], acc_b[kSbTiles];
  __syncthreads();
  float La = ldsL[0][r16], Lq = ldsL[0][16 + r16];  // log2 denominators of this lane's query column, even / odd tile
  // (the last chunk stands behind the loop: every iteration inside has the same shape, so no value has two
  // homes at the loop's end)
  if (has_keys) DYNTS_SB_MM(acc_a, lds[0], 0)
  for (int ch = 0; ch + 1 < n_chunks; ++ch) {
    const int nb = (ch + 1) & 1;
    if (has_keys) {
      DYNTS_SB_MM(acc_b, lds[ch & 1], 1)
      DYNTS_SB_SUM(acc_a, La)
    }
    DYNTS_SB_PARK(nb)
    if (ch + 2 < n_chunks) { DYNTS_SB_FETCH() }
    __syncthreads();
    const float Lq_cur = Lq;
    La = ldsL[nb][r16];
    Lq = ldsL[nb][16 + r16];
    if (has_keys) {
      DYNTS_SB_MM(acc_a, lds[nb], 0)
      DYNTS_SB_SUM(acc_b, Lq_cur)
    }
  }
  if (has_keys) {
    DYNTS_SB_MM(acc_b, lds[(n_chunks - 1) & 1], 1)
    DYNTS_SB_SUM(acc_a, La)
    DYNTS_SB_SUM(acc_b, Lq)
  }
#undef DYNTS_SB_MM
#undef DYNTS_SB_SUM
#undef DYNTS_SB_FETCH
#undef DYNTS_SB_PARK
  if (!has_keys) return;

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
