// Eviction (Sec. 4.2): stable in-place gather of the retained rows, plus the small
// bookkeeping kernels (prompt fill, append) that write cache rows.
//
// In-place safety: keep_idx is strictly ascending, so source >= destination for every row.
// A workgroup walks its unit in ascending tiles of kCompactRows destinations; it loads the
// whole tile's source rows into registers, meets at a barrier, then stores.  The sources of
// any later tile lie at or beyond the end of this tile's destinations, so no row is
// overwritten before it has been read.  Rows before the first evicted slot do not move and
// are skipped.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dynts {

constexpr int kCompactThreads = 256;
constexpr int kCompactUnroll = 4;
// A workgroup moves one column slice of this many bytes of every row: whole 128-byte lines, so that no line is
// fetched by two workgroups (64-byte slices read 2.8 bytes per byte written on the 32-layer workload).
#ifndef DYNTS_COMPACT_SLICE
#define DYNTS_COMPACT_SLICE 128
#endif
constexpr int kCompactSliceBytes = DYNTS_COMPACT_SLICE;

struct CompactParams {
  uint16_t *K, *V;          // [Nb][Hkv][cap][D]
  float *S;                 // [Nb][Hkv][cap]
  int32_t *pos;             // [Nb][Hkv][cap]
  int32_t *seq_len;         // [Nb]
  const uint8_t *trigger;   // [Nb] or null
  const int32_t *keep_idx;  // [Nb][Hkv][keep_stride]
  const int32_t *new_len;   // [Nb]
  int Hkv, cap, keep_stride;
};

__device__ __forceinline__ int clamp_slot(int v, int cap) { return v < 0 ? 0 : (v >= cap ? cap - 1 : v); }

// First destination whose source differs.  keep_idx[i] == i holds on a prefix only, so the boundary is found by
// cutting the range 256 ways at a time, every thread probing one position: two or three rounds of one load
// each, where a bisection by one thread makes eleven dependent loads.  Called by all threads of the workgroup.
__device__ __forceinline__ int first_moved(const int32_t *ku, int m) {
  const int tid = threadIdx.x;
  int lo = 0, hi = m;  // the boundary lies in [lo, hi]
  while (lo < hi) {
    const int step = (hi - lo + kCompactThreads - 1) / kCompactThreads;
    const int idx = lo + tid * step;
    const int c = __syncthreads_count(idx < hi && ku[idx] == idx);  // probes 0 .. c-1 hold, probe c does not
    if (c == 0) {
      hi = lo;
    } else {
      const int up = lo + c * step;
      lo = lo + (c - 1) * step + 1;
      hi = up < hi ? up : hi;
    }
  }
  return lo;
}

// grid (2 * kSlices + 2, Hkv, Nb): x < kSlices moves one column slice of the K rows,
// the next kSlices the same for V, the last two move S and pos.  Column slices are independent
// copies, so the in-place argument above holds for each of them; splitting a row over several
// workgroups shortens the chain of dependent round trips (index, row, barrier, store) that bounds
// this kernel: a trigger usually moves a few hundred rows per unit.
template <int D>
__global__ __launch_bounds__(kCompactThreads) void compact_kernel(const CompactParams p) {
  constexpr int kSlices = D * 2 / kCompactSliceBytes;   // column slices per row
  constexpr int LPS = kCompactSliceBytes / 16;          // lanes per row slice (16 bytes each)
  constexpr int ROWS = kCompactThreads / LPS;       // rows per pass
  constexpr int TILE = ROWS * kCompactUnroll;       // destinations per barrier
  const int tid = threadIdx.x;
  const int what = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (p.trigger && !p.trigger[b]) return;
  int m = p.new_len[b];
  m = m < 0 ? 0 : (m > p.cap ? p.cap : m);
  if (m > p.keep_stride) m = p.keep_stride;
  const size_t unit = (size_t)b * p.Hkv + h;
  const int32_t *ku = p.keep_idx + unit * (size_t)p.keep_stride;

  const int first = first_moved(ku, m);

  if (what < 2 * kSlices) {
    uint16_t *base = (what < kSlices ? p.K : p.V) + unit * (size_t)p.cap * D + (kCompactSliceBytes / 2) * (what % kSlices);
    const int r = tid / LPS, piece = tid % LPS;
    // Two tiles in flight: the rows of tile t+1 are requested before tile t is stored.  That is safe
    // because every source of tile t+1 lies at or beyond its own first destination, past all of
    // tile t's destinations; the barrier still separates tile t's loads from tile t's stores.
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 cur[kCompactUnroll], nxt[kCompactUnroll];
    int src[kCompactUnroll];
    // (rows past the end read slot 0 and are never stored, so every load is unconditional)
#define DYNTS_COMPACT_IDX(i0_)                                   \
  _Pragma("unroll") for (int u = 0; u < kCompactUnroll; ++u) {   \
    const int i = (i0_) + u * ROWS + r;                          \
    src[u] = i < m ? clamp_slot(ku[i], p.cap) : 0;               \
  }
#define DYNTS_COMPACT_ROWS(buf_)                                 \
  _Pragma("unroll") for (int u = 0; u < kCompactUnroll; ++u)     \
      buf_[u] = *reinterpret_cast<const u32x4 *>(base + (size_t)src[u] * D + 8 * piece);
    DYNTS_COMPACT_IDX(first)
    DYNTS_COMPACT_ROWS(cur)
    DYNTS_COMPACT_IDX(first + TILE)
    for (int i0 = first; i0 < m; i0 += TILE) {
      DYNTS_COMPACT_ROWS(nxt)
      DYNTS_COMPACT_IDX(i0 + 2 * TILE)
      __syncthreads();
#pragma unroll
      for (int u = 0; u < kCompactUnroll; ++u) {
        const int i = i0 + u * ROWS + r;
        if (i < m) *reinterpret_cast<u32x4 *>(base + (size_t)i * D + 8 * piece) = cur[u];
      }
#pragma unroll
      for (int u = 0; u < kCompactUnroll; ++u) cur[u] = nxt[u];
    }
#undef DYNTS_COMPACT_IDX
#undef DYNTS_COMPACT_ROWS
  } else {
    // S (x == 2 * kSlices) or pos (the last x): 4-byte elements, kScalarUnroll per thread and pass
    constexpr int kScalarUnroll = 8;
    constexpr int STILE = kCompactThreads * kScalarUnroll;
    uint32_t *eu = (what == 2 * kSlices ? reinterpret_cast<uint32_t *>(p.S) : reinterpret_cast<uint32_t *>(p.pos)) +
                   unit * (size_t)p.cap;
    for (int i0 = first; i0 < m; i0 += STILE) {
      int src[kScalarUnroll];
      uint32_t val[kScalarUnroll];
#pragma unroll
      for (int u = 0; u < kScalarUnroll; ++u) {
        const int i = i0 + u * kCompactThreads + tid;
        src[u] = i < m ? clamp_slot(ku[i], p.cap) : 0;
      }
#pragma unroll
      for (int u = 0; u < kScalarUnroll; ++u) {
        const int i = i0 + u * kCompactThreads + tid;
        if (i < m) val[u] = eu[src[u]];
      }
      __syncthreads();
#pragma unroll
      for (int u = 0; u < kScalarUnroll; ++u) {
        const int i = i0 + u * kCompactThreads + tid;
        if (i < m) eu[i] = val[u];
      }
    }
    if (what == 2 * kSlices && h == 0 && tid == 0) p.seq_len[b] = m;
  }
}

struct PrefillParams {
  uint16_t *K, *V;
  float *S;
  int32_t *pos, *seq_len, *next_pos, *n_prompt;
  const uint16_t *K0, *V0;  // [Nb][Hkv][m_max][D]
  const int32_t *m;         // [Nb]
  int Hkv, cap, m_max;
};

// grid (ceil(m_max / rows-per-block), Hkv, Nb)
template <int D>
__global__ __launch_bounds__(256) void prefill_kernel(const PrefillParams p) {
  constexpr int LPR = D / 8, ROWS = 256 / LPR;
  const int tid = threadIdx.x, h = blockIdx.y, b = blockIdx.z;
  int mb = p.m[b];
  mb = mb < 0 ? 0 : (mb > p.m_max ? p.m_max : mb);
  mb = mb > p.cap ? p.cap : mb;
  const size_t unit = (size_t)b * p.Hkv + h;
  const int row = blockIdx.x * ROWS + tid / LPR, piece = tid % LPR;
  if (row < mb) {
    const size_t src = (unit * p.m_max + row) * D + 8 * piece;
    const size_t dst = (unit * (size_t)p.cap + row) * D + 8 * piece;
    *reinterpret_cast<uint4 *>(p.K + dst) = *reinterpret_cast<const uint4 *>(p.K0 + src);
    *reinterpret_cast<uint4 *>(p.V + dst) = *reinterpret_cast<const uint4 *>(p.V0 + src);
    if (piece == 0) {
      p.S[unit * (size_t)p.cap + row] = INFINITY;
      p.pos[unit * (size_t)p.cap + row] = row;
    }
  }
  if (blockIdx.x == 0 && h == 0 && tid == 0) {
    p.seq_len[b] = mb;
    p.next_pos[b] = mb;
    p.n_prompt[b] = mb;
  }
}

struct AppendParams {
  uint16_t *K, *V;
  float *S;
  int32_t *pos, *seq_len, *next_pos;
  const uint16_t *k_new, *v_new;  // [Nb][Hkv][D]
  const float *s_new;             // [Nb][Hkv] or null
  const uint8_t *active;
  int32_t *status;
  int Hkv, cap;
};

// grid (Nb), block Hkv * D/8 threads rounded up to 64: every thread copies 16 bytes of K and of V.
// seq_len/next_pos are advanced by thread 0 after a barrier so that all heads read the old length.
template <int D>
__global__ void append_kernel(const AppendParams p) {
  constexpr int LPR = D / 8;
  const int b = blockIdx.x, tid = threadIdx.x;
  if (p.active && !p.active[b]) return;
  const int n = p.seq_len[b];
  const int np = p.next_pos[b];
  if (n < 0 || n >= p.cap) {
    if (tid == 0) atomicOr(p.status, 1);
    return;
  }
  const int h = tid / LPR, piece = tid % LPR;
  if (h < p.Hkv) {
    const size_t unit = (size_t)b * p.Hkv + h;
    const size_t dst = (unit * (size_t)p.cap + n) * D + 8 * piece;
    *reinterpret_cast<uint4 *>(p.K + dst) = *reinterpret_cast<const uint4 *>(p.k_new + unit * D + 8 * piece);
    *reinterpret_cast<uint4 *>(p.V + dst) = *reinterpret_cast<const uint4 *>(p.v_new + unit * D + 8 * piece);
    if (piece == 0) {
      p.S[unit * (size_t)p.cap + n] = p.s_new ? p.s_new[unit] : 0.f;
      p.pos[unit * (size_t)p.cap + n] = np;
    }
  }
  __syncthreads();
  if (tid == 0) {
    p.seq_len[b] = n + 1;
    p.next_pos[b] = np + 1;
  }
}

}  // namespace dynts
