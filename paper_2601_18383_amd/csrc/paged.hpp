// Paged (block-table) cache layout: the K and V rows of all (layer, sequence, KV head) units live in two
// page pools [n_pages][kPageSlots][D]; slot j of a unit is row j % kPageSlots of page
// block_table[unit][j / kPageSlots].  Scores and positions stay dense per unit (8 bytes per slot).
// Pages come from and go back to a device-side free stack: appends (and the prompt fill) pop, the trim after
// a compaction pushes; one kernel only ever pops or only ever pushes, so the stack needs no more than an
// atomic counter.  Eviction therefore returns memory that other sequences can take.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attend.hpp"
#include "compact.hpp"

namespace dynts {

struct PagedView {
  uint16_t *K, *V;          // pools
  int32_t *block_table;     // layer base, [Nb][Hkv][max_pages]
  int32_t *free_stack, *free_top;
  int max_pages, n_pages;
};

__device__ __forceinline__ int safe_page(int pg, int n_pages) { return pg < 0 ? 0 : (pg >= n_pages ? n_pages - 1 : pg); }

// element offset of slot j of a unit inside a pool
template <int D>
__device__ __forceinline__ size_t paged_row(const int32_t *tb, int j, int max_pages, int n_pages) {
  int pi = j / kPageSlots;
  pi = pi < max_pages ? pi : max_pages - 1;
  return ((size_t)safe_page(tb[pi], n_pages) * kPageSlots + j % kPageSlots) * D;
}

// One thread per unit takes the pages for slots [have[b], want[b]) of its unit (have = NULL: 0).
// Returns with status bit 2 (value 4) latched when the pool runs dry; the unit then keeps what it got.
// grid (ceil(Nb * Hkv / 64)), 64 threads.
__global__ void paged_alloc_kernel(PagedView pv, const int32_t *have, const int32_t *want, int want_max, int Nb, int Hkv,
                                   int32_t *status) {
  const int u = blockIdx.x * 64 + threadIdx.x;
  if (u >= Nb * Hkv) return;
  const int b = u / Hkv;
  int lo = have ? have[b] : 0, hi = want[b];
  hi = hi < 0 ? 0 : (hi > want_max ? want_max : hi);
  lo = lo < 0 ? 0 : lo;
  int32_t *tb = pv.block_table + (size_t)u * pv.max_pages;
  for (int pi = (lo + kPageSlots - 1) / kPageSlots; pi < (hi + kPageSlots - 1) / kPageSlots && pi < pv.max_pages; ++pi) {
    const int idx = atomicSub(pv.free_top, 1) - 1;
    if (idx < 0) {
      atomicAdd(pv.free_top, 1);
      atomicOr(status, 4);
      return;
    }
    tb[pi] = pv.free_stack[idx];
  }
}

// Question window into paged storage (pages already allocated).  grid (ceil(m_max / rows-per-block), Hkv, Nb).
template <int D>
__global__ __launch_bounds__(256) void paged_prefill_kernel(const PrefillParams p, PagedView pv) {
  constexpr int LPR = D / 8, ROWS = 256 / LPR;
  const int tid = threadIdx.x, h = blockIdx.y, b = blockIdx.z;
  int mb = p.m[b];
  mb = mb < 0 ? 0 : (mb > p.m_max ? p.m_max : mb);
  mb = mb > p.cap ? p.cap : mb;
  const size_t unit = (size_t)b * p.Hkv + h;
  const int32_t *tb = pv.block_table + unit * pv.max_pages;
  const int row = blockIdx.x * ROWS + tid / LPR, piece = tid % LPR;
  if (row < mb) {
    const size_t src = (unit * p.m_max + row) * D + 8 * piece;
    const size_t dst = paged_row<D>(tb, row, pv.max_pages, pv.n_pages) + 8 * piece;
    *reinterpret_cast<uint4 *>(pv.K + dst) = *reinterpret_cast<const uint4 *>(p.K0 + src);
    *reinterpret_cast<uint4 *>(pv.V + dst) = *reinterpret_cast<const uint4 *>(p.V0 + src);
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

// Append into paged storage; a slot that opens a page takes one from the free stack.  grid (Nb), block
// Hkv * D/8 threads rounded up to 64.
template <int D>
__global__ void paged_append_kernel(const AppendParams p, PagedView pv) {
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
    int32_t *tb = pv.block_table + unit * pv.max_pages;
    const int pi = n / kPageSlots;
    int pg = 0;
    if (piece == 0) {
      if (n % kPageSlots == 0) {
        const int idx = atomicSub(pv.free_top, 1) - 1;
        if (idx >= 0) {
          pg = pv.free_stack[idx];
          tb[pi] = pg;
        } else {
          atomicAdd(pv.free_top, 1);
          atomicOr(p.status, 4);
          pg = -1;
        }
      } else {
        pg = tb[pi];
      }
    }
    pg = __shfl(pg, (tid & 63) / LPR * LPR);  // from the first lane of this head's group
    if (pg >= 0 && pg < pv.n_pages) {
      const size_t dst = ((size_t)pg * kPageSlots + n % kPageSlots) * D + 8 * piece;
      *reinterpret_cast<uint4 *>(pv.K + dst) = *reinterpret_cast<const uint4 *>(p.k_new + unit * D + 8 * piece);
      *reinterpret_cast<uint4 *>(pv.V + dst) = *reinterpret_cast<const uint4 *>(p.v_new + unit * D + 8 * piece);
    }
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

// Eviction in paged storage: the same stable in-place gather as compact_kernel (a slot's storage is unique,
// so "sources lie at or beyond destinations" protects rows exactly as in the dense layout), every row found
// through the block table.  seq_len is left to paged_trim_kernel, which still needs the old length.
// grid (2 * kSlices + 2, Hkv, Nb), 256 threads.
template <int D>
__global__ __launch_bounds__(kCompactThreads) void paged_compact_kernel(const CompactParams p, PagedView pv) {
  constexpr int kSlices = D * 2 / kCompactSliceBytes;
  constexpr int LPS = kCompactSliceBytes / 16;
  constexpr int ROWS = kCompactThreads / LPS;
  constexpr int TILE = ROWS * kCompactUnroll;
  const int tid = threadIdx.x;
  const int what = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (p.trigger && !p.trigger[b]) return;
  int m = p.new_len[b];
  m = m < 0 ? 0 : (m > p.cap ? p.cap : m);
  if (m > p.keep_stride) m = p.keep_stride;
  const size_t unit = (size_t)b * p.Hkv + h;
  const int32_t *ku = p.keep_idx + unit * (size_t)p.keep_stride;
  const int32_t *tb = pv.block_table + unit * pv.max_pages;
  const int first = first_moved(ku, m);

  if (what < 2 * kSlices) {
    uint16_t *pool = (what < kSlices ? pv.K : pv.V) + (kCompactSliceBytes / 2) * (what % kSlices);
    const int r = tid / LPS, piece = tid % LPS;
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    for (int i0 = first; i0 < m; i0 += TILE) {
      u32x4_t buf[kCompactUnroll];
      size_t src[kCompactUnroll];
#pragma unroll
      for (int u = 0; u < kCompactUnroll; ++u) {
        const int i = i0 + u * ROWS + r;
        src[u] = paged_row<D>(tb, i < m ? clamp_slot(ku[i], p.cap) : 0, pv.max_pages, pv.n_pages);
      }
#pragma unroll
      for (int u = 0; u < kCompactUnroll; ++u) buf[u] = *reinterpret_cast<const u32x4_t *>(pool + src[u] + 8 * piece);
      __syncthreads();
#pragma unroll
      for (int u = 0; u < kCompactUnroll; ++u) {
        const int i = i0 + u * ROWS + r;
        if (i < m) *reinterpret_cast<u32x4_t *>(pool + paged_row<D>(tb, i, pv.max_pages, pv.n_pages) + 8 * piece) = buf[u];
      }
      __syncthreads();  // (the next tile's loads must not overtake these stores within the workgroup)
    }
  } else {
    uint32_t *eu = (what == 2 * kSlices ? reinterpret_cast<uint32_t *>(p.S) : reinterpret_cast<uint32_t *>(p.pos)) +
                   unit * (size_t)p.cap;
    for (int i0 = first; i0 < m; i0 += kCompactThreads) {
      const int i = i0 + tid;
      uint32_t val = 0;
      if (i < m) val = eu[clamp_slot(ku[i], p.cap)];
      __syncthreads();
      if (i < m) eu[i] = val;
    }
  }
}

// After a paged compaction: give the pages past the new length back and set the new length.  One thread per
// sequence (all KV heads of a sequence have the same lengths).  grid (ceil(Nb / 64)), 64 threads.
__global__ void paged_trim_kernel(PagedView pv, const uint8_t *trigger, const int32_t *new_len, int32_t *seq_len, int Nb,
                                  int Hkv, int cap, int keep_stride) {
  const int b = blockIdx.x * 64 + threadIdx.x;
  if (b >= Nb) return;
  if (trigger && !trigger[b]) return;
  int m = new_len[b];
  m = m < 0 ? 0 : (m > cap ? cap : m);
  if (m > keep_stride) m = keep_stride;
  int n = seq_len[b];
  n = n < 0 ? 0 : (n > cap ? cap : n);
  const int keep_pages = (m + kPageSlots - 1) / kPageSlots;
  int old_pages = (n + kPageSlots - 1) / kPageSlots;
  old_pages = old_pages < pv.max_pages ? old_pages : pv.max_pages;
  const int k = old_pages - keep_pages;
  if (k > 0) {
    const int base = atomicAdd(pv.free_top, k * Hkv);
    for (int h = 0; h < Hkv; ++h) {
      const int32_t *tb = pv.block_table + ((size_t)b * Hkv + h) * pv.max_pages;
      for (int j = 0; j < k; ++j) pv.free_stack[base + h * k + j] = tb[keep_pages + j];
    }
  }
  seq_len[b] = m;
}

}  // namespace dynts
