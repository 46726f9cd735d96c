// Top-k selection inside the selection window (Sec. 4.2) for gfx950: one workgroup per
// (sequence, KV head).  An 8-bit radix select over order-preserving integer keys finds the
// k-th largest score exactly; ties at the cut go to the lowest slots (= lowest positions,
// slots are kept in position order); two block scans turn the keep flags into the ascending
// list of retained slots.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dynts {

constexpr int kSelThreads = 256;

struct SelectParams {
  const float *S;           // [Nb][Hkv][cap]
  const int32_t *seq_len;   // [Nb]
  const int32_t *n_prompt;  // [Nb]
  const uint8_t *trigger;   // [Nb] or null
  int32_t *keep_idx;        // [Nb][Hkv][keep_stride]
  int32_t *new_len;         // [Nb]
  int32_t *status;          // bit 1 latched when keep_stride is too small for a sequence
  int Hkv, cap, window, k_keep, keep_stride;
};

// fp32 -> uint32 whose unsigned order is the IEEE order; -0 and +0 map to the same key
__device__ __forceinline__ uint32_t score_key(float s) {
  uint32_t u = __float_as_uint(s);
  if ((u << 1) == 0u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exclusive prefix sum of one int per thread over the workgroup; also returns the total
__device__ __forceinline__ int block_exclusive_scan(int v, int *sh /*[kSelThreads/64 + 1]*/, int &total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  __syncthreads();  // sh may still be read from a previous call
  if (lane == 63) sh[wave] = incl;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelThreads / 64; ++w) {
    int c = sh[w];
    if (w < wave) base += c;
    tot += c;
  }
  total = tot;
  return base + incl - v;
}

template <bool USE_LDS>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelectParams p) {
  extern __shared__ uint32_t keys[];  // candidate keys when USE_LDS
  __shared__ uint32_t hist[256];
  __shared__ int sh_scan[kSelThreads / 64 + 1];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_remaining;

  const int tid = threadIdx.x;
  const int h = blockIdx.x, b = blockIdx.y;
  int n = p.seq_len[b];
  n = n < 0 ? 0 : (n > p.cap ? p.cap : n);
  if (p.trigger && !p.trigger[b]) {
    if (h == 0 && tid == 0) p.new_len[b] = n;
    return;
  }
  int M = p.n_prompt[b];
  M = M < 0 ? 0 : (M > n ? n : M);
  const int lo = M;
  const int hi = (n - p.window > lo) ? n - p.window : lo;
  const int nc = hi - lo;
  const int kk = nc < p.k_keep ? nc : p.k_keep;
  const int out_len = M + kk + (n - hi);
  if (out_len > p.keep_stride) {  // cannot list the retained slots: leave the sequence as it is
    if (h == 0 && tid == 0) {
      p.new_len[b] = n;
      atomicOr(p.status, 2);
    }
    return;
  }
  if (h == 0 && tid == 0) p.new_len[b] = out_len;

  const size_t unit = (size_t)b * p.Hkv + h;
  const float *Su = p.S + unit * (size_t)p.cap + lo;
  int32_t *ku = p.keep_idx + unit * (size_t)p.keep_stride;

  for (int i = tid; i < M; i += kSelThreads) ku[i] = i;
  for (int i = tid; i < n - hi; i += kSelThreads) ku[M + kk + i] = hi + i;
  if (kk == 0) return;
  if (kk == nc) {
    for (int i = tid; i < nc; i += kSelThreads) ku[M + i] = lo + i;
    return;
  }

  if (USE_LDS) {
    for (int j = tid; j < nc; j += kSelThreads) keys[j] = score_key(Su[j]);
  }
  auto key = [&](int j) -> uint32_t { return USE_LDS ? keys[j] : score_key(Su[j]); };

  // ---- radix select: the kk-th largest key, 8 bits per pass from the top ---------------
  uint32_t prefix = 0;
  int remaining = kk;
#pragma unroll 1
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t himask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
    hist[tid] = 0;  // kSelThreads == 256 bins
    __syncthreads();
    for (int j = tid; j < nc; j += kSelThreads) {
      uint32_t u = key(j);
      if ((u & himask) == prefix) atomicAdd(&hist[(u >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid < 64) {
      // lane L owns bins 255-4L .. 252-4L, walked from the top
      const int top = 255 - 4 * tid;
      int c0 = hist[top], c1 = hist[top - 1], c2 = hist[top - 2], c3 = hist[top - 3];
      int tot = c0 + c1 + c2 + c3;
      int incl = tot;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        int up = __shfl_up(incl, off);
        if (tid >= off) incl += up;
      }
      int excl = incl - tot;
      if (excl < remaining && remaining <= incl) {
        int r = remaining - excl, bin, above;
        if (r <= c0) { bin = top; above = excl; }
        else if (r <= c0 + c1) { bin = top - 1; above = excl + c0; }
        else if (r <= c0 + c1 + c2) { bin = top - 2; above = excl + c0 + c1; }
        else { bin = top - 3; above = excl + c0 + c1 + c2; }
        sh_prefix = prefix | ((uint32_t)bin << shift);
        sh_remaining = remaining - above;
      }
    }
    __syncthreads();
    prefix = sh_prefix;
    remaining = sh_remaining;
  }
  const uint32_t T = prefix;       // key of the kk-th largest score
  const int take_eq = remaining;   // how many slots with that key are kept (lowest slots first)

  // ---- flags -> ascending output, each thread owns a contiguous run of candidates --------
  const int per = (nc + kSelThreads - 1) / kSelThreads;
  const int j0 = tid * per < nc ? tid * per : nc;
  const int j1 = j0 + per < nc ? j0 + per : nc;
  int eq = 0;
  for (int j = j0; j < j1; ++j) eq += (key(j) == T);
  int tot_unused;
  int eq_rank = block_exclusive_scan(eq, sh_scan, tot_unused);
  int kept = 0, er = eq_rank;
  for (int j = j0; j < j1; ++j) {
    uint32_t u = key(j);
    kept += (u > T) || (u == T && er < take_eq);
    er += (u == T);
  }
  int off = block_exclusive_scan(kept, sh_scan, tot_unused);
  er = eq_rank;
  for (int j = j0; j < j1; ++j) {
    uint32_t u = key(j);
    bool k = (u > T) || (u == T && er < take_eq);
    er += (u == T);
    if (k) {
      if (off < kk) ku[M + off] = lo + j;  // off < kk always holds for NaN-free scores
      ++off;
    }
  }
}

}  // namespace dynts
