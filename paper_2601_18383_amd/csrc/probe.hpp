// Measurement aid: a plain read stream, 16 bytes per lane per load, nothing else.  Its rate on a
// buffer of the cache's size is what the memory system delivers to the simplest possible kernel,
// the second denominator (next to the published peak) for the attention kernel's bandwidth.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attend.hpp"

namespace dynts {

constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 4;

// Grid-stride over n16 16-byte words; the XOR of everything read is stored only if it equals
// `magic`, which keeps the loads alive without adding write traffic.
__global__ __launch_bounds__(kProbeThreads) void read_stream_kernel(const uint32_t *__restrict__ buf, size_t n16,
                                                                    uint32_t magic, uint32_t *sink) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 *p = reinterpret_cast<const u32x4 *>(buf);
  const size_t tid = (size_t)blockIdx.x * kProbeThreads + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * kProbeThreads;
  u32x4 acc = {0u, 0u, 0u, 0u};
  size_t i = tid;
  for (; i + (kProbeUnroll - 1) * stride < n16; i += kProbeUnroll * stride) {
    u32x4 v[kProbeUnroll];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) v[u] = p[i + u * stride];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) acc ^= v[u];
  }
  for (; i < n16; i += stride) acc ^= p[i];
  const uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (x == magic) sink[0] = x;
}

// Second measurement aid: how many 2^x the vector ALUs deliver.  Every lane runs `iters` rounds of eight
// independent v_exp_f32 (arguments stay in (0, 1], nothing else in the loop); nothing is written unless the sum
// equals `magic`.  The block-scoring kernels need one exponential per (query row, slot) and pass, which is what
// bounds them besides the matrix cores.
__global__ __launch_bounds__(kProbeThreads) void exp2_rate_kernel(int iters, float magic, float *sink) {
  float a[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = 1.0f / (float)(1 + ((threadIdx.x + i) & 15));
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = __builtin_amdgcn_exp2f(a[i]) - 1.0f;  // 2^a - 1 stays in (0, 1]
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += a[i];
  if (s == magic) sink[0] = s;
}

// Third measurement aid: the instruction mix of the block-scoring kernels with no memory access at all.  Per round
// a wave issues what one streamed 16-row tile costs it there: 16 v_mfma_f32_16x16x32_bf16 on four independent
// accumulators (WHAT & 1) and 16 x (multiply-add, 2^x, add) on independent registers (WHAT & 2), in one basic
// block, so that the compiler interleaves them as it does in the kernels.  The time per round is what a SIMD
// needs for a tile when nothing but instruction issue and the two pipes limit it.
template <int WHAT>
__global__ __launch_bounds__(kProbeThreads) void issue_mix_kernel(int iters, float c, float L, float magic, float *sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      a[i][e] = (__bf16)(0.001f * (float)(lane + i + e));
      b[i][e] = (__bf16)(0.002f * (float)(lane - i + e));
    }
  f32x4 acc[4];
  float sum[16], x[16];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    sum[i] = 0.f;
    x[i] = 0.01f * (float)(lane + i);
  }
  for (int it = 0; it < iters; ++it) {
    if (WHAT & 1) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) acc[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[kt], b[ks], acc[kt], 0, 0, 0);
    }
    if (WHAT & 2) {
#pragma unroll
      for (int i = 0; i < 16; ++i) sum[i] += fast_exp2(fmaf(x[i], c, L));
      // (the arguments are not loop-invariant as far as the compiler can tell)
      asm volatile("" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]));
      asm volatile("" : "+v"(x[8]), "+v"(x[9]), "+v"(x[10]), "+v"(x[11]), "+v"(x[12]), "+v"(x[13]), "+v"(x[14]), "+v"(x[15]));
    }
  }
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) r += sum[i];
#pragma unroll
  for (int i = 0; i < 4; ++i) r += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  if (r == magic) sink[0] = r;
}

}  // namespace dynts
