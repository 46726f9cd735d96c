// Measurement aid: a plain read stream, 16 bytes per lane per load, nothing else.  Its rate on a
// buffer of the cache's size is what the memory system delivers to the simplest possible kernel,
// the second denominator (next to the published peak) for the attention kernel's bandwidth.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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

}  // namespace dynts
