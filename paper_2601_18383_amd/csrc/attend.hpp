// Decode attention + deferred importance-score accumulation for gfx950 (wave64, MFMA).
//
// One workgroup (4 waves) owns a contiguous chunk of one (sequence, KV head) cache; each
// wave walks 32-slot tiles of that chunk on its own:
//   * K rows go straight from HBM into MFMA A-operand registers (16-byte loads; lane
//     (r, kg) holds row r, columns 32*ks + 8*kg .. +7), and one v_mfma_f32_16x16x32_bf16
//     per 32 columns gives the logits of 16 slots x 16 (padded) query heads of the group,
//     so the K tile is read once for the whole GQA group (Eq. attn-score).
//   * the same K registers are multiplied with the PREVIOUS step's query; with that step's
//     final softmax statistics this yields its attention weights exactly, which are summed
//     over the group and added to S (Eq. importance-score, running form) -- the score
//     update rides on this step's pass over K instead of a second pass or a logit spill.
//   * V rows are staged through a wave-private LDS tile (coalesced 16-byte loads in,
//     column reads out) to form the transposed MFMA operand; softmax weights are split
//     into bf16 hi + lo parts so the P.V product keeps ~16 bits of the weights
//     (Eq. attn-o), accumulation is fp32 throughout.
//   * online softmax state (running max, sum, output) is per wave; the four waves are
//     combined in LDS and one partial per workgroup goes to the workspace; a small merge
//     kernel combines the splits, writes `out`, and saves the query and the statistics the
//     next step's score update needs.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dynts {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;           // waves per workgroup
constexpr int kTile = 32;           // cache slots one wave handles per iteration
constexpr int kThreads = kWaves * 64;
constexpr int kChunkQuantum = kWaves * kTile;  // chunk sizes are multiples of this

struct AttendParams {
  uint16_t *K, *V;          // layer base, [Nb][Hkv][cap][D]
  float *S;                 // [Nb][Hkv][cap]
  int32_t *pos;             // [Nb][Hkv][cap]
  const int32_t *seq_len;   // [Nb]
  const int32_t *n_prompt;  // [Nb]
  const int32_t *next_pos;  // [Nb]
  const uint16_t *q;        // [Nb][Hq][D]
  const uint16_t *k_new, *v_new;  // [Nb][Hkv][D] (fused append) or null
  const float *s_new;       // [Nb][Hkv] or null
  const uint8_t *active;    // [Nb] or null
  const uint16_t *qprev;    // [Nb][Hq][D] query of the deferred update
  const float *mlprev;      // [Nb][Hq][2] (max in log2 units, sum) of the deferred update
  const int32_t *nprev;     // [Nb] slots the deferred update covers (0 = none)
  float *part_o;            // [Nb][Hkv][nsplit][G][D]
  float *part_ml;           // [Nb][Hkv][nsplit][G][2]
  int32_t *ncur;            // [Nb] slots attended this call (0 = skipped), for the merge
  int32_t *status;
  int Nb, Hq, Hkv, G, cap, chunk, nsplit;
  float scale_log2;         // softmax scale * log2(e)
};

__device__ __forceinline__ bf16x8 load_bf16x8(const uint16_t *p) {
  return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(p));
}
__device__ __forceinline__ void store_bf16x8(uint16_t *p, bf16x8 v) {
  *reinterpret_cast<uint4 *>(p) = __builtin_bit_cast(uint4, v);
}

template <int D, bool ATTEND, bool PENDING, bool APPEND>
__global__ __launch_bounds__(kThreads) void attend_partial_kernel(const AttendParams p) {
  constexpr int KS = D / 32;              // MFMA k-steps per K row
  constexpr int CB = D / 16;              // 16-column blocks of the output
  constexpr int PIECES = D / 8;           // 16-byte pieces per row
  constexpr int VROWS = 64 / PIECES;      // rows covered by one wave-wide 16-byte load
  constexpr int VIT = kTile / VROWS;
  constexpr int VSTRIDE = 2 * D + 8;      // bytes per staged V row (+8: column reads hit distinct banks)
  constexpr int OSTRIDE = D + 4;          // floats per row of the cross-wave output reduction
  static_assert(kWaves * kTile * VSTRIDE == 64 * OSTRIDE * 4, "LDS tile is reused for the reduction");
  __shared__ __align__(16) unsigned char smem[kWaves * kTile * VSTRIDE];
  __shared__ float sm_m[kWaves][16];
  __shared__ float sm_l[kWaves][16];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kg = lane >> 4;  // r16: row within a 16-slot sub-tile == query head index g
  const int g = r16;
  const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int G = p.G;

  const bool act = p.active ? (p.active[b] != 0) : true;
  int n_old = p.seq_len[b];
  n_old = n_old < 0 ? 0 : (n_old > p.cap ? p.cap : n_old);
  int n_now = 0;
  bool appending = false;
  if (ATTEND && act) {
    if (APPEND) {
      if (n_old < p.cap) {
        n_now = n_old + 1;
        appending = true;
      } else if (tid == 0 && split == 0 && h == 0) {
        atomicOr(p.status, 1);
      }
    } else {
      n_now = n_old;
    }
  }
  int n_prev = PENDING ? p.nprev[b] : 0;
  n_prev = n_prev < 0 ? 0 : (n_prev > p.cap ? p.cap : n_prev);
  const int M = p.n_prompt[b];
  const int n_vis = n_now > n_prev ? n_now : n_prev;
  if (ATTEND && tid == 0 && split == 0 && h == 0) p.ncur[b] = n_now;

  const int r0 = split * p.chunk;
  const int r1 = (r0 + p.chunk < n_vis) ? r0 + p.chunk : n_vis;
  if (r0 >= r1) return;

  const size_t unit = (size_t)b * p.Hkv + h;
  uint16_t *Kb = p.K + unit * (size_t)p.cap * D;
  uint16_t *Vb = p.V + unit * (size_t)p.cap * D;
  float *Sb = p.S + unit * (size_t)p.cap;
  const uint16_t *knew = APPEND ? p.k_new + unit * D : nullptr;
  const uint16_t *vnew = APPEND ? p.v_new + unit * D : nullptr;

  // query fragments (MFMA B operand): lane (g, kg) holds q[g][32*ks + 8*kg .. +7]
  bf16x8 qf[KS], qpf[KS];
  const size_t qoff = ((size_t)b * p.Hq + (size_t)h * G + g) * D + 8 * kg;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = bf16x8{};
    qpf[ks] = bf16x8{};
    if (g < G) {
      if (ATTEND) qf[ks] = load_bf16x8(p.q + qoff + 32 * ks);
      if (PENDING) qpf[ks] = load_bf16x8(p.qprev + qoff + 32 * ks);
    }
  }
  float mprev = 0.f, inv_lprev = 0.f;
  if (PENDING && g < G && n_prev > 0) {
    const float *ml = p.mlprev + ((size_t)b * p.Hq + (size_t)h * G + g) * 2;
    mprev = ml[0];
    inv_lprev = 1.0f / ml[1];
  }

  float m_run = -INFINITY, l_run = 0.f;
  f32x4 oacc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) oacc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};

  unsigned char *vst = smem + wave * (kTile * VSTRIDE);

  for (int t = r0 + kTile * wave; t < r1; t += kChunkQuantum) {
    const bool tile_att = ATTEND && t < n_now;  // wave-uniform
    // ---- loads --------------------------------------------------------------------
    bf16x8 kf[2][KS];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      int row = t + 16 * s + r16;
      int rowc = row < n_vis ? row : n_vis - 1;
      const uint16_t *src = (APPEND && appending && rowc == n_old) ? knew : Kb + (size_t)rowc * D;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kf[s][ks] = load_bf16x8(src + 32 * ks + 8 * kg);
      if (APPEND && appending && row == n_old) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) store_bf16x8(Kb + (size_t)n_old * D + 32 * ks + 8 * kg, kf[s][ks]);
      }
    }
    uint4 vf[VIT];
    if (tile_att) {
#pragma unroll
      for (int it = 0; it < VIT; ++it) {
        int row = t + VROWS * it + lane / PIECES;
        int rowc = row < n_now ? row : n_now - 1;
        const uint16_t *src = (APPEND && appending && rowc == n_old) ? vnew : Vb + (size_t)rowc * D;
        vf[it] = *reinterpret_cast<const uint4 *>(src + 8 * (lane % PIECES));
        if (APPEND && appending && row == n_old)
          *reinterpret_cast<uint4 *>(Vb + (size_t)n_old * D + 8 * (lane % PIECES)) = vf[it];
      }
    }
    if (APPEND && appending && lane == 0 && t <= n_old && n_old < t + kTile) {
      Sb[n_old] = p.s_new ? p.s_new[unit] : 0.f;
      p.pos[unit * (size_t)p.cap + n_old] = p.next_pos[b];
    }

    // ---- deferred score update: weights of the previous query on these slots -------
    if (PENDING && t < n_prev) {
      f32x4 accp[2];
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        accp[s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          accp[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[s][ks], qpf[ks], accp[s], 0, 0, 0);
      }
      float mine = 0.f;
#pragma unroll
      for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float a = (g < G) ? exp2f(accp[s][i] * p.scale_log2 - mprev) * inv_lprev : 0.f;
          a += __shfl_xor(a, 1);
          a += __shfl_xor(a, 2);
          a += __shfl_xor(a, 4);
          a += __shfl_xor(a, 8);
          if (r16 == 4 * s + i) mine = a;
        }
      }
      if (r16 < 8) {
        int tok = t + 16 * (r16 >> 2) + 4 * kg + (r16 & 3);
        if (tok < n_prev && tok >= M) Sb[tok] += mine;
      }
    }

    // ---- attention for the current query -----------------------------------------
    if (tile_att) {
      f32x4 acc[2];
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          acc[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[s][ks], qf[ks], acc[s], 0, 0, 0);
      }
      // acc[s][i] = logit(slot t + 16 s + 4 kg + i, head g)
      float x[8];
      float mx = -INFINITY;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        int tok = t + 16 * (e >> 2) + 4 * kg + (e & 3);
        x[e] = tok < n_now ? acc[e >> 2][e & 3] * p.scale_log2 : -INFINITY;
        mx = fmaxf(mx, x[e]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx);  // finite: the tile holds at least one valid slot
      const float corr = exp2f(m_run - m_new);  // m_run = -inf on the first tile -> 0
      m_run = m_new;
      bf16x8 ph, pl;
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float pe = exp2f(x[e] - m_new);
        psum += pe;
        __bf16 hi = (__bf16)pe;
        ph[e] = hi;
        pl[e] = (__bf16)(pe - (float)hi);
      }
      l_run = l_run * corr + psum;
      if (__any(corr != 1.0f)) {
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) oacc[cb] *= corr;
      }
      // stage V rows: the wave's own tile, read back column-wise below
#pragma unroll
      for (int it = 0; it < VIT; ++it) {
        unsigned char *dst = vst + (VROWS * it + lane / PIECES) * VSTRIDE + 16 * (lane % PIECES);
        *reinterpret_cast<uint2 *>(dst) = make_uint2(vf[it].x, vf[it].y);
        *reinterpret_cast<uint2 *>(dst + 8) = make_uint2(vf[it].z, vf[it].w);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        // V^T operand: lane (c = 16 cb + r16, kg) holds V[t + 16 s + 4 kg + i][c] in element 4 s + i
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
          int ea = 2 * e2, eb = 2 * e2 + 1;
          int rowa = 16 * (ea >> 2) + 4 * kg + (ea & 3);
          int rowb = 16 * (eb >> 2) + 4 * kg + (eb & 3);
          uint32_t lo = *reinterpret_cast<const uint16_t *>(vst + rowa * VSTRIDE + 2 * (16 * cb + r16));
          uint32_t hi = *reinterpret_cast<const uint16_t *>(vst + rowb * VSTRIDE + 2 * (16 * cb + r16));
          w[e2] = lo | (hi << 16);
        }
        bf16x8 vt = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
        oacc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, ph, oacc[cb], 0, 0, 0);
        oacc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, pl, oacc[cb], 0, 0, 0);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  }

  if (!ATTEND) return;
  if (r0 >= n_now) return;  // chunk only carried a deferred update (workgroup-uniform)

  // ---- combine the four waves, emit one partial per workgroup ------------------------
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (kg == 0) {
    sm_m[wave][g] = m_run;
    sm_l[wave][g] = l_run;
  }
  __syncthreads();
  float mstar = sm_m[0][g];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) mstar = fmaxf(mstar, sm_m[w][g]);
  const float f = (m_run == -INFINITY) ? 0.f : exp2f(m_run - mstar);
  float *ored = reinterpret_cast<float *>(smem);
  if (g < G) {
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      f32x4 v = oacc[cb] * f;
      *reinterpret_cast<f32x4 *>(ored + (wave * 16 + g) * OSTRIDE + 16 * cb + 4 * kg) = v;
    }
  }
  __syncthreads();
  const size_t pbase = (unit * p.nsplit + split) * (size_t)G;
  for (int idx = tid; idx < G * D; idx += kThreads) {
    int gg = idx / D, c = idx % D;
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) sum += ored[(w * 16 + gg) * OSTRIDE + c];
    p.part_o[(pbase + gg) * D + c] = sum;
  }
  if (tid < G) {
    float ms = sm_m[0][tid];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) ms = fmaxf(ms, sm_m[w][tid]);
    float ls = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      float mw = sm_m[w][tid];
      ls += (mw == -INFINITY) ? 0.f : sm_l[w][tid] * exp2f(mw - ms);
    }
    p.part_ml[(pbase + tid) * 2 + 0] = ms;
    p.part_ml[(pbase + tid) * 2 + 1] = ls;
  }
}

struct MergeParams {
  const float *part_o, *part_ml;
  const int32_t *ncur;      // [Nb]
  const uint16_t *q;        // [Nb][Hq][D]
  float *out;               // [Nb][Hq][D]
  float *lse;               // [Nb][Hq] or null
  uint16_t *qprev;          // [Nb][Hq][D] or null (no score bookkeeping)
  float *mlprev;            // [Nb][Hq][2]
  int32_t *nprev;           // [Nb]
  int32_t *seq_len, *next_pos;  // [Nb]; advanced when the step appended
  int Hq, Hkv, G, chunk, nsplit, appended;
};

// grid (Hq, Nb), block D threads: combine the split partials of one query head.
template <int D>
__global__ __launch_bounds__(D) void attend_merge_kernel(const MergeParams p) {
  const int hq = blockIdx.x, b = blockIdx.y, c = threadIdx.x;
  const int h = hq / p.G, gg = hq % p.G;
  const int n_now = p.ncur[b];
  if (n_now > 0) {
    const int ns = (n_now + p.chunk - 1) / p.chunk;
    const size_t base = (((size_t)b * p.Hkv + h) * p.nsplit) * p.G + gg;
    float m = -INFINITY;
    for (int s = 0; s < ns; ++s) m = fmaxf(m, p.part_ml[(base + (size_t)s * p.G) * 2]);
    float L = 0.f, o = 0.f;
    for (int s = 0; s < ns; ++s) {
      const size_t row = base + (size_t)s * p.G;
      float w = exp2f(p.part_ml[row * 2] - m);
      L += p.part_ml[row * 2 + 1] * w;
      o += p.part_o[row * D + c] * w;
    }
    const size_t orow = (size_t)b * p.Hq + hq;
    p.out[orow * D + c] = o / L;
    if (p.lse && c == 0) p.lse[orow] = (m + log2f(L)) * 0.6931471805599453f;
    if (p.qprev) {
      p.qprev[orow * D + c] = p.q[orow * D + c];
      if (c == 0) {
        p.mlprev[orow * 2] = m;
        p.mlprev[orow * 2 + 1] = L;
      }
    }
  }
  if (hq == 0 && c == 0) {
    if (p.qprev) p.nprev[b] = n_now;
    if (p.appended && n_now > 0) {
      p.seq_len[b] = n_now;
      p.next_pos[b] += 1;
    }
  }
}

}  // namespace dynts
