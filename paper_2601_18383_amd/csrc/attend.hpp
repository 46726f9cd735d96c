// Decode attention + deferred importance-score accumulation for gfx950 (wave64, MFMA).
//
// The cache of one (sequence, KV head) is shared out over nsplit workgroups of W waves (8 by
// default).  Wave number wi of the nsplit*W takes the 32-slot tile that starts at slot 32*wi -- its
// loads are issued before the kernel knows the sequence length -- and then an equal, contiguous
// share of the slots behind those first tiles, 32 at a time, with the next tile's loads already
// in flight while it works on the current one:
//   * K rows go straight from HBM into MFMA operand registers (16-byte loads; lane (r, kg)
//     holds row r, columns 32*ks + 8*kg .. +7).  One v_mfma_f32_16x16x32_bf16 per 32 columns
//     gives the logits of 16 slots x 16 (padded) query heads of the group, so a K tile is read
//     once for the whole GQA group (Eq. attn-score).
//   * the same K registers are multiplied with the PREVIOUS step's query (operands swapped, so
//     a lane ends up with 4 heads of one slot); with that step's final softmax statistics this
//     gives its attention weights exactly, which are summed over the group and added to S
//     (Eq. importance-score, running form).  The score update thus rides on this step's pass
//     over K instead of a second pass or a spill of logits.
//   * V rows are staged through a wave-private LDS tile (coalesced 16-byte loads in,
//     ds_read_b64_tr_b16 transposing reads out) to form the V^T MFMA operand; the softmax
//     weights are split into bf16 hi + lo parts so P.V keeps ~16 bits of each weight
//     (Eq. attn-o); accumulation is fp32 throughout.
//   * online-softmax state (running max, sum, output) is per wave; the waves of a workgroup are
//     combined in LDS.  With nsplit == 1 the result is finished on the spot; otherwise the partial
//     goes to the workspace and the LAST workgroup of the (sequence, KV head) to arrive
//     (device-scope counter) merges the partials, writes `out`, and saves the query and the
//     statistics that the next step's score update needs.  Every workgroup checks in on a
//     per-sequence counter as it starts; the last one to do so advances seq_len / next_pos.
//     No second kernel, no host round trip.
//   * with APPEND the new token's K/V row is written to its slot by one workgroup and enters the
//     softmax as the initial state of the first wave (max = q.k_new, sum = 1, output = v_new), so
//     no wave has to wait for the row to become visible.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dynts {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef short i16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTile = 32;           // cache slots one wave handles per iteration
// A workgroup has W waves (4 or 8).

struct AttendParams {
  uint16_t *K, *V;          // layer base, [Nb][Hkv][cap][D]
  float *S;                 // [Nb][Hkv][cap]
  int32_t *pos;             // [Nb][Hkv][cap]
  int32_t *seq_len;         // [Nb]
  const int32_t *n_prompt;  // [Nb]
  int32_t *next_pos;        // [Nb]
  const uint16_t *q;        // [Nb][Hq][D]
  const uint16_t *k_new, *v_new;  // [Nb][Hkv][D] (fused append) or null
  const float *s_new;       // [Nb][Hkv] or null
  const uint8_t *active;    // [Nb] or null
  float *out;               // [Nb][Hq][D]
  float *lse;               // [Nb][Hq] or null
  const uint16_t *qprev;    // [Nb][Hq][D] query of the deferred update (read)
  uint16_t *qnext;          // [Nb][Hq][D] where this call's query is kept for the next deferred update
  float *mlprev;            // [Nb][Hq][2] (max in log2 units, sum) of the deferred update
  int32_t *nprev;           // [Nb] slots the deferred update covers (0 = none)
  uint64_t *part_o;         // [Nb][Hkv][nsplit][G][D]  (tag << 32 | fp32 bits)
  uint64_t *part_ml;        // [Nb][Hkv][nsplit][G][2]
  uint32_t tag;             // this launch's serial number (never 0)
  int score_tiles;          // updated scores are written out every so many tiles of a wave (1 .. 16)
  // When a trigger is known to follow this step, the step's own scaled logits (log2 units) are kept,
  // [Nb][Hkv][G][cap_pad] fp32, so that its score update can be applied from them (apply_spill_kernel) instead of
  // a second pass over K.  Null: not kept.
  float *spill;
  int cap_pad;              // cap rounded up to a whole tile: row pitch of the kept logits (a tile's store stays inside its row)
  uint32_t *unit_cnt;       // [Nb][Hkv] ticket counters, zero between launches
  uint32_t *seq_cnt;        // [Nb]      arrival counters, zero between launches
  int32_t *status;
  int Nb, Hq, Hkv, G, cap, nsplit;
  int track;                // 1: scores are accumulated from attention (save q and statistics)
  float scale_log2;         // softmax scale * log2(e)
  // paged layout only: K and V are page pools [n_pages][kPageSlots][D]; slot j of a unit lives in page
  // block_table[unit][j / kPageSlots], row j % kPageSlots
  const int32_t *block_table;  // layer base, [Nb][Hkv][max_pages]
  int32_t *block_table_w;      // the same, for the appender
  int32_t *free_stack;         // [n_pages] page ids; entries below *free_top are free
  int32_t *free_top;
  int max_pages, n_pages;
};

constexpr int kPageSlots = 64;  // slots per page: two tiles, so a tile never straddles pages


__device__ __forceinline__ u32x4 load_u32x4(const uint16_t *p) { return *reinterpret_cast<const u32x4 *>(p); }
__device__ __forceinline__ void store_u32x4(uint16_t *p, u32x4 v) { *reinterpret_cast<u32x4 *>(p) = v; }
__device__ __forceinline__ bf16x8 load_bf16x8(const uint16_t *p) {
  return __builtin_bit_cast(bf16x8, load_u32x4(p));
}
__device__ __forceinline__ void store_bf16x8(uint16_t *p, bf16x8 v) {
  store_u32x4(p, __builtin_bit_cast(u32x4, v));
}

// K rows of the 32-slot tile at t as MFMA operand fragments; rows past `end` repeat row end-1.
// Addresses are a uniform base plus a 32-bit byte offset (a unit's cache is far below 4 GiB), which
// keeps the per-tile address arithmetic to a clamp and a multiply-add per 16 rows.
template <int D>
__device__ __forceinline__ void load_k_tile(bf16x8 (&kf)[2][D / 32], const uint16_t *Kb, int t, int r16, int kg,
                                            int end) {
  const char *base = reinterpret_cast<const char *>(Kb);
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    int row = t + 16 * s + r16;
    row = row < end ? row : end - 1;
    const uint32_t off = (uint32_t)row * (uint32_t)(2 * D) + 16u * (uint32_t)kg;
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks)
      kf[s][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(base + off + 64 * ks));
  }
}

// V rows of the tile, whole rows across 16-byte pieces (coalesced); rows past `end` repeat row end-1
template <int D>
__device__ __forceinline__ void load_v_tile(u32x4 (&vf)[kTile / (64 / (D / 8))], const uint16_t *Vb, int t,
                                            int lane, int end) {
  constexpr int PIECES = D / 8, VROWS = 64 / PIECES;
  const char *base = reinterpret_cast<const char *>(Vb);
  const uint32_t lane_off = 16u * (uint32_t)(lane % PIECES);
#pragma unroll
  for (int it = 0; it < kTile / VROWS; ++it) {
    int row = t + VROWS * it + lane / PIECES;
    row = row < end ? row : end - 1;
    vf[it] = *reinterpret_cast<const u32x4 *>(base + ((uint32_t)row * (uint32_t)(2 * D) + lane_off));
  }
}
// Cross-workgroup traffic inside one launch (split partials, arrival counters) consists of relaxed
// agent-scope atomics only, which compile to sc1 accesses that are written through to, and read
// from, the level all XCDs share.  A split partial is handed over WITHOUT any ordering between
// different words: every 32-bit value travels in one 64-bit word together with the launch's tag
// (a serial number no earlier launch of this process used), stored and loaded with single 64-bit
// atomic accesses, so a word is either this launch's value or recognisably stale.  The workgroup
// that draws the last ticket of a (sequence, KV head) merges: it re-reads a word until its tag is
// this launch's.  That loop ends: a workgroup draws its ticket only when it is running, it issues its
// stores without ever waiting for another workgroup, and issued stores become visible.  There is no
// fence, no wait for store acknowledgements and no cache-wide write-back; no ordinary cached access
// ever touches these words during a launch.
__device__ __forceinline__ void tagged_store(uint64_t *p, float v, uint32_t tag) {
  __hip_atomic_store(p, ((uint64_t)tag << 32) | (uint64_t)__float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t tagged_load(const uint64_t *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Draw a ticket from a device counter, the answer to be looked at later.  The address is made to look
// lane-dependent: for a uniform address the compiler rewrites the operation into its wave-aggregated
// form, whose broadcast of the result waits for the atomic -- and for every load issued before it --
// on the spot.
__device__ __forceinline__ uint32_t draw_ticket(uint32_t *counter) {
  uint32_t zero = 0;
  asm volatile("" : "+v"(zero));
  return __hip_atomic_fetch_add(counter + zero, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool tag_is(uint64_t w, uint32_t tag) { return (uint32_t)(w >> 32) == tag; }
__device__ __forceinline__ float tagged_value(uint64_t w) { return __uint_as_float((uint32_t)w); }

// 2^x by the hardware instruction alone (v_exp_f32, ~1 ulp).  Arguments here are <= 0 up to
// rounding; results below 2^-126 flush to zero, which is far under what the sums resolve.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// BURST: updated scores leave in bursts through LDS (see flush_scores) instead of tile by tile.
// SPILL: the step keeps its logits (AttendParams::spill) for a trigger that follows.
template <int D, int W, bool ATTEND, bool PENDING, bool APPEND, bool PAGED = false, bool BURST = false, bool SPILL = false>
__global__ __launch_bounds__(W * 64, 2) void attend_kernel(const AttendParams p) {
  constexpr int kWaves = W, kThreads = W * 64;
  constexpr int KS = D / 32;              // MFMA k-steps per K row
  constexpr int CB = D / 16;              // 16-column blocks of the output
  constexpr int PIECES = D / 8;           // 16-byte pieces per row
  constexpr int VROWS = 64 / PIECES;      // rows covered by one wave-wide 16-byte load
  constexpr int VIT = kTile / VROWS;
  constexpr int VSTRIDE = 2 * D + 32;     // bytes per staged V row (+32: transposing reads hit distinct banks)
  constexpr int OSTRIDE = D + 4;          // floats per row of the cross-wave output reduction
  static_assert(kWaves * kTile * VSTRIDE >= kWaves * 16 * OSTRIDE * 4, "LDS tile is reused for the reduction");
  __shared__ __align__(16) unsigned char smem[kWaves * kTile * VSTRIDE];
  __shared__ float sm_m[kWaves][16];
  __shared__ float sm_l[kWaves][16];
  __shared__ float sm_fin[2][16];
  __shared__ uint32_t sm_flag;
  __shared__ int32_t sm_hdr[5];
  // updated scores of up to kScoreTiles consecutive tiles per wave, written out together (see flush_scores)
  constexpr int kScoreTiles = 16;
  __shared__ __align__(16) float sm_score[PENDING && BURST ? kWaves : 1][PENDING && BURST ? kScoreTiles * kTile : 4];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kg = lane >> 4;
  const int g = r16;  // query head (within the group) of this lane's logits
  // Workgroup -> (unit, chunk).  Consecutive workgroup ids go to the 8 XCDs in turn; the chunks of one
  // (sequence, KV head) unit get ids that are 8 apart, so that they normally run on ONE XCD and their
  // hand-off of partials travels through that XCD's L2 (measured: a round trip between workgroups costs
  // about 0.55 us inside an XCD, 0.7 - 0.9 us across).  Nothing depends on the placement but speed.
  // grid = round_up(units, 8) * nsplit; the padding workgroups leave at once.
  const int wg = blockIdx.x, per_grp = 8 * p.nsplit;
  const int split = (wg % per_grp) >> 3, u_lin = (wg / per_grp) * 8 + (wg & 7);
  if (u_lin >= p.Nb * p.Hkv) return;
  const int b = u_lin / p.Hkv, h = u_lin - b * p.Hkv;
  const int G = p.G;

  const size_t unit = (size_t)b * p.Hkv + h;
  // dense: this unit's rows; paged: the pools
  uint16_t *Kb = PAGED ? p.K : p.K + unit * (size_t)p.cap * D;
  uint16_t *Vb = PAGED ? p.V : p.V + unit * (size_t)p.cap * D;
  const int32_t *tb = PAGED ? p.block_table + unit * (size_t)p.max_pages : nullptr;
  // Paged addressing of one tile: the tile start is first pulled back into the tile that holds row end-1
  // (so every clamped row stays in ONE page); the tile is then loaded relative to that page: base = pool +
  // page * 64 rows, rows and the clamp counted from the page's first slot.
  auto page_of = [&](int tp) -> int {
    int pi = tp / kPageSlots;
    pi = pi < p.max_pages ? pi : p.max_pages - 1;
    int pg = tb[pi];
    return pg < 0 ? 0 : (pg >= p.n_pages ? p.n_pages - 1 : pg);  // never followed out of the pool
  };
  auto clamp_tile = [&](int tt, int end) -> int {
    const int last_tile = (end - 1) & ~(kTile - 1);
    return tt < last_tile ? tt : last_tile;
  };
  auto page_base = [&](int pg) -> size_t { return (size_t)pg * kPageSlots * D; };  // element offset of a page
  float *Sb = p.S + unit * (size_t)p.cap;
  unsigned char *vst = smem + wave * (kTile * VSTRIDE);
  const int vrow_l = lane / PIECES, vpiece = lane % PIECES;
  // Work split of one (sequence, KV head) over its nsplit * W waves: wave wi first takes tile wi
  // (a position known before the sequence length is, so its loads can leave at once); the slots
  // past those first tiles are then cut into contiguous ranges of whole tiles, one per wave, from
  // the actual length, so the waves move (nearly) the same number of bytes whatever the length.
  const int NW = p.nsplit * kWaves;
  const int wi = split * kWaves + wave;
  int t = kTile * wi;

  // ---- request everything the prologue needs in one go -----------------------------------
  // Loads return in order, so the few scalars (lengths, activity) go first; right behind them
  // the first tile, whose addresses depend on kernel arguments only (rows clamped to the end
  // of the allocation; what lies past the sequence is masked once its length is known); then
  // the query and the statistics.
  //
  // The per-sequence words.  seq_len, nprev and next_pos are REWRITTEN during this launch, by the last
  // workgroup of the sequence to check in, so only wave 0 reads them (the wave of the thread that checks
  // in, which it does after these loads have returned); the other waves get them through LDS behind the
  // barrier below.  Lanes 0..4 of wave 0 fetch one word each with a vector load, so nothing waits here
  // (uniform addresses would become scalar loads that the wave must wait for before its tile loads).
  int hdr_word = 1;  // lane 4 without a mask: active
  if (tid < 4) {
    const int32_t *src = tid == 0 ? p.seq_len : (tid == 1 ? p.nprev : (tid == 2 ? p.next_pos : p.n_prompt));
    hdr_word = src[b];
  } else if (tid == 4 && p.active) {
    hdr_word = (int)p.active[b];
  }
  __builtin_amdgcn_sched_barrier(0);
  bf16x8 kf[2][KS];
  u32x4 vf[VIT];
  float s_old = 0.f;
  if (!PAGED) load_k_tile<D>(kf, Kb, t, r16, kg, p.cap);
  if (PENDING) {
    const int tok = t + (lane & (kTile - 1));
    s_old = Sb[tok < p.cap ? tok : p.cap - 1];
  }
  if (ATTEND && !PAGED) load_v_tile<D>(vf, Vb, t, lane, p.cap);
  if (PAGED) {
    // The first tile's page is looked up right away and its 32 rows fetched whole (a tile lies inside one
    // page, and a page id is clamped into the pool, so the addresses are valid whatever the length turns
    // out to be; rows past the sequence hold finite stale data and meet masked logits and zero weights).
    const size_t b0 = page_base(page_of(t));
    const int tr = t & (kPageSlots - 1);
    load_k_tile<D>(kf, Kb + b0, tr, r16, kg, tr + kTile);
    if (ATTEND) load_v_tile<D>(vf, Vb + b0, tr, lane, tr + kTile);
  }
  __builtin_amdgcn_sched_barrier(0);

  // query fragments: lane (g, kg) holds q[g][32*ks + 8*kg .. +7]
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
  // statistics of the deferred update for heads 4*kg .. 4*kg+3 (the rows this lane gets from
  // the swapped-operand MFMA)
  float mprev[4], inv_lprev[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    mprev[i] = 0.f;
    inv_lprev[i] = 0.f;
    const int gg = 4 * kg + i;
    if (PENDING && gg < G) {
      const float *ml = p.mlprev + ((size_t)b * p.Hq + (size_t)h * G + gg) * 2;
      mprev[i] = ml[0];
      inv_lprev[i] = ml[1];
    }
  }

  // the wave that takes the appended token asks for its row (and what goes with it) right away
  const bool new_wave = APPEND && split == 0 && wave == 0;
  bf16x8 kn[KS];
  uint2 vn[CB];
  int pos_new = 0;
  float s_init = 0.f;
  if (new_wave) {
    const uint16_t *knew = p.k_new + unit * D;
    const uint16_t *vnew = p.v_new + unit * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kn[ks] = load_bf16x8(knew + 32 * ks + 8 * kg);  // every operand row is k_new
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) vn[cb] = *reinterpret_cast<const uint2 *>(vnew + 16 * cb + 4 * kg);
    if (p.s_new) s_init = p.s_new[unit];
  }

  // hand the three per-sequence words from wave 0 to the whole workgroup.  Everything above was only
  // ISSUED (the tile loads are still in flight across this barrier); wave 0 waits for its three words,
  // which it would have had to do next anyway.
  if (tid < 5) sm_hdr[tid] = hdr_word;
  __syncthreads();
  const int len_raw = sm_hdr[0];
  const int prev_raw = PENDING ? sm_hdr[1] : 0;
  const int pos_new_all = APPEND ? sm_hdr[2] : 0;
  const int M = sm_hdr[3];
  const int act_raw = sm_hdr[4];
  pos_new = pos_new_all;

  // ---- what this launch does for sequence b (identical in every workgroup of b) ---------
  // n_rows cache slots are attended from the cache; when a token is appended in the same
  // pass its row is taken from k_new / v_new up front (below), so the tiles never see it.
  const bool act = act_raw != 0;
  int n_old = len_raw;
  n_old = n_old < 0 ? 0 : (n_old > p.cap ? p.cap : n_old);
  int n_now = 0, n_rows = 0;
  bool appending = false;
  if (ATTEND && act) {
    if (APPEND) {
      if (n_old < p.cap) {
        n_now = n_old + 1;
        n_rows = n_old;
        appending = true;
      } else if (tid == 0 && split == 0 && h == 0) {
        atomicOr(p.status, 1);
      }
    } else {
      n_now = n_rows = n_old;
    }
  }
  int n_prev = prev_raw;
  n_prev = n_prev < 0 ? 0 : (n_prev > p.cap ? p.cap : n_prev);
  const int n_vis = n_rows > n_prev ? n_rows : n_prev;
  // workgroups of this unit that produce an attention partial (chunk 0 always does when the
  // sequence is attended: it owns the appended token), and that have any work at all
  // (a workgroup has work iff its first wave's first tile starts inside the sequence)
  constexpr int kFirst = kWaves * kTile;  // slots covered by a workgroup's first tiles
  auto wgs_for = [&](int n) { int c = (n + kFirst - 1) / kFirst; return c < p.nsplit ? c : p.nsplit; };
  const int chunks_now = n_now > 0 ? (wgs_for(n_rows) > 1 ? wgs_for(n_rows) : 1) : 0;
  const int chunks_prev = wgs_for(n_prev);
  const int chunks_vis = chunks_now > chunks_prev ? chunks_now : chunks_prev;
#pragma unroll
  for (int i = 0; i < 4; ++i)  // inv_l = 0 switches padded heads and idle sequences off
    inv_lprev[i] = (PENDING && 4 * kg + i < G && n_prev > 0) ? 1.0f / inv_lprev[i] : 0.f;

  // Every workgroup of the sequence checks in once its reads of seq_len / nprev / next_pos have come
  // back: thread 0 checks in, and its own wave made those reads and has already consumed their values
  // (they went through LDS above), so the atomic is issued after they completed.  The last workgroup
  // to check in advances the three words -- by then no workgroup of the sequence has a read of them
  // outstanding.  The check-in is issued early and its answer looked at later, so it costs no round
  // trip at the end of the workgroup.
  uint32_t seq_ticket = 0xffffffffu;
  auto seq_checkin = [&]() {
    if (ATTEND && tid == 0) seq_ticket = draw_ticket(&p.seq_cnt[b]);
  };
  auto seq_settle = [&]() {
    if (ATTEND && tid == 0 && seq_ticket == (uint32_t)p.nsplit * p.Hkv - 1) {
      __hip_atomic_store(&p.seq_cnt[b], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (p.track) p.nprev[b] = n_now;
      if (APPEND && appending) {
        p.seq_len[b] = n_now;
        p.next_pos[b] = pos_new_all + 1;
      }
    }
  };

  if (split >= chunks_vis) {
    seq_checkin();
    seq_settle();
    return;
  }
  // this wave's contiguous range [ra, rb) behind the first tiles
  const int base = kTile * NW;
  int per = n_vis > base ? (n_vis - base + NW - 1) / NW : 0;
  // whole tiles per wave: only the last wave with work ends on a partial tile (measured 1-3 % faster than
  // byte-equal ranges that end mid-tile everywhere), and in the paged layout no tile straddles two pages
  per = (per + kTile - 1) & ~(kTile - 1);
  // (handed out from the last wave down: the range that comes up short or empty goes to the unit's first
  // waves, of which wave 0 also takes the appended token; 0.5 % on the many-unit workloads)
  const int ra = base + (NW - 1 - wi) * per;
  const int rb = ra + per < n_vis ? ra + per : n_vis;

  // keep this call's query for the next deferred score update (its own buffer: the old one is
  // still being read by the other workgroups of this launch)
  if (ATTEND && p.track && split == 0 && wave == 0 && g < G && n_now > 0) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) store_bf16x8(p.qnext + qoff + 32 * ks, qf[ks]);
  }

  float m_run = -INFINITY, l_run = 0.f;
  f32x4 oacc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) oacc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // ---- fused append: the new token is this wave's starting softmax state -----------------
  // One wave of the unit takes the appended token: its logit is q.k_new for every head, its
  // weight relative to itself is 1, so the running state starts as (max = logit, sum = 1,
  // output = v_new).  The same wave writes the row into the cache.  All of it overlaps the
  // wait for the first tile.
  if (new_wave && appending) {
    f32x4 a0 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) a0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kn[ks], qf[ks], a0, 0, 0, 0);
    m_run = a0[0] * p.scale_log2;
    l_run = kg == 0 ? 1.f : 0.f;  // per-lane partial sums are added over kg at the end
    if (SPILL && kg == 0 && g < G) p.spill[(unit * G + g) * (size_t)p.cap_pad + n_old] = m_run;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
      const bf16x4 v4 = __builtin_bit_cast(bf16x4, vn[cb]);
      oacc[cb] = f32x4{(float)v4[0], (float)v4[1], (float)v4[2], (float)v4[3]};
    }
    size_t new_row = (size_t)n_old * D;  // element offset of the new row from Kb / Vb
    bool have_row = true;
    if (PAGED) {
      // the slot's page: a fresh one from the free stack when the slot opens a page
      int pg = 0;
      if (lane == 0) {
        const int pi = n_old / kPageSlots;
        if (n_old % kPageSlots == 0) {
          const int idx = atomicSub(p.free_top, 1) - 1;
          if (idx >= 0) {
            pg = p.free_stack[idx];
            p.block_table_w[unit * (size_t)p.max_pages + pi] = pg;
          } else {  // pool exhausted: give the ticket back, drop the row, say so
            atomicAdd(p.free_top, 1);
            atomicOr(p.status, 4);
            pg = -1;
          }
        } else {
          pg = tb[pi];
        }
      }
      pg = __builtin_amdgcn_readfirstlane(pg);
      have_row = pg >= 0 && pg < p.n_pages;
      new_row = ((size_t)(have_row ? pg : 0) * kPageSlots + n_old % kPageSlots) * D;
    }
    if (r16 == 0 && have_row) {
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) *reinterpret_cast<uint2 *>(Vb + new_row + 16 * cb + 4 * kg) = vn[cb];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) store_bf16x8(Kb + new_row + 32 * ks + 8 * kg, kn[ks]);
    }
    if (lane == 0) {
      Sb[n_old] = s_init;
      p.pos[unit * (size_t)p.cap + n_old] = pos_new;
    }
  }

  seq_checkin();

  // the first tile was fetched before the length was known: keep rows past the sequence out of P.V
  if (ATTEND && !PAGED && t + kTile > n_rows) {
#pragma unroll
    for (int it = 0; it < VIT; ++it) vf[it] = (t + VROWS * it + vrow_l < n_rows) ? vf[it] : u32x4{0u, 0u, 0u, 0u};
  }
  // Row clamps of the prefetches: a prefetch must not pull another wave's rows, so rows are
  // clamped to the end of this wave's own range (or, with no range, of its first tile); the
  // clamp row is always a valid row of the allocation.
  const int own_end = ra < rb ? rb : (t + kTile < n_vis ? t + kTile : n_vis);
  const int k_last = own_end > 0 ? own_end : 1;
  const int v_end = own_end < n_rows ? own_end : n_rows;
  // (paged: V rows are clamped like K rows, so that one page serves both; slots below n_vis are allocated,
  // and whatever lies past n_rows meets a zero weight)
  const int v_last = PAGED ? k_last : (v_end > 0 ? v_end : 1);
  // paged: the page of the next tile to fetch is looked up one tile ahead of its use
  int pg_nxt = 0;
  if (PAGED) pg_nxt = page_of(clamp_tile(ra, k_last));

  // ---- updated scores leave in bursts -----------------------------------------------------------
  // A tile updates 32 scores (128 bytes).  Written tile by tile these are small writes scattered through
  // the read stream, which cost the memory system far more than their bytes (measured: 4 % of the launch
  // for 1.2 % of the traffic).  So, when the launch says so (score_tiles > 1: the cache is larger than
  // the memory-side cache; below that the single writes are absorbed and bursts at the end of a workgroup
  // only lengthen its tail), a wave parks them in LDS and writes a run of consecutive tiles with
  // 16 bytes per lane at once: when the run breaks, when score_tiles have gathered, and when the wave is
  // done.  sc_base: first slot of the run, sc_n: tiles in it, [sc_lo, sc_hi): the slots that may be written
  // (thinking slots below the end of the deferred update and of this wave's share).
  float *sbuf = sm_score[PENDING && BURST ? wave : 0];
  int sc_base = 0, sc_n = 0, sc_lo = 0, sc_hi = 0;
  auto flush_scores = [&]() {
    if (!PENDING || !BURST || sc_n == 0) return;
    wave_lds_fence();
    for (int c0 = 0; c0 < sc_n * kTile; c0 += 256) {
      const int off = c0 + 4 * lane;
      if (off < sc_n * kTile) {
        const f32x4 v = *reinterpret_cast<const f32x4 *>(sbuf + off);
        const int s0 = sc_base + off;
        float *dst = Sb + s0;
        if (s0 >= sc_lo && s0 + 4 <= sc_hi && (reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
          *reinterpret_cast<f32x4 *>(dst) = v;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (s0 + i >= sc_lo && s0 + i < sc_hi) dst[i] = v[i];
        }
      }
    }
    wave_lds_fence();  // the buffer is written again
    sc_n = 0;
  };

  // ---- one 32-slot tile of this wave -------------------------------------------------------
  // Branch-free apart from two wave-uniform guards; the next tile's loads are issued
  // unconditionally (clamped), so the loop never drains its outstanding loads.
  // t: first slot of the tile; hi: end of the slots of this tile that belong to this wave;
  // tn: first slot of the wave's next tile (any value when there is none: the loads are clamped)
  auto tile = [&](int t, int hi, int tn) {
    const int att_hi = hi < n_rows ? hi : n_rows;
    const int pend_hi = hi < n_prev ? hi : n_prev;

    // logits for the current query (A = K rows, B = q) and for the previous one (swapped:
    // accp[s][i] = logit(slot t + 16 s + r16, head 4 kg + i))
    f32x4 acc[2], accp[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
      accp[s] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if (ATTEND) acc[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[s][ks], qf[ks], acc[s], 0, 0, 0);
        if (PENDING) accp[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qpf[ks], kf[s][ks], accp[s], 0, 0, 0);
      }
    }
    const float s_cur = s_old;
    // where the next tile is fetched from: (base, first row, row clamp), page-relative in the paged layout
    size_t nb = 0;
    int nt = tn, nk_end = k_last, nv_end = v_last;
    if (PAGED) {
      const int tnp = clamp_tile(tn, k_last), page_start = tnp & ~(kPageSlots - 1);
      nb = page_base(pg_nxt);
      nt = tnp - page_start;
      nk_end = k_last - page_start;
      nv_end = v_last - page_start;
      pg_nxt = page_of(clamp_tile(tn + kTile, k_last));
    }
    load_k_tile<D>(kf, Kb + nb, nt, r16, kg, nk_end);
    if (PENDING) {
      const int tok = tn + (lane & (kTile - 1));
      s_old = Sb[tok < p.cap ? tok : p.cap - 1];
    }

    // ---- deferred score update: S[slot] += sum over the group of alpha_prev[g][slot] --------
    if (PENDING && t < pend_hi) {
      float part[2];
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        float a = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) a += fast_exp2(accp[s][i] * p.scale_log2 - mprev[i]) * inv_lprev[i];
        if (G > 4) a += __shfl_xor(a, 16);
        if (G > 8) a += __shfl_xor(a, 32);
        part[s] = a;
      }
      if (G <= 8) {  // lanes of row group 0 (and 1) hold the sums; hand sub-tile 1 to row group 1
        const float other = __shfl(part[1], r16);
        if (kg == 1) part[1] = other;
      }
      // lane < 32 holds the new score of slot t + lane (sub-tile kg, row r16): write it, or park it
      const float s_upd = s_cur + (kg == 0 ? part[0] : part[1]);
      if (!BURST) {
        const int tok = t + lane;
        if (lane < kTile && tok < pend_hi && tok >= M) Sb[tok] = s_upd;
      } else {
        if (sc_n > 0 && (t != sc_base + kTile * sc_n || sc_n >= p.score_tiles)) flush_scores();
        if (sc_n == 0) {
          sc_base = t;
          sc_lo = t > M ? t : M;
        }
        if (lane < kTile) sbuf[kTile * sc_n + lane] = s_upd;
        ++sc_n;
        sc_hi = pend_hi;
      }
    }

    // ---- attention for the current query --------------------------------------------------
    if (ATTEND && t < att_hi) {
      // acc[s][i] = logit(slot t + 16 s + 4 kg + i, head g)
      float x[8];
      float mx = -INFINITY;
      if (t + kTile <= att_hi) {  // wave-uniform: a full tile needs no masks
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          x[e] = acc[e >> 2][e & 3] * p.scale_log2;
          mx = fmaxf(mx, x[e]);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int tok = t + 16 * (e >> 2) + 4 * kg + (e & 3);
          x[e] = tok < att_hi ? acc[e >> 2][e & 3] * p.scale_log2 : -INFINITY;
          mx = fmaxf(mx, x[e]);
        }
      }
      if (SPILL && g < G) {  // this lane's 8 logits of head g: slots t + 16 s + 4 kg .. +3
        // (only slots this tile attends: the slot behind them may be the appended token's, kept by its own wave)
        float *sp = p.spill + (unit * G + g) * (size_t)p.cap_pad + t + 4 * kg;
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const int s_lo = t + 16 * s2 + 4 * kg;
          if (s_lo + 4 <= att_hi) {
            *reinterpret_cast<f32x4 *>(sp + 16 * s2) = f32x4{x[4 * s2], x[4 * s2 + 1], x[4 * s2 + 2], x[4 * s2 + 3]};
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (s_lo + i < att_hi) sp[16 * s2 + i] = x[4 * s2 + i];
          }
        }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx);     // finite: the tile holds at least one valid slot
      const float corr = fast_exp2(m_run - m_new);  // m_run = -inf on the first tile -> 0
      m_run = m_new;
      bf16x8 ph, pl;
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float pe = fast_exp2(x[e] - m_new);
        psum += pe;
        const __bf16 hi = (__bf16)pe;
        ph[e] = hi;
        pl[e] = (__bf16)(pe - (float)hi);
      }
      l_run = l_run * corr + psum;
      {
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) oacc[cb] *= corr;
      }
      // stage this tile's V rows in the wave's LDS tile, then fetch the next tile's
#pragma unroll
      for (int it = 0; it < VIT; ++it)
        *reinterpret_cast<u32x4 *>(vst + (VROWS * it + vrow_l) * VSTRIDE + 16 * vpiece) = vf[it];
      wave_lds_fence();
      load_v_tile<D>(vf, Vb + nb, nt, lane, nv_end);
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        // V^T operand: lane (c = 16 cb + r16, kg) gets V[t + 16 s + 4 kg + i][c] as element 4 s + i.
        // ds_read_b64_tr_b16: within 16 lanes, lane i's element e comes from source lane
        // 4 e + i/4, element i%4; so source lane j points at row (j / 4), columns 4 (j % 4) .. +3.
        const unsigned char *src = vst + (4 * kg + (r16 >> 2)) * VSTRIDE + 2 * (16 * cb + 4 * (r16 & 3));
        i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) i16x4 *)(src));
        i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) i16x4 *)(src + 16 * VSTRIDE));
        i16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        const bf16x8 vt = __builtin_bit_cast(bf16x8, both);
        oacc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, ph, oacc[cb], 0, 0, 0);
        oacc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, pl, oacc[cb], 0, 0, 0);
      }
      wave_lds_fence();
    }
  };

  if (t < n_vis) tile(t, t + kTile < n_vis ? t + kTile : n_vis, ra);
  seq_settle();
  for (t = ra; t < rb; t += kTile) tile(t, rb, t + kTile);
  flush_scores();

  if (!ATTEND) return;
  // with several chunks per unit: draw this workgroup's ticket now, so that the round trip of the atomic
  // overlaps the combine below.  (The holder of the last ticket merges, whenever it gets there.)
  uint32_t unit_ticket = 0;
  if (chunks_vis > 1 && tid == 0) unit_ticket = draw_ticket(&p.unit_cnt[unit]);
  const bool has_partial = split < chunks_now;  // workgroup-uniform; false: the chunk only carried a deferred update
  if (chunks_vis == 1 && !has_partial) return;

  // Merging (several chunks per unit): thread tid owns output elements tid + k * kThreads, in its own partial
  // and in the merge; chunks are merged kMergeGroup at a time, in chunk order.  Asking for a group means:
  // every thread requests its elements of the group's partials, and threads 0 .. 16 * kMergeGroup - 1 the
  // (max, sum) of one (chunk, head) each; this workgroup's own partial never comes from memory.
  constexpr int NE = (16 * D + kThreads - 1) / kThreads;  // output elements per thread at the largest group size
  constexpr int kMergeGroup = 4;
  const int ne = (G * D + kThreads - 1) / kThreads;
  const size_t ubase = unit * p.nsplit * (size_t)G;
  uint64_t ask_o[NE][kMergeGroup], ask_m = 0, ask_l = 0;
  auto ask_group = [&](int s0) {
#pragma unroll
    for (int k = 0; k < NE; ++k) {
      const int idx = tid + k * kThreads;
#pragma unroll
      for (int j = 0; j < kMergeGroup; ++j) {
        const int sj = s0 + j;
        ask_o[k][j] = (uint64_t)p.tag << 32;  // nothing to wait for
        if (k < ne && idx < G * D && sj < chunks_now && !(has_partial && sj == split))
          ask_o[k][j] = tagged_load(&p.part_o[(ubase + (size_t)sj * G + idx / D) * D + idx % D]);
      }
    }
    ask_m = ask_l = (uint64_t)p.tag << 32;
    if (tid < 16 * kMergeGroup) {
      const int sj = s0 + (tid >> 4), gg = tid & 15;
      if (sj < chunks_now && gg < G && !(has_partial && sj == split)) {
        const uint64_t *src = &p.part_ml[(ubase + (size_t)sj * G + gg) * 2];
        ask_m = tagged_load(src);
        ask_l = tagged_load(src + 1);
      }
    }
  };
  auto group_fresh = [&]() {
    bool ok = tag_is(ask_m, p.tag) && tag_is(ask_l, p.tag);
#pragma unroll
    for (int k = 0; k < NE; ++k)
#pragma unroll
      for (int j = 0; j < kMergeGroup; ++j) ok = ok && tag_is(ask_o[k][j], p.tag);
    return ok;
  };

  // ---- combine the four waves ------------------------------------------------------------
  float *ored = reinterpret_cast<float *>(smem);
  if (has_partial) {
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
  if (g < G) {
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      f32x4 v = oacc[cb] * f;
      *reinterpret_cast<f32x4 *>(ored + (wave * 16 + g) * OSTRIDE + 16 * cb + 4 * kg) = v;
    }
  }
  if (tid < G) {
    float ms = sm_m[0][tid];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) ms = fmaxf(ms, sm_m[w][tid]);
    float ls = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float mw = sm_m[w][tid];
      ls += (mw == -INFINITY) ? 0.f : sm_l[w][tid] * exp2f(mw - ms);
    }
    sm_fin[0][tid] = ms;
    sm_fin[1][tid] = ls;
  }
  __syncthreads();
  }

  const size_t orow0 = (size_t)b * p.Hq + (size_t)h * G;  // first query head of this group
  if (chunks_vis == 1) {
    // the chunk is the whole cache: finish here
    for (int idx = tid; idx < G * D; idx += kThreads) {
      const int gg = idx / D, c = idx % D;
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) sum += ored[(w * 16 + gg) * OSTRIDE + c];
      p.out[(orow0 + gg) * D + c] = sum / sm_fin[1][gg];
    }
    if (tid < G) {
      if (p.lse) p.lse[orow0 + tid] = (sm_fin[0][tid] + log2f(sm_fin[1][tid])) * 0.6931471805599453f;
      if (p.track) {
        p.mlprev[(orow0 + tid) * 2] = sm_fin[0][tid];
        p.mlprev[(orow0 + tid) * 2 + 1] = sm_fin[1][tid];
      }
    }
    return;
  }

  // ---- several chunks: publish the partial, the holder of the last ticket merges ----------------
  float own_o[NE];
#pragma unroll
  for (int k = 0; k < NE; ++k) own_o[k] = 0.f;
  if (has_partial) {
    const size_t pbase = (unit * p.nsplit + split) * (size_t)G;
#pragma unroll
    for (int k = 0; k < NE; ++k) {
      const int idx = tid + k * kThreads;
      if (k < ne && idx < G * D) {
        const int gg = idx / D, c = idx % D;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) sum += ored[(w * 16 + gg) * OSTRIDE + c];
        own_o[k] = sum;
        tagged_store(&p.part_o[(pbase + gg) * D + c], sum, p.tag);
      }
    }
    if (tid < G) {
      tagged_store(&p.part_ml[(pbase + tid) * 2 + 0], sm_fin[0][tid], p.tag);
      tagged_store(&p.part_ml[(pbase + tid) * 2 + 1], sm_fin[1][tid], p.tag);
    }
  }
  // the ticket was drawn when this workgroup's first wave left its tile loop; its answer is looked at now
  if (tid == 0) sm_flag = unit_ticket;
  __syncthreads();
  const bool merger = sm_flag == (uint32_t)chunks_vis - 1;
  if (!merger) return;
  if (tid == 0) __hip_atomic_store(&p.unit_cnt[unit], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (chunks_now == 0) return;

  __shared__ float sm_pm[kMergeGroup][16], sm_pl[kMergeGroup][16];
  float m_e[NE], L_e[NE], o_e[NE];
#pragma unroll
  for (int k = 0; k < NE; ++k) {
    m_e[k] = -INFINITY;
    L_e[k] = 0.f;
    o_e[k] = 0.f;
  }
  for (int s0 = 0; s0 < chunks_now; s0 += kMergeGroup) {
    ask_group(s0);
    while (!group_fresh()) ask_group(s0);  // a word that is not this launch's yet is on its way: ask again
    if (tid < 16 * kMergeGroup) {
      const int j = tid >> 4, gg = tid & 15, sj = s0 + j;
      if (sj < chunks_now && gg < G) {
        const bool mine = has_partial && sj == split;
        sm_pm[j][gg] = mine ? sm_fin[0][gg] : tagged_value(ask_m);
        sm_pl[j][gg] = mine ? sm_fin[1][gg] : tagged_value(ask_l);
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < NE; ++k) {
      const int idx = tid + k * kThreads;
      if (k < ne && idx < G * D) {
        const int gg = idx / D;
#pragma unroll
        for (int j = 0; j < kMergeGroup; ++j) {
          if (s0 + j < chunks_now) {
            const float ms = sm_pm[j][gg], ls = sm_pl[j][gg];
            const float ov = (has_partial && s0 + j == split) ? own_o[k] : tagged_value(ask_o[k][j]);
            const float mn = fmaxf(m_e[k], ms);  // finite: a chunk that has a partial has attended a slot
            const float fa = fast_exp2(m_e[k] - mn), fb = fast_exp2(ms - mn);
            L_e[k] = L_e[k] * fa + ls * fb;
            o_e[k] = o_e[k] * fa + ov * fb;
            m_e[k] = mn;
          }
        }
      }
    }
    if (s0 + kMergeGroup < chunks_now) __syncthreads();  // the statistics' LDS is written again
  }
#pragma unroll
  for (int k = 0; k < NE; ++k) {
    const int idx = tid + k * kThreads;
    if (k < ne && idx < G * D) {
      const int gg = idx / D, c = idx % D;
      p.out[(orow0 + gg) * D + c] = o_e[k] / L_e[k];
      if (c == 0) {
        if (p.lse) p.lse[orow0 + gg] = (m_e[k] + log2f(L_e[k])) * 0.6931471805599453f;
        if (p.track) {
          p.mlprev[(orow0 + gg) * 2] = m_e[k];
          p.mlprev[(orow0 + gg) * 2 + 1] = L_e[k];
        }
      }
    }
  }
}

// The score update of a step whose logits were kept (AttendParams::spill): S[slot] += sum over the group of
// 2^(logit - max) / sum, for the thinking slots that step attended, with that step's final softmax
// statistics -- the same arithmetic as the deferred update inside attend_kernel, fed from 4 * G bytes per slot
// instead of a K row.  grid (ceil(cap / (256 * kApplyPerThread)), Hkv * Nb), 256 threads.
constexpr int kApplyPerThread = 4;
__global__ __launch_bounds__(256) void apply_spill_kernel(float *S, const float *spill, const float *mlprev,
                                                          const int32_t *nprev, const int32_t *n_prompt, int Hkv, int Hq,
                                                          int G, int cap, int cap_pad) {
  const int unit = blockIdx.y, b = unit / Hkv, h = unit - b * Hkv;
  const int n = nprev[b] < cap ? nprev[b] : cap, M = n_prompt[b];
  const int j0 = (blockIdx.x * 256 + threadIdx.x) * kApplyPerThread;
  if (j0 >= n || j0 + kApplyPerThread <= M) return;
  float add[kApplyPerThread];
#pragma unroll
  for (int i = 0; i < kApplyPerThread; ++i) add[i] = 0.f;
  for (int g = 0; g < G; ++g) {
    const float *ml = mlprev + ((size_t)b * Hq + (size_t)h * G + g) * 2;
    const float m = ml[0], inv_l = 1.0f / ml[1];
    const f32x4 x = *reinterpret_cast<const f32x4 *>(spill + ((size_t)unit * G + g) * cap_pad + j0);
#pragma unroll
    for (int i = 0; i < kApplyPerThread; ++i) add[i] += fast_exp2(x[i] - m) * inv_l;
  }
  float *Su = S + (size_t)unit * cap;
#pragma unroll
  for (int i = 0; i < kApplyPerThread; ++i)
    if (j0 + i < n && j0 + i >= M) Su[j0 + i] += add[i];
}

}  // namespace dynts
