// Host side of the C ABI declared in include/dynts.h: argument checks, workspace layout and
// kernel launches.  Nothing here allocates device memory or synchronises the host.
#include "../../include/dynts.h"

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "attend.hpp"
#include "compact.hpp"
#include "paged.hpp"
#include "predictor.hpp"
#include "probe.hpp"
#include "score_block.hpp"
#include "select.hpp"

namespace {

constexpr size_t kAlign = 256;
constexpr int kSelectLdsMax = 16384;  // candidates whose keys are cached in LDS (64 KiB)

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Plan {
  int G = 0, waves = 0, chunk = 0, nsplit = 0;
  size_t off_part_o = 0, off_part_ml = 0, off_unit_cnt = 0, off_seq_cnt = 0, off_qprev = 0, off_mlprev = 0, off_nprev = 0, off_spill = 0;
  int cap_pad = 0;
  size_t bytes = 0;
};

int check_config(const dynts_config *c) {
  if (!c) return DYNTS_ENULL;
  if (c->n_layers <= 0 || c->batch <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0) return DYNTS_EINVAL;
  if (c->budget < 0 || c->window < 0 || c->evict_every <= 0 || c->capacity <= 0) return DYNTS_EINVAL;
  if (c->score_mode != DYNTS_SCORE_ACCUMULATE && c->score_mode != DYNTS_SCORE_EXTERNAL) return DYNTS_EINVAL;
  if (!(c->softmax_scale >= 0.f) || std::isinf(c->softmax_scale)) return DYNTS_EINVAL;
  if (c->head_dim != 64 && c->head_dim != 128) return DYNTS_ESHAPE;
  if (c->n_q_heads % c->n_kv_heads) return DYNTS_ESHAPE;
  if (c->n_q_heads / c->n_kv_heads > 16) return DYNTS_ESHAPE;
  if (c->n_kv_heads * (c->head_dim / 8) > 1024) return DYNTS_ESHAPE;
  if (c->batch > 65535 || c->n_kv_heads > 65535) return DYNTS_ESHAPE;
  if (c->capacity > (1 << 22)) return DYNTS_ESHAPE;  // row offsets inside a unit are 32-bit byte offsets
  if ((long long)c->capacity < (long long)c->budget + c->window + c->evict_every) return DYNTS_ECAPACITY;
  return DYNTS_OK;
}

// Split every (sequence, KV head) cache into chunks, one workgroup per chunk.  Workgroups have
// 8 waves (one per compute unit fits) when that still fills the chip, else 4; chunks are whole
// multiples of the workgroup's tile quantum.  The aim is about one 8-wave workgroup per compute
// unit: few enough that every wave loops over many tiles with its loads in flight, and that
// the split partials stay small.
Plan make_plan(const dynts_config &c, int target_wgs, int waves) {
  Plan p;
  p.G = c.n_q_heads / c.n_kv_heads;
  const long long units = (long long)c.batch * c.n_kv_heads;
  const long long target = target_wgs > 0 ? target_wgs : 256;  // workgroups wanted (256 compute units)
  p.waves = waves == 4 ? 4 : 8;
  const int quantum = p.waves * dynts::kTile;
  const int quanta = (c.capacity + quantum - 1) / quantum;
  long long want = (target + units / 2) / units;
  if (want < 1) want = 1;
  if (want > quanta) want = quanta;
  const int per = (int)((quanta + want - 1) / want);  // quanta per chunk
  p.chunk = per * quantum;
  p.nsplit = (c.capacity + p.chunk - 1) / p.chunk;
  const size_t rows = (size_t)units * p.nsplit * p.G;
  size_t off = 0;
  p.off_part_o = off;  off = align_up(off + rows * c.head_dim * sizeof(uint64_t));  // value + tag per word
  p.off_part_ml = off; off = align_up(off + rows * 2 * sizeof(uint64_t));
  p.off_unit_cnt = off; off = align_up(off + (size_t)units * sizeof(uint32_t));
  p.off_seq_cnt = off; off = align_up(off + (size_t)c.batch * sizeof(uint32_t));
  const size_t LB = (size_t)c.n_layers * c.batch;
  p.off_qprev = off;   off = align_up(off + 2 * LB * c.n_q_heads * c.head_dim * sizeof(uint16_t));  // two copies, used in turn
  p.off_mlprev = off;  off = align_up(off + LB * c.n_q_heads * 2 * sizeof(float));
  p.off_nprev = off;   off = align_up(off + LB * sizeof(int32_t));
  // the logits of one step of one layer, kept when a trigger is known to follow (score_mode accumulate only)
  p.cap_pad = (c.capacity + dynts::kTile - 1) / dynts::kTile * dynts::kTile;
  p.off_spill = off;
  if (c.score_mode == DYNTS_SCORE_ACCUMULATE) off = align_up(off + (size_t)units * p.G * p.cap_pad * sizeof(float));
  p.bytes = off;
  return p;
}

}  // namespace

struct dynts_ctx {
  dynts_config cfg;
  Plan plan;
  float scale_log2;
  bool bound = false;
  uint16_t *K = nullptr, *V = nullptr;
  float *S = nullptr;
  int32_t *pos = nullptr, *seq_len = nullptr, *next_pos = nullptr, *n_prompt = nullptr, *status = nullptr;
  unsigned char *ws = nullptr;
  std::vector<unsigned char> pending;  // per layer: a score update is owed (1: by a pass over K, 2: from kept logits)
  std::vector<unsigned char> hint;     // per layer: a trigger follows the next fused step, keep its logits
  int spill_layer = -1;                // the layer whose kept logits are waiting to be applied, or -1
  std::vector<unsigned char> qslot;    // per layer: which copy of the saved query is current
  hipEvent_t ev_start = nullptr, ev_stop = nullptr;
  std::vector<hipEvent_t> ev_list_start, ev_list_stop;  // one pair per coming attend launch
  size_t ev_list_next = 0;
  // paged layout (dynts_bind_paged): K and V above are the page pools
  bool paged = false;
  int32_t *block_table = nullptr, *free_stack = nullptr, *free_top = nullptr;
  int max_pages = 0, n_pages = 0;
};

namespace {

int launch_status() { return hipGetLastError() == hipSuccess ? DYNTS_OK : DYNTS_EHIP; }

// Serial number of an attend launch: the tag its split partials carry.  One counter for the whole
// process, so that two contexts which share scratch memory can never mistake each other's words for
// their own; 0 is skipped (zero-filled scratch must read as stale).
uint32_t next_launch_tag() {
  static std::atomic<uint32_t> serial{0};
  uint32_t t = serial.fetch_add(1, std::memory_order_relaxed) + 1;
  if (t == 0) t = serial.fetch_add(1, std::memory_order_relaxed) + 1;
  return t;
}

int check_call(const dynts_ctx *ctx, int32_t layer) {
  if (!ctx) return DYNTS_ENULL;
  if (!ctx->bound) return DYNTS_ENOTBOUND;
  if (layer < 0 || layer >= ctx->cfg.n_layers) return DYNTS_EINVAL;
  return DYNTS_OK;
}

struct LayerView {
  uint16_t *K, *V;
  float *S;
  int32_t *pos, *seq_len, *next_pos;
  uint16_t *qprev, *qnext;
  float *mlprev;
  int32_t *nprev;
  int32_t *block_table;  // paged layout: this layer's [Nb][Hkv][max_pages]
};

LayerView layer_view(const dynts_ctx *ctx, int layer) {
  const dynts_config &c = ctx->cfg;
  const size_t units = (size_t)c.batch * c.n_kv_heads;
  const size_t rows = units * c.capacity;
  LayerView v;
  v.K = ctx->paged ? ctx->K : ctx->K + (size_t)layer * rows * c.head_dim;
  v.V = ctx->paged ? ctx->V : ctx->V + (size_t)layer * rows * c.head_dim;
  v.block_table = ctx->paged ? ctx->block_table + (size_t)layer * units * ctx->max_pages : nullptr;
  v.S = ctx->S + (size_t)layer * rows;
  v.pos = ctx->pos + (size_t)layer * rows;
  v.seq_len = ctx->seq_len + (size_t)layer * c.batch;
  v.next_pos = ctx->next_pos + (size_t)layer * c.batch;
  const size_t LBq = (size_t)layer * c.batch * c.n_q_heads;
  uint16_t *qbuf = reinterpret_cast<uint16_t *>(ctx->ws + ctx->plan.off_qprev) + 2 * LBq * c.head_dim;
  const size_t qsz = (size_t)c.batch * c.n_q_heads * c.head_dim;
  v.qprev = qbuf + (ctx->qslot[layer] ? qsz : 0);
  v.qnext = qbuf + (ctx->qslot[layer] ? 0 : qsz);
  v.mlprev = reinterpret_cast<float *>(ctx->ws + ctx->plan.off_mlprev) + LBq * 2;
  v.nprev = reinterpret_cast<int32_t *>(ctx->ws + ctx->plan.off_nprev) + (size_t)layer * c.batch;
  return v;
}

// start/stop (may be null) are attached to the dispatch itself, so their timestamps are the
// kernel's own begin and end
template <int D, int W, bool ATTEND, bool PENDING, bool APPEND>
void launch_partial(const dynts::AttendParams &p, dim3 grid, hipStream_t st, hipEvent_t start, hipEvent_t stop) {
  const bool burst = PENDING && p.score_tiles > 1;  // score writes in bursts: a kernel variant of its own (registers)
  const bool spill = ATTEND && p.spill != nullptr;   // so is the step that keeps its logits
#define DYNTS_LAUNCH(PAGED, BURST, SPILL)                                                                           \
  hipExtLaunchKernelGGL((dynts::attend_kernel<D, W, ATTEND, PENDING, APPEND, PAGED, BURST, SPILL>), grid,            \
                        dim3(W * 64), 0, st, start, stop, 0, p)
#define DYNTS_LAUNCH2(PAGED, BURST)              \
  if (spill) DYNTS_LAUNCH(PAGED, BURST, ATTEND); \
  else DYNTS_LAUNCH(PAGED, BURST, false)
  if (p.block_table) {
    if (burst) { DYNTS_LAUNCH2(true, PENDING); }
    else { DYNTS_LAUNCH2(true, false); }
  } else {
    if (burst) { DYNTS_LAUNCH2(false, PENDING); }
    else { DYNTS_LAUNCH2(false, false); }
  }
#undef DYNTS_LAUNCH2
#undef DYNTS_LAUNCH
}

template <int D, int W>
void launch_partial_d(const dynts::AttendParams &p, dim3 grid, hipStream_t st, hipEvent_t e0, hipEvent_t e1,
                      bool attend, bool pending, bool append) {
  if (!attend) return launch_partial<D, W, false, true, false>(p, grid, st, e0, e1);
  if (pending) {
    if (append) return launch_partial<D, W, true, true, true>(p, grid, st, e0, e1);
    return launch_partial<D, W, true, true, false>(p, grid, st, e0, e1);
  }
  if (append) return launch_partial<D, W, true, false, true>(p, grid, st, e0, e1);
  return launch_partial<D, W, true, false, false>(p, grid, st, e0, e1);
}

// scratch of one attend launch: split partials (tagged words) and ticket counters (zero between launches)
struct Transient {
  uint64_t *part_o, *part_ml;
  uint32_t *unit_cnt, *seq_cnt;
};

// attend (optionally with fused append) and/or the deferred score update of one layer
int run_attend(dynts_ctx *ctx, int layer, const uint16_t *q, const uint16_t *k_new, const uint16_t *v_new,
               const float *s_new, const uint8_t *active, float *out, float *lse, bool attend,
               bool apply_pending, bool append, hipStream_t st, const Transient *transient = nullptr,
               bool keep_logits = false) {
  // transient: where the split partials and the counters of this launch live (default: the head of the
  // workspace); what must survive from one step to the next is always in the workspace
  const dynts_config &c = ctx->cfg;
  const Plan &pl = ctx->plan;
  Transient tr;
  if (transient) {
    tr = *transient;
  } else {
    tr.part_o = reinterpret_cast<uint64_t *>(ctx->ws + pl.off_part_o);
    tr.part_ml = reinterpret_cast<uint64_t *>(ctx->ws + pl.off_part_ml);
    tr.unit_cnt = reinterpret_cast<uint32_t *>(ctx->ws + pl.off_unit_cnt);
    tr.seq_cnt = reinterpret_cast<uint32_t *>(ctx->ws + pl.off_seq_cnt);
  }
  const LayerView lv = layer_view(ctx, layer);
  const bool track = c.score_mode == DYNTS_SCORE_ACCUMULATE;

  dynts::AttendParams p;
  p.K = lv.K; p.V = lv.V; p.S = lv.S; p.pos = lv.pos;
  p.seq_len = lv.seq_len; p.n_prompt = ctx->n_prompt; p.next_pos = lv.next_pos;
  p.q = q; p.k_new = k_new; p.v_new = v_new; p.s_new = s_new; p.active = active;
  p.out = out; p.lse = lse;
  p.qprev = lv.qprev; p.qnext = lv.qnext; p.mlprev = lv.mlprev; p.nprev = lv.nprev;
  p.part_o = tr.part_o;
  p.part_ml = tr.part_ml;
  p.tag = next_launch_tag();
  // score writes: tile by tile while the layer's K and V fit the memory-side cache (256 MB), in bursts beyond
  const double kv_bytes = 4.0 * c.batch * c.n_kv_heads * (double)c.capacity * c.head_dim;
  p.score_tiles = kv_bytes > 192e6 ? 16 : 1;
  p.spill = keep_logits ? reinterpret_cast<float *>(ctx->ws + pl.off_spill) : nullptr;
  p.cap_pad = pl.cap_pad;
  p.unit_cnt = tr.unit_cnt;
  p.seq_cnt = tr.seq_cnt;
  p.status = ctx->status;
  p.Nb = c.batch; p.Hq = c.n_q_heads; p.Hkv = c.n_kv_heads; p.G = pl.G; p.cap = c.capacity;
  p.nsplit = pl.nsplit; p.track = track ? 1 : 0; p.scale_log2 = ctx->scale_log2;
  p.block_table = lv.block_table; p.block_table_w = lv.block_table; p.free_stack = ctx->free_stack;
  p.free_top = ctx->free_top; p.max_pages = ctx->max_pages; p.n_pages = ctx->n_pages;

  // one-dimensional grid: units rounded up to the 8 XCDs, times the chunks per unit (mapped inside the kernel)
  const long long units8 = ((long long)c.batch * c.n_kv_heads + 7) / 8 * 8;
  if (units8 * pl.nsplit > 0x7fffffffLL) return DYNTS_ESHAPE;
  const dim3 grid((unsigned)(units8 * pl.nsplit));
  hipEvent_t e0 = ctx->ev_start, e1 = ctx->ev_stop;
  if (attend && ctx->ev_list_next < ctx->ev_list_start.size()) {
    e0 = ctx->ev_list_start[ctx->ev_list_next];
    e1 = ctx->ev_list_stop[ctx->ev_list_next];
    ++ctx->ev_list_next;
  }
  if (c.head_dim == 128) {
    if (pl.waves == 8) launch_partial_d<128, 8>(p, grid, st, e0, e1, attend, apply_pending, append);
    else launch_partial_d<128, 4>(p, grid, st, e0, e1, attend, apply_pending, append);
  } else {
    if (pl.waves == 8) launch_partial_d<64, 8>(p, grid, st, e0, e1, attend, apply_pending, append);
    else launch_partial_d<64, 4>(p, grid, st, e0, e1, attend, apply_pending, append);
  }
  const int rc = launch_status();
  if (rc == DYNTS_OK && attend && track) ctx->qslot[layer] ^= 1;  // the query just saved becomes the current one
  return rc;
}


// the score update of `layer` from its kept logits (pending == 2)
int apply_spill(dynts_ctx *ctx, int layer, hipStream_t st) {
  const dynts_config &c = ctx->cfg;
  const Plan &pl = ctx->plan;
  const LayerView lv = layer_view(ctx, layer);
  const dim3 grid((c.capacity + 256 * dynts::kApplyPerThread - 1) / (256 * dynts::kApplyPerThread), c.n_kv_heads * c.batch);
  hipLaunchKernelGGL(dynts::apply_spill_kernel, grid, dim3(256), 0, st, lv.S,
                     reinterpret_cast<const float *>(ctx->ws + pl.off_spill), lv.mlprev, lv.nprev, ctx->n_prompt,
                     c.n_kv_heads, c.n_q_heads, pl.G, c.capacity, pl.cap_pad);
  const int rc = launch_status();
  if (rc == DYNTS_OK) {
    ctx->pending[layer] = 0;
    ctx->spill_layer = -1;
  }
  return rc;
}

// One fused step (attention, the score update owed by the previous step, optionally the append) with the
// bookkeeping of owed updates.  With a trigger announced for this layer (dynts_hint_trigger) the step keeps its
// logits, and its own update is later applied from them instead of from a second pass over K.
int fused_step(dynts_ctx *ctx, int layer, const uint16_t *q, const uint16_t *k_new, const uint16_t *v_new,
               const float *s_new, const uint8_t *active, float *out, float *lse, bool append, hipStream_t st,
               const Transient *transient) {
  const bool track = ctx->cfg.score_mode == DYNTS_SCORE_ACCUMULATE;
  const bool keep = track && ctx->hint[layer];
  ctx->hint[layer] = 0;
  int rc = DYNTS_OK;
  if (ctx->pending[layer] == 2) rc = apply_spill(ctx, layer, st);
  if (rc == DYNTS_OK && keep && ctx->spill_layer >= 0) rc = apply_spill(ctx, ctx->spill_layer, st);  // the buffer is reused
  if (rc != DYNTS_OK) return rc;
  rc = run_attend(ctx, layer, q, k_new, v_new, s_new, active, out, lse, true, ctx->pending[layer] == 1, append, st,
                  transient, keep);
  if (rc == DYNTS_OK) {
    ctx->pending[layer] = track ? (keep ? 2 : 1) : 0;
    if (keep) ctx->spill_layer = layer;
  }
  return rc;
}

// ---- Importance Predictor ---------------------------------------------------------------------------
struct MlpPlan {
  int bt;      // batch tiles of 16
  int nsplit;  // workgroups along K (each covers mlp_slice_steps k-steps)
};

MlpPlan mlp_plan(int batch, int K, int parts) {
  MlpPlan pl;
  pl.bt = batch <= 16 ? 1 : batch <= 32 ? 2 : batch <= 64 ? 4 : 8;
  const int slice = dynts::mlp_slice_steps(pl.bt, parts);
  pl.nsplit = (K / 32 + slice - 1) / slice;
  return pl;
}

int check_predictor(const dynts_predictor *w, int batch) {
  if (!w) return DYNTS_ENULL;
  if (batch <= 0 || batch > 128) return DYNTS_EINVAL;
  if (w->d <= 0 || w->m1 <= 0 || w->m2 <= 0) return DYNTS_EINVAL;
  if (w->d % 32 || w->m1 % 32 || w->m2 % 16) return DYNTS_ESHAPE;
  if (w->activation < DYNTS_ACT_NONE || w->activation > DYNTS_ACT_SILU) return DYNTS_EINVAL;
  if (w->packed != 0 && w->packed != 1) return DYNTS_EINVAL;
  return DYNTS_OK;
}

struct MlpScratch {
  size_t off_p1, off_yhi, off_ylo, off_p2, off_part, off_cnt, total;
};

MlpScratch mlp_scratch(const dynts_predictor *w, int batch, const MlpPlan &l1, const MlpPlan &l2) {
  MlpScratch sc;
  size_t off = 0;
  sc.off_p1 = off;
  off += align_up((size_t)l1.nsplit * batch * w->m1 * sizeof(float));
  sc.off_yhi = off;
  off += align_up((size_t)batch * w->m1 * sizeof(uint16_t));
  sc.off_ylo = off;
  off += align_up((size_t)batch * w->m1 * sizeof(uint16_t));
  sc.off_p2 = off;
  off += align_up((size_t)l2.nsplit * batch * w->m2 * sizeof(float));
  sc.off_part = off;
  off += align_up((size_t)batch * ((w->m2 + 255) / 256) * sizeof(uint64_t));  // tagged words
  sc.off_cnt = off;
  off += align_up((size_t)batch * sizeof(uint32_t));
  sc.total = off;
  return sc;
}

template <int PARTS, bool PACKED>
void launch_mlp_gemm(const dynts::MlpGemmParams &p, const MlpPlan &pl, hipStream_t st, hipEvent_t e0, hipEvent_t e1) {
  const dim3 grid((p.m + dynts::kMlpFeaturesPerWg - 1) / dynts::kMlpFeaturesPerWg, pl.nsplit);
  const dim3 block(dynts::kMlpThreads);
  switch (pl.bt) {
    case 1: hipExtLaunchKernelGGL((dynts::mlp_gemm_kernel<1, PARTS, PACKED>), grid, block, 0, st, e0, e1, 0, p); break;
    case 2: hipExtLaunchKernelGGL((dynts::mlp_gemm_kernel<2, PARTS, PACKED>), grid, block, 0, st, e0, e1, 0, p); break;
    case 4: hipExtLaunchKernelGGL((dynts::mlp_gemm_kernel<4, PARTS, PACKED>), grid, block, 0, st, e0, e1, 0, p); break;
    default: hipExtLaunchKernelGGL((dynts::mlp_gemm_kernel<8, PARTS, PACKED>), grid, block, 0, st, e0, e1, 0, p); break;
  }
}

// ---- scratch that nobody allocates (dynts_decode_step_static) ----------------------------------------
// One array per GPU, part of the loaded code object, alive until the process ends.  Host code never uses the
// array's name as an address: it asks the runtime for the device address once per device and keeps it.
constexpr size_t kStaticScratchBytes = DYNTS_STATIC_SCRATCH_BYTES;
constexpr size_t kStaticCounters = size_t(1) << 20;  // the first MiB holds counters only
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

__global__ void static_scratch_clear_kernel(uint32_t *words, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) words[i] = 0u;
}

constexpr int kMaxDevices = 64;
std::mutex static_scratch_mutex;
unsigned char *static_scratch_ptr[kMaxDevices] = {};

// Device address of this GPU's array (the current device), looked up and cleared on first use.  nullptr on error.
unsigned char *static_scratch(hipStream_t st) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(static_scratch_mutex);
  if (!static_scratch_ptr[dev]) {
    unsigned char *ptr = nullptr;
    if (hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    // counters must start at zero (launches leave them at zero afterwards); the whole array, once, with a
    // fill kernel on the caller's stream -- stream order puts it before the first launch that uses the array
    hipLaunchKernelGGL(static_scratch_clear_kernel, dim3(256), dim3(256), 0, st, reinterpret_cast<uint32_t *>(ptr),
                       kStaticScratchBytes / sizeof(uint32_t));
    if (hipGetLastError() != hipSuccess) return nullptr;
    static_scratch_ptr[dev] = ptr;
  }
  return static_scratch_ptr[dev];
}

}  // namespace

extern "C" {

int dynts_version(void) { return 100; }

const char *dynts_strerror(int code) {
  switch (code) {
    case DYNTS_OK: return "ok";
    case DYNTS_EINVAL: return "argument out of range";
    case DYNTS_ENULL: return "required pointer is null";
    case DYNTS_ESHAPE: return "unsupported shape (head_dim must be 64 or 128, group size <= 16, n_q_heads % n_kv_heads == 0)";
    case DYNTS_ECAPACITY: return "capacity or index stride too small";
    case DYNTS_ENOTBOUND: return "no buffers bound (call dynts_bind)";
    case DYNTS_EWORKSPACE: return "workspace too small or misaligned";
    case DYNTS_EHIP: return "HIP runtime error at kernel launch";
    case DYNTS_EPENDING: return "a score update is outstanding (call dynts_update_scores first)";
    default: return "unknown error";
  }
}

int dynts_create(const dynts_config *cfg, dynts_ctx **out) {
  if (!out) return DYNTS_ENULL;
  *out = nullptr;
  int rc = check_config(cfg);
  if (rc != DYNTS_OK) return rc;
  dynts_ctx *ctx = new (std::nothrow) dynts_ctx();
  if (!ctx) return DYNTS_EINVAL;
  ctx->cfg = *cfg;
  ctx->plan = make_plan(*cfg, 0, 0);
  const float scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
  ctx->scale_log2 = scale * 1.4426950408889634f;
  ctx->pending.assign((size_t)cfg->n_layers, 0);
  ctx->hint.assign((size_t)cfg->n_layers, 0);
  ctx->qslot.assign((size_t)cfg->n_layers, 0);
  *out = ctx;
  return DYNTS_OK;
}

int dynts_destroy(dynts_ctx *ctx) {
  if (!ctx) return DYNTS_ENULL;
  delete ctx;
  return DYNTS_OK;
}

int dynts_set_launch_shape(dynts_ctx *ctx, int32_t target_workgroups, int32_t waves_per_workgroup) {
  if (!ctx) return DYNTS_ENULL;
  if (target_workgroups < 0 || (waves_per_workgroup != 0 && waves_per_workgroup != 4 && waves_per_workgroup != 8))
    return DYNTS_EINVAL;
  ctx->plan = make_plan(ctx->cfg, target_workgroups, waves_per_workgroup);
  ctx->bound = false;  // the workspace layout changed
  return DYNTS_OK;
}

size_t dynts_ctx_workspace_bytes(const dynts_ctx *ctx) { return ctx ? ctx->plan.bytes : 0; }

size_t dynts_workspace_bytes(const dynts_config *cfg) {
  if (check_config(cfg) != DYNTS_OK) return 0;
  return make_plan(*cfg, 0, 0).bytes;
}

int dynts_bind(dynts_ctx *ctx, uint16_t *K, uint16_t *V, float *S, int32_t *pos, int32_t *seq_len,
               int32_t *next_pos, int32_t *n_prompt, void *workspace, size_t workspace_bytes, int32_t *status) {
  if (!ctx || !K || !V || !S || !pos || !seq_len || !next_pos || !n_prompt || !workspace || !status) return DYNTS_ENULL;
  if (workspace_bytes < ctx->plan.bytes || (reinterpret_cast<uintptr_t>(workspace) % kAlign)) return DYNTS_EWORKSPACE;
  if ((reinterpret_cast<uintptr_t>(K) | reinterpret_cast<uintptr_t>(V)) % 16) return DYNTS_EINVAL;
  ctx->K = K; ctx->V = V; ctx->S = S; ctx->pos = pos; ctx->seq_len = seq_len; ctx->next_pos = next_pos;
  ctx->n_prompt = n_prompt; ctx->ws = static_cast<unsigned char *>(workspace); ctx->status = status;
  ctx->paged = false; ctx->block_table = nullptr; ctx->free_stack = nullptr; ctx->free_top = nullptr;
  ctx->max_pages = ctx->n_pages = 0;
  ctx->pending.assign(ctx->pending.size(), 0);
  ctx->hint.assign(ctx->hint.size(), 0);
  ctx->spill_layer = -1;
  ctx->qslot.assign(ctx->qslot.size(), 0);
  ctx->bound = true;
  return DYNTS_OK;
}

int dynts_bind_paged(dynts_ctx *ctx, uint16_t *K_pool, uint16_t *V_pool, int32_t n_pages, int32_t *block_table,
                     int32_t max_pages, int32_t *free_stack, int32_t *free_top, float *S, int32_t *pos,
                     int32_t *seq_len, int32_t *next_pos, int32_t *n_prompt, void *workspace, size_t workspace_bytes,
                     int32_t *status) {
  if (!ctx || !block_table || !free_stack || !free_top) return DYNTS_ENULL;
  if (n_pages <= 0 || max_pages <= 0) return DYNTS_EINVAL;
  if ((long long)max_pages * dynts::kPageSlots < ctx->cfg.capacity) return DYNTS_ECAPACITY;
  const int rc = dynts_bind(ctx, K_pool, V_pool, S, pos, seq_len, next_pos, n_prompt, workspace, workspace_bytes, status);
  if (rc != DYNTS_OK) return rc;
  ctx->paged = true; ctx->block_table = block_table; ctx->free_stack = free_stack; ctx->free_top = free_top;
  ctx->max_pages = max_pages; ctx->n_pages = n_pages;
  return DYNTS_OK;
}

int dynts_prefill(dynts_ctx *ctx, int32_t layer, const uint16_t *K0, const uint16_t *V0, int32_t m_max,
                  const int32_t *m, void *stream) {
  int rc = check_call(ctx, layer);
  if (rc != DYNTS_OK) return rc;
  if (!K0 || !V0 || !m) return DYNTS_ENULL;
  if (m_max <= 0) return DYNTS_EINVAL;
  if (m_max > ctx->cfg.capacity) return DYNTS_ECAPACITY;
  if ((reinterpret_cast<uintptr_t>(K0) | reinterpret_cast<uintptr_t>(V0)) % 16) return DYNTS_EINVAL;
  const dynts_config &c = ctx->cfg;
  const LayerView lv = layer_view(ctx, layer);
  dynts::PrefillParams p{lv.K, lv.V, lv.S, lv.pos, lv.seq_len, lv.next_pos, ctx->n_prompt, K0, V0, m,
                         c.n_kv_heads, c.capacity, m_max};
  const int rows = 256 / (c.head_dim / 8);
  const dim3 grid((m_max + rows - 1) / rows, c.n_kv_heads, c.batch);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (ctx->paged) {
    const dynts::PagedView pv{lv.K, lv.V, lv.block_table, ctx->free_stack, ctx->free_top, ctx->max_pages, ctx->n_pages};
    const int units = c.batch * c.n_kv_heads;
    hipLaunchKernelGGL(dynts::paged_alloc_kernel, dim3((units + 63) / 64), dim3(64), 0, st, pv, nullptr, m, m_max,
                       c.batch, c.n_kv_heads, ctx->status);
    if (c.head_dim == 128) hipLaunchKernelGGL((dynts::paged_prefill_kernel<128>), grid, dim3(256), 0, st, p, pv);
    else hipLaunchKernelGGL((dynts::paged_prefill_kernel<64>), grid, dim3(256), 0, st, p, pv);
  } else if (c.head_dim == 128) {
    hipLaunchKernelGGL((dynts::prefill_kernel<128>), grid, dim3(256), 0, st, p);
  } else {
    hipLaunchKernelGGL((dynts::prefill_kernel<64>), grid, dim3(256), 0, st, p);
  }
  ctx->pending[layer] = 0;
  if (ctx->spill_layer == layer) ctx->spill_layer = -1;
  return launch_status();
}

int dynts_append(dynts_ctx *ctx, int32_t layer, const uint16_t *k_new, const uint16_t *v_new, const float *s_new,
                 const uint8_t *active, void *stream) {
  int rc = check_call(ctx, layer);
  if (rc != DYNTS_OK) return rc;
  if (!k_new || !v_new) return DYNTS_ENULL;
  const dynts_config &c = ctx->cfg;
  if (c.score_mode == DYNTS_SCORE_EXTERNAL && !s_new) return DYNTS_ENULL;
  if ((reinterpret_cast<uintptr_t>(k_new) | reinterpret_cast<uintptr_t>(v_new)) % 16) return DYNTS_EINVAL;
  const LayerView lv = layer_view(ctx, layer);
  dynts::AppendParams p{lv.K, lv.V, lv.S, lv.pos, lv.seq_len, lv.next_pos, k_new, v_new,
                        c.score_mode == DYNTS_SCORE_EXTERNAL ? s_new : nullptr, active, ctx->status,
                        c.n_kv_heads, c.capacity};
  const int threads = (c.n_kv_heads * (c.head_dim / 8) + 63) / 64 * 64;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (ctx->paged) {
    const dynts::PagedView pv{lv.K, lv.V, lv.block_table, ctx->free_stack, ctx->free_top, ctx->max_pages, ctx->n_pages};
    if (c.head_dim == 128) hipLaunchKernelGGL((dynts::paged_append_kernel<128>), dim3(c.batch), dim3(threads), 0, st, p, pv);
    else hipLaunchKernelGGL((dynts::paged_append_kernel<64>), dim3(c.batch), dim3(threads), 0, st, p, pv);
  } else if (c.head_dim == 128) {
    hipLaunchKernelGGL((dynts::append_kernel<128>), dim3(c.batch), dim3(threads), 0, st, p);
  } else {
    hipLaunchKernelGGL((dynts::append_kernel<64>), dim3(c.batch), dim3(threads), 0, st, p);
  }
  return launch_status();
}

int dynts_decode_attend(dynts_ctx *ctx, int32_t layer, const uint16_t *q, const uint8_t *active, float *out,
                        float *lse, void *stream) {
  int rc = check_call(ctx, layer);
  if (rc != DYNTS_OK) return rc;
  if (!q || !out) return DYNTS_ENULL;
  if (reinterpret_cast<uintptr_t>(q) % 16) return DYNTS_EINVAL;
  if (ctx->pending[layer] == 2) {  // kept logits would lose their statistics to this call: apply them first
    rc = apply_spill(ctx, layer, static_cast<hipStream_t>(stream));
    if (rc != DYNTS_OK) return rc;
  }
  rc = run_attend(ctx, layer, q, nullptr, nullptr, nullptr, active, out, lse, true, false, false,
                  static_cast<hipStream_t>(stream));
  if (rc == DYNTS_OK) ctx->pending[layer] = ctx->cfg.score_mode == DYNTS_SCORE_ACCUMULATE;
  return rc;
}

int dynts_update_scores(dynts_ctx *ctx, int32_t layer, void *stream) {
  int rc = check_call(ctx, layer);
  if (rc != DYNTS_OK) return rc;
  if (!ctx->pending[layer]) return DYNTS_OK;
  if (ctx->pending[layer] == 2) return apply_spill(ctx, layer, static_cast<hipStream_t>(stream));
  rc = run_attend(ctx, layer, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, false, true, false,
                  static_cast<hipStream_t>(stream));
  if (rc == DYNTS_OK) ctx->pending[layer] = 0;
  return rc;
}

int dynts_decode_attend_update(dynts_ctx *ctx, int32_t layer, const uint16_t *q, const uint8_t *active,
                               float *out, float *lse, void *stream) {
  int rc = check_call(ctx, layer);
  if (rc != DYNTS_OK) return rc;
  if (!q || !out) return DYNTS_ENULL;
  if (reinterpret_cast<uintptr_t>(q) % 16) return DYNTS_EINVAL;
  return fused_step(ctx, layer, q, nullptr, nullptr, nullptr, active, out, lse, false, static_cast<hipStream_t>(stream),
                    nullptr);
}

int dynts_decode_step(dynts_ctx *ctx, int32_t layer, const uint16_t *q, const uint16_t *k_new,
                      const uint16_t *v_new, const float *s_new, const uint8_t *active, float *out, float *lse,
                      void *stream) {
  int rc = check_call(ctx, layer);
  if (rc != DYNTS_OK) return rc;
  if (!q || !out || !k_new || !v_new) return DYNTS_ENULL;
  const bool ext = ctx->cfg.score_mode == DYNTS_SCORE_EXTERNAL;
  if (ext && !s_new) return DYNTS_ENULL;
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_new) | reinterpret_cast<uintptr_t>(v_new)) % 16)
    return DYNTS_EINVAL;
  return fused_step(ctx, layer, q, k_new, v_new, ext ? s_new : nullptr, active, out, lse, true,
                    static_cast<hipStream_t>(stream), nullptr);
}

int dynts_decode_step_static(dynts_ctx *ctx, int32_t layer, const uint16_t *q, const uint16_t *k_new,
                             const uint16_t *v_new, const float *s_new, const uint8_t *active, float *out, float *lse,
                             void *stream) {
  int rc = check_call(ctx, layer);
  if (rc != DYNTS_OK) return rc;
  if (!q || !out || !k_new || !v_new) return DYNTS_ENULL;
  const bool ext = ctx->cfg.score_mode == DYNTS_SCORE_EXTERNAL;
  if (ext && !s_new) return DYNTS_ENULL;
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_new) | reinterpret_cast<uintptr_t>(v_new)) % 16)
    return DYNTS_EINVAL;
  // Layout of the static array, the same for every context so that what one call leaves fits the next:
  //   [0, 512 KiB)      ticket counters of the (sequence, KV head) units -- every launch leaves them at zero
  //   [512 KiB, 1 MiB)  check-in counters of the sequences               -- likewise
  //   [1 MiB, 8 MiB)    split partials: tagged words, a stale one is recognised whoever wrote it
  const dynts_config &c = ctx->cfg;
  const Plan &pl = ctx->plan;
  const size_t units = (size_t)c.batch * c.n_kv_heads, rows = units * pl.nsplit * pl.G;
  const size_t part_o_bytes = align_up(rows * c.head_dim * sizeof(uint64_t)), part_ml_bytes = rows * 2 * sizeof(uint64_t);
  if (units * sizeof(uint32_t) > kStaticCounters / 2 || (size_t)c.batch * sizeof(uint32_t) > kStaticCounters / 2 ||
      part_o_bytes + part_ml_bytes > kStaticScratchBytes - kStaticCounters)
    return DYNTS_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  unsigned char *base = static_scratch(st);
  if (!base) return DYNTS_EHIP;
  Transient tr;
  tr.unit_cnt = reinterpret_cast<uint32_t *>(base);
  tr.seq_cnt = reinterpret_cast<uint32_t *>(base + kStaticCounters / 2);
  tr.part_o = reinterpret_cast<uint64_t *>(base + kStaticCounters);
  tr.part_ml = reinterpret_cast<uint64_t *>(base + kStaticCounters + part_o_bytes);
  return fused_step(ctx, layer, q, k_new, v_new, ext ? s_new : nullptr, active, out, lse, true, st, &tr);
}

int dynts_hint_trigger(dynts_ctx *ctx, int32_t layer) {
  const int rc = check_call(ctx, layer);
  if (rc != DYNTS_OK) return rc;
  ctx->hint[layer] = 1;
  return DYNTS_OK;
}

int dynts_select_evict(dynts_ctx *ctx, int32_t layer, const uint8_t *trigger, int32_t k_keep, int32_t *keep_idx,
                       int32_t keep_stride, int32_t *new_len, void *stream) {
  int rc = check_call(ctx, layer);
  if (rc != DYNTS_OK) return rc;
  if (!keep_idx || !new_len) return DYNTS_ENULL;
  if (keep_stride <= 0) return DYNTS_ECAPACITY;
  const dynts_config &c = ctx->cfg;
  if (k_keep < 0) k_keep = c.budget;
  rc = dynts_update_scores(ctx, layer, stream);
  if (rc != DYNTS_OK) return rc;
  const LayerView lv = layer_view(ctx, layer);
  dynts::SelectParams p{lv.S, lv.seq_len, ctx->n_prompt, trigger, keep_idx, new_len, ctx->status,
                        c.n_kv_heads, c.capacity, c.window, k_keep, keep_stride};
  const dim3 grid(c.n_kv_heads, c.batch);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (c.capacity <= kSelectLdsMax)
    hipLaunchKernelGGL((dynts::select_kernel<true>), grid, dim3(dynts::kSelThreads), (size_t)c.capacity * 4, st, p);
  else
    hipLaunchKernelGGL((dynts::select_kernel<false>), grid, dim3(dynts::kSelThreads), 0, st, p);
  return launch_status();
}

int dynts_compact(dynts_ctx *ctx, int32_t layer, const uint8_t *trigger, const int32_t *keep_idx,
                  int32_t keep_stride, const int32_t *new_len, void *stream) {
  int rc = check_call(ctx, layer);
  if (rc != DYNTS_OK) return rc;
  if (!keep_idx || !new_len) return DYNTS_ENULL;
  if (keep_stride <= 0) return DYNTS_ECAPACITY;
  if (ctx->pending[layer]) return DYNTS_EPENDING;
  const dynts_config &c = ctx->cfg;
  const LayerView lv = layer_view(ctx, layer);
  dynts::CompactParams p{lv.K, lv.V, lv.S, lv.pos, lv.seq_len, trigger, keep_idx, new_len,
                         c.n_kv_heads, c.capacity, keep_stride};
  const dim3 grid(2 * (c.head_dim * 2 / dynts::kCompactSliceBytes) + 2, c.n_kv_heads, c.batch);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (ctx->paged) {
    const dynts::PagedView pv{lv.K, lv.V, lv.block_table, ctx->free_stack, ctx->free_top, ctx->max_pages, ctx->n_pages};
    if (c.head_dim == 128) hipLaunchKernelGGL((dynts::paged_compact_kernel<128>), grid, dim3(dynts::kCompactThreads), 0, st, p, pv);
    else hipLaunchKernelGGL((dynts::paged_compact_kernel<64>), grid, dim3(dynts::kCompactThreads), 0, st, p, pv);
    hipLaunchKernelGGL(dynts::paged_trim_kernel, dim3((c.batch + 63) / 64), dim3(64), 0, st, pv, trigger, new_len,
                       lv.seq_len, c.batch, c.n_kv_heads, c.capacity, keep_stride);
  } else if (c.head_dim == 128) {
    hipLaunchKernelGGL((dynts::compact_kernel<128>), grid, dim3(dynts::kCompactThreads), 0, st, p);
  } else {
    hipLaunchKernelGGL((dynts::compact_kernel<64>), grid, dim3(dynts::kCompactThreads), 0, st, p);
  }
  return launch_status();
}

int dynts_set_kernel_events(dynts_ctx *ctx, void *start, void *stop) {
  if (!ctx) return DYNTS_ENULL;
  if ((start == nullptr) != (stop == nullptr)) return DYNTS_EINVAL;
  ctx->ev_start = static_cast<hipEvent_t>(start);
  ctx->ev_stop = static_cast<hipEvent_t>(stop);
  return DYNTS_OK;
}

int dynts_set_kernel_event_list(dynts_ctx *ctx, void *const *starts, void *const *stops, int32_t n) {
  if (!ctx) return DYNTS_ENULL;
  if (n < 0) return DYNTS_EINVAL;
  if (n > 0 && (!starts || !stops)) return DYNTS_ENULL;
  ctx->ev_list_start.clear();
  ctx->ev_list_stop.clear();
  ctx->ev_list_next = 0;
  for (int i = 0; i < n; ++i) {
    if (!starts[i] || !stops[i]) return DYNTS_ENULL;
    ctx->ev_list_start.push_back(static_cast<hipEvent_t>(starts[i]));
    ctx->ev_list_stop.push_back(static_cast<hipEvent_t>(stops[i]));
  }
  return DYNTS_OK;
}

size_t dynts_score_block_scratch_bytes(const dynts_config *cfg, int32_t n_queries) {
  if (!cfg || check_config(cfg) != DYNTS_OK || n_queries <= 0 || n_queries > (1 << 20)) return 0;
  const size_t rpad = align_up((size_t)n_queries * (cfg->n_q_heads / cfg->n_kv_heads));
  return align_up((size_t)cfg->batch * cfg->n_kv_heads * rpad * sizeof(float));
}

int dynts_score_block(dynts_ctx *ctx, int32_t layer, const uint16_t *q_blk, const uint16_t *k_blk,
                      int32_t n_queries, const uint8_t *active, float *dst, int32_t accumulate, void *scratch,
                      size_t scratch_bytes, void *stream) {
  int rc = check_call(ctx, layer);
  if (rc != DYNTS_OK) return rc;
  if (!q_blk || !scratch) return DYNTS_ENULL;
  if (n_queries <= 0 || n_queries > (1 << 20)) return DYNTS_EINVAL;
  if (reinterpret_cast<uintptr_t>(q_blk) % 16 || reinterpret_cast<uintptr_t>(k_blk) % 16) return DYNTS_EINVAL;
  const dynts_config &c = ctx->cfg;
  const size_t need = dynts_score_block_scratch_bytes(&c, n_queries);
  if (scratch_bytes < need || reinterpret_cast<uintptr_t>(scratch) % 4) return DYNTS_EWORKSPACE;
  const LayerView lv = layer_view(ctx, layer);
  const int G = c.n_q_heads / c.n_kv_heads;
  dynts::ScoreBlockParams p{};
  p.K = lv.K;
  p.q_blk = q_blk;
  p.k_blk = k_blk;
  p.seq_len = lv.seq_len;
  p.n_prompt = ctx->n_prompt;
  p.active = active;
  p.stats = static_cast<float *>(scratch);
  p.dst = dst ? dst : lv.S;
  p.Nb = c.batch;
  p.T = n_queries;
  p.Hq = c.n_q_heads;
  p.Hkv = c.n_kv_heads;
  p.G = G;
  p.cap = c.capacity;
  p.Rpad = (int)align_up((size_t)n_queries * G);
  p.skip_prompt = dst ? 0 : 1;
  p.accumulate = accumulate ? 1 : 0;
  p.scale_log2 = ctx->scale_log2;
  p.block_table = lv.block_table; p.max_pages = ctx->max_pages; p.n_pages = ctx->n_pages;
  const long long R = (long long)n_queries * G;
  // (1-D grids: blocks per unit x units rounded up to the 8 XCDs, mapped inside the kernels)
  const long long units8 = ((long long)c.batch * c.n_kv_heads + 7) / 8 * 8;
  const long long b1 = (R + dynts::kSbRowsPerWg - 1) / dynts::kSbRowsPerWg;
  const long long b2 = (c.capacity + dynts::kSbRowsPerWg - 1) / dynts::kSbRowsPerWg;
  if (b1 * units8 > 0x7fffffffLL || b2 * units8 > 0x7fffffffLL) return DYNTS_EINVAL;
  if ((long long)n_queries * c.n_q_heads * c.head_dim * 2 > 0x7fffffffLL) return DYNTS_EINVAL;  // 32-bit row offsets
  const dim3 g1((unsigned)(b1 * units8)), g2((unsigned)(b2 * units8));
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (c.head_dim == 128) {
    hipLaunchKernelGGL(dynts::score_block_stats_kernel<128>, g1, dim3(dynts::kSbWaves * 64), 0, st, p);
    hipLaunchKernelGGL(dynts::score_block_colsum_kernel<128>, g2, dim3(dynts::kSbWaves * 64), 0, st, p);
  } else {
    hipLaunchKernelGGL(dynts::score_block_stats_kernel<64>, g1, dim3(dynts::kSbWaves * 64), 0, st, p);
    hipLaunchKernelGGL(dynts::score_block_colsum_kernel<64>, g2, dim3(dynts::kSbWaves * 64), 0, st, p);
  }
  return launch_status();
}

int dynts_predictor_pack(const uint16_t *W, int32_t m, int32_t K, uint16_t *W_packed, void *stream) {
  if (!W || !W_packed) return DYNTS_ENULL;
  if (m <= 0 || K <= 0) return DYNTS_EINVAL;
  if (m % 16 || K % 32) return DYNTS_ESHAPE;
  if (reinterpret_cast<uintptr_t>(W) % 16 || reinterpret_cast<uintptr_t>(W_packed) % 16 || W == W_packed) return DYNTS_EINVAL;
  const size_t pieces = (size_t)m * K / 8;
  hipLaunchKernelGGL(dynts::mlp_pack_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), W, m, K, W_packed);
  return launch_status();
}

size_t dynts_predict_scratch_bytes(const dynts_predictor *w, int32_t batch) {
  if (check_predictor(w, batch) != DYNTS_OK) return 0;
  const MlpPlan l1 = mlp_plan(batch, w->d, 1), l2 = mlp_plan(batch, w->m1, 2);
  return mlp_scratch(w, batch, l1, l2).total;
}

int dynts_predict_scores(const dynts_predictor *w, const uint16_t *h, int32_t batch, float *s_out, int32_t n_rep,
                         void *scratch, size_t scratch_bytes, void *start, void *stop, void *stream) {
  int rc = check_predictor(w, batch);
  if (rc != DYNTS_OK) return rc;
  if (!h || !s_out || !scratch || !w->W1 || !w->W2 || !w->w3) return DYNTS_ENULL;
  if (n_rep <= 0 || n_rep > 256) return DYNTS_EINVAL;
  if ((start == nullptr) != (stop == nullptr)) return DYNTS_EINVAL;
  if (reinterpret_cast<uintptr_t>(h) % 16 || reinterpret_cast<uintptr_t>(w->W1) % 16 ||
      reinterpret_cast<uintptr_t>(w->W2) % 16)
    return DYNTS_EINVAL;
  const MlpPlan l1 = mlp_plan(batch, w->d, 1), l2 = mlp_plan(batch, w->m1, 2);
  const MlpScratch sc = mlp_scratch(w, batch, l1, l2);
  if (scratch_bytes < sc.total || reinterpret_cast<uintptr_t>(scratch) % kAlign) return DYNTS_EWORKSPACE;
  unsigned char *base = static_cast<unsigned char *>(scratch);
  float *P1 = reinterpret_cast<float *>(base + sc.off_p1), *P2 = reinterpret_cast<float *>(base + sc.off_p2);
  uint16_t *yhi = reinterpret_cast<uint16_t *>(base + sc.off_yhi), *ylo = reinterpret_cast<uint16_t *>(base + sc.off_ylo);
  hipStream_t st = static_cast<hipStream_t>(stream);
  // the optional events bracket the whole call: start on the first kernel, stop on the last
  dynts::MlpGemmParams g1{w->W1, h, nullptr, P1, batch, w->m1, w->d};
  if (w->packed) launch_mlp_gemm<1, true>(g1, l1, st, static_cast<hipEvent_t>(start), nullptr);
  else launch_mlp_gemm<1, false>(g1, l1, st, static_cast<hipEvent_t>(start), nullptr);
  const size_t n1 = (size_t)batch * w->m1 / 4;
  hipLaunchKernelGGL(dynts::mlp_reduce_act_kernel, dim3((unsigned)((n1 + 255) / 256)), dim3(256), 0, st, P1, w->b1,
                     l1.nsplit, batch, w->m1, w->activation, yhi, ylo, reinterpret_cast<uint32_t *>(base + sc.off_cnt));
  dynts::MlpGemmParams g2{w->W2, yhi, ylo, P2, batch, w->m2, w->m1};
  if (w->packed) launch_mlp_gemm<2, true>(g2, l2, st, nullptr, nullptr);
  else launch_mlp_gemm<2, false>(g2, l2, st, nullptr, nullptr);
  hipExtLaunchKernelGGL(dynts::mlp_reduce_dot_kernel, dim3((w->m2 + 255) / 256, batch), dim3(256), 0, st, nullptr,
                        static_cast<hipEvent_t>(stop), 0, P2, w->b2, l2.nsplit, batch, w->m2, w->activation, w->w3,
                        w->b3, reinterpret_cast<uint64_t *>(base + sc.off_part), next_launch_tag(),
                        reinterpret_cast<uint32_t *>(base + sc.off_cnt), s_out, n_rep);
  return launch_status();
}

int dynts_probe_read_stream(const void *buf, size_t bytes, int32_t n_workgroups, uint32_t magic, uint32_t *sink,
                            void *start, void *stop, void *stream) {
  if (!buf || !sink) return DYNTS_ENULL;
  if (bytes == 0 || bytes % 16 != 0 || n_workgroups <= 0 || n_workgroups > (1 << 20)) return DYNTS_EINVAL;
  if ((reinterpret_cast<uintptr_t>(buf) & 15) != 0) return DYNTS_EINVAL;
  if ((start == nullptr) != (stop == nullptr)) return DYNTS_EINVAL;
  hipExtLaunchKernelGGL(dynts::read_stream_kernel, dim3(n_workgroups), dim3(dynts::kProbeThreads), 0,
                        static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(start),
                        static_cast<hipEvent_t>(stop), 0, static_cast<const uint32_t *>(buf), bytes / 16, magic, sink);
  return launch_status();
}

int dynts_probe_exp_rate(int32_t n_workgroups, int32_t iters, float *sink, void *start, void *stop, void *stream) {
  if (!sink) return DYNTS_ENULL;
  if (n_workgroups <= 0 || n_workgroups > (1 << 20) || iters <= 0) return DYNTS_EINVAL;
  if ((start == nullptr) != (stop == nullptr)) return DYNTS_EINVAL;
  hipExtLaunchKernelGGL(dynts::exp2_rate_kernel, dim3(n_workgroups), dim3(dynts::kProbeThreads), 0,
                        static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(start),
                        static_cast<hipEvent_t>(stop), 0, iters, -12345.678f, sink);
  return launch_status();
}

int dynts_probe_issue_mix(int32_t n_workgroups, int32_t iters, int32_t what, float *sink, void *start, void *stop,
                          void *stream) {
  if (!sink) return DYNTS_ENULL;
  if (n_workgroups <= 0 || n_workgroups > (1 << 20) || iters <= 0 || what < 1 || what > 3) return DYNTS_EINVAL;
  if ((start == nullptr) != (stop == nullptr)) return DYNTS_EINVAL;
  const dim3 grid(n_workgroups), block(dynts::kProbeThreads);
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipEvent_t e0 = static_cast<hipEvent_t>(start), e1 = static_cast<hipEvent_t>(stop);
  const float c = 0.1f, L = -3.f, magic = -12345.678f;
  if (what == 1) hipExtLaunchKernelGGL(dynts::issue_mix_kernel<1>, grid, block, 0, st, e0, e1, 0, iters, c, L, magic, sink);
  else if (what == 2) hipExtLaunchKernelGGL(dynts::issue_mix_kernel<2>, grid, block, 0, st, e0, e1, 0, iters, c, L, magic, sink);
  else hipExtLaunchKernelGGL(dynts::issue_mix_kernel<3>, grid, block, 0, st, e0, e1, 0, iters, c, L, magic, sink);
  return launch_status();
}

int dynts_decode_loop(dynts_ctx *ctx, int32_t n_steps, const uint16_t *q, const uint16_t *k_new,
                      const uint16_t *v_new, const float *s_new, const uint8_t *active, const uint8_t *evict_steps,
                      const uint8_t *trigger, float *out, size_t out_step_stride, int32_t *keep_idx,
                      int32_t *new_len, void *stream) {
  int rc = check_call(ctx, 0);
  if (rc != DYNTS_OK) return rc;
  if (n_steps < 0) return DYNTS_EINVAL;
  if (!q || !k_new || !v_new || !out) return DYNTS_ENULL;
  const dynts_config &c = ctx->cfg;
  const bool ext = c.score_mode == DYNTS_SCORE_EXTERNAL;
  if (ext && !s_new) return DYNTS_ENULL;
  if (evict_steps && (!keep_idx || !new_len)) return DYNTS_ENULL;
  const size_t q_layer = (size_t)c.batch * c.n_q_heads * c.head_dim;
  const size_t kv_layer = (size_t)c.batch * c.n_kv_heads * c.head_dim;
  for (int i = 0; i < n_steps; ++i) {
    const uint8_t *act = active ? active + (size_t)i * c.batch : nullptr;
    const float *sn = ext ? s_new + (size_t)i * c.batch * c.n_kv_heads : nullptr;
    for (int l = 0; l < c.n_layers; ++l) {
      const size_t sl = (size_t)i * c.n_layers + l;
      if (evict_steps && evict_steps[i]) ctx->hint[l] = 1;  // the trigger below follows this step
      rc = dynts_decode_step(ctx, l, q + sl * q_layer, k_new + sl * kv_layer, v_new + sl * kv_layer, sn, act,
                             out + (size_t)i * out_step_stride + (size_t)l * q_layer, nullptr, stream);
      if (rc != DYNTS_OK) return rc;
      if (evict_steps && evict_steps[i]) {
        const uint8_t *trig = trigger ? trigger + (size_t)i * c.batch : nullptr;
        rc = dynts_select_evict(ctx, l, trig, c.budget, keep_idx, c.capacity, new_len, stream);
        if (rc != DYNTS_OK) return rc;
        rc = dynts_compact(ctx, l, trig, keep_idx, c.capacity, new_len, stream);
        if (rc != DYNTS_OK) return rc;
      }
    }
  }
  return DYNTS_OK;
}

}  // extern "C"
