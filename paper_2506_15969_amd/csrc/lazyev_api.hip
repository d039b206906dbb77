// Host side of the C ABI declared in include/lazyev.h: argument checks, the host mirror of
// each layer's cache length (it evolves deterministically: +1 per decode step, back to B at an
// eviction, so no device read-back is ever needed), workspace carve-up and kernel launches.
#include "lazyev.h"
#include "lazyev_bench.h"

#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "kernels.h"

namespace lazyev {
int decode_chunk_max();
int decode_split_max();
int decode_slice_max();
}  // namespace lazyev

using lazyev::Workspace;

// Gather list of lazyev_evict_static: the library's own device memory, one copy per GPU, held
// until the process ends.  In host code the name is only a handle for hipGetSymbolAddress; the
// address a kernel can use is looked up once per device (static_scratch_of below).
constexpr size_t kStaticScratchEntries = LAZYEV_STATIC_SCRATCH_ENTRIES;
static __device__ __align__(256) int32_t scratch[kStaticScratchEntries];

struct lazyev_ctx {
  lazyev_config cfg;
  int32_t capacity, group, units;
  int32_t chunk, n_split_max, variant, target_blocks;
  bool target_blocks_set;                          // by the caller: then taken literally
  float scale;
  hipStream_t stream;
  Workspace ws;
  std::vector<int32_t> len, last_step;
  std::vector<int64_t> n_evict_events, n_evicted;
  int last_hip_error;
  int device;                       // the device that was current at lazyev_init
  int32_t *static_scratch;          // that device's copy of `scratch` (see static_scratch_of)
  uint32_t launch_seq;              // fused kernel: launches so far (the stamp of handed-over partials)
  uint32_t spin_ticks;              // fused kernel: longest wait for such a partial, 10 ns ticks
  // fused kernel: the call whose tracking has not been applied yet, and the buffer pair in turn
  lazyev::TrackArgs pend;
  int32_t pend_layer;               // the layer of that call
  int cur_buf;
  // activation log (see TrackArgs::bitlog): per layer, the calls whose tracking has been left as
  // one bit per cache entry and not yet applied to TS / MRI; null when the shape has no log
  uint32_t *bitlog;
  int32_t log_words, log_slots;
  std::vector<int32_t> log_n;       // per layer: logged calls
  std::vector<int32_t> log_t;       // [layer][log_slots]: their steps
  std::vector<int32_t> log_n_old;   // [layer][log_slots]: the entries they appended
  // the last decode call, if the fused kernel ran it: its logits and statistics are still in
  // the workspace (what an eviction that ranks by that step's weights reads)
  int32_t last_layer;
  const float *last_logits, *last_stat;
  int32_t last_p_stride;
  float *prefill_stat;              // workspace of lazyev_prefill_track
  // per-sequence timing (lazyev_admit / lazyev_retire): prompt length (-1: empty slot) and the
  // global step before each sequence's first one; device copies in the workspace.  Off until
  // the first admit or retire: until then every sequence has the configuration's prompt, t0 = 0.
  bool slots_on;
  std::vector<int32_t> slot_prompt, slot_t0;
  int32_t *dev_slot_prompt, *dev_slot_t0, *dev_seq_len;
  std::vector<int32_t> evict_applied;              // per layer: last step whose due eviction ran
  // profiling aid: event triples of the calls that were armed, kind 0 = decode, 1 = evict
  int32_t prof_armed;
  struct Timed { int kind; hipEvent_t ev[3]; };
  std::vector<Timed> prof;
};

namespace {

constexpr int kMinChunk = 64;
constexpr int kTile = 32;            // finest split granularity the partial arrays are sized for
constexpr size_t kAlign = 256;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

bool config_ok(const lazyev_config *c) {
  if (!c) return false;
  if (c->n_layers < 1 || c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1) return false;
  if (c->n_q_heads % c->n_kv_heads != 0) return false;
  const int g = c->n_q_heads / c->n_kv_heads;
  if (g < 1 || g > 8) return false;
  if (c->head_dim != 64 && c->head_dim != 128) return false;
  if (c->window < 1 || c->budget <= c->window || c->prompt_len < 0) return false;
  if (c->dtype != LAZYEV_DTYPE_FP32 && c->dtype != LAZYEV_DTYPE_BF16) return false;
  if (c->score_flags & ~(LAZYEV_SCORE_H1 | LAZYEV_SCORE_H2 | LAZYEV_SCORE_H2_DECREASING |
                         LAZYEV_SCORE_CURRENT_ATTENTION))
    return false;
  if ((c->score_flags & LAZYEV_SCORE_CURRENT_ATTENTION) &&
      (c->dtype != LAZYEV_DTYPE_BF16 || c->head_dim != 128))
    return false;
  if (!(c->alpha >= 0.0f) || !(c->softmax_scale >= 0.0f)) return false;   // also rejects NaN
  const long long cap = static_cast<long long>(c->prompt_len > c->budget ? c->prompt_len : c->budget) + c->window;
  if (cap > (1ll << 20)) return false;
  if (static_cast<long long>(c->batch) * c->n_kv_heads > 65535) return false;   // grid.y / grid.z
  return true;
}

int32_t capacity_of(const lazyev_config *c) {
  return (c->prompt_len > c->budget ? c->prompt_len : c->budget) + c->window;
}

// Entries per unit in a logits buffer of the fused kernel: the capacity in whole sub-tiles plus
// the slack its per-block regions of candidate records need (65 slots for each of up to 64 blocks).
size_t fused_p_stride(int32_t capacity) { return static_cast<size_t>((capacity + 15) / 16 * 16) + 65 * 64; }

struct Layout {
  size_t part_acc, part_ml, p_tilde, logits1, stat, prefill_stat, src_index, sel_keys, bitlog, activations, rows_moved, ticket, records, fault, hist, slots, total;
  int32_t log_words, log_slots;     // 0: no activation log for this shape
  int32_t n_split_max;
};

Layout layout_of(const lazyev_config *c) {
  Layout l;
  const size_t cap = capacity_of(c);
  const size_t units = static_cast<size_t>(c->batch) * c->n_kv_heads;
  const size_t g = c->n_q_heads / c->n_kv_heads;
  l.n_split_max = static_cast<int32_t>((cap + kTile - 1) / kTile);
  size_t off = 0;
  l.part_acc = off; off = align_up(off + units * l.n_split_max * g * c->head_dim * sizeof(float));
  l.part_ml = off;  off = align_up(off + units * l.n_split_max * 2 * g * sizeof(float));
  // two logits buffers of [units][fused_p_stride][8] floats; the split + merge kernels use the
  // first as [batch][n_q_heads][C16]
  const size_t logits_bytes = units * fused_p_stride(static_cast<int32_t>(cap)) * 8 * sizeof(float);
  l.p_tilde = off;  off = align_up(off + logits_bytes);
  l.logits1 = off;  off = align_up(off + logits_bytes);
  l.stat = off;     off = align_up(off + 2 * units * 16 * sizeof(float));
  // softmax statistics of every (unit, head, prompt position) for the tracking over the prompt
  l.prefill_stat = off;                            // (the longest prompt a slot can hold: capacity - window)
  off = align_up(off + units * 8 * ((cap - c->window + 15) / 16 * 16) * sizeof(float));
  l.src_index = off; off = align_up(off + static_cast<size_t>(c->n_layers) * units * cap * sizeof(int32_t));   // (all layers may be evicted in one go)
  // score keys of the selection, only if an eviction can have more candidates than LDS holds
  l.sel_keys = off;
  if (cap - c->window > static_cast<size_t>(lazyev::evict_lds_candidates()))
    off = align_up(off + static_cast<size_t>(c->n_layers) * units * cap * sizeof(unsigned long long));
  // activation log of the single-launch kernel: [layer][unit][slot][one bit per cache entry], as
  // many slots as calls lie between two evictions (at most kLogSlotsMax; a full log is applied)
  l.bitlog = off;
  l.log_words = 0; l.log_slots = 0;
  if (c->dtype == LAZYEV_DTYPE_BF16 && c->head_dim == 128 &&
      (cap + 31) / 32 <= static_cast<size_t>(lazyev::decode_fused_log_words_max())) {
    l.log_words = static_cast<int32_t>((cap + 31) / 32);
    l.log_slots = c->window < lazyev::kLogSlotsMax ? c->window : lazyev::kLogSlotsMax;
    off = align_up(off + static_cast<size_t>(c->n_layers) * l.log_slots * units * l.log_words * sizeof(uint32_t));
  }
  l.activations = off; off = align_up(off + static_cast<size_t>(c->n_layers) * units * lazyev::decode_slice_max() * sizeof(unsigned long long));
  l.rows_moved = off; off = align_up(off + static_cast<size_t>(c->n_layers) * units * sizeof(unsigned long long));
  l.ticket = off; off = align_up(off + units * sizeof(int32_t));
  // fused kernel, units of 2..4 blocks: three stamped records of partials per unit (zero at first:
  // no launch has the number 0), and the word a block raises when it gives up waiting for one
  l.records = off; off = align_up(off + units * 3 * lazyev::decode_fused_record_bytes());
  l.fault = off; off = align_up(off + sizeof(int32_t));
  l.hist = off; off = align_up(off + LAZYEV_MAX_HIST_BINS * sizeof(unsigned long long));
  l.slots = off; off = align_up(off + 3 * static_cast<size_t>(c->batch) * sizeof(int32_t));
  l.total = off;
  return l;
}

// Returns the three events of an armed call (created here), or null when not armed.
hipEvent_t *arm_events(lazyev_ctx *ctx, int kind) {
  if (ctx->prof_armed <= 0) return nullptr;
  lazyev_ctx::Timed t;
  t.kind = kind;
  for (int i = 0; i < 3; ++i)
    if (hipEventCreate(&t.ev[i]) != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(t.ev[j]);
      return nullptr;
    }
  try {
    ctx->prof.push_back(t);
  } catch (const std::bad_alloc &) {               // the call then goes untimed
    for (int i = 0; i < 3; ++i) (void)hipEventDestroy(t.ev[i]);
    return nullptr;
  }
  ctx->prof_armed -= 1;
  return ctx->prof.back().ev;
}

void drop_events(lazyev_ctx *ctx) {
  for (auto &t : ctx->prof)
    for (int i = 0; i < 3; ++i) (void)hipEventDestroy(t.ev[i]);
  ctx->prof.clear();
}

// Device address of `scratch` on the current device, looked up on the first call per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int32_t *g_scratch_ptr[kMaxDevices];

hipError_t static_scratch_of(int *device, int32_t **ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<int32_t *>(p);
  }
  *device = dev;
  *ptr = g_scratch_ptr[dev];
  return hipSuccess;
}

int fail_hip(lazyev_ctx *ctx, hipError_t e) {
  ctx->last_hip_error = static_cast<int>(e);
  return LAZYEV_EHIP;
}

// ---- per-sequence timing
lazyev::Slots slots_of(const lazyev_ctx *ctx) {
  lazyev::Slots sl;
  sl.prompt_len = ctx->slots_on ? ctx->dev_slot_prompt : nullptr;
  sl.t0 = ctx->slots_on ? ctx->dev_slot_t0 : nullptr;
  sl.budget = ctx->cfg.budget;
  sl.window = ctx->cfg.window;
  return sl;
}

// Does sequence s take part in global step t, and with how many cached entries before its append?
bool slot_active(const lazyev_ctx *ctx, int s, int32_t t, int32_t *n_old) {
  const int32_t P = ctx->slot_prompt[s], tau = t - ctx->slot_t0[s];
  if (P < 0 || tau < 1) return false;
  *n_old = lazyev::slot_n_old(P, tau, ctx->cfg.budget, ctx->cfg.window);
  return true;
}

// Is an eviction due for sequence s after global step t (Sec. 4), and from how many entries?
bool slot_due(const lazyev_ctx *ctx, int s, int32_t t, int32_t *n) {
  int32_t n_old;
  if (!slot_active(ctx, s, t, &n_old)) return false;
  *n = n_old + 1;
  return (t - ctx->slot_t0[s]) % ctx->cfg.window == 0 && *n > ctx->cfg.budget;
}

// Entries sequence s holds in `layer` now (after the layer's last step and, if it ran, that
// step's eviction); 0 for an empty or not yet started slot's generated part.
int32_t slot_len_now(const lazyev_ctx *ctx, int layer, int s) {
  const int32_t t = ctx->last_step[layer];
  if (ctx->slot_prompt[s] < 0) return 0;
  int32_t n_old;
  if (!slot_active(ctx, s, t, &n_old)) return ctx->slot_prompt[s];
  int32_t n;
  if (slot_due(ctx, s, t, &n) && ctx->evict_applied[layer] == t) return ctx->cfg.budget;
  return n_old + 1;
}

// With per-sequence timing: when at most 8 sequences are due after step t, an eviction launch
// covers only their units.
void fill_due(const lazyev_ctx *ctx, int32_t t, lazyev::EvictArgs &a) {
  a.n_due = 0;
  if (!ctx->slots_on) return;
  int32_t n_tmp;
  for (int s = 0; s < ctx->cfg.batch; ++s) {
    if (!slot_due(ctx, s, t, &n_tmp)) continue;
    if (a.n_due == 8) { a.n_due = 0; return; }     // many: one block per unit, the others return at once
    a.due_seq[a.n_due++] = s;
  }
}

// Applies the logged calls of layers l0 .. l1 - 1, which all hold the same calls, to TS / MRI.
hipError_t flush_log_range(lazyev_ctx *ctx, int l0, int l1) {
  const int n = ctx->log_n[l0];
  if (n == 0) return hipSuccess;
  lazyev::FlushArgs f;
  std::memset(&f, 0, sizeof(f));
  const size_t slab = static_cast<size_t>(ctx->units) * ctx->capacity;
  f.ts = ctx->cfg.ts + static_cast<size_t>(l0) * slab;
  f.mri = ctx->cfg.mri + static_cast<size_t>(l0) * slab;
  f.pos = ctx->cfg.pos + static_cast<size_t>(l0) * slab;
  f.prompt_len = ctx->cfg.prompt_len;
  f.bitlog = ctx->bitlog + static_cast<size_t>(l0) * ctx->log_slots * ctx->units * ctx->log_words;
  f.units = ctx->units; f.capacity = ctx->capacity;
  f.log_words = ctx->log_words; f.log_slots = ctx->log_slots;
  f.n_calls = n;
  for (int s = 0; s < n; ++s) {
    f.t[s] = ctx->log_t[static_cast<size_t>(l0) * ctx->log_slots + s];
    f.n_old[s] = ctx->log_n_old[static_cast<size_t>(l0) * ctx->log_slots + s];
  }
  const hipError_t e = lazyev::launch_track_flush(f, l1 - l0, ctx->stream);
  if (e == hipSuccess)
    for (int l = l0; l < l1; ++l) ctx->log_n[l] = 0;
  return e;
}

// Applies every layer's logged calls: consecutive layers that hold the same calls (the usual
// case: all of them) in one launch.
hipError_t flush_logs(lazyev_ctx *ctx) {
  if (!ctx->bitlog) return hipSuccess;
  const int L = ctx->cfg.n_layers;
  for (int l0 = 0; l0 < L;) {
    int l1 = l0 + 1;
    const int n = ctx->log_n[l0];
    while (l1 < L && ctx->log_n[l1] == n &&
           std::equal(ctx->log_t.begin() + static_cast<size_t>(l0) * ctx->log_slots,
                      ctx->log_t.begin() + static_cast<size_t>(l0) * ctx->log_slots + n,
                      ctx->log_t.begin() + static_cast<size_t>(l1) * ctx->log_slots) &&
           std::equal(ctx->log_n_old.begin() + static_cast<size_t>(l0) * ctx->log_slots,
                      ctx->log_n_old.begin() + static_cast<size_t>(l0) * ctx->log_slots + n,
                      ctx->log_n_old.begin() + static_cast<size_t>(l1) * ctx->log_slots) &&
           static_cast<long long>(l1 + 1 - l0) * ctx->units <= 65535)
      ++l1;
    const hipError_t e = flush_log_range(ctx, l0, l1);
    if (e != hipSuccess) return e;
    l0 = l1;
  }
  return hipSuccess;
}

// Applies all tracking that is still outstanding, in the order of the calls: the logged calls
// of every layer, then the last fused decode call if its tracking is still pending.  Everything
// that reads TS / MRI (an eviction, lazyev_stats, the histogram, a caller who asks for the
// weights) comes through here first.
hipError_t flush_tracking(lazyev_ctx *ctx) {
  hipError_t e = flush_logs(ctx);
  if (e != hipSuccess || !ctx->pend.valid) return e;
  ctx->pend.bitlog = nullptr;                      // (applied at once)
  e = lazyev::launch_track(ctx->pend, ctx->stream);
  if (e == hipSuccess) ctx->pend.valid = 0;
  return e;
}

}  // namespace

extern "C" {

int32_t lazyev_capacity(const lazyev_config *cfg) { return config_ok(cfg) ? capacity_of(cfg) : 0; }

size_t lazyev_workspace_size(const lazyev_config *cfg) {
  return config_ok(cfg) ? layout_of(cfg).total : 0;
}

int lazyev_init(const lazyev_config *cfg, lazyev_ctx **out) {
  if (!out) return LAZYEV_EINVAL;
  *out = nullptr;
  if (!config_ok(cfg)) return LAZYEV_EINVAL;
  if (!cfg->k_cache || !cfg->v_cache || !cfg->ts || !cfg->mri || !cfg->pos) return LAZYEV_EINVAL;
  const Layout l = layout_of(cfg);
  if (!cfg->workspace || cfg->workspace_bytes < l.total ||
      reinterpret_cast<uintptr_t>(cfg->workspace) % kAlign != 0)
    return LAZYEV_EWORKSPACE;

  lazyev_ctx *ctx = new (std::nothrow) lazyev_ctx();
  if (!ctx) return LAZYEV_ENOMEM;
  try {                                            // (the host mirrors are std::vectors)
    ctx->slot_prompt.assign(cfg->batch, cfg->prompt_len);
    ctx->slot_t0.assign(cfg->batch, 0);
    ctx->evict_applied.assign(cfg->n_layers, 0);
    ctx->len.assign(cfg->n_layers, cfg->prompt_len);
    ctx->last_step.assign(cfg->n_layers, 0);
    ctx->n_evict_events.assign(cfg->n_layers, 0);
    ctx->n_evicted.assign(cfg->n_layers, 0);
    ctx->log_n.assign(cfg->n_layers, 0);
    ctx->log_t.assign(static_cast<size_t>(cfg->n_layers) * (l.log_slots > 0 ? l.log_slots : 1), 0);
    ctx->log_n_old.assign(ctx->log_t.size(), 0);
  } catch (const std::bad_alloc &) {
    delete ctx;
    return LAZYEV_ENOMEM;
  }
  ctx->cfg = *cfg;
  ctx->capacity = capacity_of(cfg);
  ctx->group = cfg->n_q_heads / cfg->n_kv_heads;
  ctx->units = cfg->batch * cfg->n_kv_heads;
  ctx->n_split_max = l.n_split_max;
  ctx->chunk = 128;
  ctx->variant = 1;
  ctx->target_blocks = 512;          // two blocks per compute unit
  ctx->target_blocks_set = false;
  while ((ctx->capacity + ctx->chunk - 1) / ctx->chunk > lazyev::decode_split_max()) ctx->chunk *= 2;
  ctx->scale = cfg->softmax_scale > 0.0f ? cfg->softmax_scale
                                         : 1.0f / std::sqrt(static_cast<float>(cfg->head_dim));
  ctx->stream = static_cast<hipStream_t>(cfg->stream);
  char *base = static_cast<char *>(cfg->workspace);
  ctx->ws.part_acc = reinterpret_cast<float *>(base + l.part_acc);
  ctx->ws.part_ml = reinterpret_cast<float *>(base + l.part_ml);
  ctx->ws.p_tilde = reinterpret_cast<float *>(base + l.p_tilde);
  ctx->ws.logits[0] = ctx->ws.p_tilde;
  ctx->ws.logits[1] = reinterpret_cast<float *>(base + l.logits1);
  ctx->ws.stat[0] = reinterpret_cast<float *>(base + l.stat);
  ctx->ws.stat[1] = ctx->ws.stat[0] + static_cast<size_t>(cfg->batch) * cfg->n_kv_heads * 16;
  std::memset(&ctx->pend, 0, sizeof(ctx->pend));
  ctx->cur_buf = 0;
  ctx->last_layer = -1;
  ctx->last_logits = ctx->last_stat = nullptr;
  ctx->last_p_stride = 0;
  ctx->prefill_stat = reinterpret_cast<float *>(base + l.prefill_stat);
  ctx->ws.src_index = reinterpret_cast<int32_t *>(base + l.src_index);
  ctx->ws.sel_keys = l.bitlog > l.sel_keys ? reinterpret_cast<unsigned long long *>(base + l.sel_keys) : nullptr;
  ctx->bitlog = l.log_slots > 0 ? reinterpret_cast<uint32_t *>(base + l.bitlog) : nullptr;
  ctx->log_words = l.log_words;
  ctx->log_slots = l.log_slots;
  ctx->pend_layer = -1;
  ctx->ws.activations = reinterpret_cast<unsigned long long *>(base + l.activations);
  ctx->ws.rows_moved = reinterpret_cast<unsigned long long *>(base + l.rows_moved);
  ctx->ws.ticket = reinterpret_cast<int32_t *>(base + l.ticket);
  ctx->ws.part_rec = reinterpret_cast<unsigned long long *>(base + l.records);
  ctx->ws.fault = reinterpret_cast<int32_t *>(base + l.fault);
  ctx->launch_seq = 0;
  ctx->spin_ticks = 2000000;           // 20 ms of the 100 MHz counter
  ctx->ws.hist = reinterpret_cast<unsigned long long *>(base + l.hist);
  ctx->dev_slot_prompt = reinterpret_cast<int32_t *>(base + l.slots);
  ctx->dev_slot_t0 = ctx->dev_slot_prompt + cfg->batch;
  ctx->dev_seq_len = ctx->dev_slot_t0 + cfg->batch;
  ctx->slots_on = false;
  ctx->last_hip_error = 0;
  ctx->prof_armed = 0;
  if (ctx->chunk > lazyev::decode_chunk_max()) { delete ctx; return LAZYEV_EINVAL; }
  if (static_scratch_of(&ctx->device, &ctx->static_scratch) != hipSuccess) { delete ctx; return LAZYEV_EHIP; }

  // activation counters, moved-row counters, tickets, records and the fault word lie next to each other
  hipError_t e = hipMemsetAsync(ctx->ws.activations, 0, l.total - l.activations, ctx->stream);
  if (e == hipSuccess)
    e = lazyev::launch_init_state(cfg->ts, cfg->mri, cfg->pos,
                                  static_cast<int64_t>(cfg->n_layers) * ctx->units, ctx->capacity,
                                  cfg->prompt_len, ctx->stream);
  if (e != hipSuccess) { delete ctx; return LAZYEV_EHIP; }
  *out = ctx;
  return LAZYEV_OK;
}

int lazyev_set_chunk(lazyev_ctx *ctx, int32_t chunk) {
  if (!ctx || chunk < kMinChunk || chunk > lazyev::decode_chunk_max() || (chunk & (chunk - 1)))
    return LAZYEV_EINVAL;
  if ((ctx->capacity + chunk - 1) / chunk > lazyev::decode_split_max()) return LAZYEV_EINVAL;
  ctx->chunk = chunk;
  return LAZYEV_OK;
}

int lazyev_set_target_blocks(lazyev_ctx *ctx, int32_t n_blocks) {
  if (!ctx || n_blocks < 1) return LAZYEV_EINVAL;
  ctx->target_blocks = n_blocks;
  ctx->target_blocks_set = true;
  return LAZYEV_OK;
}

int lazyev_set_spin_ticks(lazyev_ctx *ctx, uint32_t ticks) {
  if (!ctx) return LAZYEV_EINVAL;
  ctx->spin_ticks = ticks;
  return LAZYEV_OK;
}

int lazyev_set_variant(lazyev_ctx *ctx, int32_t variant) {
  if (!ctx || variant < 0 || variant > 6 || variant == 2 || variant == 3) return LAZYEV_EINVAL;
  ctx->variant = variant;
  return LAZYEV_OK;
}

int lazyev_decode_step(lazyev_ctx *ctx, int32_t layer, int32_t t, const void *q, const void *k_new,
                       const void *v_new, void *out, float *p_out, const float *p_override) {
  if (!ctx || !q || !k_new || !v_new || !out) return LAZYEV_EINVAL;
  const lazyev_config &c = ctx->cfg;
  if (layer < 0 || layer >= c.n_layers) return LAZYEV_EINVAL;
  if (t != ctx->last_step[layer] + 1) return LAZYEV_EINVAL;
  int32_t n_old = ctx->len[layer];
  if (ctx->slots_on) {
    // per-sequence timing: a due eviction of the layer's previous step must have run, and the
    // launch is sized for the longest cache among the sequences that take this step
    const int32_t tp = ctx->last_step[layer];
    int32_t n_tmp;
    if (tp >= 1 && ctx->evict_applied[layer] != tp)
      for (int s2 = 0; s2 < c.batch; ++s2)
        if (slot_due(ctx, s2, tp, &n_tmp)) return LAZYEV_ECAPACITY;
    n_old = -1;
    for (int s2 = 0; s2 < c.batch; ++s2)
      if (slot_active(ctx, s2, t, &n_tmp) && n_tmp > n_old) n_old = n_tmp;
    if (n_old < 0) {                               // no sequence takes this step
      ctx->last_step[layer] = t;
      return LAZYEV_OK;
    }
  }
  if (n_old >= ctx->capacity) return LAZYEV_ECAPACITY;

  const size_t esz = c.dtype == LAZYEV_DTYPE_FP32 ? 4 : 2;
  const size_t slab = static_cast<size_t>(ctx->units) * ctx->capacity;
  lazyev::DecodeArgs a;
  std::memset(&a, 0, sizeof(a));
  a.batch = c.batch; a.n_q_heads = c.n_q_heads; a.n_kv_heads = c.n_kv_heads;
  a.head_dim = c.head_dim; a.group = ctx->group; a.capacity = ctx->capacity;
  a.n_old = n_old; a.t = t; a.prompt_len = c.prompt_len;
  // which attention kernel: see lazyev_set_variant
  const bool mfma_shape = c.dtype == LAZYEV_DTYPE_BF16 && c.head_dim == 128;
  // (5 and 6 are 4 with the logits always / never written in full)
  const int kind = (mfma_shape && ctx->variant != 0) ? 4 : 0;
  bool compact = false;
  if (ctx->slots_on && kind != 4) return LAZYEV_EINVAL;   // only the single-launch kernel knows slots
  a.slots = slots_of(ctx);
  if (kind == 4) {
    // fused kernel: n_split blocks of four waves per unit, every wave a run of 16-entry sub-tiles
    const int n_sub = (n_old + 1 + 15) / 16;
    int n_split = (ctx->target_blocks + ctx->units / 2) / ctx->units;
    if (!ctx->target_blocks_set) {
      // one block per compute unit, whatever the cache length: measured at 128 units over caches
      // of 1088 .. 6144 entries against 1.5 and 2 blocks per compute unit (2448 / 3248 / 4144 /
      // 5048 entries: 28.3 / 36.5 / 44.5 / 55.9 us per call against 30.2 / 37.4 / 46.4 / 57.0 with
      // two per compute unit; three blocks per two compute units are worst, 39.3 at 3248).  A
      // second stream block on a compute unit doubles the bytes its waves keep in flight, which
      // this memory system answers with a wider spread of the blocks' ends, not with more
      // bandwidth; a wave whose run then exceeds the sub-tiles it keeps logits of in LDS leaves
      // its candidate lists segment by segment.
      n_split = (256 + ctx->units - 1) / ctx->units;
    }
    if (n_split > (n_sub + 3) / 4) n_split = (n_sub + 3) / 4;
    if (n_split > lazyev::decode_fused_split_max()) n_split = lazyev::decode_fused_split_max();
    if (n_split > ctx->n_split_max) n_split = ctx->n_split_max;
    if (n_split < 1) n_split = 1;
    a.n_split = n_split;
    a.chunk = 16;
    a.logits_out = ctx->ws.logits[ctx->cur_buf];
    a.stat_out = ctx->ws.stat[ctx->cur_buf];
    if (p_out || p_override) {                     // the caller looks at the weights of this call at once:
      const hipError_t ef = flush_tracking(ctx);   // everything older is applied first, in order
      if (ef != hipSuccess) return fail_hip(ctx, ef);
    }
    a.track = ctx->pend;                           // the previous call's tracking rides along
    if (a.track.valid && ctx->bitlog && !ctx->slots_on && ctx->pend_layer >= 0) {
      // ... as one bit per cache entry in the next free slot of its layer's log (a full log is
      // applied first)
      const int ly = ctx->pend_layer;
      if (ctx->log_n[ly] == ctx->log_slots) {
        const hipError_t ef = flush_log_range(ctx, ly, ly + 1);
        if (ef != hipSuccess) return fail_hip(ctx, ef);
      }
      const int slot = ctx->log_n[ly];
      a.track.bitlog = ctx->bitlog + (static_cast<size_t>(ly) * ctx->units * ctx->log_slots + slot) * ctx->log_words;
      a.track.log_words = ctx->log_words;
      a.track.log_unit_stride = ctx->log_slots * ctx->log_words;
      ctx->log_t[static_cast<size_t>(ly) * ctx->log_slots + slot] = a.track.t;
      ctx->log_n_old[static_cast<size_t>(ly) * ctx->log_slots + slot] = a.track.n_old;
    }
    a.p_stride = static_cast<int32_t>(fused_p_stride(ctx->capacity));
    // candidate lists instead of every logit, unless somebody reads the logits as such (the
    // caller through p_out / p_override, or an eviction that ranks by this call's weights): the
    // lists are built by waves of their own beside the merge, so they cost a call nothing and
    // save traffic at every cache length (measured 129 .. 4160 entries)
    compact = ctx->variant != 5 && !p_out && !p_override &&
              !(c.score_flags & LAZYEV_SCORE_CURRENT_ATTENTION) &&
              lazyev::decode_fused_compact_fits(n_old, n_split, a.p_stride, ctx->group);
  }
  if (kind != 4) {
    a.chunk = ctx->chunk;
    a.n_split = (n_old + 1 + ctx->chunk - 1) / ctx->chunk;
  }
  a.n_split_max = ctx->n_split_max;
  if (kind != 4) a.p_stride = (ctx->capacity + 15) / 16 * 16;
  a.variant = compact ? 6 : kind;
  a.alpha = c.alpha; a.scale = ctx->scale; a.dtype = c.dtype;
  a.q = q; a.k_new = k_new; a.v_new = v_new; a.out = out;
  a.k_cache = static_cast<char *>(c.k_cache) + static_cast<size_t>(layer) * slab * c.head_dim * esz;
  a.v_cache = static_cast<char *>(c.v_cache) + static_cast<size_t>(layer) * slab * c.head_dim * esz;
  a.ts = c.ts + static_cast<size_t>(layer) * slab;
  a.mri = c.mri + static_cast<size_t>(layer) * slab;
  a.pos = c.pos + static_cast<size_t>(layer) * slab;
  a.p_out = p_out; a.p_override = p_override;
  a.ws = ctx->ws;
  a.ticket = ctx->ws.ticket;
  if (kind == 4) {
    // the number of this launch stamps the partials its blocks hand over; 0 is what the records
    // hold before any launch, so after a wrap-around they are cleared and the count restarts
    if (++ctx->launch_seq == 0) {
      const hipError_t ec = lazyev::launch_clear_records(
          ctx->ws.part_rec, static_cast<size_t>(ctx->units) * 3 * lazyev::decode_fused_record_bytes() / 8, ctx->stream);
      if (ec != hipSuccess) return fail_hip(ctx, ec);
      ctx->launch_seq = 1;
    }
    a.seq = ctx->launch_seq;
    a.spin_ticks = ctx->spin_ticks;
  }
  a.activation_counter = ctx->ws.activations + static_cast<size_t>(layer) * ctx->units * lazyev::decode_slice_max();

  if (kind != 4) {                                 // the other kernels track in the same call
    const hipError_t ef = flush_tracking(ctx);
    if (ef != hipSuccess) return fail_hip(ctx, ef);
  }
  const hipError_t e = lazyev::launch_decode(a, ctx->stream, arm_events(ctx, 0));
  if (e != hipSuccess) return fail_hip(ctx, e);
  ctx->len[layer] = n_old + 1;
  ctx->last_step[layer] = t;
  ctx->last_layer = kind == 4 ? layer : -1;
  if (kind == 4 && a.track.valid && a.track.bitlog) ctx->log_n[ctx->pend_layer] += 1;   // (that call is in the log now)
  if (kind == 4) {
    ctx->pend_layer = layer;
    ctx->last_logits = a.logits_out; ctx->last_stat = a.stat_out; ctx->last_p_stride = a.p_stride;
    lazyev::TrackArgs &k = ctx->pend;              // this call's tracking: with the next launch
    std::memset(&k, 0, sizeof(k));
    k.valid = 1;
    k.n_old = n_old; k.t = t; k.prompt_len = c.prompt_len;
    k.capacity = ctx->capacity; k.group = ctx->group; k.n_q_heads = c.n_q_heads;
    k.n_kv_heads = c.n_kv_heads; k.units = ctx->units; k.p_stride = a.p_stride;
    k.alpha = c.alpha;
    k.ts = a.ts; k.mri = a.mri; k.pos = a.pos;
    k.logits = a.logits_out; k.stat = a.stat_out;
    k.compact = compact ? 1 : 0; k.n_parts = a.n_split;
    k.p_out = p_out; k.p_override = p_override;
    k.activation_counter = a.activation_counter;
    k.slots = a.slots;
    ctx->cur_buf ^= 1;
    if (p_out || p_override) {                     // the caller looks at the weights now
      const hipError_t ef = flush_tracking(ctx);
      if (ef != hipSuccess) return fail_hip(ctx, ef);
    }
  }
  return LAZYEV_OK;
}

int lazyev_prefill_track(lazyev_ctx *ctx, int32_t layer, const void *q_prompt, float *p_out,
                         const float *p_override) {
  if (!ctx || !q_prompt) return LAZYEV_EINVAL;
  const lazyev_config &c = ctx->cfg;
  if (layer < 0 || layer >= c.n_layers) return LAZYEV_EINVAL;
  if (ctx->slots_on || c.prompt_len < 1) return LAZYEV_EINVAL;
  if (ctx->last_step[layer] != 0) return LAZYEV_EINVAL;       // the layer has already decoded
  const size_t slab = static_cast<size_t>(ctx->units) * ctx->capacity;
  lazyev::PrefillArgs a;
  std::memset(&a, 0, sizeof(a));
  a.batch = c.batch; a.n_q_heads = c.n_q_heads; a.n_kv_heads = c.n_kv_heads; a.group = ctx->group;
  a.head_dim = c.head_dim; a.dtype = c.dtype;
  a.capacity = ctx->capacity; a.prompt_len = c.prompt_len;
  a.p16 = (c.prompt_len + 15) / 16 * 16;
  a.counter_stride = lazyev::decode_slice_max();
  a.alpha = c.alpha; a.scale = ctx->scale;
  a.q_prompt = q_prompt;
  a.k_cache = static_cast<char *>(c.k_cache) +
              static_cast<size_t>(layer) * slab * c.head_dim * (c.dtype == LAZYEV_DTYPE_FP32 ? 4 : 2);
  a.ts = c.ts + static_cast<size_t>(layer) * slab;
  a.mri = c.mri + static_cast<size_t>(layer) * slab;
  a.stat = ctx->prefill_stat;
  a.p_out = p_out; a.p_override = p_override;
  a.activation_counter = ctx->ws.activations + static_cast<size_t>(layer) * ctx->units * lazyev::decode_slice_max();
  const hipError_t e = lazyev::launch_prefill_track(a, ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, e);
  return LAZYEV_OK;
}

int lazyev_prefill_track_seq(lazyev_ctx *ctx, int32_t layer, int32_t seq, const void *q_prompt, float *p_out,
                             const float *p_override) {
  if (!ctx || !q_prompt) return LAZYEV_EINVAL;
  const lazyev_config &c = ctx->cfg;
  if (layer < 0 || layer >= c.n_layers || seq < 0 || seq >= c.batch) return LAZYEV_EINVAL;
  if (c.dtype != LAZYEV_DTYPE_BF16 || c.head_dim != 128 || ctx->group > 8) return LAZYEV_EINVAL;
  if (!ctx->slots_on || ctx->slot_prompt[seq] < 1) return LAZYEV_EINVAL;
  if (ctx->last_step[layer] > ctx->slot_t0[seq]) return LAZYEV_EINVAL;   // the sequence has already decoded here
  const int32_t P = ctx->slot_prompt[seq];
  const size_t slab = static_cast<size_t>(ctx->units) * ctx->capacity;
  const size_t first = static_cast<size_t>(seq) * c.n_kv_heads;          // the sequence's first unit
  lazyev::PrefillArgs a;
  std::memset(&a, 0, sizeof(a));
  a.batch = 1; a.n_q_heads = c.n_q_heads; a.n_kv_heads = c.n_kv_heads; a.group = ctx->group;
  a.head_dim = c.head_dim; a.dtype = c.dtype;
  a.capacity = ctx->capacity; a.prompt_len = P;
  a.p16 = (P + 15) / 16 * 16;
  a.counter_stride = lazyev::decode_slice_max();
  a.alpha = c.alpha; a.scale = ctx->scale;
  a.q_prompt = q_prompt;
  a.k_cache = static_cast<char *>(c.k_cache) + (static_cast<size_t>(layer) * slab + first * ctx->capacity) * c.head_dim * 2;
  a.ts = c.ts + static_cast<size_t>(layer) * slab + first * ctx->capacity;
  a.mri = c.mri + static_cast<size_t>(layer) * slab + first * ctx->capacity;
  a.stat = ctx->prefill_stat;
  a.p_out = p_out; a.p_override = p_override;
  a.activation_counter = ctx->ws.activations +
                         (static_cast<size_t>(layer) * ctx->units + first) * lazyev::decode_slice_max();
  const hipError_t e = lazyev::launch_prefill_track(a, ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, e);
  return LAZYEV_OK;
}

// The eviction check of one layer.  `gather`: where the units' gather lists go (null: the
// workspace's area).
static int evict_layer(lazyev_ctx *ctx, int32_t layer, int32_t t, int32_t *n_evicted, int32_t *gather) {
  if (n_evicted) *n_evicted = 0;
  if (!ctx) return LAZYEV_EINVAL;
  const lazyev_config &c = ctx->cfg;
  if (layer < 0 || layer >= c.n_layers) return LAZYEV_EINVAL;
  if (t < 1 || t != ctx->last_step[layer]) return LAZYEV_EINVAL;
  int32_t n = ctx->len[layer];
  if (ctx->slots_on) {                             // due for any sequence?  sized for the longest of those
    n = 0;
    int32_t n_tmp;
    for (int s2 = 0; s2 < c.batch; ++s2)
      if (slot_due(ctx, s2, t, &n_tmp) && n_tmp > n) n = n_tmp;
    if (n == 0 || ctx->evict_applied[layer] == t) return LAZYEV_OK;
  } else if (t % c.window != 0 || n <= c.budget) {
    return LAZYEV_OK;                              // not due (Sec. 4)
  }

  const size_t esz = c.dtype == LAZYEV_DTYPE_FP32 ? 4 : 2;
  const size_t slab = static_cast<size_t>(ctx->units) * ctx->capacity;
  lazyev::EvictArgs a;
  std::memset(&a, 0, sizeof(a));
  a.units = ctx->units; a.units_per_layer = ctx->units; a.head_dim = c.head_dim; a.dtype = c.dtype; a.capacity = ctx->capacity;
  a.n = n; a.budget = c.budget; a.window = c.window; a.t = t; a.score_flags = c.score_flags;
  a.k_cache = static_cast<char *>(c.k_cache) + static_cast<size_t>(layer) * slab * c.head_dim * esz;
  a.v_cache = static_cast<char *>(c.v_cache) + static_cast<size_t>(layer) * slab * c.head_dim * esz;
  a.ts = c.ts + static_cast<size_t>(layer) * slab;
  a.mri = c.mri + static_cast<size_t>(layer) * slab;
  a.pos = c.pos + static_cast<size_t>(layer) * slab;
  a.ws = ctx->ws;
  if (gather) a.ws.src_index = gather;
  a.rows_moved = ctx->ws.rows_moved + static_cast<size_t>(layer) * ctx->units;
  a.n_kv_heads = c.n_kv_heads;
  a.slots = slots_of(ctx);
  fill_due(ctx, t, a);
  if (c.score_flags & LAZYEV_SCORE_CURRENT_ATTENTION) {
    // the weights of step t: only there if this layer's decode call was the last one
    if (ctx->last_layer != layer || !ctx->last_logits) return LAZYEV_EINVAL;
    a.logits = ctx->last_logits; a.stat = ctx->last_stat;
    a.group = ctx->group; a.p_stride = ctx->last_p_stride;
  }
  const hipError_t ef = flush_tracking(ctx);       // scores use TS and MRI of step t (Alg. 1 order)
  if (ef != hipSuccess) return fail_hip(ctx, ef);
  const hipError_t e = lazyev::launch_evict(a, ctx->stream, arm_events(ctx, 1));
  if (e != hipSuccess) return fail_hip(ctx, e);
  if (n_evicted) *n_evicted = n - c.budget;
  ctx->n_evict_events[layer] += 1;
  ctx->n_evicted[layer] += n - c.budget;
  ctx->evict_applied[layer] = t;
  ctx->len[layer] = c.budget;
  if (ctx->slots_on) {
    ctx->len[layer] = 0;
    for (int s2 = 0; s2 < c.batch; ++s2) {
      const int32_t ls = slot_len_now(ctx, layer, s2);
      if (ls > ctx->len[layer]) ctx->len[layer] = ls;
    }
  }
  ctx->last_layer = -1;                            // the stored logits no longer match the slots
  return LAZYEV_OK;
}

int lazyev_evict(lazyev_ctx *ctx, int32_t layer, int32_t t, int32_t *n_evicted) {
  return evict_layer(ctx, layer, t, n_evicted, nullptr);
}

int lazyev_evict_static(lazyev_ctx *ctx, int32_t layer, int32_t t, int32_t *n_evicted) {
  if (n_evicted) *n_evicted = 0;
  if (!ctx) return LAZYEV_EINVAL;
  // one gather-list entry per cache entry of the layer; the selection keeps its keys in LDS
  if (static_cast<size_t>(ctx->units) * ctx->capacity > kStaticScratchEntries ||
      ctx->capacity - ctx->cfg.window > lazyev::evict_lds_candidates())
    return LAZYEV_ESCRATCH;
  int dev = -1;
  const hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(ctx, e);
  if (dev != ctx->device || !ctx->static_scratch) return LAZYEV_EINVAL;   // (the array is per device)
  return evict_layer(ctx, layer, t, n_evicted, ctx->static_scratch);
}

int lazyev_evict_all(lazyev_ctx *ctx, int32_t t, int32_t *n_evicted) {
  if (n_evicted) *n_evicted = 0;
  if (!ctx) return LAZYEV_EINVAL;
  const lazyev_config &c = ctx->cfg;
  const int L = c.n_layers;
  // One launch pair for all layers when they stand at the same point (same step, same length,
  // none evicted yet at this step) and the score does not need a layer's own last decode call;
  // otherwise layer by layer.
  bool together = L > 1 && !(c.score_flags & LAZYEV_SCORE_CURRENT_ATTENTION) &&
                  static_cast<long long>(L) * ctx->units <= 65535;
  for (int l = 0; l < L && together; ++l)
    together = ctx->last_step[l] == t && ctx->len[l] == ctx->len[0] && ctx->evict_applied[l] != t;
  if (!together) {
    for (int l = 0; l < L; ++l) {
      int32_t n1 = 0;
      const int rc = lazyev_evict(ctx, l, t, &n1);
      if (rc != LAZYEV_OK) return rc;
      if (n_evicted && n1 > *n_evicted) *n_evicted = n1;
    }
    return LAZYEV_OK;
  }
  if (t < 1) return LAZYEV_EINVAL;
  int32_t n = ctx->len[0];
  if (ctx->slots_on) {                             // due for any sequence?  sized for the longest of those
    n = 0;
    int32_t n_tmp;
    for (int s2 = 0; s2 < c.batch; ++s2)
      if (slot_due(ctx, s2, t, &n_tmp) && n_tmp > n) n = n_tmp;
    if (n == 0) return LAZYEV_OK;
  } else if (t % c.window != 0 || n <= c.budget) {
    return LAZYEV_OK;                              // not due (Sec. 4)
  }
  lazyev::EvictArgs a;
  std::memset(&a, 0, sizeof(a));
  a.units = L * ctx->units; a.units_per_layer = ctx->units;
  a.head_dim = c.head_dim; a.dtype = c.dtype; a.capacity = ctx->capacity;
  a.n = n; a.budget = c.budget; a.window = c.window; a.t = t; a.score_flags = c.score_flags;
  a.k_cache = c.k_cache; a.v_cache = c.v_cache;    // layer 0; the other layers' slabs follow
  a.ts = c.ts; a.mri = c.mri; a.pos = c.pos;
  a.ws = ctx->ws;
  a.rows_moved = ctx->ws.rows_moved;
  a.n_kv_heads = c.n_kv_heads;
  a.slots = slots_of(ctx);
  fill_due(ctx, t, a);
  const hipError_t ef = flush_tracking(ctx);       // scores use TS and MRI of step t (Alg. 1 order)
  if (ef != hipSuccess) return fail_hip(ctx, ef);
  const hipError_t e = lazyev::launch_evict(a, ctx->stream, arm_events(ctx, 1));
  if (e != hipSuccess) return fail_hip(ctx, e);
  if (n_evicted) *n_evicted = n - c.budget;
  for (int l = 0; l < L; ++l) {
    ctx->n_evict_events[l] += 1;
    ctx->n_evicted[l] += n - c.budget;
    ctx->evict_applied[l] = t;
    ctx->len[l] = c.budget;
    if (ctx->slots_on) {
      ctx->len[l] = 0;
      for (int s2 = 0; s2 < c.batch; ++s2) {
        const int32_t ls = slot_len_now(ctx, l, s2);
        if (ls > ctx->len[l]) ctx->len[l] = ls;
      }
    }
  }
  ctx->last_layer = -1;                            // the stored logits no longer match the slots
  return LAZYEV_OK;
}

int lazyev_stats(lazyev_ctx *ctx, lazyev_stats_t *out) {
  if (!ctx || !out || out->n_layers != ctx->cfg.n_layers) return LAZYEV_EINVAL;
  const int L = ctx->cfg.n_layers;
  hipError_t e = flush_tracking(ctx);
  if (e != hipSuccess) return fail_hip(ctx, e);
  e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, e);
  // did a block of a decode call give up waiting for another block's partial?
  int32_t fault = 0;
  e = hipMemcpy(&fault, ctx->ws.fault, sizeof(fault), hipMemcpyDeviceToHost);
  if (e == hipSuccess && fault != 0) e = hipMemset(ctx->ws.fault, 0, sizeof(fault));
  if (e != hipSuccess) return fail_hip(ctx, e);
  if (fault != 0) return LAZYEV_EEXCHANGE;
  try {
  if (out->n_activations) {
    const size_t per_layer = static_cast<size_t>(ctx->units) * lazyev::decode_slice_max();
    std::vector<unsigned long long> tmp(per_layer * L);
    e = hipMemcpy(tmp.data(), ctx->ws.activations, tmp.size() * sizeof(unsigned long long),
                  hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail_hip(ctx, e);
    for (int i = 0; i < L; ++i) {
      unsigned long long sum = 0;
      for (size_t k = 0; k < per_layer; ++k) sum += tmp[i * per_layer + k];
      out->n_activations[i] = static_cast<int64_t>(sum);
    }
  }
  if (out->n_rows_moved) {
    std::vector<unsigned long long> tmp(static_cast<size_t>(ctx->units) * L);
    e = hipMemcpy(tmp.data(), ctx->ws.rows_moved, tmp.size() * sizeof(unsigned long long),
                  hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail_hip(ctx, e);
    for (int i = 0; i < L; ++i) {
      unsigned long long sum = 0;
      for (int k = 0; k < ctx->units; ++k) sum += tmp[static_cast<size_t>(i) * ctx->units + k];
      out->n_rows_moved[i] = static_cast<int64_t>(sum);
    }
  }
  } catch (const std::bad_alloc &) {
    return LAZYEV_ENOMEM;
  }
  for (int i = 0; i < L; ++i) {
    if (out->len) out->len[i] = ctx->len[i];
    if (out->last_step) out->last_step[i] = ctx->last_step[i];
    if (out->n_evict_events) out->n_evict_events[i] = ctx->n_evict_events[i];
    if (out->n_evicted) out->n_evicted[i] = ctx->n_evicted[i];
  }
  return LAZYEV_OK;
}

int lazyev_mri_histogram(lazyev_ctx *ctx, int32_t layer, int32_t n_bins, int64_t *hist) {
  if (!ctx || !hist || n_bins < 2 || n_bins > LAZYEV_MAX_HIST_BINS || layer < -1 ||
      layer >= ctx->cfg.n_layers)
    return LAZYEV_EINVAL;
  hipError_t e = flush_tracking(ctx);
  if (e == hipSuccess) e = hipMemsetAsync(ctx->ws.hist, 0, n_bins * sizeof(unsigned long long), ctx->stream);
  const int l0 = layer < 0 ? 0 : layer, l1 = layer < 0 ? ctx->cfg.n_layers : layer + 1;
  for (int l = l0; l < l1 && e == hipSuccess; ++l) {
    const int32_t *mri_l = ctx->cfg.mri + static_cast<size_t>(l) * ctx->units * ctx->capacity;
    if (!ctx->slots_on) {
      e = lazyev::launch_mri_histogram(mri_l, ctx->units, ctx->capacity, ctx->len[l], n_bins,
                                       ctx->ws.hist, ctx->stream);
      continue;
    }
    // per-sequence lengths of this layer go to the device first (a rare, synchronous call)
    std::vector<int32_t> lens;
    try {
      lens.resize(ctx->cfg.batch);
    } catch (const std::bad_alloc &) {
      return LAZYEV_ENOMEM;
    }
    int32_t n_max = 0;
    for (int s2 = 0; s2 < ctx->cfg.batch; ++s2) {
      lens[s2] = slot_len_now(ctx, l, s2);
      if (lens[s2] > n_max) n_max = lens[s2];
    }
    e = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess)
      e = hipMemcpy(ctx->dev_seq_len, lens.data(), lens.size() * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess)
      e = lazyev::launch_mri_histogram_slots(mri_l, ctx->units, ctx->capacity, ctx->cfg.n_kv_heads,
                                             ctx->dev_seq_len, n_max, n_bins, ctx->ws.hist, ctx->stream);
  }
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e == hipSuccess)
    e = hipMemcpy(hist, ctx->ws.hist, n_bins * sizeof(unsigned long long), hipMemcpyDeviceToHost);
  return e == hipSuccess ? LAZYEV_OK : fail_hip(ctx, e);
}

int lazyev_window_from_histogram(const int64_t *hist, int32_t n_bins, double quantile, int32_t *window) {
  if (!hist || !window || n_bins < 2 || !(quantile > 0.0) || !(quantile <= 1.0)) return LAZYEV_EINVAL;
  // entries that recurred at least once (bin 0 = never re-activated)
  int64_t total = 0;
  for (int32_t m = 1; m < n_bins; ++m) {
    if (hist[m] < 0) return LAZYEV_EINVAL;
    total += hist[m];
  }
  *window = 0;
  if (total == 0) return LAZYEV_OK;
  // the ceil(quantile * total)-th smallest MRI (inverted-CDF quantile), in binary64
  const double need = std::ceil(quantile * static_cast<double>(total));
  int64_t seen = 0;
  for (int32_t m = 1; m < n_bins; ++m) {
    seen += hist[m];
    if (static_cast<double>(seen) >= need) { *window = m; return LAZYEV_OK; }
  }
  *window = n_bins - 1;
  return LAZYEV_OK;
}

// Common part of lazyev_admit and lazyev_retire.
static int change_slot(lazyev_ctx *ctx, int32_t seq, int32_t prompt_len, int32_t t0) {
  const lazyev_config &c = ctx->cfg;
  hipError_t e = flush_tracking(ctx);              // pending tracking still belongs to the old occupant
  if (e != hipSuccess) return fail_hip(ctx, e);
  if (!ctx->slots_on) {                            // first use: the device copies of the timing records
    e = hipStreamSynchronize(ctx->stream);
    if (e == hipSuccess)
      e = hipMemcpy(ctx->dev_slot_prompt, ctx->slot_prompt.data(), c.batch * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess)
      e = hipMemcpy(ctx->dev_slot_t0, ctx->slot_t0.data(), c.batch * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail_hip(ctx, e);
    ctx->slots_on = true;
  }
  e = lazyev::launch_init_slot(c.ts, c.mri, c.pos, c.n_layers, c.batch, c.n_kv_heads, ctx->capacity,
                               seq, prompt_len, ctx->dev_slot_prompt, ctx->dev_slot_t0, t0, ctx->stream);
  if (e != hipSuccess) return fail_hip(ctx, e);
  ctx->slot_prompt[seq] = prompt_len;
  ctx->slot_t0[seq] = t0;
  ctx->last_layer = -1;
  for (int l = 0; l < c.n_layers; ++l) {           // what lazyev_stats reports as the layer's length
    ctx->len[l] = 0;
    for (int s2 = 0; s2 < c.batch; ++s2) {
      const int32_t ls = slot_len_now(ctx, l, s2);
      if (ls > ctx->len[l]) ctx->len[l] = ls;
    }
  }
  return LAZYEV_OK;
}

int32_t lazyev_cached_before_step(int32_t prompt_len, int32_t local_step, int32_t budget, int32_t window) {
  if (prompt_len < 0 || local_step < 1 || window < 1 || budget <= window) return -1;
  return lazyev::slot_n_old(prompt_len, local_step, budget, window);
}

int lazyev_admit(lazyev_ctx *ctx, int32_t seq, int32_t prompt_len, int32_t t0) {
  if (!ctx) return LAZYEV_EINVAL;
  const lazyev_config &c = ctx->cfg;
  if (seq < 0 || seq >= c.batch || prompt_len < 0 || prompt_len > ctx->capacity - c.window) return LAZYEV_EINVAL;
  if (c.dtype != LAZYEV_DTYPE_BF16 || c.head_dim != 128 || (ctx->variant != 1 && ctx->variant < 4))
    return LAZYEV_EINVAL;
  for (int l = 0; l < c.n_layers; ++l)
    if (t0 < ctx->last_step[l]) return LAZYEV_EINVAL;   // its first step lies ahead of every layer
  return change_slot(ctx, seq, prompt_len, t0);
}

int lazyev_retire(lazyev_ctx *ctx, int32_t seq) {
  if (!ctx) return LAZYEV_EINVAL;
  const lazyev_config &c = ctx->cfg;
  if (seq < 0 || seq >= c.batch) return LAZYEV_EINVAL;
  if (c.dtype != LAZYEV_DTYPE_BF16 || c.head_dim != 128 || (ctx->variant != 1 && ctx->variant < 4))
    return LAZYEV_EINVAL;
  return change_slot(ctx, seq, -1, 0);
}

int lazyev_score_pairs(const int32_t *delta_t, const int32_t *mri, double *score, int64_t n,
                       int32_t score_flags, void *stream) {
  if (n < 0 || (n > 0 && (!delta_t || !mri || !score))) return LAZYEV_EINVAL;
  if (score_flags & ~(LAZYEV_SCORE_H1 | LAZYEV_SCORE_H2 | LAZYEV_SCORE_H2_DECREASING)) return LAZYEV_EINVAL;
  const hipError_t e = lazyev::launch_score_pairs(delta_t, mri, score, n, score_flags,
                                                  static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LAZYEV_OK : LAZYEV_EHIP;
}

int32_t lazyev_log_words(lazyev_ctx *ctx) { return ctx && ctx->bitlog ? ctx->log_words : 0; }

int lazyev_log_peek(lazyev_ctx *ctx, int32_t layer, int32_t back, int32_t unit, uint32_t *words, int32_t *t) {
  if (!ctx || !words || layer < 0 || layer >= ctx->cfg.n_layers || back < 0 || unit < 0 || unit >= ctx->units)
    return LAZYEV_EINVAL;
  if (!ctx->bitlog || back >= ctx->log_n[layer]) return LAZYEV_EINVAL;
  const int slot = ctx->log_n[layer] - 1 - back;
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (e == hipSuccess)
    e = hipMemcpy(words,
                  ctx->bitlog + ((static_cast<size_t>(layer) * ctx->units + unit) * ctx->log_slots + slot) * ctx->log_words,
                  ctx->log_words * sizeof(uint32_t), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail_hip(ctx, e);
  if (t) *t = ctx->log_t[static_cast<size_t>(layer) * ctx->log_slots + slot];
  return LAZYEV_OK;
}

int lazyev_profile_arm(lazyev_ctx *ctx, int32_t n_calls) {
  if (!ctx || n_calls < 0) return LAZYEV_EINVAL;
  ctx->prof_armed = n_calls;
  return LAZYEV_OK;
}

int lazyev_profile_read(lazyev_ctx *ctx, double ms_total[4], int64_t launches[4]) {
  if (!ctx || !ms_total || !launches) return LAZYEV_EINVAL;
  for (int i = 0; i < 4; ++i) { ms_total[i] = 0.0; launches[i] = 0; }
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) { drop_events(ctx); return fail_hip(ctx, e); }
  for (auto &t : ctx->prof) {
    for (int i = 0; i < 2; ++i) {
      float ms = 0.f;
      e = hipEventElapsedTime(&ms, t.ev[i], t.ev[i + 1]);
      if (e != hipSuccess) { drop_events(ctx); return fail_hip(ctx, e); }
      ms_total[2 * t.kind + i] += ms;
      launches[2 * t.kind + i] += 1;
    }
  }
  drop_events(ctx);
  return LAZYEV_OK;
}

void lazyev_destroy(lazyev_ctx *ctx) {
  if (!ctx) return;
  drop_events(ctx);
  delete ctx;
}

const char *lazyev_strerror(int code) {
  switch (code) {
    case LAZYEV_OK: return "ok";
    case LAZYEV_EINVAL: return "invalid argument (shape, null pointer, budget <= window, step or layer out of order)";
    case LAZYEV_ECAPACITY: return "cache full (a due eviction was skipped)";
    case LAZYEV_EWORKSPACE: return "workspace missing, misaligned or too small";
    case LAZYEV_EHIP: return "HIP runtime error";
    case LAZYEV_ENOMEM: return "out of host memory";
    case LAZYEV_ESCRATCH: return "shape beyond the static scratch of lazyev_evict_static";
    case LAZYEV_EEXCHANGE: return "a block of a decode call gave up waiting for another block's partial result";
    default: return "unknown lazyev error code";
  }
}

int lazyev_last_hip_error(const lazyev_ctx *ctx) { return ctx ? ctx->last_hip_error : 0; }

}  // extern "C"
