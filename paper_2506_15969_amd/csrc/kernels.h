// Internal launch interface between the host API (lazyev_api.hip) and the kernel files.
// Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lazyev {

// Workspace carve-up, all offsets 256-byte aligned.  One layer call uses it at a time (calls
// are ordered by the stream), so nothing here is per layer except the counters.
struct Workspace {
  float    *part_acc;     // [units][n_split_max][G][D]  un-normalised partial outputs
  float    *part_ml;      // [units][n_split_max][2][G]  partial row max, partial row sum
  float    *p_tilde;      // [batch][n_q_heads][p_stride] exp(s - partial max) of every entry
                          // (split + merge kernels); the first logits buffer lies over it
  float    *logits[2];    // [units][p_stride][8]        fused kernel: scaled logits, double-buffered
  float    *stat[2];      // [units][8][2]               fused kernel: softmax max and 1 / sum per head
  int32_t  *src_index;    // [units][C]                  eviction: source entry of survivor j
  unsigned long long *sel_keys;     // [n_layers][units][C] eviction: score keys of a unit with more candidates
                                    // than LDS holds; null when the capacity rules that out
  unsigned long long *activations;  // [n_layers][units][slice_max]  running activation counts
  unsigned long long *rows_moved;   // [n_layers][units]             entries an eviction moved to a new slot
  int32_t  *ticket;       // [units]                     fused kernel: blocks of the unit done so far
  unsigned long long *part_rec;     // [units][3][fused record]  fused kernel, units of 2..4 blocks: the
                                    // partials of all blocks but the last as stamped records
  int32_t  *fault;        // [1]                         set when a block gave up waiting for a record
  unsigned long long *hist;         // [LAZYEV_MAX_HIST_BINS]  MRI histogram under construction
};

// Per-sequence timing.  Sequence s entered with prompt_len[s] cached rows (prompt_len[s] < 0: the
// slot is empty) and takes its first decode step at global step t0[s] + 1; its local step is
// tau = t - t0[s].  Null pointers: every sequence has the call's own n_old / t / prompt_len.
struct Slots {
  const int32_t *prompt_len, *t0;
  int32_t budget, window;
};

// Entries a sequence holds before the append of its local step tau >= 1, with every due
// eviction applied (Sec. 4: one is due after local step e when e % W == 0 and more than B
// entries are cached; it leaves exactly B).
__host__ __device__ inline int32_t slot_n_old(int32_t prompt_len, int32_t tau, int32_t budget,
                                              int32_t window) {
  // first local step after which an eviction fires
  const int32_t first = prompt_len > budget
                            ? window
                            : window * ((budget - prompt_len + 1 + window - 1) / window);
  const int32_t last = window * ((tau - 1) / window);     // latest multiple of W before step tau
  return last >= first ? budget + (tau - 1 - last) : prompt_len + tau - 1;
}

// Tracking of one finished decode call (Alg. 1 first loop, Eq. 1) from its stored logits and
// softmax statistics; the fused kernel runs it one call late.
struct TrackArgs {
  int32_t valid;
  int32_t n_old, t, prompt_len;
  int32_t capacity, group, n_q_heads, n_kv_heads, units;
  int32_t p_stride;                 // entries per unit in the logits buffer
  float   alpha;
  int32_t *ts, *mri, *pos;          // the call's layer slab
  const float *logits, *stat;
  float *p_out;
  const float *p_override;
  unsigned long long *activation_counter;   // the call's layer
  Slots slots;                      // with slots: n_old is the largest of the sequences', t global
  // compact != 0 (fused kernel, groups of at most 7 heads): the logits buffer holds, per block
  // of the call (n_parts per unit), only the entries that can reach alpha ("candidates").
  // Block b of a unit owns the slots [b * cap, (b + 1) * cap) of the unit's p_stride slots of 8
  // floats, cap = fused_part_cap(n_old, n_parts): slot 0 holds the number of records (as an
  // integer), slot 1 + r record r = the entry's 7 logits and, in the 8th place, its index.
  int32_t compact, n_parts;
  // Activation log (fused kernel, uniform batches).  Not null: the tracking blocks do not touch
  // TS / MRI of the active entries (a 128-byte line read and written for every 4-byte word) but
  // leave ONE BIT per cache entry of the unit, bit i = entry i was active in this call, as
  // log_words 32-bit words here; track_flush_kernel applies the logged calls of a layer in step
  // order (Eq. 1) before anything reads TS / MRI, and starts the entries those calls appended.
  uint32_t *bitlog;                 // this call's words of unit 0; unit u's follow at u * log_unit_stride
  int32_t log_words, log_unit_stride;   // (a unit's slots lie together: stride = log_slots * log_words)
};

// The logged calls of one or several layers applied to TS / MRI (Alg. 1 first loop, Eq. 1, in the
// order of the calls).  Block b works on layer b / units, unit b % units.
constexpr int kLogSlotsMax = 256;
struct FlushArgs {
  int32_t *ts, *mri, *pos;          // first layer's slab; the other layers' follow
  int32_t prompt_len;
  const uint32_t *bitlog;           // [layer][units][log_slots][log_words], first layer of the launch
  int32_t units, capacity, log_words, log_slots;
  int32_t n_calls;                  // logged calls to apply: slots 0 .. n_calls - 1
  int32_t t[kLogSlotsMax];          // step of the call in slot s (what TS becomes)
  int32_t n_old[kLogSlotsMax];      // the entry that call appended (it starts with TS = t, MRI = 0, pos = P + t - 1)
};

struct DecodeArgs {
  int32_t batch, n_q_heads, n_kv_heads, head_dim, group;
  int32_t capacity;       // C
  int32_t n_old;          // N before the append; the new entry goes to slot n_old
  int32_t t, prompt_len;
  int32_t chunk, n_split; // entries per split block, number of split blocks per unit
  int32_t n_split_max;    // stride of the partial arrays
  int32_t p_stride;       // row stride of p_tilde (C rounded up to a multiple of 4)
  int32_t variant;        // attention kernel actually launched: 0 vector ALU + merge,
                          // 4 fused MFMA, 6 fused MFMA leaving candidate lists (see TrackArgs)
  float   alpha, scale;
  int32_t dtype;
  const void *q, *k_new, *v_new;
  void *out;
  void *k_cache, *v_cache;          // this layer's slab
  int32_t *ts, *mri, *pos;          // this layer's slab
  float *p_out;
  const float *p_override;
  Workspace ws;
  unsigned long long *activation_counter;   // this layer's [units][slice_max] counters
  int32_t *ticket;                          // [units], zero between launches
  uint32_t seq;                             // fused kernel: number of this launch (never 0), the stamp of its records
  uint32_t spin_ticks;                      // fused kernel: longest wait for a record, in 10 ns ticks
  // fused kernel: where this call's logits and statistics go, and the previous call to track
  float *logits_out, *stat_out;
  TrackArgs track;
  Slots slots;                              // with slots: n_old is the largest of the sequences', t global
};

struct EvictArgs {
  int32_t units;          // units of the launch: batch * n_kv_heads, times the number of layers
                          // when consecutive layers (whose slabs follow one another) go together
  int32_t units_per_layer;  // batch * n_kv_heads
  int32_t head_dim, dtype;
  int32_t capacity;       // C
  int32_t n, budget, window, t;
  int32_t score_flags;
  void *k_cache, *v_cache;
  int32_t *ts, *mri, *pos;
  Workspace ws;
  unsigned long long *rows_moved;   // this layer's [units] counters
  // score = the last call's attention weights (score_flags bit 32): its logits and statistics
  const float *logits, *stat;
  int32_t group, p_stride;
  int32_t n_kv_heads;
  Slots slots;            // with slots: n is the largest of the due sequences', t global
  // with slots, when few sequences are due: only their units are launched.  Block index i then
  // stands for layer i / (n_due * n_kv_heads), due sequence (i / n_kv_heads) % n_due and KV head
  // i % n_kv_heads.  n_due = 0: one block per unit as usual.
  int32_t n_due;
  int32_t due_seq[8];
};

// The unit a block of an eviction launch works on.
__host__ __device__ inline int32_t evict_unit_of(const EvictArgs &a, int32_t i) {
  if (a.n_due <= 0) return i;
  const int32_t per_layer = a.n_due * a.n_kv_heads;
  const int32_t layer = i / per_layer, r = i % per_layer;
  return layer * a.units_per_layer + a.due_seq[r / a.n_kv_heads] * a.n_kv_heads + r % a.n_kv_heads;
}

// Tracking over the prompt (Alg. 1 first loop and Eq. 1 on the prompt's causal attention).
struct PrefillArgs {
  int32_t batch, n_q_heads, n_kv_heads, group;
  int32_t head_dim, dtype;          // 64 or 128; 0 fp32, 1 bf16
  int32_t capacity, prompt_len;
  int32_t p16;                      // positions per (unit, head) row of `stat`, >= prompt_len
  int32_t counter_stride;           // activation counters per unit
  float   alpha, scale;
  const void *q_prompt;             // [batch][prompt_len][n_q_heads][head_dim], the cache's type
  const void *k_cache;              // the layer's slab
  int32_t *ts, *mri;                // the layer's slab
  float *stat;                      // [units][group][p16]: -(log-sum-exp of the scaled logits) / scale per
                                    // (head, position), workspace
  float *p_out;                     // [batch][n_q_heads][prompt_len][prompt_len] or null
  const float *p_override;          // same shape or null
  unsigned long long *activation_counter;   // the layer's [units][counter_stride] or null
};
hipError_t launch_prefill_track(const PrefillArgs &a, hipStream_t stream);

// `ev`, when not null, points at three events recorded before the first kernel, between the two
// kernels and after the second (per-kernel timing for the profiling aid).
hipError_t launch_decode(const DecodeArgs &a, hipStream_t stream, hipEvent_t *ev);
// One launch per call: split blocks, the last block of a unit merges and tracks (bf16, d 128).
hipError_t launch_decode_fused(const DecodeArgs &a, hipStream_t stream, hipEvent_t *ev);
int decode_fused_split_max();
// Most sub-tiles of 16 entries one wave of a call with n_split blocks per unit takes, and how
// many of them a wave keeps in LDS at a time.
int decode_fused_wave_run(int n_sub, int n_split);
int decode_fused_run_max();
// Can a call with these sizes leave candidate lists (they fit the logits buffer, a wave's logits
// stay in LDS to the end of its run, and the 8th logit place is free for the entry index)?
bool decode_fused_compact_fits(int n_old, int n_split, int p_stride, int group);
int decode_fused_head_pad();
size_t decode_fused_record_bytes();           // one stamped record; a unit has 3
hipError_t launch_clear_records(unsigned long long *rec, size_t n_words, hipStream_t stream);
hipError_t launch_track(const TrackArgs &k, hipStream_t stream);
hipError_t launch_track_flush(const FlushArgs &f, int n_layers, hipStream_t stream);
int decode_fused_log_words_max();                // cache entries / 32 up to which the fused kernel can log
hipError_t launch_evict(const EvictArgs &a, hipStream_t stream, hipEvent_t *ev);
int evict_lds_candidates();   // candidates per unit whose keys the selection keeps in LDS
hipError_t launch_init_state(int32_t *ts, int32_t *mri, int32_t *pos, int64_t n_units,
                             int32_t capacity, int32_t prompt_len, hipStream_t stream);
// One sequence starts over: TS = 0, MRI = 0, pos = i for its first prompt_len entries in every layer.
hipError_t launch_init_slot(int32_t *ts, int32_t *mri, int32_t *pos, int32_t n_layers, int32_t batch,
                            int32_t n_kv_heads, int32_t capacity, int32_t seq, int32_t prompt_len,
                            int32_t *dev_prompt_len, int32_t *dev_t0, int32_t t0, hipStream_t stream);
hipError_t launch_mri_histogram(const int32_t *mri, int64_t n_units, int32_t capacity, int32_t n,
                                int32_t n_bins, unsigned long long *hist, hipStream_t stream);
// seq_len (device, [batch]): entries of each sequence, used instead of n when not null
hipError_t launch_mri_histogram_slots(const int32_t *mri, int64_t n_units, int32_t capacity,
                                      int32_t n_kv_heads, const int32_t *seq_len, int32_t n_max,
                                      int32_t n_bins, unsigned long long *hist, hipStream_t stream);
hipError_t launch_score_pairs(const int32_t *dt, const int32_t *mri, double *score, int64_t n,
                              int32_t flags, hipStream_t stream);

}  // namespace lazyev
