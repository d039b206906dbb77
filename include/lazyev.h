/*
 * lazyev -- decode-time hot path of LazyEviction (arXiv 2506.15969) for AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer is marked (host) or (device).  The library owns no device memory:
 * caches, statistics arrays and the workspace are allocated by the caller (for example as
 * torch tensors) and must stay valid until lazyev_destroy.  All calls enqueue work on the
 * stream given at init and return without waiting, except lazyev_stats and
 * lazyev_mri_histogram, which wait for it.
 * Calls on one context must come from one thread at a time.
 *
 * A "unit" is one (layer, sequence, KV head).  Each unit has its own cache of N entries
 * (N is the same for all units of a layer), its own recurrence statistics and its own
 * survivor set.  Notation of the paper: B budget, W observation window, alpha activation
 * threshold, t decode step (1-based), TS timestamp vector, MRI maximum recurrence interval.
 *
 * Layouts (row-major, C = lazyev_capacity(cfg) entries per unit):
 *   k_cache, v_cache   [n_layers][batch][n_kv_heads][C][head_dim]   fp32 or bf16
 *   ts, mri, pos       [n_layers][batch][n_kv_heads][C]             int32
 *   q, out             [batch][n_q_heads][head_dim]                 same dtype as the caches
 *   k_new, v_new       [batch][n_kv_heads][head_dim]
 *   p_out, p_override  [batch][n_q_heads][C]                        fp32
 * Query head h reads KV head h / (n_q_heads / n_kv_heads).
 */
#ifndef LAZYEV_H
#define LAZYEV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LAZYEV_OK          0
#define LAZYEV_EINVAL     -1   /* bad shape, null pointer, B <= W, step or layer out of order   */
#define LAZYEV_ECAPACITY  -2   /* decode_step on a full cache (a due eviction was skipped)        */
#define LAZYEV_EWORKSPACE -3   /* workspace missing or smaller than lazyev_workspace_size        */
#define LAZYEV_EHIP       -4   /* a HIP runtime call failed; lazyev_last_hip_error has the code  */
#define LAZYEV_ENOMEM     -5   /* host memory for the context or a read-back buffer ran out      */
#define LAZYEV_ESCRATCH   -6   /* lazyev_evict_static: the shape exceeds the library's static scratch */
#define LAZYEV_EEXCHANGE  -7   /* lazyev_stats: a block of an earlier decode call gave up waiting for
                                  another block's partial result; that call's outputs are invalid   */

#define LAZYEV_DTYPE_FP32  0
#define LAZYEV_DTYPE_BF16  1

#define LAZYEV_SCORE_H1    1   /* use the H1 term of Eq. 3 */
#define LAZYEV_SCORE_H2    2   /* use the H2 term of Eq. 3 */
/* With LAZYEV_SCORE_H2: use 1 - H2 (and 1 at MRI = 1, 0 at MRI = 0) in place of H2.  The H2 of
 * Sec. 4 item 2 as printed grows with MRI; the sentence introducing it and App. D describe a
 * term that falls with MRI.  Default is the printed formula; this bit selects the other reading. */
#define LAZYEV_SCORE_H2_DECREASING 16
/* Rank the candidates by the attention weight they received at the eviction's own step (largest
 * over the query group) instead of Eq. 3: the rule of the current-attention methods the paper
 * compares against (Sec. 2 (2); App. C "Baselines").  With window = 1 this is their per-step
 * greedy eviction, with a larger window the same rule behind an observation window.  Replaces
 * the H1 / H2 bits.  bf16, head_dim 128 only, and lazyev_evict must directly follow the
 * lazyev_decode_step of the same layer (the weights of older calls are gone). */
#define LAZYEV_SCORE_CURRENT_ATTENTION 32

/* Number of eviction candidates (cache entries outside the last W) per unit whose score keys
 * the selection kernel holds in LDS.  An eviction with more candidates (a prompt far beyond the
 * budget) ranks through the workspace instead: same result, slower selection. */
#define LAZYEV_LDS_CANDIDATES 8192

/* Largest number of bins of lazyev_mri_histogram. */
#define LAZYEV_MAX_HIST_BINS 8192

typedef struct lazyev_ctx lazyev_ctx;              /* opaque, host memory */

typedef struct {
  int32_t n_layers, batch, n_q_heads, n_kv_heads;  /* n_q_heads % n_kv_heads == 0, group <= 8 */
  int32_t head_dim;                                /* 64 or 128                                */
  int32_t budget, window, prompt_len;              /* B > W >= 1 (Sec. 4: B >> W); P >= 0      */
  float   alpha;                                   /* activation test is p >= alpha (Alg. 1)   */
  float   softmax_scale;                           /* 0 selects 1/sqrt(head_dim) (Eq. 4)       */
  int32_t dtype;                                   /* LAZYEV_DTYPE_*: storage of K, V, q, out  */
  int32_t score_flags;                             /* LAZYEV_SCORE_* bits (Table 4 ablation)   */
  void    *k_cache, *v_cache;                      /* (device) see layouts                     */
  int32_t *ts, *mri, *pos;                         /* (device) see layouts                     */
  void    *workspace;                              /* (device) scratch, 256-byte aligned       */
  size_t  workspace_bytes;
  void    *stream;                                 /* hipStream_t; NULL = the default stream   */
} lazyev_config;

typedef struct {
  int32_t  n_layers;            /* in: length of the arrays below                               */
  int32_t *len;                 /* (host, nullable) out: current N of each layer                 */
  int32_t *last_step;           /* (host, nullable) out: last decode step seen by each layer     */
  int64_t *n_evict_events;      /* (host, nullable) out: evictions that fired, per layer         */
  int64_t *n_evicted;           /* (host, nullable) out: entries removed per unit, summed over
                                   the layer's events (with per-sequence timing, where the due
                                   units of an event may differ: the largest per event)         */
  int64_t *n_activations;       /* (host, nullable) out: (entry, step) pairs with p >= alpha,
                                   summed over the layer's units                                */
  int64_t *n_rows_moved;        /* (host, nullable) out: surviving entries that an eviction moved
                                   to a lower slot, summed over the layer's units and events:
                                   each is one K row and one V row read and written             */
} lazyev_stats_t;

/* Entries of cache per unit: C = max(prompt_len, budget) + window.  0 if cfg is invalid. */
int32_t lazyev_capacity(const lazyev_config *cfg /*host*/);

/* Bytes of workspace the configuration needs (split partials, two buffers of per-entry logits,
 * gather lists, counters, tickets).  0 if cfg is invalid. */
size_t lazyev_workspace_size(const lazyev_config *cfg /*host*/);

/* Creates a context.  The caller has already written the prompt's K/V rows to entries
 * 0..P-1 of every unit.  Enqueues: TS = 0, MRI = 0, pos = i for those entries (the state a
 * token has "as if last important when prefill ended"; the paper starts MRI at 0, Sec. 4),
 * and clears the counters.  N = P for every layer.
 * Errors: EINVAL, EWORKSPACE, EHIP, ENOMEM. */
int lazyev_init(const lazyev_config *cfg /*host*/, lazyev_ctx **out /*host*/);

/* Optional start state from the prompt (the paper starts its clock at the first generated
 * token and is silent on the prompt): runs the tracking loop of Alg. 1 and Eq. 1 over the
 * prompt's own causal attention in `layer`.  Prompt position i (0-based, P positions) is the
 * query of step i + 1 - P <= 0 over the keys 0..i; entry i is born with TS = i + 1 - P, MRI = 0
 * and is updated by every later position whose probability for it reaches alpha in any head of
 * its group, exactly as a decode step would.  Decoding continues at step 1; the activations are
 * added to the layer's count.  Replaces the TS = 0, MRI = 0 that lazyev_init gave the prompt
 * entries; call it after lazyev_init and before the layer's first decode step.
 * q_prompt (device): [batch][P][n_q_heads][head_dim], the prompt's queries in the cache's dtype.
 * p_out / p_override (device, nullable): [batch][n_q_heads][P][P] fp32, row = query position,
 *   column = key; only the lower triangle (key <= query) is written / read; meaning as in
 *   lazyev_decode_step.
 * bf16 with head_dim 128 runs on the matrix cores; fp32 or head_dim 64 on a plain vector-ALU
 * path meant for small prompts.  Not with lazyev_admit / retire.
 * Errors: EINVAL (shape, order, null, P = 0), EHIP. */
int lazyev_prefill_track(lazyev_ctx *ctx, int32_t layer, const void *q_prompt /*device*/,
                         float *p_out /*device, nullable*/,
                         const float *p_override /*device, nullable*/);

/* The same for ONE sequence of a batch with per-sequence timing (lazyev_admit): the prompt of
 * slot `seq` (its prompt_len positions, rows already in the caches) is tracked on the slot's own
 * clock, position i as local step i + 1 - prompt_len.  Call it after lazyev_admit and before the
 * sequence's first decode step in `layer`.
 * q_prompt (device): [prompt_len][n_q_heads][head_dim]; p_out / p_override: [n_q_heads][P][P].
 * Errors: EINVAL (no per-sequence timing, empty slot or prompt, the sequence has decoded in the
 * layer, shape), EHIP. */
int lazyev_prefill_track_seq(lazyev_ctx *ctx, int32_t layer, int32_t seq, const void *q_prompt /*device*/,
                             float *p_out /*device, nullable*/,
                             const float *p_override /*device, nullable*/);

/* One decode step of one layer (Eq. 4; Alg. 1 tracking loop; Eq. 1):
 *   appends (k_new, v_new) as entry N with TS = t, MRI = 0, pos = P + t - 1;
 *   out[h] = softmax(scale * q[h] K^T) V over the N+1 entries of the head's unit;
 *   an entry is active if any query head of its group has probability >= alpha (fp32 compare);
 *   active entries get MRI = max(MRI, t - TS), then TS = t.
 * `out` and the appended K/V rows are complete when the call's work on the stream is.  The
 * single-launch attention kernel (see lazyev_set_variant) works out which entries were active
 * with the NEXT call on the context (any layer) and keeps that as one bit per entry; the updates
 * of ts / mri of a layer's calls are applied together, in the order of the calls, before
 * anything reads them: by lazyev_evict / lazyev_evict_all, lazyev_stats, lazyev_mri_histogram,
 * lazyev_admit / lazyev_retire, after at most min(W, 256) calls of the layer, and at once when
 * p_out or p_override is given.  A caller that reads ts / mri / pos itself calls lazyev_stats
 * first.
 * t must be the layer's previous step + 1 (first step is 1).
 * p_out (device, nullable): receives the fp32 probabilities the threshold test used, entries
 *   [0, N+1) of each row.
 * p_override (device, nullable): probabilities to threshold INSTEAD of the computed ones (the
 *   attention output is unaffected); lets a checker feed identical weights to two
 *   implementations.
 * Errors: EINVAL (order, range, null), ECAPACITY (N == C), EHIP. */
int lazyev_decode_step(lazyev_ctx *ctx, int32_t layer, int32_t t,
                       const void *q /*device*/, const void *k_new /*device*/,
                       const void *v_new /*device*/, void *out /*device*/,
                       float *p_out /*device, nullable*/,
                       const float *p_override /*device, nullable*/);

/* Lagged eviction check after decode step t of a layer (Sec. 4; Eq. 3; Eq. 6; Alg. 1):
 * does nothing unless t % W == 0 and N > B.  Otherwise every unit scores entries 0..N-W-1
 * with I = H1 + H2 in binary64, keeps the B-W best (ties: the more recent entry wins) and
 * the last W, and moves K, V, TS, MRI, pos of the survivors to entries 0..B-1 in their
 * original order.  N becomes B.
 * n_evicted (host, nullable): entries removed per unit (N - B, or 0).
 * t must equal the layer's last decode step.
 * Errors: EINVAL, EHIP. */
int lazyev_evict(lazyev_ctx *ctx, int32_t layer, int32_t t, int32_t *n_evicted /*host*/);

/* lazyev_evict for callers that must not allocate and cannot hand over a scratch area of their
 * own for this call: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and the same result as lazyev_evict; the one
 * difference is where the kernels' scratch buffer lives.  The selection kernel leaves a gather
 * list (source entry of every survivor, one int32 per cache entry of the layer's units) that the
 * row-move kernel then walks; lazyev_evict keeps it in the caller's workspace, this call keeps
 * it in a device array of LAZYEV_STATIC_SCRATCH_ENTRIES int32 (4 MiB) that is part of the
 * library image: every GPU the library runs on holds its own copy from load time until the
 * process ends.  The call allocates nothing, neither device nor host memory.
 * Limits: batch * n_kv_heads * capacity <= LAZYEV_STATIC_SCRATCH_ENTRIES and at most
 * LAZYEV_LDS_CANDIDATES candidates per unit (capacity - window); beyond them LAZYEV_ESCRATCH and
 * nothing is launched.  The device that was current at lazyev_init must be current (EINVAL).
 * All contexts of a process share one array per GPU and the array keeps the previous call's
 * list: nothing in it has to start at zero (a call overwrites every entry it later reads), but
 * two such calls whose kernels overlap on one GPU (different streams) race.  The per-layer
 * counters lazyev_stats reports stay in the caller's workspace.
 * Errors: those of lazyev_evict, ESCRATCH. */
#define LAZYEV_STATIC_SCRATCH_ENTRIES (1 << 20)
int lazyev_evict_static(lazyev_ctx *ctx, int32_t layer, int32_t t, int32_t *n_evicted /*host*/);

/* The same check (Sec. 4 "MRI-Centric Eviction"; Eq. 3; Eq. 6; the eviction branch of Alg. 1)
 * for EVERY layer after decode step t (every layer must have taken step t).  The paper states
 * Alg. 1 for one attention module; the modules of a model are independent of one another.
 * Where the layers stand at the same point, which is the normal course of a model, the
 * selection and the row move of all layers go in one launch each (the units of different
 * layers are independent); otherwise this is lazyev_evict layer by layer.  Results are those
 * of the per-layer calls.  n_evicted: entries removed per unit of a layer (the largest, if the
 * layers differ).  Errors: those of lazyev_evict. */
int lazyev_evict_all(lazyev_ctx *ctx, int32_t t, int32_t *n_evicted /*host*/);

/* The bookkeeping of Alg. 1 as the host sees it: cache length per layer (the saw-tooth of
 * Fig. 6: at most B + W entries, exactly B after an eviction, Sec. 4 / Eq. 6), evictions that
 * fired, entries removed, activations (entries with A_t[i] >= alpha, first loop of Alg. 1) and
 * rows the compaction moved.  Applies any tracking still pending, waits for the stream, then
 * fills the non-null arrays of *out.  The TS / MRI / pos arrays themselves belong to the caller,
 * who reads them directly after this call (there is no copy-out argument).
 * Errors: EINVAL, EHIP, ENOMEM; EEXCHANGE when a decode call since the last lazyev_stats could
 * not complete its exchange between blocks (not expected on a working GPU; reported once). */
int lazyev_stats(lazyev_ctx *ctx, lazyev_stats_t *out /*host*/);

/* Per-sequence timing, for a batch whose sequences do not start together (the paper decodes one
 * sequence at a time and says nothing about batches; what follows applies Alg. 1 to every
 * sequence on its own clock).  Until the first of these two calls every sequence has the
 * configuration's prompt_len and starts at step 1.
 *
 * lazyev_admit: batch slot `seq` is taken by a sequence whose prompt_len K/V rows the caller
 *   has written (or will have written, on the context's stream, before the sequence's first
 *   step) to entries 0..prompt_len-1 of the slot's units in every layer.  Its first decode step
 *   is the call with t = t0 + 1; every quantity of Alg. 1 then runs on the sequence's local
 *   step t - t0: TS, the W-step schedule, pos = prompt_len + local step - 1.  Enqueues the
 *   state of lazyev_init for the slot in every layer.  A slot that is already taken starts over.
 *   Needs prompt_len <= capacity - window and t0 >= every layer's last decode step.
 * lazyev_retire: the slot is empty from now on: its units take no part in later calls (their
 *   output rows are not written) until it is admitted again.
 *
 * With per-sequence timing in use: lazyev_decode_step skips sequences whose first step lies
 * ahead; lazyev_evict runs for the sequences whose local step is a multiple of W and whose cache
 * exceeds the budget (n_evicted: the largest number removed from one unit) and must be called
 * after every step at which that holds for some sequence (the next lazyev_decode_step of the
 * layer returns ECAPACITY otherwise); lazyev_stats reports the longest cache of each layer.
 * bf16, head_dim 128 and the default attention kernel only.
 * A caller that wants the prompt itself tracked (TS / MRI from the prompt's own attention, and
 * eviction while a prompt longer than the budget is read) admits the sequence with prompt_len 0
 * and feeds the prompt tokens as decode steps.
 * Both apply pending tracking first.  Errors: EINVAL, EHIP. */
int lazyev_admit(lazyev_ctx *ctx, int32_t seq, int32_t prompt_len, int32_t t0);
/* Entries a sequence holds before the append of its local step (>= 1) when every due eviction has
 * run: the closed form host and kernels share (a due eviction leaves exactly `budget` entries,
 * Sec. 4 / Eq. 6, so the length depends on nothing else).  Host only.  -1 for bad arguments. */
int32_t lazyev_cached_before_step(int32_t prompt_len, int32_t local_step, int32_t budget, int32_t window);
int lazyev_retire(lazyev_ctx *ctx, int32_t seq);

/* Distribution of the Maximum Recurrence Interval (Eq. 1) over the cached entries, the
 * statistic from which the observation window W is chosen offline (Sec. 3, Fig. 2(c); Sec. 4
 * "Observation Window": W = the MRI below which 80 % of the tokens fall; run it on a context
 * whose budget covers the whole generation so that no token has been evicted).
 * hist[m] = number of entries 0..N-1, over all units of `layer` (-1: of every layer), whose MRI
 * is m, for m < n_bins - 1; hist[n_bins - 1] counts MRI >= n_bins - 1.  hist[0] are the entries
 * never re-activated since they were appended.
 * Applies any tracking still pending and waits for the stream.
 * Errors: EINVAL (2 <= n_bins <= LAZYEV_MAX_HIST_BINS, layer range, null), EHIP, ENOMEM. */
int lazyev_mri_histogram(lazyev_ctx *ctx, int32_t layer, int32_t n_bins, int64_t *hist /*host*/);

/* Observation window from such a histogram (Sec. 4 "Observation Window": W is set to the MRI
 * below which 80 % of the tokens fall): over the entries that were re-activated at least once
 * (MRI >= 1; an entry with MRI = 0 never recurred), the smallest W with at least `quantile` of
 * them at MRI <= W.  *window = 0 if no entry was ever re-activated; an answer of n_bins - 1 means
 * the histogram was too short.  Host arithmetic only, no GPU work.
 * Errors: EINVAL (null, n_bins < 2, quantile outside (0, 1], a negative count). */
int lazyev_window_from_histogram(const int64_t *hist /*host*/, int32_t n_bins, double quantile,
                                 int32_t *window /*host*/);

/* Score of Eq. 3 for n (t - TS, MRI) pairs, on the device, with the same code the eviction
 * uses; result as binary64.  For checking the scoring arithmetic in isolation.
 * Errors: EINVAL, EHIP. */
int lazyev_score_pairs(const int32_t *delta_t /*device*/, const int32_t *mri /*device*/,
                       double *score /*device*/, int64_t n, int32_t score_flags,
                       void *stream);

void lazyev_destroy(lazyev_ctx *ctx);              /* frees host memory only; NULL is allowed */
const char *lazyev_strerror(int code);
int lazyev_last_hip_error(const lazyev_ctx *ctx);  /* hipError_t of the last EHIP, else 0 */

#ifdef __cplusplus
}
#endif
#endif /* LAZYEV_H */
