// Decode step of one layer in ONE launch (bf16, head_dim 128): append, attention (Eq. 4 of the
// paper) and, one call behind, the recurrence tracking of Alg. 1 / Eq. 1.
//
// A unit's cache is cut into 16-entry sub-tiles, dealt to the 4 * n_split stream waves of the
// unit's n_split blocks in turn (fused_wave_map: the waves of a unit read one moving window of the
// cache together, which keeps DRAM pages open).  Per sub-tile a wave
//   loads      K and V as whole 256-byte rows (16 lanes per row), non-temporal; the next
//              sub-tile is requested while the current one is multiplied, the first one from the
//              arguments a wave is handed in registers, before the argument block is read
//   K layout   K rows go through a wave-private LDS area to reach the MFMA operand layout
//   S^T = K Q^T   v_mfma_f32_16x16x32_bf16, the G query rows padded to 16 columns
//   logits     scaled logits are kept in LDS as [entry][8 heads]; what the tracking needs of
//              them goes to the workspace when the wave's run ends (a store among the loads
//              would hold up the in-order load counter)
//   softmax    per wave: reference maximum m, sum l, output accumulator O.  The reference is
//              raised only when a logit exceeds it by more than 8, so rescaling O is rare;
//              exp(s - m) <= e^8 stays far from overflow
//   O += P V   v_mfma_f32_16x16x16_bf16 after an in-lane 4x8 transpose of the V rows
// The four stream waves of a block merge their (m, l, O) in LDS into one partial per block.
// What follows the stream is serial code of single waves, where instructions, not bytes, set
// the time: no branches where a select does, addresses worked out beforehand.
//
// Partials of a unit.  One block: its partial is the result.  2 .. 4 blocks (the usual split):
// the unit's last block finishes the unit, the others hand it their partial as a record of
// stamped 64-bit words (see "hand-over" below): no acknowledgement is waited for, nothing is
// signalled, one memory round trip.  More blocks: partials are published with device-scope
// stores, and the block that takes the LAST ticket of its unit (a counter in the workspace,
// taken after the block's stores have completed) merges them; the ticket resets itself.  In all
// cases the partials are merged in block order, and the finishing block leaves the unit's
// softmax statistics (max, 1 / sum per head) for the tracking.
//
// Tracking.  The activation test of Alg. 1 needs p = exp(s - m) / l with the statistics of the
// WHOLE unit, which exist only when the unit's last block is done.  Doing it there puts a
// chain of dependent memory round trips at the end of every launch, so it is deferred: the
// NEXT launch carries, behind its stream blocks, as many tracking blocks (spread over the
// compute units the same way) that apply the previous call's tracking from the stored logits
// and statistics (>= alpha test over the query group, TS / MRI update, start of the appended
// entry) while the new call streams; lazyev_evict and lazyev_stats apply what is pending
// through track_kernel.  Logits and statistics are double-buffered.
// In a uniform batch the tracking blocks do not touch TS / MRI themselves (a 128-byte line read
// and written for every 4-byte word of an active entry, beside the stream): they leave one bit
// per cache entry in the layer's activation log, and track_flush_kernel applies the logged calls
// in step order before anything reads TS / MRI (TrackArgs::bitlog).
//
// Candidate lists (kernel instances <true, ..>, groups of at most 7 heads; every call whose
// logits nobody reads as such).  A block knows, once its four stream waves are done, its own
// share of every head's softmax denominator, which bounds the
// true denominator from below: an entry whose weight relative to the BLOCK's denominator
// stays under alpha in every head cannot reach alpha.  The block then writes only the other
// entries ("candidates", about a tenth on the benchmark workloads; the appended entry always)
// as records (7 logits, entry index) into its own region of the logits buffer, and the
// tracking applies the exact test to the records: the same state bit for bit.  A wave whose run
// is longer than the sub-tiles it keeps in LDS (instances <true, true, ..>) writes the candidates
// of every full segment while it streams, with the cut that the block's waves' running sums give
// at that moment, and only the last segment after the stream.  Where all blocks of the launch
// fit the chip at once with eight waves each (instances <.., .., true>), four more waves per
// block ("list waves") sleep through the stream and build the lists beside the merge.
//
// MFMA operand layouts (lane l, c = l % 16, g = l / 16):
//   16x16x32: A[row c][k = 8g..8g+7]  B[k = 8g..8g+7][col c]  C[row 4g+i][col c]
//   16x16x16: A[row c][k = 4g..4g+3]  B[k = 4g..4g+3][col c]  C[row 4g+i][col c]
// so a lane that owns head c and entries 4g..4g+3 of a sub-tile after the first product already
// holds the A operand of the second.
#include "kernels.h"

#include <type_traits>

namespace lazyev {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int D = 128;
constexpr int KC = D / 32;
constexpr int kFusedSplitMax = 64;      // blocks per unit
constexpr float kRaise = 8.0f;          // the reference maximum moves when exceeded by this much
constexpr int kTrackRows = 3;           // entries per thread per tracking batch
constexpr int kHeadPad = 8;             // logits and statistics are stored for 8 heads per unit
constexpr int kRunMax = 20;             // sub-tiles whose logits a wave keeps in LDS (10 KB) before it writes them out
// How a unit's n_sub sub-tiles of 16 entries are dealt to the kWaves * n_split waves of its
// n_split blocks: wave wv (= kWaves * (n_split - 1 - split) + wave) takes wv, wv + kWaves * n_split,
// ..., so the waves of a unit read one moving window of the cache together (measured against a
// region of consecutive sub-tiles per block: 28.6 against 29.2 us per call on the 2048-entry
// workload).  The unit's LAST block comes first in that order: when the sub-tiles do not divide
// evenly its waves take the longer runs, and it is the block that finishes a unit of 2..4 blocks,
// so the other blocks' partials are on their way while it still streams.
struct WaveMap { int first, step, cnt; };
__host__ __device__ inline WaveMap fused_wave_map(int n_sub, int n_split, int split, int wave) {
  WaveMap m;
  m.first = (n_split - 1 - split) * kWaves + wave;
  m.step = kWaves * n_split;
  m.cnt = m.first < n_sub ? (n_sub - m.first + m.step - 1) / m.step : 0;
  return m;
}
// Most sub-tiles one wave takes.
__host__ __device__ inline int fused_wave_run(int n_sub, int n_split) {
  return (n_sub + kWaves * n_split - 1) / (kWaves * n_split);
}

#ifdef LAZYEV_TIMELINE
// Measuring build only (liblazyev_timeline.so, see build.py): every block of the LAST launch
// leaves time stamps of the constant 100 MHz counter: 0 block start, 1 first sub-tile multiplied,
// 2 end of wave 0's stream, 3 all four waves done, 4 ticket taken, 5 block end; word 6: the XCD the
// block ran on (hardware register XCC_ID); word 7: 1 if the block finished its unit.  Read with
// lazyev_timeline_read.
__device__ unsigned long long lz_stamp[2048 * 8];
#define STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x < 2048) lz_stamp[blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
#define STAMPV(i, v) do { if (threadIdx.x == 0 && blockIdx.x < 2048) lz_stamp[blockIdx.x * 8 + (i)] = (v); } while (0)
__device__ inline unsigned long long xcc_id() {
  unsigned x;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
  return x & 15u;
}
#else
#define STAMP(i) do {} while (0)
#define STAMPV(i, v) do {} while (0)
#endif

typedef unsigned short bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2_t;

__device__ __forceinline__ bf16_t float_to_bf16(float f) {   // round to nearest even
  unsigned u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}

// x + (x of lane ^ 16) + (the same of lane ^ 32), and the maximum likewise: the sum / maximum over
// the four lanes c, c + 16, c + 32, c + 48.  v_permlane16_swap / v_permlane32_swap exchange 16-
// and 32-lane halves between two registers in the vector ALU; applied to two copies of x they
// leave the two summands of every lane side by side (same pairs, same roundings as the
// shuffles through the LDS crossbar they replace, which cost a wave a round trip each).
__device__ __forceinline__ float sum_over_lane_groups(float x) {
  auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float max_over_lane_groups(float x) {
  auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// K and V rows of one sub-tile as a wave holds them: 4 + 4 loads of 16 bytes per lane.
struct SubTile {
  u32x4_t k[KC];
  u32x4_t v[4];
};

// What one block writes for another block of the SAME launch to read (the partials) is
// stored at device ("agent") scope: the stores write through the XCD-local L2, so no whole-cache
// write-back is needed to publish them.  Publishing is: every wave waits until its stores have
// completed (wait_own_stores), the block barrier, then one relaxed device-scope atomic on the
// unit's ticket.  The block that takes the last ticket reads the partials with device-scope loads
// (which do not use possibly stale cached copies); a cache-invalidating acquire fence followed
// by ordinary loads measured five times slower.
// Waits until every global store (and load) this wave has issued is complete.  A block barrier
// alone does not: the compiler only drains the LDS counter before s_barrier.
__device__ __forceinline__ void wait_own_stores() {
  __asm__ volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0); expcnt and lgkmcnt untouched
  __asm__ volatile("" ::: "memory");
}

__device__ __forceinline__ void store_f32_device(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_f32_device(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ----------------------------------------------------------------------------- tracking
// Alg. 1 (first loop) and Eq. 1 for a share of one unit of a finished decode call:
// probabilities from the stored logits and statistics, >= alpha over the query group, TS / MRI
// update, start of the appended entry.  Part `part` of `n_parts` takes the entries
// track_entry(part, n_parts, r), r = 0, 1, ...
struct TrackBatch {
  float4 sa[kTrackRows], sb[kTrackRows];
};

// Entry that thread `tid` of part `part` (of n_parts) handles in round r: the parts own the
// 16-entry sub-tiles exactly as the stream blocks of a launch with n_parts blocks per unit do
// (fused_wave_map), so a tracking block that runs on the XCD of the stream block with the same
// index finds the logits that block wrote in its L2.  Beyond the part's share: a number no
// cache reaches.
__device__ __forceinline__ int track_entry(int n_sub, int part, int n_parts, int r) {
  const int j = r * (kBlock / 16) + (static_cast<int>(threadIdx.x) >> 4);   // wave j % kWaves, its sub-tile j / kWaves
  const WaveMap m = fused_wave_map(n_sub, n_parts, part, j % kWaves);
  const int it = j / kWaves;
  return it < m.cnt ? (m.first + it * m.step) * 16 + (static_cast<int>(threadIdx.x) & 15) : 0x7FFFFFF0;
}
// Rounds of kBlock entries that cover the largest part.
__device__ __forceinline__ int track_rounds(int n_sub, int n_parts) {
  return (kWaves * fused_wave_run(n_sub, n_parts) + kBlock / 16 - 1) / (kBlock / 16);
}

__device__ __forceinline__ void track_load(const TrackArgs &k, int unit, int part, int n_parts, int r0,
                                           TrackBatch &b) {
  const float *lg = k.logits + static_cast<size_t>(unit) * k.p_stride * kHeadPad;
  const int n1 = k.n_old + 1;
  const int n_sub = (n1 + 15) >> 4;
#pragma unroll
  for (int r = 0; r < kTrackRows; ++r) {
    const int i = track_entry(n_sub, part, n_parts, r0 + r);
    b.sa[r] = b.sb[r] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < n1) {
      b.sa[r] = *reinterpret_cast<const float4 *>(lg + static_cast<size_t>(i) * kHeadPad);
      b.sb[r] = *reinterpret_cast<const float4 *>(lg + static_cast<size_t>(i) * kHeadPad + 4);
    }
  }
}

// The activation test and the TS / MRI update of entry i (Alg. 1, Eq. 1); true if active.
// log_mask (LDS, or null): the call is logged; an active entry then only sets its bit there.
__device__ __forceinline__ bool track_one(const TrackArgs &k, int unit, int i, const float (&s)[kHeadPad],
                                          const float (&m)[kHeadPad], const float (&invl)[kHeadPad],
                                          unsigned *log_mask) {
  const int seq = unit / k.n_kv_heads, kvh = unit % k.n_kv_heads;
  const int G = k.group;
  const size_t head0 = static_cast<size_t>(seq) * k.n_q_heads + static_cast<size_t>(kvh) * G;
  int32_t *ts = k.ts + static_cast<size_t>(unit) * k.capacity;
  int32_t *mri = k.mri + static_cast<size_t>(unit) * k.capacity;
  bool act = false;
#pragma unroll
  for (int h = 0; h < kHeadPad; ++h) {
    if (h < G) {
      float p = __expf(s[h] - m[h]) * invl[h];
      const size_t at = (head0 + h) * k.capacity + i;
      if (k.p_out) k.p_out[at] = p;
      if (k.p_override) p = k.p_override[at];
      act = act || (p >= k.alpha);
    }
  }
  if (i == k.n_old) {                              // the appended entry starts here (Sec. 4)
    if (!log_mask) {                               // (of a logged call: when the log is applied)
      ts[i] = k.t;
      mri[i] = 0;
      k.pos[static_cast<size_t>(unit) * k.capacity + i] = k.prompt_len + k.t - 1;
    }
  } else if (act) {                                // few entries are active: TS / MRI are read only here
    if (log_mask) {
      atomicOr(log_mask + (i >> 5), 1u << (i & 31));
    } else {
      const int32_t gap = k.t - ts[i];
      if (gap > mri[i]) mri[i] = gap;              // Eq. 1
      ts[i] = k.t;                                 // Alg. 1
    }
  }
  return act;
}

__device__ __forceinline__ unsigned track_apply(const TrackArgs &k, int unit, int part, int n_parts,
                                                int r0, const TrackBatch &b, const float (&m)[kHeadPad],
                                                const float (&invl)[kHeadPad], unsigned *log_mask) {
  const int seq = unit / k.n_kv_heads, kvh = unit % k.n_kv_heads;
  const int G = k.group;
  const int n_old = k.n_old, n1 = k.n_old + 1;
  const int n_sub = (n1 + 15) >> 4;
  const size_t head0 = static_cast<size_t>(seq) * k.n_q_heads + static_cast<size_t>(kvh) * G;
  int32_t *ts = k.ts + static_cast<size_t>(unit) * k.capacity;
  int32_t *mri = k.mri + static_cast<size_t>(unit) * k.capacity;
  unsigned n_act = 0;
#pragma unroll
  for (int r = 0; r < kTrackRows; ++r) {
    const int i = track_entry(n_sub, part, n_parts, r0 + r);
    if (i >= n1) continue;
    const float s[kHeadPad] = {b.sa[r].x, b.sa[r].y, b.sa[r].z, b.sa[r].w,
                               b.sb[r].x, b.sb[r].y, b.sb[r].z, b.sb[r].w};
    bool act = false;
#pragma unroll
    for (int h = 0; h < kHeadPad; ++h) {
      if (h < G) {
        float p = __expf(s[h] - m[h]) * invl[h];
        const size_t at = (head0 + h) * k.capacity + i;
        if (k.p_out) k.p_out[at] = p;
        if (k.p_override) p = k.p_override[at];
        act = act || (p >= k.alpha);
      }
    }
    if (i == n_old) {                              // the appended entry starts here (Sec. 4)
      if (!log_mask) {                             // (of a logged call: when the log is applied)
        ts[i] = k.t;
        mri[i] = 0;
        k.pos[static_cast<size_t>(unit) * k.capacity + i] = k.prompt_len + k.t - 1;
      }
    } else if (act) {                              // few entries are active: TS / MRI are read only here
      if (log_mask) {
        atomicOr(log_mask + (i >> 5), 1u << (i & 31));
      } else {
        const int32_t gap = k.t - ts[i];
        if (gap > mri[i]) mri[i] = gap;            // Eq. 1
        ts[i] = k.t;                               // Alg. 1
      }
    }
    n_act += act ? 1u : 0u;
  }
  return n_act;
}

// Slots of a block's region of candidate records in a call with n_parts blocks per unit: one
// for the count and one for each entry the block can own.
__host__ __device__ inline int fused_part_cap(int n_old, int n_parts) {
  const int n_sub = (n_old + 1 + 15) >> 4;
  return fused_wave_run(n_sub, n_parts) * (kWaves * 16) + 1;
}

// Tracking from the candidate records of the call's blocks b = part, part + step, ...
__device__ __forceinline__ unsigned track_records(const TrackArgs &k, int unit, int part, int step,
                                                  const float (&m)[kHeadPad], const float (&invl)[kHeadPad],
                                                  unsigned *log_mask) {
  const int cap = fused_part_cap(k.n_old, k.n_parts);
  unsigned n_act = 0;
  for (int b = part; b < k.n_parts; b += step) {
    const float *region = k.logits + (static_cast<size_t>(unit) * k.p_stride + static_cast<size_t>(b) * cap) * kHeadPad;
    const int n = *reinterpret_cast<const int32_t *>(region);
    for (int r = threadIdx.x; r < n; r += kBlock) {
      const float4 sa = *reinterpret_cast<const float4 *>(region + static_cast<size_t>(1 + r) * kHeadPad);
      const float4 sb = *reinterpret_cast<const float4 *>(region + static_cast<size_t>(1 + r) * kHeadPad + 4);
      const float s[kHeadPad] = {sa.x, sa.y, sa.z, sa.w, sb.x, sb.y, sb.z, 0.f};
      n_act += track_one(k, unit, __float_as_int(sb.w), s, m, invl, log_mask) ? 1u : 0u;
    }
  }
  return n_act;
}

// With per-sequence timing: the call's arguments as they hold for one unit (its own cache length,
// local step and prompt length).  False: the unit's sequence takes no part in that call.
__device__ __forceinline__ bool track_for_unit(const TrackArgs &k, int unit, TrackArgs &ku) {
  ku = k;
  if (!k.slots.prompt_len) return true;
  const int seq = unit / k.n_kv_heads;
  const int32_t P = k.slots.prompt_len[seq], tau = k.t - k.slots.t0[seq];
  if (P < 0 || tau < 1) return false;
  ku.n_old = slot_n_old(P, tau, k.slots.budget, k.slots.window);
  ku.t = tau;
  ku.prompt_len = P;
  return true;
}

__device__ __forceinline__ void track_stats(const TrackArgs &k, int unit, float (&m)[kHeadPad],
                                            float (&invl)[kHeadPad]) {
  const float *st = k.stat + static_cast<size_t>(unit) * (2 * kHeadPad);
#pragma unroll
  for (int h = 0; h < kHeadPad; ++h) { m[h] = st[2 * h]; invl[h] = st[2 * h + 1]; }
}

// Adds up the block's activation count; every (unit, part) owns one counter slot.
__device__ void track_count(const TrackArgs &k, int unit, int part, unsigned n_act, unsigned *cnt_lds) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int o = 32; o > 0; o >>= 1) n_act += __shfl_xor(n_act, o);
  if (lane == 0) cnt_lds[wave] = n_act;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned total = 0;
    for (int w = 0; w < kWaves; ++w) total += cnt_lds[w];
    if (total) k.activation_counter[unit * 64 + part] += total;
  }
}

// Tracking alone (lazyev_evict, lazyev_stats, or a caller that wants the weights at once).
__global__ __launch_bounds__(kBlock) void track_kernel(const TrackArgs k_all, int n_parts) {
  __shared__ unsigned cnt_lds[kWaves];
  const int unit = blockIdx.x / n_parts, part = blockIdx.x % n_parts;
  TrackArgs k;
  if (!track_for_unit(k_all, unit, k)) return;
  float m[kHeadPad], invl[kHeadPad];
  track_stats(k, unit, m, invl);
  unsigned n_act = 0;
  if (k.compact) {
    n_act = track_records(k, unit, part, n_parts, m, invl, nullptr);
  } else {
    const int rounds = track_rounds((k.n_old + 1 + 15) >> 4, n_parts);
    for (int r0 = 0; r0 < rounds; r0 += kTrackRows) {
      TrackBatch b;
      track_load(k, unit, part, n_parts, r0, b);
      n_act += track_apply(k, unit, part, n_parts, r0, b, m, invl, nullptr);
    }
  }
  track_count(k, unit, part, n_act, cnt_lds);
}

// The logged calls of a layer applied to TS / MRI: one thread per cache entry, the calls in step
// order.  An entry's bit in the words of a call says that it was active there (TrackArgs::bitlog).
// Block b works on the kFlushSpan entries from kFlushSpan * (b % spans) on of unit (b / spans) % units
// of layer b / spans / units, spans = blocks per unit.  The span's 32 words of every logged call
// go to LDS first (all requested together: one memory round trip), then every thread walks the
// calls for its four entries.
constexpr int kFlushSpan = 4 * kBlock;
__global__ __launch_bounds__(kBlock) void track_flush_kernel(const FlushArgs f) {
  __shared__ uint32_t lw[kLogSlotsMax * (kFlushSpan / 32)];
  __shared__ int32_t lt[kLogSlotsMax];             // the calls' steps (an indexed read of the argument block costs a scalar load each time)
  __shared__ int32_t lo[kLogSlotsMax];             // the entries the calls appended
  constexpr int kSpanWords = kFlushSpan / 32;
  const int spans = (f.capacity + kFlushSpan - 1) / kFlushSpan;
  const int span = blockIdx.x % spans, lu = blockIdx.x / spans;
  const int layer = lu / f.units, unit = lu % f.units;
  const size_t slab = (static_cast<size_t>(layer) * f.units + unit) * f.capacity;
  const uint32_t *log = f.bitlog + (static_cast<size_t>(layer) * f.units + unit) * f.log_slots * f.log_words +
                        span * kSpanWords;           // (a unit's slots lie together: a stream of n_calls * log_words words)
  const size_t slot_stride = static_cast<size_t>(f.log_words);
  const int n_words = min(kSpanWords, f.log_words - span * kSpanWords);
  for (int x = threadIdx.x; x < f.n_calls * kSpanWords; x += kBlock) {
    const int s = x / kSpanWords, j = x % kSpanWords;
    lw[x] = j < n_words ? log[s * slot_stride + j] : 0u;
  }
  for (int s = threadIdx.x; s < f.n_calls; s += kBlock) { lt[s] = f.t[s]; lo[s] = f.n_old[s]; }
  int32_t ts[4], mri[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {                    // (requested while the words travel)
    const int i = span * kFlushSpan + e * kBlock + static_cast<int>(threadIdx.x);
    ts[e] = mri[e] = 0;
    if (i < f.capacity) { ts[e] = f.ts[slab + i]; mri[e] = f.mri[slab + i]; }
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int il = e * kBlock + static_cast<int>(threadIdx.x), i = span * kFlushSpan + il;
    if (i >= f.capacity) continue;
    const uint32_t *w = lw + (il >> 5);
    bool touched = false;
    const int sh = il & 31;
    // An entry that one of the calls appended starts there (Sec. 4): no earlier call has a bit for
    // it, so it is started before the bits are walked.  (Calls of consecutive steps append
    // consecutive entries: the first guess is right unless steps were left out.)
    {
      int s_new = i - lo[0];
      if (s_new < 0 || s_new >= f.n_calls || lo[s_new] != i) {
        s_new = -1;
        if (i >= lo[0] && i <= lo[f.n_calls - 1])
          for (int s = 0; s < f.n_calls; ++s) s_new = lo[s] == i ? s : s_new;
      }
      if (s_new >= 0) {
        ts[e] = lt[s_new];
        mri[e] = 0;
        f.pos[slab + i] = f.prompt_len + lt[s_new] - 1;
        touched = true;
      }
    }
    for (int s0 = 0; s0 < f.n_calls; s0 += 32) {   // 32 calls at a time: in which of them was the entry active?
      unsigned calls = 0;
      const int n32 = min(32, f.n_calls - s0);
#pragma unroll
      for (int d = 0; d < 32; ++d)                 // (no branch in here: the LDS reads overlap; reads beyond the
        calls |= ((w[min(s0 + d, f.n_calls - 1) * kSpanWords] >> sh) & 1u) << d;   // last call repeat it and are masked)
      calls &= n32 == 32 ? ~0u : (1u << n32) - 1u;
      while (calls) {                              // ... and those, in step order
        const int s = s0 + __builtin_ctz(calls);
        calls &= calls - 1;
        const int32_t t_s = lt[s];
        const int32_t gap = t_s - ts[e];
        if (gap > mri[e]) mri[e] = gap;            // Eq. 1
        ts[e] = t_s;                               // Alg. 1
        touched = true;
      }
    }
    if (touched) { f.ts[slab + i] = ts[e]; f.mri[slab + i] = mri[e]; }
  }
}

// --------------------------------------------------------------------- last block of a unit
// A block's partial as another block reads it: four consecutive output elements (one head) and
// that head's (max, sum).  The loads are device-scope (sc1) like load_f32_device, but 16 bytes
// wide, which the atomic builtins do not offer; one asm statement issues all loads of a group
// and waits for them, so no register is touched while a load is still in flight.
template <int GW>
struct PartialGroup {
  f32x4_t o[GW];
  float m[GW], l[GW];
};

__device__ __forceinline__ void load_partials(PartialGroup<2> &g, const float *const (&po)[2],
                                              const float *const (&pm)[2], const float *const (&pl)[2]) {
  __asm__ volatile(
      "global_load_dwordx4 %0, %6, off sc1\n"
      "global_load_dwordx4 %1, %7, off sc1\n"
      "global_load_dword %2, %8, off sc1\n"
      "global_load_dword %3, %9, off sc1\n"
      "global_load_dword %4, %10, off sc1\n"
      "global_load_dword %5, %11, off sc1\n"
      "s_waitcnt vmcnt(0)\n"
      : "=&v"(g.o[0]), "=&v"(g.o[1]), "=&v"(g.m[0]), "=&v"(g.m[1]), "=&v"(g.l[0]), "=&v"(g.l[1])
      : "v"(po[0]), "v"(po[1]), "v"(pm[0]), "v"(pm[1]), "v"(pl[0]), "v"(pl[1])
      : "memory");
}

__device__ __forceinline__ void load_partials(PartialGroup<4> &g, const float *const (&po)[4],
                                              const float *const (&pm)[4], const float *const (&pl)[4]) {
  __asm__ volatile(
      "global_load_dwordx4 %0, %12, off sc1\n"
      "global_load_dwordx4 %1, %13, off sc1\n"
      "global_load_dwordx4 %2, %14, off sc1\n"
      "global_load_dwordx4 %3, %15, off sc1\n"
      "global_load_dword %4, %16, off sc1\n"
      "global_load_dword %5, %17, off sc1\n"
      "global_load_dword %6, %18, off sc1\n"
      "global_load_dword %7, %19, off sc1\n"
      "global_load_dword %8, %20, off sc1\n"
      "global_load_dword %9, %21, off sc1\n"
      "global_load_dword %10, %22, off sc1\n"
      "global_load_dword %11, %23, off sc1\n"
      "s_waitcnt vmcnt(0)\n"
      : "=&v"(g.o[0]), "=&v"(g.o[1]), "=&v"(g.o[2]), "=&v"(g.o[3]), "=&v"(g.m[0]), "=&v"(g.m[1]),
        "=&v"(g.m[2]), "=&v"(g.m[3]), "=&v"(g.l[0]), "=&v"(g.l[1]), "=&v"(g.l[2]), "=&v"(g.l[3])
      : "v"(po[0]), "v"(po[1]), "v"(po[2]), "v"(po[3]), "v"(pm[0]), "v"(pm[1]), "v"(pm[2]),
        "v"(pm[3]), "v"(pl[0]), "v"(pl[1]), "v"(pl[2]), "v"(pl[3])
      : "memory");
}

// Running merge of partials in block order.  Every product and sum is written out with its
// rounding (no contraction left to the compiler), so that all kernel instances produce the same
// bits from the same partials.
struct Merge {
  float m = -INFINITY, l = 0.f;
  float o[4] = {0.f, 0.f, 0.f, 0.f};
  __device__ __forceinline__ void fold(float mj, float lj, const f32x4_t &oj) {
#pragma clang fp contract(off)
    const float m_new = fmaxf(m, mj);
    // a block without entries has max = -inf, sum = 0, values = 0: its factor is 0
    const float fr = m == -INFINITY ? 0.f : __expf(m - m_new);
    const float fj = mj == -INFINITY ? 0.f : __expf(mj - m_new);
    l = fmaf(l, fr, lj * fj);
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = fmaf(o[i], fr, oj[i] * fj);
    m = m_new;
  }
};

// The merged row of a unit: thread t writes output elements 4t .. 4t+3 (all of head h) and, as
// the owner of a head's first elements, the head's softmax statistics for the tracking.
__device__ __forceinline__ void write_unit_row(const DecodeArgs &a, int unit, const Merge &mg, int e0, int h) {
  const int G = a.group;
  if (e0 >= G * D) return;
  const int seq = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const size_t head0 = static_cast<size_t>(seq) * a.n_q_heads + static_cast<size_t>(kvh) * G;
  const float invl = 1.0f / mg.l;
  u32x2_t w;
  w[0] = static_cast<unsigned>(float_to_bf16(mg.o[0] * invl)) |
         (static_cast<unsigned>(float_to_bf16(mg.o[1] * invl)) << 16);
  w[1] = static_cast<unsigned>(float_to_bf16(mg.o[2] * invl)) |
         (static_cast<unsigned>(float_to_bf16(mg.o[3] * invl)) << 16);
  *reinterpret_cast<u32x2_t *>(static_cast<bf16_t *>(a.out) + head0 * D + e0) = w;
  if (e0 % D == 0) {
    float *st = a.stat_out + static_cast<size_t>(unit) * (2 * kHeadPad) + 2 * h;
    st[0] = mg.m;
    st[1] = invl;
  }
}

// ------------------------------------------------ hand-over of partials, units of 2..4 blocks
// The unit's LAST block (highest block index) always finishes the unit; the others hand their
// partial over as a record of 64-bit words, each = (number of the launch << 32) | value bits,
// written and read with 64-bit device-scope atomics.  A word that shows this launch's number
// holds this launch's value, whatever else is still on its way, so the writer neither waits for
// its stores nor signals, and the reader needs no second round trip after a flag: it reads the
// words it needs until all of them carry the number.  Blocks are started in index order and the
// writers wait for nothing, so the reader's wait ends; it is bounded all the same (spin_ticks of
// the 100 MHz counter), after which the block raises the workspace's fault word and goes on.
// Rows 0..3 of 256 words hold the output elements (element 4 t + i of thread t in word
// i * 256 + t: one store instruction of a wave writes 512 contiguous bytes), row 4 the heads'
// maxima (words 0..7) and sums (words 8..15).
constexpr int kRecWords = 5 * kBlock;
constexpr int kHandOverMax = 4;                    // blocks per unit up to which partials are handed over

__device__ __forceinline__ void rec_store(unsigned long long *p, float v, unsigned seq) {
  __hip_atomic_store(p, (static_cast<unsigned long long>(seq) << 32) | __float_as_uint(v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
// What one thread reads of another block's record: its four output elements, its head's max and sum.
struct RecPart { unsigned long long w[6]; };
__device__ __forceinline__ void rec_load(RecPart &r, const unsigned long long *rec, int t_own, int h) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
    r.w[i] = __hip_atomic_load(rec + i * kBlock + t_own, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  r.w[4] = __hip_atomic_load(rec + 4 * kBlock + h, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  r.w[5] = __hip_atomic_load(rec + 4 * kBlock + kHeadPad + h, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool rec_valid(const RecPart &r, unsigned seq) {
  bool ok = true;
#pragma unroll
  for (int i = 0; i < 6; ++i) ok = ok && static_cast<unsigned>(r.w[i] >> 32) == seq;
  return ok;
}
__device__ __forceinline__ float rec_value(unsigned long long w) { return __uint_as_float(static_cast<unsigned>(w)); }

__global__ void clear_records_kernel(unsigned long long *rec, size_t n_words) {
  for (size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x; i < n_words;
       i += static_cast<size_t>(gridDim.x) * blockDim.x)
    rec[i] = 0;
}

// Merges the unit's block partials (in block order, so the result does not depend on which
// block came last) into the output row and stores the unit's softmax statistics.  Thread t
// owns output elements 4t .. 4t+3 (all of one head); GW partials per memory round trip.
// The calling block is partial `own_j` itself and has it in registers (own_o: its four output
// elements, own_m / own_l: its head's max and sum): those are used instead of what memory holds
// in that place.  kOwn: the unit has no other block and nothing is loaded at all.
template <int GW, bool kOwn>
__device__ void finish_unit(const DecodeArgs &a, int unit, int n_split, int own_j, const f32x4_t &own_o,
                            float own_m, float own_l) {
  const int tid = threadIdx.x;
  const int G = a.group;
  const float *ml = a.ws.part_ml + static_cast<size_t>(unit) * a.n_split_max * (2 * G);
  const float *pa = a.ws.part_acc + static_cast<size_t>(unit) * a.n_split_max * (G * D);
  const int e0 = 4 * tid;
  const int ec = min(e0, G * D - 4);               // threads beyond the group's rows load a valid place
  const int h = ec / D;

  Merge mg;
  for (int j0 = 0; j0 < n_split; j0 += GW) {
    // all loads unconditional (indices clamped to real partials) and issued together
    PartialGroup<GW> g;
    const float *po[GW], *pm[GW], *pl[GW];
#pragma unroll
    for (int jj = 0; jj < GW; ++jj) {
      const int j = min(j0 + jj, n_split - 1);
      po[jj] = pa + static_cast<size_t>(j) * (G * D) + ec;
      pm[jj] = ml + j * (2 * G) + h;
      pl[jj] = ml + j * (2 * G) + G + h;
    }
    if (!kOwn) load_partials(g, po, pm, pl);
#pragma unroll
    for (int jj = 0; jj < GW; ++jj) {
      if (j0 + jj >= n_split) break;               // uniform
      if (j0 + jj == own_j) { g.o[jj] = own_o; g.m[jj] = own_m; g.l[jj] = own_l; }   // (never read back)
      mg.fold(g.m[jj], g.l[jj], g.o[jj]);
    }
  }
  write_unit_row(a, unit, mg, e0, h);
}

// ------------------------------------------------------------------------------- the kernel
// kCompact: this call leaves candidate lists instead of every logit.
// The leading scalar arguments repeat what a stream wave needs to request its first sub-tile
// (the same values are in `a`): scalar kernel arguments are handed to a wave in registers at its
// start (kernel-argument preload, see build.py), a struct has to be fetched from memory first.
// kLong (with kCompact): a wave's run is longer than the kRunMax sub-tiles whose logits it keeps
// in LDS; every kRunMax sub-tiles it then writes the candidates among them, found with the cut
// that the block's four waves' running statistics give at that moment (a lower bound of the
// final denominator at any time, so the cut only errs towards more candidates).
// kListWaves (with kCompact): blocks of 2 * kWaves waves.  The second four ("list waves") sleep at
// the block barrier while the first four stream, and then build the candidate lists from the
// logits in LDS while the first four merge, exchange and finish the unit; that phase is serial
// code of one wave per SIMD, so a second wave per SIMD takes the lists off its path.  Used when
// all blocks of the launch are resident at once with eight waves each (a stream block and a
// tracking block per compute unit: every instance keeps to 128 registers per lane); a launch of
// more blocks runs four-wave blocks whose stream waves build their own lists.
// kSplit > 0: the instance is for units of exactly kSplit blocks (the benchmark workloads' 2 and
// 4).  What follows the stream is serial code of single waves, and a split known at compile
// time takes the ticket route, the loops over a variable number of partials and the divisions
// by the split out of it.
template <bool kCompact, bool kLong = false, bool kListWaves = false, int kSplit = 0>
__global__ __launch_bounds__(kListWaves ? 2 * kBlock : kBlock, 4) void decode_fused_kernel(
    const bf16_t *k_cache, const bf16_t *v_cache, const bf16_t *k_new_all, const bf16_t *v_new_all, const int n_old_call, const int n_split_call, const int capacity,
    const int units_call, const int slots_on, const DecodeArgs a) {
  const int n_split = kSplit > 0 ? kSplit : n_split_call;   // (a constant where the instance fixes it)
  __shared__ float m_lds[kWaves][16], lsum_lds[kWaves][16];
  // one 16-row K sub-tile per wave while streaming; afterwards the wave's output accumulator
  __shared__ u32x4_t stage_lds[kWaves][16 * 16];
  extern __shared__ float logit_lds[];             // [kWaves][min(run, kRunMax)][16 entries][8 heads]
  __shared__ unsigned cnt_lds[kWaves];
  __shared__ int last_flag;
  __shared__ unsigned cand_total;                  // candidate records of this block so far
  __shared__ float run_lse[kWaves][kHeadPad];      // kLong: each wave's latest log-sum-exp per head (one word: no torn reads)

  STAMP(0);
#ifdef LAZYEV_TIMELINE
  STAMPV(6, xcc_id());
#endif
  if (static_cast<int>(blockIdx.x) >= n_split * units_call) {
    // tracking of the previous call: n_split blocks per unit, spread over the compute units
    // like the stream blocks
    if (kListWaves && threadIdx.x >= kBlock) return;  // (the tracking has no use for list waves)
    const int tb = blockIdx.x - n_split * units_call;
    const int unit = tb / n_split, part = tb % n_split;
    TrackArgs k;
    if (!track_for_unit(a.track, unit, k)) return;
    float m[kHeadPad], invl[kHeadPad];
    track_stats(k, unit, m, invl);
    unsigned n_act = 0;
    // a logged call: the active entries' bits are collected in LDS (the K staging area, which
    // a tracking block has no other use for) ...
    unsigned *log_mask = nullptr;
    if (k.bitlog) {
      log_mask = reinterpret_cast<unsigned *>(&stage_lds[0][0]);
      for (int j = threadIdx.x; j < k.log_words; j += kBlock) log_mask[j] = 0;
      __syncthreads();
    }
    if (k.compact) {
      n_act = track_records(k, unit, part, n_split, m, invl, log_mask);
    } else {
      const int rounds = track_rounds((k.n_old + 1 + 15) >> 4, n_split);
      for (int r0 = 0; r0 < rounds; r0 += kTrackRows) {
        TrackBatch b;
        track_load(k, unit, part, n_split, r0, b);
        n_act += track_apply(k, unit, part, n_split, r0, b, m, invl, log_mask);
      }
    }
    if (k.bitlog) {
      // ... and every word of the unit is written by the one block whose entries it covers: word
      // j holds sub-tiles 2j and 2j + 1, which the wave map gives to one block (an even wave and
      // the next one); with candidate records that is a block of the logged call's own split,
      // whose records this tracking block reads if the block's index is its own modulo n_split
      __syncthreads();
      const int parts = k.compact ? k.n_parts : n_split;
      uint32_t *dst = k.bitlog + static_cast<size_t>(unit) * k.log_unit_stride;
      for (int j = threadIdx.x; j < k.log_words; j += kBlock) {
        const int wv = (2 * j) % (kWaves * parts);
        const int owner = (parts - 1 - wv / kWaves) % n_split;
        if (owner == part) dst[j] = log_mask[j];
      }
    }
    track_count(k, unit, part, n_act, cnt_lds);
    STAMP(5);
    return;
  }
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // wave-uniform: scalar branches below
  if (kCompact && tid == 0) cand_total = 0;        // (the block barrier after the stream orders it)
  if constexpr (kLong) {                           // (here the waves add to it while they stream)
    if (tid < kWaves * kHeadPad) run_lse[tid / kHeadPad][tid % kHeadPad] = -INFINITY;   // nothing seen yet
    __syncthreads();
  }
  const int c = lane & 15, g = lane >> 4;
  const int unit = blockIdx.x / n_split, split = blockIdx.x % n_split;
  int n_old = n_old_call;
  if (slots_on) {                                  // per-sequence timing: this unit's own length
    const int seq_s = unit / a.n_kv_heads;
    const int32_t P = a.slots.prompt_len[seq_s], tau = a.t - a.slots.t0[seq_s];
    if (P < 0 || tau < 1) return;                  // the whole unit sits this call out
    n_old = slot_n_old(P, tau, a.slots.budget, a.slots.window);
  }
  const int n1 = n_old + 1;
  const int n_sub = (n1 + 15) >> 4;
  // A unit of one block needs no exchange: its partial is the whole result.  Units of up to
  // kHandOverMax blocks hand their partials over to the unit's last block; longer splits take
  // tickets and the block with the last one finishes.
  const bool alone = n_split == 1;
  const bool hand_over = n_split >= 2 && n_split <= kHandOverMax;

  // the appended row goes to slot N (the stream waves read it from k_new / v_new, nobody from the slot)
  auto append_row = [&]() {
    const bf16_t *kn = k_new_all + static_cast<size_t>(unit) * D, *vn = v_new_all + static_cast<size_t>(unit) * D;
    bf16_t *ku = const_cast<bf16_t *>(k_cache) + static_cast<size_t>(unit) * capacity * D;
    bf16_t *vu = const_cast<bf16_t *>(v_cache) + static_cast<size_t>(unit) * capacity * D;
    if (lane < 16)
      reinterpret_cast<uint4 *>(ku + static_cast<size_t>(n_old) * D)[lane] = reinterpret_cast<const uint4 *>(kn)[lane];
    else if (lane < 32)
      reinterpret_cast<uint4 *>(vu + static_cast<size_t>(n_old) * D)[lane - 16] = reinterpret_cast<const uint4 *>(vn)[lane - 16];
  };

  // ---- candidate list of the sub-tiles that stream wave w leaves in LDS (for a long run: the last
  // segment; the earlier ones went out while the wave streamed), i.e. the entries that can reach
  // alpha in some head.  p_h = exp(s_h - m_h) / l_h <= exp(s_h - mb_h) / lb_h with the block's
  // own (mb, lb), so p_h >= alpha needs s_h >= mb_h + log(alpha lb_h); 2 % slack covers the
  // rounding of the two sides.  In two steps: what does not depend on the logits (plan), and
  // the rest, after the block barrier that ends the stream (run).  Four sub-tiles per round, one
  // entry per lane.
  constexpr int kRounds = (kRunMax + 3) / 4;
  struct ScanPlan {
    const float *src[kRounds];
    int entry[kRounds];
    bool always[kRounds], may[kRounds];
    char *region;
    int group;
    float alpha98;
  };
  auto plan_scan = [&](ScanPlan &sp, int w) {
    const WaveMap wmap = fused_wave_map(n_sub, n_split, split, w);
    const int cnt_w = wmap.cnt;
    const int s0 = (kLong && cnt_w > 0) ? (cnt_w - 1) / kRunMax * kRunMax : 0;
    const int run_w = min(fused_wave_run(n_sub, n_split), kRunMax);
    const float *logits = logit_lds + static_cast<size_t>(w) * run_w * (16 * kHeadPad);
    sp.group = a.group;
    sp.alpha98 = 0.98f * a.alpha;
    sp.region = reinterpret_cast<char *>(a.logits_out + (static_cast<size_t>(unit) * a.p_stride +
                                                         static_cast<size_t>(split) * fused_part_cap(n_old, n_split)) * kHeadPad);
    const int e_in = lane & 15;
#pragma unroll
    for (int rd = 0; rd < kRounds; ++rd) {
      // (reads of a round beyond the run are clamped to its last sub-tile and not used)
      const int it = s0 + 4 * rd + (lane >> 4);
      const int itc = max(min(it, cnt_w - 1), s0);
      sp.src[rd] = logits + (itc - s0) * (16 * kHeadPad) + e_in * kHeadPad;
      sp.entry[rd] = (wmap.first + it * wmap.step) * 16 + e_in;
      sp.may[rd] = it < cnt_w && sp.entry[rd] < n1;
      sp.always[rd] = it < cnt_w && sp.entry[rd] == n_old;   // the appended entry starts its tracking there
    }
  };
  auto run_scan = [&](ScanPlan &sp) {
    // lane h < 8 works out the cut of head h, everybody reads the eight cuts
    const int hh = lane & 7;
    float mbh = m_lds[0][hh];
#pragma unroll
    for (int w2 = 1; w2 < kWaves; ++w2) mbh = fmaxf(mbh, m_lds[w2][hh]);
    float lbh = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < kWaves; ++w2) {
      const float mw = m_lds[w2][hh];
      lbh = fmaf(mw == -INFINITY ? 0.f : __expf(mw - mbh), lsum_lds[w2][hh], lbh);
    }
    // the logits of all rounds are read first ...
    f32x4_t sa[kRounds], sb[kRounds];
#pragma unroll
    for (int rd = 0; rd < kRounds; ++rd) {
      sa[rd] = *reinterpret_cast<const f32x4_t *>(sp.src[rd]);
      sb[rd] = *reinterpret_cast<const f32x4_t *>(sp.src[rd] + 4);
    }
    const float cut_h = (hh < sp.group && lbh > 0.f) ? mbh + __logf(sp.alpha98 * lbh) : INFINITY;
    float cut[kHeadPad];
#pragma unroll
    for (int h = 0; h < kHeadPad; ++h)
      cut[h] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(cut_h), h));
    unsigned long long mask[kRounds];
    unsigned n_rec = 0;
#pragma unroll
    for (int rd = 0; rd < kRounds; ++rd) {
      // s_h >= cut_h in some head  <=>  the largest s_h - cut_h is not negative
      const float d = fmaxf(fmaxf(fmaxf(sa[rd][0] - cut[0], sa[rd][1] - cut[1]), fmaxf(sa[rd][2] - cut[2], sa[rd][3] - cut[3])),
                            fmaxf(fmaxf(sb[rd][0] - cut[4], sb[rd][1] - cut[5]), sb[rd][2] - cut[6]));
      const bool cand = ((d >= 0.f) & sp.may[rd]) | sp.always[rd];
      sb[rd][3] = __int_as_float(sp.entry[rd]);    // (the 8th place: groups have at most 7 heads here)
      mask[rd] = __builtin_amdgcn_ballot_w64(cand);
      n_rec += static_cast<unsigned>(__popcll(mask[rd]));
    }
    // ... then ONE addition to the block's record count reserves the places of all of the wave's records
    if (n_rec != 0) {                              // wave-uniform
      unsigned base = 0;
      if (lane == 0) base = atomicAdd(&cand_total, n_rec);
      base = __builtin_amdgcn_readfirstlane(base) + 1;
#pragma unroll
      for (int rd = 0; rd < kRounds; ++rd) {
        if ((mask[rd] >> lane) & 1ull) {
          const unsigned at = base + __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(mask[rd] >> 32),
                                                              __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(mask[rd]), 0u));
          char *dst = sp.region + at * static_cast<unsigned>(kHeadPad * sizeof(float));   // (a 32-bit offset: under 4 GB)
          *reinterpret_cast<f32x4_t *>(dst) = sa[rd];
          *reinterpret_cast<f32x4_t *>(dst + 16) = sb[rd];
        }
        base += static_cast<unsigned>(__popcll(mask[rd]));
      }
    }
  };

  if (kListWaves && wave >= kWaves) {
    // ---- list wave kWaves + w: appends the new row (one of them), plans, sleeps at the barrier
    // that ends the stream, builds stream wave w's list
    const int w = wave - kWaves;
    if (split == 0 && w == 1) append_row();
    ScanPlan sp;
    plan_scan(sp, w);
    __asm__ volatile("" ::"s"(sp.group), "s"(sp.alpha98), "s"(sp.region));   // (fetched before the barrier, not after)
    __syncthreads();                               // the stream has ended, the waves' statistics are in LDS
    run_scan(sp);
    __syncthreads();                               // cand_total is complete
    if (!hand_over) __syncthreads();               // (the ticket route has one more)
    return;
  }

  // this wave's sub-tiles (fused_wave_map)
  const WaveMap wm = fused_wave_map(n_sub, n_split, split, wave);
  const int cnt = wm.cnt;                          // (0 for a wave beyond a short cache)
  auto sub_of = [&](int it) { return wm.first + it * wm.step; };

  const bf16_t *kc = k_cache + static_cast<size_t>(unit) * capacity * D;
  const bf16_t *vc = v_cache + static_cast<size_t>(unit) * capacity * D;
  const bf16_t *k_new = k_new_all + static_cast<size_t>(unit) * D;
  const bf16_t *v_new = v_new_all + static_cast<size_t>(unit) * D;

  auto load_k = [&](SubTile &t, int it) {
    const int sub = sub_of(it);
    // K: whole rows, 16 lanes per row (row 4j+g, 16-byte chunk c); re-laid out through LDS
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = min(sub * 16 + 4 * j + g, n_old);
      const bf16_t *src = (row == n_old) ? k_new : kc + static_cast<size_t>(row) * D;
      t.k[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(src + c * 8));
    }
  };
  auto load_v = [&](SubTile &t, int it) {
    const int sub = sub_of(it);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = min(sub * 16 + 4 * g + i, n_old);
      const bf16_t *src = (row == n_old) ? v_new : vc + static_cast<size_t>(row) * D;
      t.v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(src + c * 8));
    }
  };
  // ---- the stream starts here: the first sub-tile is requested with what the wave was handed
  // in registers, before anything is read from the argument block in memory
  SubTile buf;
  if (cnt > 0) { load_k(buf, 0); load_v(buf, 0); }

  const int G = a.group;
  const int seq = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const int hc = min(c, G - 1);
  const size_t head0 = static_cast<size_t>(seq) * a.n_q_heads + static_cast<size_t>(kvh) * G;
  const bf16_t *q_row = static_cast<const bf16_t *>(a.q) + (head0 + hc) * D + g * 8;
  const int run = min(fused_wave_run(n_sub, n_split), kRunMax);
  float *my_logits = logit_lds + static_cast<size_t>(wave) * run * (16 * kHeadPad);
  int seg0 = 0;                                    // first of this wave's sub-tiles whose logits are still in LDS
  float *logits_out = a.logits_out + static_cast<size_t>(unit) * a.p_stride * kHeadPad;

  float m_ref = -INFINITY, lsum = 0.f;
  f32x4_t o[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // B operand of the logits: Q^T, head c (zero rows beyond the group)
  u32x4_t qb[KC];
#pragma unroll
  for (int kk = 0; kk < KC; ++kk) {
    const u32x4_t v = *reinterpret_cast<const u32x4_t *>(q_row + kk * 32);
    qb[kk] = c < G ? v : u32x4_t{0, 0, 0, 0};
  }

  // kMore (a std::bool_constant): the wave has a sub-tile after this one and requests it here
  auto compute = [&](SubTile &t, int it, auto more_tag) {
    constexpr bool kMore = decltype(more_tag)::value;
    const int sub = sub_of(it);
    // K rows -> MFMA A layout (lane (c, g): row c, chunks 4kk+g).  Chunk x of row r sits at
    // slot x ^ r of the row, so both the row-wise writes and the column-wise reads touch
    // every LDS bank once.  The staging area is private to the wave: LDS operations of one
    // wave execute in order, the fences only stop the compiler from reordering them.
    u32x4_t ka[KC];
    {
      u32x4_t *stage = stage_lds[wave];
#pragma unroll
      for (int j = 0; j < 4; ++j) stage[(4 * j + g) * 16 + (c ^ (4 * j + g))] = t.k[j];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int kk = 0; kk < KC; ++kk) ka[kk] = stage[c * 16 + ((4 * kk + g) ^ c)];
    }
    // the K registers are free again: the next sub-tile's K rows travel during the arithmetic
    if constexpr (kMore) load_k(t, it + 1);
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KC; ++kk)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ka[kk]),
                                                    __builtin_bit_cast(bf16x8_t, qb[kk]), acc, 0, 0, 0);
    float s[4];
    const int e0 = sub * 16 + 4 * g;
#pragma unroll
    for (int i = 0; i < 4; ++i) s[i] = (e0 + i < n1) ? acc[i] * a.scale : -INFINITY;
    // logits of the sub-tile -> [entry][head] in LDS -> 512 contiguous bytes of the workspace
    // logits of the sub-tile -> [entry][head] in LDS; written out when the wave's run ends (a
    // store among the loads would hold up the in-order load counter)
    if (c < kHeadPad) {
      float *dst = my_logits + (it - seg0) * (16 * kHeadPad);
#pragma unroll
      for (int i = 0; i < 4; ++i) dst[(4 * g + i) * kHeadPad + c] = s[i];
    }
    float tmax = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
    tmax = max_over_lane_groups(tmax);
    if (__builtin_amdgcn_ballot_w64(tmax > m_ref + kRaise) != 0) {   // wave-uniform, rare
      const float m_new = fmaxf(m_ref, tmax);
      const float f = __expf(m_ref - m_new);       // 0 on the first sub-tile (m_ref = -inf)
      lsum *= f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float fh = __shfl(f, 4 * g + i);     // factor of head 4g+i (lane 4g+i owns it)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e][i] *= fh;
      }
      m_ref = m_new;
    }
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = __expf(s[i] - m_ref);
    lsum += (p[0] + p[1]) + (p[2] + p[3]);
    u32x2_t pw;
    pw[0] = static_cast<unsigned>(float_to_bf16(p[0])) | (static_cast<unsigned>(float_to_bf16(p[1])) << 16);
    pw[1] = static_cast<unsigned>(float_to_bf16(p[2])) | (static_cast<unsigned>(float_to_bf16(p[3])) << 16);
    const s16x4_t pa = __builtin_bit_cast(s16x4_t, pw);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const unsigned sel = (e & 1) ? 0x07060302u : 0x05040100u;
      u32x2_t vb;
      vb[0] = __builtin_amdgcn_perm(t.v[1][e >> 1], t.v[0][e >> 1], sel);
      vb[1] = __builtin_amdgcn_perm(t.v[3][e >> 1], t.v[2][e >> 1], sel);
      o[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, __builtin_bit_cast(s16x4_t, vb), o[e], 0, 0, 0);
    }
    if constexpr (kMore) load_v(t, it + 1);
  };

  // this wave's logits -> workspace, 512 bytes per sub-tile: when the run ends, and for a
  // long run every kRunMax sub-tiles
  auto flush = [&](int it0, int it1) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (int it = it0 + (lane >> 5); it < it1; it += 2)
      *reinterpret_cast<float4 *>(logits_out + static_cast<size_t>(sub_of(it)) * (16 * kHeadPad) + (lane & 31) * 4) =
          *reinterpret_cast<const float4 *>(my_logits + (it - it0) * (16 * kHeadPad) + (lane & 31) * 4);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  };
  // candidates among this wave's sub-tiles it_a .. it_b - 1 (their logits are in LDS from slot 0
  // on) under the cuts of the eight heads -> records in the block's region
  auto emit_candidates = [&](int it_a, int it_b, const float (&cut)[kHeadPad]) {
    float *region = a.logits_out + (static_cast<size_t>(unit) * a.p_stride +
                                    static_cast<size_t>(split) * fused_part_cap(n_old, n_split)) * kHeadPad;
    const int e_in = lane & 15;
    for (int it0 = it_a; it0 < it_b; it0 += 4) {   // four sub-tiles per round, one entry per lane
      const int it = it0 + (lane >> 4);
      bool cand = false;
      int entry = 0;
      f32x4_t sa = {0.f, 0.f, 0.f, 0.f}, sb = sa;
      if (it < it_b) {
        const float *src = my_logits + (it - it_a) * (16 * kHeadPad) + e_in * kHeadPad;
        sa = *reinterpret_cast<const f32x4_t *>(src);
        sb = *reinterpret_cast<const f32x4_t *>(src + 4);
        entry = sub_of(it) * 16 + e_in;
        cand = sa[0] >= cut[0] || sa[1] >= cut[1] || sa[2] >= cut[2] || sa[3] >= cut[3] ||
               sb[0] >= cut[4] || sb[1] >= cut[5] || sb[2] >= cut[6];
        cand = (cand && entry < n1) || entry == n_old;
      }
      const unsigned long long mask = __builtin_amdgcn_ballot_w64(cand);
      if (mask != 0) {                             // wave-uniform
        unsigned base = 0;
        if (lane == 0) base = atomicAdd(&cand_total, static_cast<unsigned>(__popcll(mask)));
        base = __builtin_amdgcn_readfirstlane(base);
        if (cand) {
          const unsigned at = 1 + base + __builtin_amdgcn_mbcnt_hi(static_cast<unsigned>(mask >> 32),
                                                                  __builtin_amdgcn_mbcnt_lo(static_cast<unsigned>(mask), 0u));
          sb[3] = __int_as_float(entry);
          *reinterpret_cast<f32x4_t *>(region + static_cast<size_t>(at) * kHeadPad) = sa;
          *reinterpret_cast<f32x4_t *>(region + static_cast<size_t>(at) * kHeadPad + 4) = sb;
        }
      }
    }
  };
  // kLong: the segment it_a .. it_b - 1 is complete.  The wave publishes the log-sum-exp of
  // every head over what it has seen and takes the cut from what the four waves have published
  // so far: the sums only grow, so p <= exp(s - lse) holds with the log-sum-exp of any subset of
  // the entries at any earlier time.
  auto segment_candidates = [&](int it_a, int it_b) {
    float ls = lsum;
    ls = sum_over_lane_groups(ls);
    if (g == 0 && c < kHeadPad) run_lse[wave][c] = ls > 0.f ? m_ref + __logf(ls) : -INFINITY;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int hh = lane & 7;
    float lw[kWaves];
#pragma unroll
    for (int w = 0; w < kWaves; ++w) lw[w] = run_lse[w][hh];
    float lmax = lw[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) lmax = fmaxf(lmax, lw[w]);
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w)
      if (lw[w] != -INFINITY) sum += __expf(lw[w] - lmax);
    const float cut_h = (hh < G && sum > 0.f) ? lmax + __logf(0.98f * a.alpha * sum) : INFINITY;
    float cut[kHeadPad];
#pragma unroll
    for (int h = 0; h < kHeadPad; ++h)
      cut[h] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(cut_h), h));
    emit_candidates(it_a, it_b, cut);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the LDS slots are written again next
    __builtin_amdgcn_wave_barrier();
  };
  // (the wave's last sub-tile stands outside the loop, so that the loop requests the next
  // sub-tile unconditionally: no branch between the loads, exact load counts for the waits)
  for (int it = 0; it + 1 < cnt; ++it) {
    compute(buf, it, std::true_type{});
#ifdef LAZYEV_TIMELINE
    if (it == 0) STAMP(1);
#endif
    if (it + 1 - seg0 == kRunMax) {
      if constexpr (kLong) segment_candidates(seg0, it + 1);
      else flush(seg0, it + 1);
      seg0 = it + 1;
    }
  }
  if (cnt > 0) compute(buf, cnt - 1, std::false_type{});
  STAMP(2);
  if (!kCompact) flush(seg0, cnt);
  // ---- the four waves of the block -> one partial
  lsum = sum_over_lane_groups(lsum);
  if (g == 0) { m_lds[wave][c] = m_ref; lsum_lds[wave][c] = lsum; }
  float *acc_lds = reinterpret_cast<float *>(&stage_lds[0][0]);   // [kWaves][8 * D]
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int head = 4 * g + i;
    if (head < G) {
      float *d4 = acc_lds + wave * (8 * D) + head * D + 8 * c;
      *reinterpret_cast<float4 *>(d4) = make_float4(o[0][i], o[1][i], o[2][i], o[3][i]);
      *reinterpret_cast<float4 *>(d4 + 4) = make_float4(o[4][i], o[5][i], o[6][i], o[7][i]);
    }
  }
  __syncthreads();
  STAMP(3);
  // ---- this block's partial: thread owns output elements 4 tid .. 4 tid + 3, all of one head
  // (threads beyond the group's rows work on a valid place and store nothing)
  const int e0 = 4 * tid;
  const int ec = min(e0, G * D - 4);
  const int h_own = ec / D;
  float mb_own = m_lds[0][h_own];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) mb_own = fmaxf(mb_own, m_lds[w][h_own]);
  float l_own = 0.f;
  f32x4_t v_own = {0.f, 0.f, 0.f, 0.f};
  // (no branches from here on where a select does: this phase is a single wave per SIMD running
  // serial code, every instruction counts)
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const float mw = m_lds[w][h_own];
    const float f = mw == -INFINITY ? 0.f : __expf(mw - mb_own);   // a wave without entries: factor 0
    const f32x4_t x = *reinterpret_cast<const f32x4_t *>(acc_lds + w * (8 * D) + ec);
#pragma unroll
    for (int i = 0; i < 4; ++i) v_own[i] = fmaf(f, x[i], v_own[i]);
    l_own = fmaf(f, lsum_lds[w][h_own], l_own);
  }
  // the block's max and sum of head lane % 8 (what lanes 0 .. G - 1 of wave 0 store for the unit's
  // other blocks)
  const int hh = lane & 7;
  float mbh = m_lds[0][hh];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) mbh = fmaxf(mbh, m_lds[w][hh]);
  float lbh = 0.f;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const float mw = m_lds[w][hh];
    lbh = fmaf(mw == -INFINITY ? 0.f : __expf(mw - mbh), lsum_lds[w][hh], lbh);
  }
  const bool finisher = split == n_split - 1;
  const int t_own = ec >> 2;                       // (threads beyond the group's rows read a valid place)
  const unsigned long long *recs =
      a.ws.part_rec + static_cast<size_t>(unit) * ((kHandOverMax - 1) * kRecWords);
  RecPart r[kHandOverMax - 1];                     // (read only where loaded: the finishing block's j < n_split - 1)
  if (hand_over || !alone) {
    // the heads' max and sum of this block go out from ONE wave (lane h of wave 0 holds head h's):
    // dword stores of several waves into the one cache line they share were seen to reach a
    // device-scope load late
    const float mb = mbh, l = lbh;
    if (hand_over && !finisher) {
      unsigned long long *rec = const_cast<unsigned long long *>(recs) + static_cast<size_t>(split) * kRecWords;
      if (e0 < G * D) {
#pragma unroll
        for (int i = 0; i < 4; ++i) rec_store(rec + i * kBlock + tid, v_own[i], a.seq);
      }
      if (tid < G) {
        rec_store(rec + 4 * kBlock + tid, mb, a.seq);
        rec_store(rec + 4 * kBlock + kHeadPad + tid, l, a.seq);
      }
    } else if (hand_over) {
      // a first look at the other blocks' records, requested before the work below
#pragma unroll
      for (int j = 0; j < kHandOverMax - 1; ++j)
        if (j < n_split - 1) rec_load(r[j], recs + static_cast<size_t>(j) * kRecWords, t_own, h_own);
    } else {
      // publish the partial with device-scope (write-through) stores, 16 bytes wide for the values
      const size_t part = static_cast<size_t>(unit) * a.n_split_max + split;
      float *pacc = a.ws.part_acc + part * (G * D);
      if (e0 < G * D) __asm__ volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(pacc + e0), "v"(v_own) : "memory");
      if (tid < G) {
        float *ml = a.ws.part_ml + part * (2 * G);
        store_f32_device(ml + tid, mb);
        store_f32_device(ml + G + tid, l);
      }
    }
  }
  // what only the NEXT launch needs, while the partial travels: the appended row and this wave's
  // candidate list (list waves, where the block has them, do both meanwhile)
  if constexpr (!kListWaves) {
    if (split == 0 && wave == 1) append_row();
    if constexpr (kCompact) {
      ScanPlan sp;
      plan_scan(sp, wave);
      run_scan(sp);
    }
  }
  const size_t count_at = (static_cast<size_t>(unit) * a.p_stride +
                           static_cast<size_t>(split) * fused_part_cap(n_old, n_split)) * kHeadPad;
  if (hand_over) {
    if (finisher) {
      // wait until every word this thread needs carries this launch's number
      unsigned long long t_first = 0;
      for (;;) {
        bool ok = true;
#pragma unroll
        for (int j = 0; j < kHandOverMax - 1; ++j)
          if (j < n_split - 1) ok = ok && rec_valid(r[j], a.seq);
        if (ok) break;
        const unsigned long long now = wall_clock64();
        if (t_first == 0) t_first = now;
        if (now - t_first >= a.spin_ticks) {       // (a limit of 0: no second look)
          atomicOr(a.ws.fault, 1);                 // (cannot happen otherwise, see above; the row is then wrong)
          break;
        }
#pragma unroll
        for (int j = 0; j < kHandOverMax - 1; ++j)
          if (j < n_split - 1 && !rec_valid(r[j], a.seq))
            rec_load(r[j], recs + static_cast<size_t>(j) * kRecWords, t_own, h_own);
      }
      STAMP(4);
      // in block order: the others', then this block's own.  The running merge starts from block
      // 0's partial as it is: folding it into the empty state would reproduce exactly its bits
      // (factors 0 and exp(0) = 1) at the price of a dozen instructions.
      Merge mg;
      mg.m = rec_value(r[0].w[4]);
      mg.l = rec_value(r[0].w[5]);
#pragma unroll
      for (int i = 0; i < 4; ++i) mg.o[i] = rec_value(r[0].w[i]);
#pragma unroll
      for (int j = 1; j < kHandOverMax - 1; ++j)
        if (j < n_split - 1) {
          const f32x4_t oj = {rec_value(r[j].w[0]), rec_value(r[j].w[1]), rec_value(r[j].w[2]), rec_value(r[j].w[3])};
          mg.fold(rec_value(r[j].w[4]), rec_value(r[j].w[5]), oj);
        }
      mg.fold(mb_own, l_own, v_own);
      write_unit_row(a, unit, mg, e0, h_own);
    }
    if (kCompact) {
      __syncthreads();                             // cand_total is complete
      if (tid == 0) *reinterpret_cast<int32_t *>(a.logits_out + count_at) = static_cast<int32_t>(cand_total);
    }
    STAMPV(7, static_cast<unsigned long long>(finisher));
    STAMP(5);
    return;
  }
  // ---- ticket: the last block of the unit finishes it
  if (!alone) wait_own_stores();                   // every wave's partial stores have completed ...
  __syncthreads();
  if (tid == 0) {
    int prev = 0;
    if (!alone)
      prev = __hip_atomic_fetch_add(a.ticket + unit, 1, __ATOMIC_RELAXED,
                                    __HIP_MEMORY_SCOPE_AGENT);   // ... before its ticket is taken
    last_flag = (prev == n_split - 1);
    if (!alone && prev == n_split - 1) a.ticket[unit] = 0;   // ready for the next launch
    if (kCompact) *reinterpret_cast<int32_t *>(a.logits_out + count_at) = static_cast<int32_t>(cand_total);
  }
  __syncthreads();
  STAMP(4);
  STAMPV(7, static_cast<unsigned long long>(last_flag));
  if (!last_flag) { STAMP(5); return; }
  // merge the unit's partials (this block's own from its registers) into the output row
  if (alone) finish_unit<2, true>(a, unit, n_split, split, v_own, mb_own, l_own);
  else finish_unit<4, false>(a, unit, n_split, split, v_own, mb_own, l_own);
  STAMP(5);
}

}  // namespace

#ifdef LAZYEV_TIMELINE
// (host) copies the first n_words words of the stamps of the last launch; waits for the device
extern "C" int lazyev_timeline_read(unsigned long long *out, int n_words) {
  if (!out || n_words < 0 || n_words > 2048 * 8) return -1;
  return static_cast<int>(hipMemcpyFromSymbol(out, HIP_SYMBOL(lz_stamp), sizeof(unsigned long long) * n_words));
}
#endif
int decode_fused_split_max() { return kFusedSplitMax; }
int decode_fused_wave_run(int n_sub, int n_split) { return fused_wave_run(n_sub, n_split); }
int decode_fused_run_max() { return kRunMax; }
int decode_fused_head_pad() { return kHeadPad; }
size_t decode_fused_record_bytes() { return static_cast<size_t>(kRecWords) * sizeof(unsigned long long); }

hipError_t launch_clear_records(unsigned long long *rec, size_t n_words, hipStream_t stream) {
  hipLaunchKernelGGL(clear_records_kernel, dim3(256), dim3(256), 0, stream, rec, n_words);
  return hipGetLastError();
}

bool decode_fused_compact_fits(int n_old, int n_split, int p_stride, int group) {
  if (n_split < 1 || n_split > kFusedSplitMax || group >= kHeadPad) return false;
  const int cap = fused_part_cap(n_old, n_split);
  return static_cast<long long>(cap) * n_split <= p_stride;
}

hipError_t launch_track(const TrackArgs &k, hipStream_t stream) {
  if (!k.valid || k.units < 1 || k.group > kHeadPad || !k.logits || !k.stat ||
      k.p_stride < (k.n_old + 16) / 16 * 16)
    return hipErrorInvalidValue;
  if (k.compact && !decode_fused_compact_fits(k.n_old, k.n_parts, k.p_stride, k.group)) return hipErrorInvalidValue;
  int n_parts = (k.n_old + 1 + 2 * kBlock - 1) / (2 * kBlock);   // about two entries per thread
  if (n_parts > 64) n_parts = 64;
  if (k.compact) n_parts = k.n_parts;              // one block per block of the call
  hipLaunchKernelGGL(track_kernel, dim3(k.units * n_parts), dim3(kBlock), 0, stream, k, n_parts);
  return hipGetLastError();
}

int decode_fused_log_words_max() { return static_cast<int>(sizeof(u32x4_t) * kWaves * 256 / sizeof(unsigned)); }

hipError_t launch_track_flush(const FlushArgs &f, int n_layers, hipStream_t stream) {
  if (!f.ts || !f.mri || !f.pos || !f.bitlog || f.units < 1 || n_layers < 1 || f.capacity < 1 ||
      f.log_words < (f.capacity + 31) / 32 || f.n_calls < 0 || f.n_calls > f.log_slots || f.log_slots > kLogSlotsMax)
    return hipErrorInvalidValue;
  if (f.n_calls == 0) return hipSuccess;
  const unsigned spans = static_cast<unsigned>((f.capacity + kFlushSpan - 1) / kFlushSpan);
  hipLaunchKernelGGL(track_flush_kernel, dim3(static_cast<unsigned>(n_layers) * f.units * spans), dim3(kBlock), 0, stream, f);
  return hipGetLastError();
}

// Compute units of the current device (asked once).
static int compute_units() {
  static int n = 0;
  if (n == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      n = v;
    else
      n = 256;
  }
  return n;
}

hipError_t launch_decode_fused(const DecodeArgs &a, hipStream_t stream, hipEvent_t *ev) {
  const int units = a.batch * a.n_kv_heads;
  if (a.dtype != 1 || a.head_dim != D || a.group > kHeadPad || a.n_split < 1 ||
      a.n_split > kFusedSplitMax || a.n_split > a.n_split_max || !a.ticket || !a.logits_out ||
      !a.ws.part_rec || !a.ws.fault || a.seq == 0 ||
      !a.stat_out || a.p_stride < (a.n_old + 16) / 16 * 16 ||
      (a.track.valid && (a.track.units != units || !a.track.logits || !a.track.stat ||
                         a.track.logits == a.logits_out || a.track.stat == a.stat_out)) ||
      (a.track.valid && a.track.compact &&
       !decode_fused_compact_fits(a.track.n_old, a.track.n_parts, a.track.p_stride, a.track.group)) ||
      (a.track.valid && a.track.bitlog &&
       (a.track.log_words < (a.track.capacity + 31) / 32 || a.track.log_words > decode_fused_log_words_max() ||
        a.track.log_unit_stride < a.track.log_words ||
        a.track.slots.prompt_len)) ||
      (a.variant == 6 && (a.p_out || a.p_override || !decode_fused_compact_fits(a.n_old, a.n_split, a.p_stride, a.group))))
    return hipErrorInvalidValue;
  if (ev) (void)hipEventRecord(ev[0], stream);
  const int n_sub = (a.n_old + 1 + 15) / 16;
  int run = fused_wave_run(n_sub, a.n_split);
  if (run > kRunMax) run = kRunMax;
  const size_t lds_all = static_cast<size_t>(kWaves) * run * 16 * kHeadPad * sizeof(float);
  const int sb = a.n_split * units;
  const bf16_t *kc = static_cast<const bf16_t *>(a.k_cache), *vc = static_cast<const bf16_t *>(a.v_cache);
  const bf16_t *kn = static_cast<const bf16_t *>(a.k_new), *vn = static_cast<const bf16_t *>(a.v_new);
  const int slots_on = a.slots.prompt_len ? 1 : 0;
  const bool long_run = fused_wave_run(n_sub, a.n_split) > kRunMax;
  // list waves (blocks of eight waves) where every block of the launch is resident at once: two
  // such blocks fit a compute unit
  const int n_blocks = sb + (a.track.valid ? sb : 0);
  const bool list_waves = n_blocks <= 2 * compute_units();
  const dim3 grid(n_blocks), b4(kBlock), b8(2 * kBlock);
#define LAZYEV_LAUNCH(instance, block) \
  hipLaunchKernelGGL(instance, grid, block, lds_all, stream, kc, vc, kn, vn, a.n_old, a.n_split, a.capacity, units, slots_on, a)
  if (a.variant == 6 && long_run && list_waves && a.n_split == 2) LAZYEV_LAUNCH((decode_fused_kernel<true, true, true, 2>), b8);
  else if (a.variant == 6 && long_run && list_waves) LAZYEV_LAUNCH((decode_fused_kernel<true, true, true>), b8);
  else if (a.variant == 6 && long_run) LAZYEV_LAUNCH((decode_fused_kernel<true, true, false>), b4);
  else if (a.variant == 6 && list_waves && a.n_split == 2) LAZYEV_LAUNCH((decode_fused_kernel<true, false, true, 2>), b8);
  else if (a.variant == 6 && list_waves) LAZYEV_LAUNCH((decode_fused_kernel<true, false, true>), b8);
  else if (a.variant == 6 && a.n_split == 4) LAZYEV_LAUNCH((decode_fused_kernel<true, false, false, 4>), b4);
  else if (a.variant == 6) LAZYEV_LAUNCH((decode_fused_kernel<true, false, false>), b4);
  else LAZYEV_LAUNCH((decode_fused_kernel<false, false, false>), b4);
#undef LAZYEV_LAUNCH
  const hipError_t e = hipGetLastError();
  if (ev) { (void)hipEventRecord(ev[1], stream); (void)hipEventRecord(ev[2], stream); }
  return e;
}

}  // namespace lazyev
