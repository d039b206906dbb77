// Lagged eviction of one layer (Sec. 4 "MRI-Centric Eviction", Eq. 3, Eq. 6, Alg. 1 of the
// paper), as two kernels:
//   select  one block per unit: scores every candidate entry (all but the last W) in binary64,
//           finds the (B-W)-th largest score with an 8-bit radix select over the score bit
//           patterns held in LDS (beyond 8192 candidates: in the workspace), breaks ties in favour of the more recent entry, prefix-scans
//           the keep flags into destination slots, compacts TS / MRI / pos in place and leaves
//           the gather list (source entry of every survivor) in the workspace.
//   move    blocks per (unit, K|V, 128-byte column part): walk the gather list in order and
//           move the rows whose slot changes; loads of a tile complete before its stores.
//
// This file is compiled with floating-point contraction off: the score is a fixed sequence of
// individually rounded binary64 operations so that it can be reproduced bit for bit elsewhere.
#include "kernels.h"

namespace lazyev {
namespace {

constexpr int kSelBlock = 1024;
constexpr int kSelWaves = kSelBlock / 64;
constexpr int kMoveBlock = 1024;
constexpr int kLdsCandidates = 8192;               // keys of 8 bytes in the 64 KB of dynamic LDS a launch gets
constexpr int kSmallSet = 256;                     // radix select: at most this many keys left -> ranked directly

// 2*sigmoid(-x) = 2/(1+e^x) for x >= 0.  e^x = 2^k * e^r with k = round(x/ln 2) and
// r = x - k ln 2 taken in two pieces (the high piece of ln 2 has 32 significant bits, so
// k * kLn2Hi is exact); e^r by the degree-13 Taylor polynomial in Horner form.  Every
// multiply, add and divide below is a separate round-to-nearest operation.
__device__ double two_sigmoid_neg(double x) {
#pragma clang fp contract(off)
  constexpr double kLog2e = 0x1.71547652b82fep+0;
  constexpr double kLn2Hi = 0x1.62e42fee00000p-1;
  constexpr double kLn2Lo = 0x1.a39ef35793c76p-33;
  constexpr double kCoef[14] = {1.0 / 1.0, 1.0 / 1.0, 1.0 / 2.0, 1.0 / 6.0, 1.0 / 24.0,
                                1.0 / 120.0, 1.0 / 720.0, 1.0 / 5040.0, 1.0 / 40320.0,
                                1.0 / 362880.0, 1.0 / 3628800.0, 1.0 / 39916800.0,
                                1.0 / 479001600.0, 1.0 / 6227020800.0};
  if (!(x < 700.0)) return 0.0;
  const double k = floor(x * kLog2e + 0.5);
  const double r = (x - k * kLn2Hi) - k * kLn2Lo;
  double p = kCoef[13];
#pragma unroll
  for (int n = 12; n >= 0; --n) {
    p = p * r;
    p = p + kCoef[n];
  }
  const double e = ldexp(p, static_cast<int>(k));
  return 2.0 / (1.0 + e);
}

// Eq. 3.  delta_t = t - TS >= 0, mri >= 0.
__device__ double mri_centric_score(int32_t delta_t, int32_t mri, int32_t flags) {
#pragma clang fp contract(off)
  double h1 = 0.0, h2 = 0.0;
  if (flags & 1) {
    if (mri > 0) h1 = two_sigmoid_neg(static_cast<double>(delta_t) / static_cast<double>(mri));
    else h1 = (delta_t == 0) ? 1.0 : 0.0;
  }
  if ((flags & 2) && mri > 1) h2 = two_sigmoid_neg(1.0 / (static_cast<double>(mri) - 1.0));
  // reflected second term (falls with MRI, as the prose of Sec. 4 item 2 and App. D ask)
  if ((flags & 2) && (flags & 16)) h2 = (mri >= 1) ? 1.0 - h2 : 0.0;
  return h1 + h2;
}

__global__ void score_pairs_kernel(const int32_t *dt, const int32_t *mri, double *score,
                                   int64_t n, int32_t flags) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < n) score[i] = mri_centric_score(dt[i], mri[i], flags);
}

// Counts the first n entries of every unit of a layer by MRI value; values >= n_bins - 1 share
// the last bin.  Most entries have MRI = 0: those are counted per wave, not per lane.
__global__ void mri_histogram_kernel(const int32_t *mri, int64_t n_units, int32_t capacity,
                                     int32_t n, int32_t n_bins, unsigned long long *hist) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const bool in = i < n_units * n;
  int32_t b = -1;
  if (in) {
    const int32_t m = mri[(i / n) * capacity + i % n];
    b = m < n_bins - 1 ? m : n_bins - 1;
  }
  const unsigned long long zeros = __builtin_amdgcn_ballot_w64(b == 0);
  if (zeros != 0 && (threadIdx.x & 63) == 0)
    atomicAdd(&hist[0], static_cast<unsigned long long>(__builtin_popcountll(zeros)));
  if (b > 0) atomicAdd(&hist[b], 1ull);
}

__global__ void mri_histogram_slots_kernel(const int32_t *mri, int64_t n_units, int32_t capacity,
                                           int32_t n_kv_heads, const int32_t *seq_len, int32_t n_max,
                                           int32_t n_bins, unsigned long long *hist) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  int32_t b = -1;
  if (i < n_units * n_max) {
    const int64_t unit = i / n_max;
    const int32_t slot = static_cast<int32_t>(i % n_max);
    if (slot < seq_len[unit / n_kv_heads]) {
      const int32_t m = mri[unit * capacity + slot];
      b = m < n_bins - 1 ? m : n_bins - 1;
    }
  }
  const unsigned long long zeros = __builtin_amdgcn_ballot_w64(b == 0);
  if (zeros != 0 && (threadIdx.x & 63) == 0)
    atomicAdd(&hist[0], static_cast<unsigned long long>(__builtin_popcountll(zeros)));
  if (b > 0) atomicAdd(&hist[b], 1ull);
}

// A sequence starts over in its slot: the state of lazyev_init for its units in every layer,
// and its timing record.
__global__ void init_slot_kernel(int32_t *ts, int32_t *mri, int32_t *pos, int32_t n_layers,
                                 int32_t batch, int32_t n_kv_heads, int32_t capacity, int32_t seq,
                                 int32_t prompt_len, int32_t *dev_prompt_len, int32_t *dev_t0,
                                 int32_t t0) {
  const int64_t per_layer = static_cast<int64_t>(n_kv_heads) * capacity;
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i == 0) { dev_prompt_len[seq] = prompt_len; dev_t0[seq] = t0; }
  if (i >= n_layers * per_layer) return;
  const int64_t layer = i / per_layer, r = i % per_layer;
  const int64_t at = ((layer * batch + seq) * n_kv_heads) * capacity + r;
  const int32_t slot = static_cast<int32_t>(r % capacity);
  ts[at] = 0;
  mri[at] = 0;
  pos[at] = slot < prompt_len ? slot : -1;
}

__global__ void init_state_kernel(int32_t *ts, int32_t *mri, int32_t *pos, int64_t total,
                                  int32_t capacity, int32_t prompt_len) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int32_t slot = static_cast<int32_t>(i % capacity);
  ts[i] = 0;
  mri[i] = 0;
  pos[i] = slot < prompt_len ? slot : -1;
}

// Exclusive prefix sum of one value per thread over the whole block; `total` is the block sum.
__device__ unsigned block_exclusive_scan(unsigned v, unsigned *wave_tot, unsigned &total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  unsigned base = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const unsigned x = wave_tot[w];
    all += x;
    if (w < wave) base += x;
  }
  __syncthreads();
  total = all;
  return base + incl - v;
}

// kKeysInLds: the candidates' keys fit the dynamic LDS of the launch (the usual case); otherwise
// they go through the unit's part of the workspace (same passes over global memory, slower).
template <bool kKeysInLds>
__global__ __launch_bounds__(kSelBlock) void evict_select_kernel(const EvictArgs a) {
  extern __shared__ unsigned long long keys_lds[];      // score bit pattern of each candidate
  __shared__ unsigned hist[256];
  __shared__ unsigned wave_tot[kSelWaves];
  __shared__ unsigned sel_bin, sel_rem, sel_cnt;
  __shared__ unsigned long long and_k[2], or_k[2];
  __shared__ unsigned long long small_keys[kSmallSet];   // the keys still in play, once they are few
  __shared__ unsigned small_n;
  __shared__ unsigned long long small_thr;

  const int tid = threadIdx.x;
  const int unit = evict_unit_of(a, blockIdx.x);
  int n = a.n, t = a.t;
  if (a.slots.prompt_len) {                        // per-sequence timing: is this unit's eviction due?
    const int seq = (unit % a.units_per_layer) / a.n_kv_heads;
    const int32_t P = a.slots.prompt_len[seq], tau = a.t - a.slots.t0[seq];
    if (P < 0 || tau < 1 || tau % a.window != 0) return;
    n = slot_n_old(P, tau, a.budget, a.window) + 1;
    if (n <= a.budget) return;
    t = tau;
  }
  const int n_cand = n - a.window, k_keep = a.budget - a.window;
  int32_t *ts = a.ts + static_cast<size_t>(unit) * a.capacity;
  int32_t *mri = a.mri + static_cast<size_t>(unit) * a.capacity;
  int32_t *pos = a.pos + static_cast<size_t>(unit) * a.capacity;
  int32_t *src_index = a.ws.src_index + static_cast<size_t>(unit) * a.capacity;
  unsigned long long *keys = keys_lds;
  if (!kKeysInLds) keys = a.ws.sel_keys + static_cast<size_t>(unit) * a.capacity;

  // scores (non-negative doubles order like their bit patterns)
  if (a.score_flags & 32) {
    // the weight each candidate received at this step, largest over the query group: the same
    // fp32 expression the tracking uses, widened exactly
    const float *lg = a.logits + static_cast<size_t>(unit) * a.p_stride * 8;
    const float *st = a.stat + static_cast<size_t>(unit) * 16;
    for (int i = tid; i < n_cand; i += kSelBlock) {
      const float4 sa = *reinterpret_cast<const float4 *>(lg + static_cast<size_t>(i) * 8);
      const float4 sb = *reinterpret_cast<const float4 *>(lg + static_cast<size_t>(i) * 8 + 4);
      const float sv[8] = {sa.x, sa.y, sa.z, sa.w, sb.x, sb.y, sb.z, sb.w};
      float best = 0.f;
#pragma unroll
      for (int h = 0; h < 8; ++h)
        if (h < a.group) best = fmaxf(best, __expf(sv[h] - st[2 * h]) * st[2 * h + 1]);
      keys[i] = static_cast<unsigned long long>(__double_as_longlong(static_cast<double>(best)));
    }
  } else {
    for (int i = tid; i < n_cand; i += kSelBlock)
      keys[i] = static_cast<unsigned long long>(
          __double_as_longlong(mri_centric_score(t - ts[i], mri[i], a.score_flags)));
  }
  __syncthreads();

  // Radix select of the k_keep-th largest key, most significant byte first, until at most
  // kSmallSet keys are left in play, which are then ranked directly.  Every pass also
  // forms the AND and the OR of the keys still in play: when they agree, all those keys are
  // the same value (the usual case: the threshold falls among the entries that were never
  // re-activated, which all score exactly 0) and the remaining passes are skipped.
  if (tid < 256) hist[tid] = 0;
  if (tid < 2) { and_k[tid] = ~0ull; or_k[tid] = 0ull; }
  __syncthreads();                                    // also: every key is in LDS
  unsigned long long prefix = 0, mask = 0, thr = 0;
  unsigned k_rem = static_cast<unsigned>(k_keep);     // kept among the keys still in play ...
  unsigned ties_total = static_cast<unsigned>(n_cand);   // ... of which there are this many
  bool all_equal = false;
  for (int shift = 56, pass = 0; shift >= 0; shift -= 8, ++pass) {
    const int pb = pass & 1;
    unsigned long long and_acc = ~0ull, or_acc = 0ull;
    for (int i = tid; i < n_cand; i += kSelBlock) {
      const unsigned long long key = keys[i];
      if ((key & mask) == prefix) {
        atomicAdd(&hist[static_cast<unsigned>(key >> shift) & 255u], 1u);
        and_acc &= key;
        or_acc |= key;
      }
    }
    for (int o = 32; o > 0; o >>= 1) {
      and_acc &= __shfl_xor(and_acc, o);
      or_acc |= __shfl_xor(or_acc, o);
    }
    if ((tid & 63) == 0) { atomicAnd(&and_k[pb], and_acc); atomicOr(&or_k[pb], or_acc); }
    __syncthreads();
    if (and_k[pb] == or_k[pb]) {                      // the same for every thread of the block
      thr = and_k[pb];
      all_equal = true;
      break;
    }
    const unsigned bin = 255u - static_cast<unsigned>(tid);      // descending digit order
    const unsigned v = tid < 256 ? hist[bin] : 0u;
    unsigned total;
    const unsigned above = block_exclusive_scan(v, wave_tot, total);   // keys in larger digits
    if (tid < 256 && above < k_rem && k_rem <= above + v) {
      sel_bin = bin;
      sel_rem = k_rem - above;
      sel_cnt = v;
    }
    if (tid < 256) hist[tid] = 0;                     // for the next pass (the scan's barriers lie
    if (tid == 0) { and_k[pb ^ 1] = ~0ull; or_k[pb ^ 1] = 0ull; }   // between the reads and this)
    __syncthreads();
    prefix |= static_cast<unsigned long long>(sel_bin) << shift;
    mask |= 255ull << shift;
    k_rem = sel_rem;
    ties_total = sel_cnt;
    if (shift > 0 && ties_total <= static_cast<unsigned>(kSmallSet)) {
      // Few keys left in play: instead of one pass per remaining byte, list them and let each
      // count the listed keys above it and equal to it; the k_rem-th largest is the threshold.
      if (tid == 0) small_n = 0;
      __syncthreads();
      for (int i = tid; i < n_cand; i += kSelBlock) {
        const unsigned long long key = keys[i];
        if ((key & mask) == prefix) small_keys[atomicAdd(&small_n, 1u)] = key;
      }
      __syncthreads();
      if (static_cast<unsigned>(tid) < small_n) {
        const unsigned long long key = small_keys[tid];
        unsigned gt = 0, eq = 0;
        for (unsigned j = 0; j < small_n; ++j) {
          const unsigned long long other = small_keys[j];
          gt += other > key ? 1u : 0u;
          eq += other == key ? 1u : 0u;
        }
        if (gt < k_rem && k_rem <= gt + eq) {         // (every holder of that value writes the same)
          small_thr = key;
          sel_rem = k_rem - gt;
          sel_cnt = eq;
        }
      }
      __syncthreads();
      thr = small_thr;
      k_rem = sel_rem;
      ties_total = sel_cnt;
      all_equal = true;
      break;
    }
  }
  if (!all_equal) thr = prefix;
  // thr is the threshold key; k_rem of the ties_total entries equal to it are kept, the most
  // recent ones (largest slots) first.
  const unsigned drop_ties = ties_total - k_rem;

  unsigned run_def = 0, run_tie = 0, n_moved = 0;
  for (int base = 0; base < n; base += kSelBlock) {
    const int slot = base + tid;
    const bool valid = slot < n;
    const bool cand = slot < n_cand;
    const unsigned long long key = cand ? keys[slot] : 0ull;
    const bool definite = valid && (!cand || key > thr);
    const bool tie = cand && key == thr;
    unsigned total;
    const unsigned ex = block_exclusive_scan((tie ? 65536u : 0u) | (definite ? 1u : 0u),
                                             wave_tot, total);
    const unsigned tie_rank = run_tie + (ex >> 16);
    const unsigned def_before = run_def + (ex & 0xFFFFu);
    const bool keep = definite || (tie && tie_rank >= drop_ties);
    const unsigned kept_ties_before = tie_rank > drop_ties ? tie_rank - drop_ties : 0u;
    const unsigned dst = def_before + kept_ties_before;
    int32_t v_ts = 0, v_mri = 0, v_pos = 0;
    if (keep) { v_ts = ts[slot]; v_mri = mri[slot]; v_pos = pos[slot]; }
    // every read of this pass precedes its writes: the loads have returned (the barrier alone
    // only drains the LDS counter), in every thread
    __asm__ volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0)
    __syncthreads();
    if (keep) {
      ts[dst] = v_ts; mri[dst] = v_mri; pos[dst] = v_pos;
      src_index[dst] = slot;
      if (dst != static_cast<unsigned>(slot)) n_moved += 1;
    }
    run_def += total & 0xFFFFu;
    run_tie += total >> 16;
  }
  // how many survivors change slot (what the row move has to copy); one writer per unit
  for (int o = 32; o > 0; o >>= 1) n_moved += __shfl_xor(n_moved, o);
  __syncthreads();
  if ((tid & 63) == 0) wave_tot[tid >> 6] = n_moved;
  __syncthreads();
  if (tid == 0) {
    unsigned all = 0;
    for (int w = 0; w < kSelWaves; ++w) all += wave_tot[w];
    a.rows_moved[unit] += all;
  }
}

// Moves rows of K (blockIdx.y = 0) or V (1): row j <- row src_index[j], j < budget.
// Row parts are 256 bytes (16 lanes of 16 bytes; a whole row for bf16 with d = 128) or, for
// shorter rows, 128 bytes.  A block of 1024 threads owns one part of every row of one unit and
// walks the rows in tiles of (1024 / LPP) * U; loads and stores are marked non-temporal (every
// byte is touched once: measured 14 % faster than plain ones); inside a tile every load
// completes before the first store (a destination row may be another thread's source row),
// and because sources never lie below their destinations and both grow with j, a tile's
// stores cannot touch what a later tile still has to read.  The loads of the next tile are requested before this tile
// is stored, so the block always has reads in flight.
template <int U, int LPP>                      // LPP lanes of 16 bytes per row part
__global__ __launch_bounds__(kMoveBlock) void evict_move_kernel(const EvictArgs a, int row_bytes) {
  constexpr int ROWS = kMoveBlock / LPP;       // rows per block load
  const int tid = threadIdx.x;
  const int part = blockIdx.x, unit = evict_unit_of(a, blockIdx.z);
  if (a.slots.prompt_len) {                        // only units whose eviction was due have a gather list
    const int seq = (unit % a.units_per_layer) / a.n_kv_heads;
    const int32_t P = a.slots.prompt_len[seq], tau = a.t - a.slots.t0[seq];
    if (P < 0 || tau < 1 || tau % a.window != 0 ||
        slot_n_old(P, tau, a.budget, a.window) + 1 <= a.budget)
      return;
  }
  char *slab = static_cast<char *>(blockIdx.y == 0 ? a.k_cache : a.v_cache) +
               static_cast<size_t>(unit) * a.capacity * row_bytes + part * (LPP * 16) + (tid % LPP) * 16;
  const int32_t *src_index = a.ws.src_index + static_cast<size_t>(unit) * a.capacity;

  // rows below the first evicted slot stay where they are: start at the tile that holds it
  int first = 0;
  while (first + ROWS * U < a.budget && src_index[first + ROWS * U - 1] == first + ROWS * U - 1)
    first += ROWS * U;

  typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
  struct Tile { u32x4_t v[U]; int src[U]; };
  auto load = [&](Tile &t, int tile) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = tile + u * ROWS + tid / LPP;
      t.src[u] = j < a.budget ? src_index[j] : -1;
      t.v[u] = u32x4_t{0, 0, 0, 0};
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = tile + u * ROWS + tid / LPP;
      if (t.src[u] >= 0 && t.src[u] != j)
        t.v[u] = __builtin_nontemporal_load(
            reinterpret_cast<const u32x4_t *>(slab + static_cast<size_t>(t.src[u]) * row_bytes));
    }
  };
  // the tile's loads have landed in every thread (touching the values makes the compiler wait
  // for exactly those loads), then the barrier, then its stores
  auto store = [&](Tile &t, int tile) {
#pragma unroll
    for (int u = 0; u < U; ++u) __asm__ volatile("" : "+v"(t.v[u]));
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = tile + u * ROWS + tid / LPP;
      if (t.src[u] >= 0 && t.src[u] != j)
        __builtin_nontemporal_store(t.v[u], reinterpret_cast<u32x4_t *>(slab + static_cast<size_t>(j) * row_bytes));
    }
  };

  Tile t0, t1;
  load(t0, first);
  for (int tile = first; tile < a.budget; tile += 2 * ROWS * U) {
    const bool more1 = tile + ROWS * U < a.budget;
    if (more1) load(t1, tile + ROWS * U);
    store(t0, tile);
    if (!more1) break;
    const bool more2 = tile + 2 * ROWS * U < a.budget;
    if (more2) load(t0, tile + 2 * ROWS * U);
    store(t1, tile + ROWS * U);
    if (!more2) break;
  }
}

}  // namespace

int evict_lds_candidates() { return kLdsCandidates; }

hipError_t launch_evict(const EvictArgs &a, hipStream_t stream, hipEvent_t *ev) {
  const int n_cand = a.n - a.window;
  if (n_cand <= a.budget - a.window || a.n > a.capacity) return hipErrorInvalidValue;
  if (a.units_per_layer < 1 || a.units % a.units_per_layer != 0 || a.units > 65535) return hipErrorInvalidValue;
  if (a.slots.prompt_len && (!a.slots.t0 || a.n_kv_heads < 1 || a.units_per_layer % a.n_kv_heads != 0))
    return hipErrorInvalidValue;
  if ((a.score_flags & 32) && a.units != a.units_per_layer) return hipErrorInvalidValue;
  if ((a.score_flags & 32) && (!a.logits || !a.stat || a.group < 1 || a.group > 8 || a.p_stride < a.n))
    return hipErrorInvalidValue;
  const size_t lds = static_cast<size_t>(n_cand) * sizeof(unsigned long long);
  if (n_cand > kLdsCandidates && !a.ws.sel_keys) return hipErrorInvalidValue;
  int n_blocks = a.units;                          // one per unit, or only the due sequences' units
  if (a.n_due > 0) {
    if (!a.slots.prompt_len || a.n_due > 8) return hipErrorInvalidValue;
    for (int i = 0; i < a.n_due; ++i)
      if (a.due_seq[i] < 0 || a.due_seq[i] * a.n_kv_heads >= a.units_per_layer) return hipErrorInvalidValue;
    n_blocks = a.units / a.units_per_layer * a.n_due * a.n_kv_heads;
  }
  if (ev) (void)hipEventRecord(ev[0], stream);
  if (n_cand <= kLdsCandidates)
    hipLaunchKernelGGL(evict_select_kernel<true>, dim3(n_blocks), dim3(kSelBlock), lds, stream, a);
  else
    hipLaunchKernelGGL(evict_select_kernel<false>, dim3(n_blocks), dim3(kSelBlock), 0, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (ev) (void)hipEventRecord(ev[1], stream);
  const int row_bytes = a.head_dim * (a.dtype == 0 ? 4 : 2);
  if (row_bytes % 256 == 0) {
    hipLaunchKernelGGL((evict_move_kernel<8, 16>), dim3(row_bytes / 256, 2, n_blocks), dim3(kMoveBlock),
                       0, stream, a, row_bytes);
  } else {
    hipLaunchKernelGGL((evict_move_kernel<8, 8>), dim3(row_bytes / 128, 2, n_blocks), dim3(kMoveBlock),
                       0, stream, a, row_bytes);
  }
  e = hipGetLastError();
  if (ev) (void)hipEventRecord(ev[2], stream);
  return e;
}

hipError_t launch_init_state(int32_t *ts, int32_t *mri, int32_t *pos, int64_t n_units,
                             int32_t capacity, int32_t prompt_len, hipStream_t stream) {
  const int64_t total = n_units * capacity;
  const unsigned blocks = static_cast<unsigned>((total + 255) / 256);
  hipLaunchKernelGGL(init_state_kernel, dim3(blocks), dim3(256), 0, stream, ts, mri, pos, total,
                     capacity, prompt_len);
  return hipGetLastError();
}

hipError_t launch_mri_histogram(const int32_t *mri, int64_t n_units, int32_t capacity, int32_t n,
                                int32_t n_bins, unsigned long long *hist, hipStream_t stream) {
  if (n_units <= 0 || n <= 0) return hipSuccess;
  if (n > capacity || n_bins < 2) return hipErrorInvalidValue;
  const unsigned blocks = static_cast<unsigned>((n_units * n + 255) / 256);
  hipLaunchKernelGGL(mri_histogram_kernel, dim3(blocks), dim3(256), 0, stream, mri, n_units,
                     capacity, n, n_bins, hist);
  return hipGetLastError();
}

hipError_t launch_mri_histogram_slots(const int32_t *mri, int64_t n_units, int32_t capacity,
                                      int32_t n_kv_heads, const int32_t *seq_len, int32_t n_max,
                                      int32_t n_bins, unsigned long long *hist, hipStream_t stream) {
  if (n_units <= 0 || n_max <= 0) return hipSuccess;
  if (n_max > capacity || n_bins < 2 || !seq_len || n_kv_heads < 1) return hipErrorInvalidValue;
  const unsigned blocks = static_cast<unsigned>((n_units * n_max + 255) / 256);
  hipLaunchKernelGGL(mri_histogram_slots_kernel, dim3(blocks), dim3(256), 0, stream, mri, n_units,
                     capacity, n_kv_heads, seq_len, n_max, n_bins, hist);
  return hipGetLastError();
}

hipError_t launch_init_slot(int32_t *ts, int32_t *mri, int32_t *pos, int32_t n_layers, int32_t batch,
                            int32_t n_kv_heads, int32_t capacity, int32_t seq, int32_t prompt_len,
                            int32_t *dev_prompt_len, int32_t *dev_t0, int32_t t0, hipStream_t stream) {
  if (seq < 0 || seq >= batch || prompt_len > capacity || !dev_prompt_len || !dev_t0)
    return hipErrorInvalidValue;
  // prompt_len < 0 empties the slot: only the timing record changes
  const int64_t total = prompt_len < 0 ? 1 : static_cast<int64_t>(n_layers) * n_kv_heads * capacity;
  const unsigned blocks = static_cast<unsigned>((total + 255) / 256);
  hipLaunchKernelGGL(init_slot_kernel, dim3(blocks), dim3(256), 0, stream, ts, mri, pos,
                     prompt_len < 0 ? 0 : n_layers, batch, n_kv_heads, capacity, seq, prompt_len,
                     dev_prompt_len, dev_t0, t0);
  return hipGetLastError();
}

hipError_t launch_score_pairs(const int32_t *dt, const int32_t *mri, double *score, int64_t n,
                              int32_t flags, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  const unsigned blocks = static_cast<unsigned>((n + 255) / 256);
  hipLaunchKernelGGL(score_pairs_kernel, dim3(blocks), dim3(256), 0, stream, dt, mri, score, n,
                     flags);
  return hipGetLastError();
}

}  // namespace lazyev
