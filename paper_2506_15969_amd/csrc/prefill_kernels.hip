// Recurrence tracking over the prompt (MFMA kernels for bf16 with head_dim 128, plain vector-ALU
// kernels at the end of the file for fp32 rows or head_dim 64): the first loop of Alg. 1 and Eq. 1 of
// the paper applied to the prompt's own causal attention, so that prompt entries enter the
// decode phase with a TS / MRI history instead of TS = 0, MRI = 0.  Prompt position i (0-based,
// P positions) acts as the query of step tau_i = i + 1 - P over the keys 0..i; entry i is born
// with TS = tau_i, MRI = 0; decoding continues at step 1.
//
// Two kernels, both built on S^T = K Q^T tiles of v_mfma_f32_16x16x32_bf16 (16 keys x 16
// queries of ONE head); MFMA layouts
//   A[row c][k = 8g..8g+7]  B[k = 8g..8g+7][col c]  C[row 4g+i][col c]     (lane l, c = l % 16, g = l / 16):
//   stats  the four waves of a block keep 64 queries each of one head in registers (four B
//          operands per wave, loaded straight into the layout) and walk the key tiles 0..their
//          own together, keeping the running softmax maximum and sum of every query; leaves
//          b = -(log-sum-exp of the query's scaled logits) / scale per (unit, head, position)
//          in the workspace
//   track  the four waves of a block keep 64 keys each in registers (four A operands) and walk
//          the (query tile, head) pairs from the block's own position upwards together.  The
//          weight of key j for query i in head h is p = exp(scale (q.k + b)), so the product is
//          started from b instead of 0 (accumulator input of the first MFMA) and the largest
//          q.k + b over the heads of the group decides (exp and the scaling are monotone): one
//          maximum per weight and head, one exponential and one compare with alpha per weight
//          after the group's last head.  The activations of each key are then applied in order
//          of the query position (one key per lane).
// The streamed tile (keys in the first kernel, queries in the second) is fetched once per block
// and shared through LDS, one barrier per tile: fetched per wave, the second kernel read 7 GB
// per call past the L2 for a 2048-token prompt of the benchmark's third workload.  Four
// products per streamed tile and wave (one: the matrix cores wait for operands; eight: the
// registers allow only two waves per SIMD).  Blocks start in index order, so the heaviest tiles
// get the lowest indices.  No wave waits for another block.
#include "kernels.h"

namespace lazyev {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int D = 128;
constexpr int KC = D / 32;
constexpr int kHeadMax = 8;

typedef unsigned short bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;

// 16 rows x 128 columns of bf16 at `rows` (row stride `stride` elements), rows clamped to
// `last`, as an MFMA A or B operand: lane (c, g) takes row c, columns 32 kk + 8 g .. + 7.
__device__ __forceinline__ void load_operand(u32x4_t (&x)[KC], const bf16_t *rows, int first, int last,
                                             size_t stride, int c, int g) {
  const int r = min(first + c, last);
  const bf16_t *p = rows + static_cast<size_t>(r) * stride + g * 8;
#pragma unroll
  for (int kk = 0; kk < KC; ++kk) x[kk] = *reinterpret_cast<const u32x4_t *>(p + kk * 32);
}

__device__ __forceinline__ f32x4_t logits_tile(const u32x4_t (&ka)[KC], const u32x4_t (&qb)[KC],
                                               f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f}) {
#pragma unroll
  for (int kk = 0; kk < KC; ++kk)
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ka[kk]),
                                                  __builtin_bit_cast(bf16x8_t, qb[kk]), acc, 0, 0, 0);
  return acc;
}

// The streamed tile (16 rows x 256 bytes) is fetched ONCE per block: thread t brings the 16-byte
// chunk t % 16 of row t / 16 (whole 256-byte rows per 16 lanes), the block keeps it in LDS, and
// every wave reads its MFMA operand from there.  Chunk x of row r sits at slot x ^ r of the row,
// so that the row-wise writes and the column-wise operand reads both touch every bank once.
struct SharedTile {
  u32x4_t slot[2][16 * 16];                        // double-buffered
};

__device__ __forceinline__ u32x4_t tile_fetch(const bf16_t *rows, int first, int last, size_t stride) {
  const int r = min(first + (static_cast<int>(threadIdx.x) >> 4), last);
  return *reinterpret_cast<const u32x4_t *>(rows + static_cast<size_t>(r) * stride + (threadIdx.x & 15) * 8);
}

__device__ __forceinline__ void tile_put(SharedTile &t, int buf, u32x4_t v) {
  const int r = static_cast<int>(threadIdx.x) >> 4, x = threadIdx.x & 15;
  t.slot[buf][r * 16 + (x ^ r)] = v;
}

__device__ __forceinline__ void tile_operand(const SharedTile &t, int buf, u32x4_t (&x)[KC], int c, int g) {
#pragma unroll
  for (int kk = 0; kk < KC; ++kk) x[kk] = t.slot[buf][c * 16 + ((4 * kk + g) ^ c)];
}

constexpr int NB = 4;                              // tiles a wave keeps in registers
constexpr int kSpan = 16 * NB;                     // queries (stats) or keys (track) per wave

constexpr float kLog2e = 1.4426950408889634f;

// max(a, b) of two numbers as ONE instruction (the median of a, b and +inf); fmaxf spends two
// more on making signalling NaNs quiet, and there are no NaNs here.
__device__ __forceinline__ float max_f32(float a, float b) { return __builtin_amdgcn_fmed3f(a, b, INFINITY); }

// One key tile against one query tile in the statistics kernel.  Logits are kept in units of
// log 2 (scaled by scale * log2(e)), so an exponential is one v_exp_f32.  Every lane keeps the
// running maximum and sum of ITS four key rows of every tile (the four lanes of a query column
// are merged once, at the end): no cross-lane traffic inside the loop.  kMask: the tile may
// hold keys newer than a query or positions beyond the prompt.
template <bool kMask>
__device__ __forceinline__ void stats_tile(const u32x4_t (&ka)[KC], const u32x4_t (&qb)[KC], float c2, int key0,
                                           int query, int P, float &m, float &l) {
  const f32x4_t acc = logits_tile(ka, qb);
  float s[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    s[i] = acc[i] * c2;
    if (kMask) s[i] = (key0 + i <= query && key0 + i < P) ? s[i] : -INFINITY;
  }
  const float m_new = max_f32(max_f32(max_f32(s[0], s[1]), max_f32(s[2], s[3])), m);
  if (kMask && m_new == -INFINITY) return;         // this lane has seen no key of the query yet
  const float ps = (__builtin_amdgcn_exp2f(s[0] - m_new) + __builtin_amdgcn_exp2f(s[1] - m_new)) +
                   (__builtin_amdgcn_exp2f(s[2] - m_new) + __builtin_amdgcn_exp2f(s[3] - m_new));
  l = l * __builtin_amdgcn_exp2f(m - m_new) + ps;  // first tile: l = 0 * 2^(-inf) + ps
  m = m_new;
}

// Softmax statistics of every (head, prompt position) of a unit:
// blocks = units * G * ceil(P / (4 * kSpan)); the four waves of a block hold consecutive query
// spans of one head and walk the key tiles together.
__global__ __launch_bounds__(kBlock) void prefill_stats_kernel(const PrefillArgs a) {
  __shared__ SharedTile tile;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int P = a.prompt_len, G = a.group;
  const int n_qt = (P + kWaves * kSpan - 1) / (kWaves * kSpan);
  // Blocks start in index order and late query tiles carry more work than early ones: the
  // heaviest tiles get the lowest block indices (they start first, the light ones fill the
  // end), and consecutive blocks, which go to different XCDs, hold the same tile position of
  // different (unit, head) pairs, so every XCD gets every tile position equally often.
  const int n_uh = static_cast<int>(gridDim.x) / n_qt;            // units * G
  const int qt = n_qt - 1 - static_cast<int>(blockIdx.x) / n_uh;
  const int b = static_cast<int>(blockIdx.x) % n_uh;
  const int h = b % G;
  const int unit = b / G;
  const int i0 = (qt * kWaves + wave) * kSpan;     // this wave's queries: i0 .. i0 + kSpan - 1
  const bool have = i0 < P;                        // (a wave without queries still fetches and waits with the block)
  const int seq = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const bf16_t *q = static_cast<const bf16_t *>(a.q_prompt) +
                    (static_cast<size_t>(seq) * P * a.n_q_heads + kvh * G + h) * D;
  const bf16_t *kc = static_cast<const bf16_t *>(a.k_cache) + static_cast<size_t>(unit) * a.capacity * D;
  const float c2 = a.scale * kLog2e;
  u32x4_t qb[NB][KC];
#pragma unroll
  for (int n = 0; n < NB; ++n)
    load_operand(qb[n], q, i0 + 16 * n, P - 1, static_cast<size_t>(a.n_q_heads) * D, c, g);

  float m[NB], l[NB];                              // of query i0 + 16 n + c, over this lane's key rows
#pragma unroll
  for (int n = 0; n < NB; ++n) { m[n] = -INFINITY; l[n] = 0.f; }
  const int my_last = have ? min(i0 + kSpan - 1, P - 1) >> 4 : -1;
  const int block_last = min(qt * kWaves * kSpan + kWaves * kSpan - 1, P - 1) >> 4;
  tile_put(tile, 0, tile_fetch(kc, 0, P - 1, D));
  __syncthreads();
  for (int jt = 0; jt <= block_last; ++jt) {
    // the next key tile travels during the arithmetic
    const u32x4_t next = tile_fetch(kc, min(jt + 1, block_last) * 16, P - 1, D);
    if (jt <= my_last) {
      u32x4_t ka[KC];
      tile_operand(tile, jt & 1, ka, c, g);
      // all four products, no branches inside; only the wave's last four key tiles can hold
      // keys newer than a query (or positions beyond the prompt)
      if (jt * 16 + 15 <= i0 && jt * 16 + 15 < P) {
#pragma unroll
        for (int n = 0; n < NB; ++n) stats_tile<false>(ka, qb[n], c2, jt * 16 + 4 * g, i0 + 16 * n + c, P, m[n], l[n]);
      } else {
#pragma unroll
        for (int n = 0; n < NB; ++n) stats_tile<true>(ka, qb[n], c2, jt * 16 + 4 * g, i0 + 16 * n + c, P, m[n], l[n]);
      }
    }
    tile_put(tile, (jt + 1) & 1, next);
    __syncthreads();                               // tile jt + 1 is complete, tile jt no longer read
  }
  if (!have) return;
  // the four lanes of a query column (g = 0..3) -> the column's maximum and sum; a lane that
  // saw no key of the query (possible in the first tiles of a wave) holds (-inf, 0)
#pragma unroll
  for (int n = 0; n < NB; ++n) {
#pragma unroll
    for (int o = 16; o <= 32; o <<= 1) {
      const float mo = __shfl_xor(m[n], o), lo = __shfl_xor(l[n], o);
      const float mx = fmaxf(m[n], mo);
      const float fa = m[n] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m[n] - mx);
      const float fb = mo == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mo - mx);
      l[n] = l[n] * fa + lo * fb;
      m[n] = mx;
    }
  }
  if (g == 0) {                                    // b = -(m + log2 l) / (scale log2 e): see the tracking kernel
    float *st = a.stat + (static_cast<size_t>(unit) * G + h) * a.p16;
#pragma unroll
    for (int n = 0; n < NB; ++n)
      if (i0 + 16 * n + c < P) st[i0 + 16 * n + c] = -(m[n] + __builtin_amdgcn_logf(l[n])) / c2;
  }
}

// Tracking: blocks = units * ceil(P / (4 * kSpan)); a wave owns the keys j0 .. j0 + kSpan - 1.
// kIO: the weights are exported and / or replaced (a checker's route).
template <bool kIO>
__global__ __launch_bounds__(kBlock) void prefill_track_kernel(const PrefillArgs a) {
  __shared__ SharedTile tile;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int P = a.prompt_len, G = a.group;
  const int n_kt = (P + kWaves * kSpan - 1) / (kWaves * kSpan);
  // early keys carry more work: heaviest first, as in the first kernel
  const int n_units = static_cast<int>(gridDim.x) / n_kt;
  const int kt = static_cast<int>(blockIdx.x) / n_units, unit = static_cast<int>(blockIdx.x) % n_units;
  const int j0 = (kt * kWaves + wave) * kSpan;
  const bool have = j0 < P;                        // (a wave without keys still fetches and waits with the block)
  const int seq = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const bf16_t *q = static_cast<const bf16_t *>(a.q_prompt) +
                    (static_cast<size_t>(seq) * P * a.n_q_heads + kvh * G) * D;
  const bf16_t *kc = static_cast<const bf16_t *>(a.k_cache) + static_cast<size_t>(unit) * a.capacity * D;
  const float *stat = a.stat + static_cast<size_t>(unit) * G * a.p16;
  const float c2 = a.scale * kLog2e;
  u32x4_t ka[NB][KC];
#pragma unroll
  for (int n = 0; n < NB; ++n) load_operand(ka[n], kc, j0 + 16 * n, P - 1, D, c, g);

  // lane (c, g) carries the state of key row 4 g + (c & 3) of key tile c >> 2
  const int my_key = j0 + 16 * (c >> 2) + 4 * g + (c & 3);
  int32_t ts = my_key + 1 - P, mri = 0;
  unsigned n_act = 0;
  // (query tile, head) pairs in order, the same for the four waves of the block (a wave skips
  // the query tiles before its own keys); the query tile of a pair is fetched once per block,
  // the next pair's travels during the arithmetic of the current one
  const size_t q_stride = static_cast<size_t>(a.n_q_heads) * D;
  int it = (kt * kWaves * kSpan) >> 4, h = 0;      // the block's oldest key tile
  const int my_first = j0 >> 4;
  tile_put(tile, 0, tile_fetch(q, it * 16, P - 1, q_stride));
  float bq = stat[min(it * 16 + c, P - 1)];
  __syncthreads();
  int buf = 0;
  // amax[4 n + i]: largest q.k + b over the heads seen so far of the current query tile, for key
  // row 4 g + i of key tile n and query column c (-inf: the key is newer than the query)
  float amax[4 * NB];
#pragma unroll
  for (int x = 0; x < 4 * NB; ++x) amax[x] = -INFINITY;
  unsigned over = 0;                               // kIO with injected weights: bit 4 n + i = some head's weight >= alpha
  while (it * 16 < P) {
    int h2 = h + 1, it2 = it;
    if (h2 == G) { h2 = 0; ++it2; }
    const int itn = it2 * 16 < P ? it2 : it, hn = it2 * 16 < P ? h2 : h;   // (the last pair is fetched twice)
    const u32x4_t next = tile_fetch(q + static_cast<size_t>(hn) * D, itn * 16, P - 1, q_stride);
    const float bn = stat[static_cast<size_t>(hn) * a.p16 + min(itn * 16 + c, P - 1)];
    const int qi = it * 16 + c;                    // this lane's query column
    const f32x4_t b4 = {bq, bq, bq, bq};
    if (have && it >= my_first) {
    u32x4_t qb[KC];
    tile_operand(tile, buf, qb, c, g);
    // every key of the wave exists and is no newer than any query of the tile, and every
    // query of the tile exists: nothing to mask (all but the wave's first four query tiles,
    // the prompt's last tile and its last wave)
    const bool plain = !kIO && j0 + kSpan - 1 <= it * 16 && j0 + kSpan - 1 < P && it * 16 + 15 < P;
    if (plain) {
#pragma unroll
      for (int n = 0; n < NB; ++n) {
        const f32x4_t acc = logits_tile(ka[n], qb, b4);
#pragma unroll
        for (int i = 0; i < 4; ++i) amax[4 * n + i] = max_f32(amax[4 * n + i], acc[i]);
      }
    } else {
#pragma unroll
      for (int n = 0; n < NB; ++n) {
        const f32x4_t acc = logits_tile(ka[n], qb, b4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int key = j0 + 16 * n + 4 * g + i;
          const bool seen = key <= qi && qi < P;   // (key <= qi < P implies key < P)
          if (seen) amax[4 * n + i] = max_f32(amax[4 * n + i], acc[i]);
          if (kIO) {
            if (seen) {
              const size_t at = ((static_cast<size_t>(seq) * a.n_q_heads + kvh * G + h) * P + qi) * P + key;
              if (a.p_out) a.p_out[at] = __builtin_amdgcn_exp2f(acc[i] * c2);
              if (a.p_override && a.p_override[at] >= a.alpha) over |= 1u << (4 * n + i);
            }
          }
        }
      }
    }
    if (h2 == 0) {                                 // the tile's last head: apply its activations
      // key row 4 g' + i of key tile n over the tile's 16 queries: bits 16 g' .. 16 g' + 15 of
      // the ballot of entry 4 n + i; lane (c, g) wants the one with 4 n + i = c
      unsigned long long mine = 0, any = 0;
#pragma unroll
      for (int x = 0; x < 4 * NB; ++x) {
        bool on = __builtin_amdgcn_exp2f(amax[x] * c2) >= a.alpha;       // exp2(-inf) = 0
        if (kIO && a.p_override) on = (over >> x) & 1u;
        const unsigned long long bal = __builtin_amdgcn_ballot_w64(on);
        if (c == x) mine = bal;
        any |= bal;
        amax[x] = -INFINITY;
      }
      over = 0;
      if (any != 0) {                              // (wave-uniform)
        unsigned mask = static_cast<unsigned>(mine >> (16 * g)) & 0xFFFFu;
        n_act += __popc(mask);
        while (mask) {                             // in order of the query position (Alg. 1, Eq. 1)
          const int32_t tau = it * 16 + __builtin_ctz(mask) + 1 - P;
          mask &= mask - 1;
          const int32_t gap = tau - ts;
          if (gap > mri) mri = gap;
          ts = tau;
        }
      }
    }
    }
    tile_put(tile, buf ^ 1, next);
    __syncthreads();                               // the next pair's tile is complete, this pair's no longer read
    buf ^= 1;
    bq = bn;
    it = it2;
    h = h2;
  }
  if (!have) return;
  if (my_key < P) {
    a.ts[static_cast<size_t>(unit) * a.capacity + my_key] = ts;
    a.mri[static_cast<size_t>(unit) * a.capacity + my_key] = mri;
  }
  if (a.activation_counter) {
    for (int o = 32; o > 0; o >>= 1) n_act += __shfl_xor(n_act, o);
    if (lane == 0 && n_act) atomicAdd(a.activation_counter + unit * a.counter_stride, static_cast<unsigned long long>(n_act));
  }
}

// ---- any other shape (fp32 rows, head_dim 64): the same two steps on the vector ALU, one
// thread per (unit, head, query position) and one per (unit, key).  A dot product adds its
// terms in index order in both kernels, so both see the same logit.
template <int DH, typename T>
__device__ inline void row_to_float(const T *src, float (&dst)[DH]) {
#pragma unroll
  for (int e = 0; e < DH; ++e) {
    if constexpr (sizeof(T) == 4) dst[e] = src[e];
    else dst[e] = __uint_as_float(static_cast<unsigned>(src[e]) << 16);
  }
}
template <int DH, typename T>
__device__ inline float dot_row(const float (&reg)[DH], const T *mem, bool reg_is_q) {
  float s = 0.f;
#pragma unroll 8
  for (int e = 0; e < DH; ++e) {
    float m;
    if constexpr (sizeof(T) == 4) m = mem[e];
    else m = __uint_as_float(static_cast<unsigned>(mem[e]) << 16);
    s = reg_is_q ? fmaf(reg[e], m, s) : fmaf(m, reg[e], s);
  }
  return s;
}

// stat[(unit * G + h) * p16 + i] = log-sum-exp of the scaled logits of query i of head h
template <int DH, typename T>
__global__ __launch_bounds__(256) void prefill_stats_simple_kernel(const PrefillArgs a) {
  const int P = a.prompt_len, G = a.group;
  const long long idx = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= static_cast<long long>(a.batch) * a.n_kv_heads * G * P) return;
  const int i = static_cast<int>(idx % P), h = static_cast<int>((idx / P) % G);
  const int unit = static_cast<int>(idx / (static_cast<long long>(P) * G));
  const int seq = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const T *q = static_cast<const T *>(a.q_prompt) +
               ((static_cast<size_t>(seq) * P + i) * a.n_q_heads + kvh * G + h) * DH;
  const T *k = static_cast<const T *>(a.k_cache) + static_cast<size_t>(unit) * a.capacity * DH;
  float qr[DH];
  row_to_float<DH>(q, qr);
  float m = -INFINITY, l = 0.f;
  for (int j = 0; j <= i; ++j) {
    const float sc = a.scale * dot_row<DH>(qr, k + static_cast<size_t>(j) * DH, true);
    if (sc > m) { l = l * __expf(m - sc) + 1.f; m = sc; }      // (exp(-inf) = 0 on the first key)
    else l += __expf(sc - m);
  }
  a.stat[(static_cast<size_t>(unit) * G + h) * a.p16 + i] = m + __logf(l);
}

template <int DH, typename T>
__global__ __launch_bounds__(256) void prefill_track_simple_kernel(const PrefillArgs a) {
  const int P = a.prompt_len, G = a.group;
  const long long idx = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
  const bool live = idx < static_cast<long long>(a.batch) * a.n_kv_heads * P;
  const int j = live ? static_cast<int>(idx % P) : 0;
  const int unit = live ? static_cast<int>(idx / P) : 0;
  const int seq = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  unsigned n_act = 0;
  if (live) {
    float kr[DH];
    row_to_float<DH>(static_cast<const T *>(a.k_cache) + (static_cast<size_t>(unit) * a.capacity + j) * DH, kr);
    int32_t ts = j + 1 - P, mri = 0;                 // born at its own step
    for (int i = j; i < P; ++i) {                    // in order of the query position (Alg. 1, Eq. 1)
      bool on = false;
      for (int h = 0; h < G; ++h) {
        const int head = kvh * G + h;
        const size_t at = ((static_cast<size_t>(seq) * a.n_q_heads + head) * P + i) * P + j;
        const T *q = static_cast<const T *>(a.q_prompt) + ((static_cast<size_t>(seq) * P + i) * a.n_q_heads + head) * DH;
        float pw = __expf(a.scale * dot_row<DH>(kr, q, false) - a.stat[(static_cast<size_t>(unit) * G + h) * a.p16 + i]);
        if (a.p_out) a.p_out[at] = pw;
        if (a.p_override) pw = a.p_override[at];
        on = on || pw >= a.alpha;
      }
      if (on) {
        const int32_t tau = i + 1 - P, gap = tau - ts;
        if (gap > mri) mri = gap;
        ts = tau;
        n_act += 1;
      }
    }
    a.ts[static_cast<size_t>(unit) * a.capacity + j] = ts;
    a.mri[static_cast<size_t>(unit) * a.capacity + j] = mri;
  }
  if (a.activation_counter && n_act) atomicAdd(a.activation_counter + static_cast<size_t>(unit) * a.counter_stride, static_cast<unsigned long long>(n_act));
}

template <int DH, typename T>
hipError_t launch_prefill_simple(const PrefillArgs &a, hipStream_t stream) {
  const long long units = static_cast<long long>(a.batch) * a.n_kv_heads;
  const long long n1 = (units * a.group * a.prompt_len + 255) / 256, n2 = (units * a.prompt_len + 255) / 256;
  if (n1 > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((prefill_stats_simple_kernel<DH, T>), dim3(static_cast<unsigned>(n1)), dim3(256), 0, stream, a);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((prefill_track_simple_kernel<DH, T>), dim3(static_cast<unsigned>(n2)), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_prefill_track(const PrefillArgs &a, hipStream_t stream) {
  if (a.prompt_len < 1 || a.prompt_len > a.capacity || a.group < 1 || a.group > kHeadMax ||
      a.n_q_heads != a.n_kv_heads * a.group || a.batch < 1 || a.p16 < (a.prompt_len + 15) / 16 * 16 ||
      !a.q_prompt || !a.k_cache || !a.ts || !a.mri || !a.stat || a.counter_stride < 1)
    return hipErrorInvalidValue;
  if (a.dtype == 0 && a.head_dim == 64) return launch_prefill_simple<64, float>(a, stream);
  if (a.dtype == 0 && a.head_dim == 128) return launch_prefill_simple<128, float>(a, stream);
  if (a.dtype == 1 && a.head_dim == 64) return launch_prefill_simple<64, bf16_t>(a, stream);
  if (a.dtype != 1 || a.head_dim != D) return hipErrorInvalidValue;
  const long long units = static_cast<long long>(a.batch) * a.n_kv_heads;
  const long long n_t = (a.prompt_len + kWaves * kSpan - 1) / (kWaves * kSpan);
  if (units * a.group * n_t > 0x7FFFFFFFLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(prefill_stats_kernel, dim3(static_cast<unsigned>(units * a.group * n_t)), dim3(kBlock), 0,
                     stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.p_out || a.p_override)
    hipLaunchKernelGGL(prefill_track_kernel<true>, dim3(static_cast<unsigned>(units * n_t)), dim3(kBlock), 0, stream, a);
  else
    hipLaunchKernelGGL(prefill_track_kernel<false>, dim3(static_cast<unsigned>(units * n_t)), dim3(kBlock), 0, stream, a);
  return hipGetLastError();
}

}  // namespace lazyev
