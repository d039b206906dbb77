// Decode step of one layer in ONE kernel (bf16, head_dim 128): append, attention (Eq. 4 of the
// paper) and the recurrence tracking of Alg. 1 / Eq. 1.
//
// A unit's cache is cut into 16-entry sub-tiles that are dealt out, in contiguous and nearly
// equal runs, to the 4 * n_split waves of the unit's n_split blocks.  Every wave streams its
// run once, K and V rows of a sub-tile together, with the loads of the next two sub-tiles in
// flight while the current one is multiplied:
//   S^T = K Q^T          v_mfma_f32_16x16x32_bf16, the G query rows padded to 16 columns
//   scaled logits        -> workspace (fp32; the activation test needs them once the softmax
//                           statistics of the WHOLE unit are known)
//   running softmax      per wave: reference maximum m, sum l, output accumulator O.  The
//                           reference is raised only when a logit exceeds it by more than 8,
//                           so rescaling O is rare; exp(s - m) <= e^8 stays far from overflow
//   O += P V             v_mfma_f32_16x16x16_bf16 after an in-lane 4x8 transpose of the V rows
// The four waves of a block merge their (m, l, O) in LDS and store one partial per block.  The
// block that finishes LAST for its unit (a ticket counter in the workspace, taken after the
// block's device-scope stores have completed) merges the unit's partials into the output row, turns every stored logit
// into its probability p = exp(s - m) / l, applies the >= alpha test over the query group and
// updates TS / MRI in place.  Nothing waits for another block, so the kernel cannot hang on
// scheduling order; the ticket resets itself for the next launch.
//
// Blocks of one unit can be placed on one XCD (workgroups go to the XCDs round-robin by their
// linear index); correctness does not depend on it.
//
// MFMA operand layouts (lane l, c = l % 16, g = l / 16):
//   16x16x32: A[row c][k = 8g..8g+7]  B[k = 8g..8g+7][col c]  C[row 4g+i][col c]
//   16x16x16: A[row c][k = 4g..4g+3]  B[k = 4g..4g+3][col c]  C[row 4g+i][col c]
// so a lane that owns head c and entries 4g..4g+3 of a sub-tile after the first product already
// holds the A operand of the second.
#include "kernels.h"

namespace lazyev {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int D = 128;
constexpr int KC = D / 32;
constexpr int kFusedSplitMax = 64;      // blocks per unit the finishing block can merge
constexpr float kRaise = 8.0f;          // the reference maximum moves when exceeded by this much
constexpr int kTrackRows = 4;           // entries per thread per tracking batch

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

// K and V rows of one sub-tile as a wave holds them: 4 + 4 loads of 16 bytes per lane.
struct SubTile {
  u32x4_t k[KC];
  u32x4_t v[4];
};

// The stream is straight-line code: the kernel is instantiated per run length N_IT, so the
// compiler sees every load and every use and waits with exact counters (vector memory
// operations of a wave complete in issue order), which keeps the next sub-tiles' loads in
// flight across the current sub-tile's arithmetic.  A wave whose run is shorter than N_IT
// turns the missing sub-tiles into loads of one always-valid address (one cache line, no HBM
// traffic) with their logits masked to -inf.
// What one block writes for another block of the same launch to read (logits, partials) goes
// through stores and loads at device ("agent") scope: they write through / read past the
// XCD-local L2, so no whole-cache write-back is needed to publish them.  Publishing is then:
// wait until this wave's stores have completed, block barrier, one relaxed device-scope
// atomic on the unit's ticket.
__device__ __forceinline__ void store_f32_device(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_f32_device(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_f32x4_device(float *p, const f32x4_t &v) {
  __asm__ volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}

__device__ __forceinline__ float wave_max64(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum64(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// ------------------------------------------------------------------------ finishing block
// Runs in the last block of a unit, after every block's partial and logits are visible.
__device__ void finish_unit(const DecodeArgs &a, int unit, int n_split) {
  __shared__ float w_lds[kFusedSplitMax * 8];      // partial max, later the weight of the partial
  __shared__ float l_lds[kFusedSplitMax * 8];
  __shared__ float m_s[8], invl_s[8];
  __shared__ unsigned cnt_lds[kWaves];
  constexpr int GMAX = 8;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int seq = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const int G = a.group;
  const int n_old = a.n_old, n1 = a.n_old + 1;
  const size_t head0 = static_cast<size_t>(seq) * a.n_q_heads + static_cast<size_t>(kvh) * G;
  const float *logit = a.ws.p_tilde + head0 * a.p_stride;
  const float *ml = a.ws.part_ml + static_cast<size_t>(unit) * a.n_split_max * (2 * G);
  const float *pa = a.ws.part_acc + static_cast<size_t>(unit) * a.n_split_max * (G * D);
  int32_t *ts = a.ts + static_cast<size_t>(unit) * a.capacity;
  int32_t *mri = a.mri + static_cast<size_t>(unit) * a.capacity;

  float sv[kTrackRows][GMAX];
  int32_t ts0[kTrackRows], mri0[kTrackRows];
  auto load_batch = [&](int base) {
#pragma unroll
    for (int r = 0; r < kTrackRows; ++r) {
      const int i = base + r * kBlock + tid;
#pragma unroll
      for (int h = 0; h < GMAX; ++h)
        sv[r][h] = (h < G && i < n1) ? load_f32_device(logit + static_cast<size_t>(h) * a.p_stride + i) : -INFINITY;
      ts0[r] = 0; mri0[r] = 0;
      if (i < n_old) { ts0[r] = ts[i]; mri0[r] = mri[i]; }
    }
  };
  load_batch(0);                                   // in flight across the merge of the statistics

  for (int i = tid; i < n_split * G; i += kBlock) {
    const int j = i / G, h = i - j * G;
    w_lds[i] = load_f32_device(ml + j * (2 * G) + h);
    l_lds[i] = load_f32_device(ml + j * (2 * G) + G + h);
  }
  __syncthreads();
  for (int h = wave; h < G; h += kWaves) {         // fixed order: lane-strided, then the lanes
    float m = -INFINITY;
    for (int j = lane; j < n_split; j += 64) m = fmaxf(m, w_lds[j * G + h]);
    m = wave_max64(m);
    float l = 0.f;
    for (int j = lane; j < n_split; j += 64) {
      const float mj = w_lds[j * G + h];
      if (mj != -INFINITY) l += l_lds[j * G + h] * __expf(mj - m);
    }
    l = wave_sum64(l);
    if (lane == 0) { m_s[h] = m; invl_s[h] = 1.0f / l; }
  }
  __syncthreads();
  for (int i = tid; i < n_split * G; i += kBlock) {
    const int h = i % G;
    const float mj = w_lds[i];
    w_lds[i] = (mj != -INFINITY) ? __expf(mj - m_s[h]) * invl_s[h] : 0.f;
  }
  __syncthreads();

  // output row: out[h][dd] = sum_j w[j][h] * O_j[h][dd]
  for (int e = tid; e < G * D; e += kBlock) {
    const int h = e / D;
    float v = 0.f;
    for (int j = 0; j < n_split; ++j)
      v = fmaf(w_lds[j * G + h], load_f32_device(pa + static_cast<size_t>(j) * (G * D) + e), v);
    static_cast<bf16_t *>(a.out)[head0 * D + e] = float_to_bf16(v);
  }

  // probabilities, activation test (Alg. 1) and Eq. 1
  unsigned n_act = 0;
  for (int base = 0; base < n1; base += kTrackRows * kBlock) {
    if (base) load_batch(base);
#pragma unroll
    for (int r = 0; r < kTrackRows; ++r) {
      const int i = base + r * kBlock + tid;
      if (i >= n1) continue;
      bool act = false;
#pragma unroll
      for (int h = 0; h < GMAX; ++h) {
        if (h < G) {
          float p = __expf(sv[r][h] - m_s[h]) * invl_s[h];
          const size_t at = (head0 + h) * a.capacity + i;
          if (a.p_out) a.p_out[at] = p;
          if (a.p_override) p = a.p_override[at];
          act = act || (p >= a.alpha);
        }
      }
      if (i == n_old) {                            // the appended entry starts here (Sec. 4)
        ts[i] = a.t;
        mri[i] = 0;
        a.pos[static_cast<size_t>(unit) * a.capacity + i] = a.prompt_len + a.t - 1;
      } else if (act) {
        const int32_t gap = a.t - ts0[r];
        if (gap > mri0[r]) mri[i] = gap;           // Eq. 1
        ts[i] = a.t;                               // Alg. 1
      }
      n_act += act ? 1u : 0u;
    }
  }
  for (int o = 32; o > 0; o >>= 1) n_act += __shfl_xor(n_act, o);
  if (lane == 0) cnt_lds[wave] = n_act;
  __syncthreads();
  if (tid == 0) {
    unsigned total = 0;
    for (int w = 0; w < kWaves; ++w) total += cnt_lds[w];
    if (total) a.activation_counter[unit * 64] += total;
  }
}

// ------------------------------------------------------------------------------- the kernel
template <int N_IT, int DEPTH>
__global__ __launch_bounds__(kBlock, 2) void decode_fused_kernel(const DecodeArgs a) {
  __shared__ float m_lds[kWaves][16], lsum_lds[kWaves][16];
  __shared__ float acc_lds[kWaves][8 * D];
  __shared__ u32x4_t k_stage[kWaves][16 * 16];     // one 16-row K sub-tile per wave
  __shared__ int last_flag;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: scalar branches below
  const int c = lane & 15, g = lane >> 4;
  const int G = a.group, n_split = a.n_split;
  const int units = a.batch * a.n_kv_heads;
  int unit, split;
  {
    const int b = blockIdx.x;
    if (a.xcd_map) {                               // blocks of a unit share an XCD
      const int k = b >> 3;
      unit = (b & 7) * (units >> 3) + k / n_split;
      split = k % n_split;
    } else {
      unit = b / n_split;
      split = b % n_split;
    }
  }
  const int seq = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const int hc = min(c, G - 1);
  const int n_old = a.n_old, n1 = a.n_old + 1;
  const int n_sub = (n1 + 15) >> 4;
  const size_t head0 = static_cast<size_t>(seq) * a.n_q_heads + static_cast<size_t>(kvh) * G;

  // this wave's sub-tiles: wv, wv + n_wv, wv + 2 n_wv, ...  (the waves of a unit read one
  // moving window of the cache together, which keeps DRAM pages open)
  const int n_wv = kWaves * n_split, wv = split * kWaves + wave;
  const int cnt = (n_sub - wv + n_wv - 1) / n_wv;  // <= N_IT (the host sizes N_IT for it); may be <= 0

  const bf16_t *kc = static_cast<const bf16_t *>(a.k_cache) + static_cast<size_t>(unit) * a.capacity * D;
  const bf16_t *vc = static_cast<const bf16_t *>(a.v_cache) + static_cast<size_t>(unit) * a.capacity * D;
  const bf16_t *k_new = static_cast<const bf16_t *>(a.k_new) + static_cast<size_t>(unit) * D;
  const bf16_t *v_new = static_cast<const bf16_t *>(a.v_new) + static_cast<size_t>(unit) * D;
  float *plog = a.ws.p_tilde + (head0 + hc) * a.p_stride + 4 * g;   // this lane's head, its 4 entries

  const bf16_t *q_row = static_cast<const bf16_t *>(a.q) + (head0 + hc) * D + g * 8;

  float m_ref = -INFINITY, lsum = 0.f;
  f32x4_t o[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  if (cnt > 0) {
    // B operand of the logits: Q^T, head c (zero rows beyond the group)
    u32x4_t qb[KC];
#pragma unroll
    for (int kk = 0; kk < KC; ++kk) {
      const u32x4_t v = *reinterpret_cast<const u32x4_t *>(q_row + kk * 32);
      qb[kk] = c < G ? v : u32x4_t{0, 0, 0, 0};
    }

    auto load = [&](SubTile &t, int it) {
      const bool real = it < cnt;                  // wave-uniform
      const int sub = wv + it * n_wv;
      // K: whole rows, 16 lanes per row (row 4j+g, 16-byte chunk c); re-laid out through LDS
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int row = min(sub * 16 + 4 * j + g, n_old);
        const bf16_t *src = (row == n_old) ? k_new : kc + static_cast<size_t>(row) * D;
        src = real ? src + c * 8 : q_row;
        t.k[j] = *reinterpret_cast<const u32x4_t *>(src);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = min(sub * 16 + 4 * g + i, n_old);
        const bf16_t *src = (row == n_old) ? v_new : vc + static_cast<size_t>(row) * D;
        src = (real && !(a.chunk & 16)) ? src + c * 8 : q_row;
        t.v[i] = *reinterpret_cast<const u32x4_t *>(src);
      }
    };

    unsigned dbg_x = 0;
    auto compute = [&](const SubTile &t, int it) {
      const bool real = it < cnt;
      const int sub = wv + it * n_wv;
      if (a.chunk & 32) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          dbg_x ^= t.k[j][0] ^ t.k[j][1] ^ t.k[j][2] ^ t.k[j][3] ^ t.v[j][0] ^ t.v[j][1] ^ t.v[j][2] ^ t.v[j][3];
        return;
      }
      // K rows -> MFMA A layout (lane (c, g): row c, chunks 4kk+g).  Chunk x of row r sits at
      // slot x ^ r of the row, so both the row-wise writes and the column-wise reads touch
      // every LDS bank once.  The staging area is private to the wave: LDS operations of one
      // wave execute in order, the fences only stop the compiler from reordering them.
      u32x4_t ka[KC];
      {
        u32x4_t *stage = k_stage[wave];
#pragma unroll
        for (int j = 0; j < 4; ++j) stage[(4 * j + g) * 16 + (c ^ (4 * j + g))] = t.k[j];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int kk = 0; kk < KC; ++kk) ka[kk] = stage[c * 16 + ((4 * kk + g) ^ c)];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
      f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < KC; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ka[kk]),
                                                      __builtin_bit_cast(bf16x8_t, qb[kk]), acc, 0, 0, 0);
      float s[4];
      const int e0 = sub * 16 + 4 * g;
#pragma unroll
      for (int i = 0; i < 4; ++i) s[i] = (real && e0 + i < n1) ? acc[i] * a.scale : -INFINITY;
      if (real && c < G && !(a.chunk & 2)) {
        if (a.chunk & 4) *reinterpret_cast<float4 *>(plog + sub * 16) = make_float4(s[0], s[1], s[2], s[3]);
        else store_f32x4_device(plog + sub * 16, f32x4_t{s[0], s[1], s[2], s[3]});
      }
      float tmax = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      if (__builtin_amdgcn_ballot_w64(tmax > m_ref + kRaise) != 0) {   // wave-uniform, rare
        const float m_new = fmaxf(m_ref, tmax);
        const float f = __expf(m_ref - m_new);     // 0 on the first sub-tile (m_ref = -inf)
        lsum *= f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float fh = __shfl(f, 4 * g + i);   // factor of head 4g+i (lane 4g+i owns it)
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
    };

    // ---- the stream: three sub-tile buffers, the loads of the next two in flight
    SubTile buf[DEPTH + 1];
#pragma unroll
    for (int it = 0; it < DEPTH; ++it)
      if (it < N_IT) load(buf[it], it);
#pragma unroll
    for (int it = 0; it < N_IT; ++it) {
      if (it + DEPTH < N_IT) load(buf[(it + DEPTH) % (DEPTH + 1)], it + DEPTH);
      __builtin_amdgcn_sched_barrier(0);           // the loads are issued before this sub-tile's math
      compute(buf[it % (DEPTH + 1)], it);
    }
    if (dbg_x == 0x9E3779B9u) lsum = 1.f;
  }

  // ---- the four waves of the block -> one partial
  lsum += __shfl_xor(lsum, 16);
  lsum += __shfl_xor(lsum, 32);
  if (g == 0) { m_lds[wave][c] = m_ref; lsum_lds[wave][c] = lsum; }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int head = 4 * g + i;
    if (head < G) {
      float *dst = &acc_lds[wave][head * D + 8 * c];
      *reinterpret_cast<float4 *>(dst) = make_float4(o[0][i], o[1][i], o[2][i], o[3][i]);
      *reinterpret_cast<float4 *>(dst + 4) = make_float4(o[4][i], o[5][i], o[6][i], o[7][i]);
    }
  }
  __syncthreads();
  {
    const size_t part = static_cast<size_t>(unit) * a.n_split_max + split;
    float *pacc = a.ws.part_acc + part * (G * D);
    for (int e = tid; e < G * D; e += kBlock) {
      const int h = e / D;
      float mb = m_lds[0][h];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) mb = fmaxf(mb, m_lds[w][h]);
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float mw = m_lds[w][h];
        if (mw != -INFINITY) v = fmaf(__expf(mw - mb), acc_lds[w][e], v);
      }
      store_f32_device(pacc + e, v);
    }
    if (tid < G) {
      float mb = m_lds[0][tid];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) mb = fmaxf(mb, m_lds[w][tid]);
      float l = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float mw = m_lds[w][tid];
        if (mw != -INFINITY) l = fmaf(__expf(mw - mb), lsum_lds[w][tid], l);
      }
      float *ml = a.ws.part_ml + part * (2 * G);
      store_f32_device(ml + tid, mb);
      store_f32_device(ml + G + tid, l);
    }
  }
  // the appended row goes to slot N (everybody read it from k_new / v_new)
  if (split == 0 && wave == 1) {
    if (lane < 16)
      reinterpret_cast<uint4 *>(const_cast<bf16_t *>(kc) + static_cast<size_t>(n_old) * D)[lane] =
          reinterpret_cast<const uint4 *>(k_new)[lane];
    else if (lane < 32)
      reinterpret_cast<uint4 *>(const_cast<bf16_t *>(vc) + static_cast<size_t>(n_old) * D)[lane - 16] =
          reinterpret_cast<const uint4 *>(v_new)[lane - 16];
  }

  if (a.chunk & 8) return;
  // ---- ticket: the last block of the unit finishes it
  __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's partial and logits are out ...
  __syncthreads();
  if (tid == 0) {
    const int prev = __hip_atomic_fetch_add(a.ticket + unit, 1, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_AGENT);   // ... before its ticket is
    last_flag = (prev == n_split - 1);
    if (prev == n_split - 1) a.ticket[unit] = 0;   // ready for the next launch
  }
  __syncthreads();
  if (!last_flag || (a.chunk & 1)) return;
  finish_unit(a, unit, n_split);
}

template <int N_IT>
hipError_t launch_n(const DecodeArgs &a, hipStream_t stream) {
  const int units = a.batch * a.n_kv_heads;
  if (a.chunk & 128)
    hipLaunchKernelGGL((decode_fused_kernel<N_IT, 1>), dim3(a.n_split * units), dim3(kBlock), 0, stream, a);
  else
    hipLaunchKernelGGL((decode_fused_kernel<N_IT, 2>), dim3(a.n_split * units), dim3(kBlock), 0, stream, a);
  return hipGetLastError();
}

// run lengths (sub-tiles per wave) the kernel is instantiated for
constexpr int kRuns[] = {1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 14, 16, 18, 20, 24, 28, 32};

}  // namespace

int decode_fused_split_max() { return kFusedSplitMax; }
int decode_fused_run_max() { return kRuns[sizeof(kRuns) / sizeof(kRuns[0]) - 1]; }

hipError_t launch_decode_fused(const DecodeArgs &a, hipStream_t stream, hipEvent_t *ev) {
  const int units = a.batch * a.n_kv_heads;
  if (a.dtype != 1 || a.head_dim != D || a.group > 8 || a.n_split < 1 ||
      a.n_split > kFusedSplitMax || a.n_split > a.n_split_max || !a.ticket ||
      a.p_stride < (a.n_old + 16) / 16 * 16 || (a.xcd_map && units % 8 != 0))
    return hipErrorInvalidValue;
  const int n_sub = (a.n_old + 1 + 15) / 16, n_wv = kWaves * a.n_split;
  const int run = (n_sub + n_wv - 1) / n_wv;       // longest run of a wave
  if (ev) (void)hipEventRecord(ev[0], stream);
  hipError_t e = hipErrorInvalidValue;
  switch (run <= 12 ? run : run <= 20 ? (run + 1) / 2 * 2 : (run + 3) / 4 * 4) {
    case 1: e = launch_n<1>(a, stream); break;
    case 2: e = launch_n<2>(a, stream); break;
    case 3: e = launch_n<3>(a, stream); break;
    case 4: e = launch_n<4>(a, stream); break;
    case 5: e = launch_n<5>(a, stream); break;
    case 6: e = launch_n<6>(a, stream); break;
    case 7: e = launch_n<7>(a, stream); break;
    case 8: e = launch_n<8>(a, stream); break;
    case 9: e = launch_n<9>(a, stream); break;
    case 10: e = launch_n<10>(a, stream); break;
    case 11: e = launch_n<11>(a, stream); break;
    case 12: e = launch_n<12>(a, stream); break;
    case 14: e = launch_n<14>(a, stream); break;
    case 16: e = launch_n<16>(a, stream); break;
    case 18: e = launch_n<18>(a, stream); break;
    case 20: e = launch_n<20>(a, stream); break;
    case 24: e = launch_n<24>(a, stream); break;
    case 28: e = launch_n<28>(a, stream); break;
    case 32: e = launch_n<32>(a, stream); break;
    default: break;                                 // run too long: the host raises n_split first
  }
  if (ev) { (void)hipEventRecord(ev[1], stream); (void)hipEventRecord(ev[2], stream); }
  return e;
}

}  // namespace lazyev
