// Decode step of one layer: append, split attention over the cache (Eq. 4 of the paper),
// combine of the split partials, and the recurrence tracking of Alg. 1 / Eq. 1.
//
// Two kernels per call:
//   split   grid (n_split, units): a block owns `chunk` consecutive entries of one unit.  It
//           streams their K rows (16 bytes per lane, whole rows contiguous across lanes), forms
//           the G logits per entry in fp32, takes the block-local softmax (max, exp, sum),
//           streams the V rows and accumulates the un-normalised partial output.  It leaves
//           the partial (max, sum, output) and exp(s - local max) of every entry in the
//           workspace.  The block holding slot N also stores the appended K/V row.
//   combine grid (n_slice, units): merges the partials into the output row, turns every
//           entry's local exponential into its probability, applies the >= alpha test over
//           the query group and updates TS / MRI in place.
#include "kernels.h"

namespace lazyev {
namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
constexpr int kChunkMax = 256;     // entries per split block (one per thread in the softmax phase)
constexpr int kSliceMax = 64;      // combine blocks per unit (and activation-count slots)
constexpr int kSplitMaxLds = 512;  // split partials the combine kernel can weight in LDS

typedef unsigned short bf16_t;

__device__ __forceinline__ bf16_t float_to_bf16(float f) {   // round to nearest even
  unsigned u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kPerLane = 4;
  __device__ static void unpack(const uint4 &v, float *f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  __device__ static void store(float *p, float x) { *p = x; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kPerLane = 8;
  __device__ static void unpack(const uint4 &v, float *f) {
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
    f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
    f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
  }
  __device__ static void store(bf16_t *p, float x) { *p = float_to_bf16(x); }
};

// Barrier for data exchanged through LDS only: waits for this wave's LDS operations, not for
// its global loads and stores (which __syncthreads would also drain).
__device__ __forceinline__ void lds_barrier() {
  __asm__ volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0), vmcnt and expcnt untouched
  __builtin_amdgcn_s_barrier();
  __asm__ volatile("" ::: "memory");
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// ------------------------------------------------------------------------------------ split
template <typename T, int D, int G>
__global__ __launch_bounds__(kBlock) void decode_split_kernel(const DecodeArgs a) {
  constexpr int EPL = Elem<T>::kPerLane;     // elements in a lane's 16 bytes
  constexpr int LPR = D / EPL;               // lanes per row
  constexpr int RPW = 64 / LPR;              // rows per wave load
  constexpr int ROWS = kWaves * RPW;         // rows per block load
  constexpr int U = 4;                       // row loads kept in flight per lane

  __shared__ float s_lds[G][kChunkMax];
  __shared__ float red_lds[kWaves][8];
  __shared__ float acc_lds[kWaves][G * D];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane % LPR, r = lane / LPR;
  const int unit = blockIdx.y, split = blockIdx.x;
  const int seq = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const int n1 = a.n_old + 1;
  const int tok0 = split * a.chunk;
  const int tok1 = min(n1, tok0 + a.chunk);
  const int n_loc = tok1 - tok0;

  const T *kc = static_cast<const T *>(a.k_cache) + static_cast<size_t>(unit) * a.capacity * D;
  const T *vc = static_cast<const T *>(a.v_cache) + static_cast<size_t>(unit) * a.capacity * D;
  const T *k_new = static_cast<const T *>(a.k_new) + static_cast<size_t>(unit) * D;
  const T *v_new = static_cast<const T *>(a.v_new) + static_cast<size_t>(unit) * D;

  // the block that owns slot N stores the appended row (nobody reads it from the cache now)
  if (a.n_old >= tok0 && a.n_old < tok1) {
    if (tid < LPR) {
      reinterpret_cast<uint4 *>(const_cast<T *>(kc) + static_cast<size_t>(a.n_old) * D)[tid] =
          reinterpret_cast<const uint4 *>(k_new)[tid];
    } else if (tid >= 64 && tid < 64 + LPR) {
      reinterpret_cast<uint4 *>(const_cast<T *>(vc) + static_cast<size_t>(a.n_old) * D)[tid - 64] =
          reinterpret_cast<const uint4 *>(v_new)[tid - 64];
    }
  }

  // this lane's slice of the G query rows
  float qf[G][EPL];
  {
    const T *q = static_cast<const T *>(a.q) +
                 (static_cast<size_t>(seq) * a.n_q_heads + static_cast<size_t>(kvh) * G) * D;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      uint4 v = reinterpret_cast<const uint4 *>(q + g * D)[c];
      Elem<T>::unpack(v, qf[g]);
    }
  }

  // ---- logits
  for (int base = tok0 + wave * RPW + r; base < tok1; base += ROWS * U) {
    uint4 kv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tok = base + u * ROWS;
      kv[u] = make_uint4(0, 0, 0, 0);
      if (tok < tok1) {
        const T *row = (tok < a.n_old) ? kc + static_cast<size_t>(tok) * D : k_new;
        kv[u] = reinterpret_cast<const uint4 *>(row)[c];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tok = base + u * ROWS;
      float kf[EPL];
      Elem<T>::unpack(kv[u], kf);
      float dot[G];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) s = fmaf(qf[g][e], kf[e], s);
        dot[g] = s;
      }
#pragma unroll
      for (int o = LPR / 2; o > 0; o >>= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) dot[g] += __shfl_xor(dot[g], o);
      }
      if (c == 0 && tok < tok1) {
#pragma unroll
        for (int g = 0; g < G; ++g) s_lds[g][tok - tok0] = dot[g] * a.scale;
      }
    }
  }
  __syncthreads();

  // ---- block-local softmax: thread tid owns entry tok0 + tid
  float sv[G];
#pragma unroll
  for (int g = 0; g < G; ++g) sv[g] = (tid < n_loc) ? s_lds[g][tid] : -INFINITY;
  float m_loc[G], l_loc[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float v = wave_max(sv[g]);
    if (lane == 0) red_lds[wave][g] = v;
  }
  __syncthreads();
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float v = red_lds[0][g];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) v = fmaxf(v, red_lds[w][g]);
    m_loc[g] = v;
  }
  __syncthreads();
  {
    float *p_tilde = a.ws.p_tilde +
                     (static_cast<size_t>(seq) * a.n_q_heads + static_cast<size_t>(kvh) * G) * a.p_stride;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float e = (tid < n_loc) ? expf(sv[g] - m_loc[g]) : 0.f;
      if (tid < n_loc) {
        s_lds[g][tid] = e;
        p_tilde[static_cast<size_t>(g) * a.p_stride + tok0 + tid] = e;
      }
      float v = wave_sum(e);
      if (lane == 0) red_lds[wave][g] = v;
    }
  }
  __syncthreads();
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float v = red_lds[0][g];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) v += red_lds[w][g];
    l_loc[g] = v;
  }

  // ---- partial output
  float acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;

  for (int base = tok0 + wave * RPW + r; base < tok1; base += ROWS * U) {
    uint4 vv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tok = base + u * ROWS;
      vv[u] = make_uint4(0, 0, 0, 0);
      if (tok < tok1) {
        const T *row = (tok < a.n_old) ? vc + static_cast<size_t>(tok) * D : v_new;
        vv[u] = reinterpret_cast<const uint4 *>(row)[c];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tok = base + u * ROWS;
      if (tok < tok1) {
        float vf[EPL];
        Elem<T>::unpack(vv[u], vf);
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const float p = s_lds[g][tok - tok0];
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, vf[e], acc[g][e]);
        }
      }
    }
  }
  // rows of one wave, then the waves
#pragma unroll
  for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] += __shfl_xor(acc[g][e], o);
  }
  if (r == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc_lds[wave][g * D + c * EPL + e] = acc[g][e];
  }
  __syncthreads();
  const size_t part = static_cast<size_t>(unit) * a.n_split_max + split;
  float *pa = a.ws.part_acc + part * (G * D);
  for (int i = tid; i < G * D; i += kBlock) {
    float v = acc_lds[0][i];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) v += acc_lds[w][i];
    pa[i] = v;
  }
  if (tid == 0) {
    float *ml = a.ws.part_ml + part * (2 * G);
#pragma unroll
    for (int g = 0; g < G; ++g) {
      ml[g] = m_loc[g];
      ml[G + g] = l_loc[g];
    }
  }
}

// ---------------------------------------------------------------------------------- combine
// One block handles kBlock consecutive entries of one unit and a share of the output row.
// Every global value a thread needs is requested before the first barrier so that the whole
// kernel costs about one memory round trip.
template <typename T, int D>
__global__ __launch_bounds__(kBlock) void decode_combine_kernel(const DecodeArgs a) {
  __shared__ float m_s[16], invl_s[16];
  __shared__ unsigned cnt_lds[kWaves];
  extern __shared__ float dyn_lds[];             // two arrays of [n_split][G]
  constexpr int GMAX = 8;
  constexpr int PRE = 24;                        // partial outputs requested before the barrier

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int unit = blockIdx.y, slice = blockIdx.x, n_slice = gridDim.x;
  const int seq = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const int G = a.group, n_split = a.n_split;
  const int n1 = a.n_old + 1;
  const float *ml = a.ws.part_ml + static_cast<size_t>(unit) * a.n_split_max * (2 * G);
  const size_t head0 = static_cast<size_t>(seq) * a.n_q_heads + static_cast<size_t>(kvh) * G;
  const float *p_tilde = a.ws.p_tilde + head0 * a.p_stride;
  int32_t *ts = a.ts + static_cast<size_t>(unit) * a.capacity;
  int32_t *mri = a.mri + static_cast<size_t>(unit) * a.capacity;
  float *w_lds = dyn_lds;                        // partial max, later the weight of the partial
  float *l_lds = dyn_lds + n_split * G;          // partial sum

  // requests first: this thread's share of the partial outputs ...
  const int per = (G * D + n_slice - 1) / n_slice;
  const int e0 = slice * per + tid;
  const bool has_out = tid < per && e0 < G * D;
  const float *pa = a.ws.part_acc + static_cast<size_t>(unit) * a.n_split_max * (G * D) + e0;
  float px[PRE];
#pragma unroll
  for (int j = 0; j < PRE; ++j)
    px[j] = (has_out && j < n_split) ? pa[static_cast<size_t>(j) * (G * D)] : 0.f;
  // ... this thread's entry ...
  const int i0 = slice * kBlock + tid;
  float pt[GMAX];
  int32_t ts0 = 0, mri0 = 0;
#pragma unroll
  for (int g = 0; g < GMAX; ++g)
    pt[g] = (g < G && i0 < n1) ? p_tilde[static_cast<size_t>(g) * a.p_stride + i0] : 0.f;
  if (i0 < a.n_old) { ts0 = ts[i0]; mri0 = mri[i0]; }
  // ... and the partial statistics of the unit
  for (int i = tid; i < n_split * G; i += kBlock) {
    const int j = i / G, g = i - j * G;
    w_lds[i] = ml[j * (2 * G) + g];
    l_lds[i] = ml[j * (2 * G) + G + g];
  }
  __syncthreads();
  for (int g = wave; g < G; g += kWaves) {
    float m = -INFINITY;
    for (int j = lane; j < n_split; j += 64) m = fmaxf(m, w_lds[j * G + g]);
    m = wave_max(m);
    float l = 0.f;
    for (int j = lane; j < n_split; j += 64) l += l_lds[j * G + g] * expf(w_lds[j * G + g] - m);
    l = wave_sum(l);
    if (lane == 0) { m_s[g] = m; invl_s[g] = 1.0f / l; }
  }
  __syncthreads();
  for (int i = tid; i < n_split * G; i += kBlock) {
    const int g = i % G;
    w_lds[i] = expf(w_lds[i] - m_s[g]) * invl_s[g];
  }
  __syncthreads();

  // output row: out[g][dd] = sum_j w[j][g] * acc_j[g][dd]; the slices share the G*D elements
  if (has_out) {
    const int g = e0 / D;
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < PRE; ++j)
      if (j < n_split) v = fmaf(w_lds[j * G + g], px[j], v);
    for (int j = PRE; j < n_split; ++j) v = fmaf(w_lds[j * G + g], pa[static_cast<size_t>(j) * (G * D)], v);
    Elem<T>::store(static_cast<T *>(a.out) + head0 * D + e0, v);
  }
  for (int k = tid + kBlock; k < per; k += kBlock) {     // only when G*D > n_slice * kBlock
    const int e = slice * per + k;
    if (e < G * D) {
      const int g = e / D;
      const float *pe = a.ws.part_acc + static_cast<size_t>(unit) * a.n_split_max * (G * D) + e;
      float v = 0.f;
      for (int j = 0; j < n_split; ++j) v = fmaf(w_lds[j * G + g], pe[static_cast<size_t>(j) * (G * D)], v);
      Elem<T>::store(static_cast<T *>(a.out) + head0 * D + e, v);
    }
  }

  // probabilities, activation test (Alg. 1) and Eq. 1 for this block's entries
  unsigned n_act = 0;
  for (int i = i0; i < n1; i += n_slice * kBlock) {
    if (i != i0) {                               // only when a unit has more than 64 blocks' worth
#pragma unroll
      for (int g = 0; g < GMAX; ++g)
        pt[g] = g < G ? p_tilde[static_cast<size_t>(g) * a.p_stride + i] : 0.f;
      if (i < a.n_old) { ts0 = ts[i]; mri0 = mri[i]; }
    }
    const int j = i / a.chunk;
    bool act = false;
#pragma unroll
    for (int g = 0; g < GMAX; ++g) {
      if (g < G) {
        float p = pt[g] * w_lds[j * G + g];
        const size_t at = (head0 + g) * a.capacity + i;
        if (a.p_out) a.p_out[at] = p;
        if (a.p_override) p = a.p_override[at];
        act = act || (p >= a.alpha);
      }
    }
    if (i == a.n_old) {                          // the appended entry starts here (Sec. 4)
      ts[i] = a.t;
      mri[i] = 0;
      a.pos[static_cast<size_t>(unit) * a.capacity + i] = a.prompt_len + a.t - 1;
    } else if (act) {
      const int32_t gap = a.t - ts0;
      if (gap > mri0) mri[i] = gap;              // Eq. 1
      ts[i] = a.t;                               // Alg. 1
    }
    n_act += act ? 1u : 0u;
  }
  // activation count: every (unit, slice) block owns one slot, so no atomics are needed
  for (int o = 32; o > 0; o >>= 1) n_act += __shfl_xor(n_act, o);
  if (lane == 0) cnt_lds[wave] = n_act;
  __syncthreads();
  if (tid == 0) {
    unsigned total = 0;
    for (int w = 0; w < kWaves; ++w) total += cnt_lds[w];
    if (total) a.activation_counter[unit * kSliceMax + slice] += total;
  }
}

template <typename T, int D, int G>
hipError_t launch_typed(const DecodeArgs &a, hipStream_t stream, hipEvent_t *ev) {
  const int units = a.batch * a.n_kv_heads;
  dim3 grid_s(a.n_split, units);
  if (ev) (void)hipEventRecord(ev[0], stream);
  hipLaunchKernelGGL((decode_split_kernel<T, D, G>), grid_s, dim3(kBlock), 0, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (ev) (void)hipEventRecord(ev[1], stream);
  const int n1 = a.n_old + 1;
  int n_slice = (n1 + kBlock - 1) / kBlock;
  if (n_slice > kSliceMax) n_slice = kSliceMax;
  dim3 grid_c(n_slice, units);
  hipLaunchKernelGGL((decode_combine_kernel<T, D>), grid_c, dim3(kBlock),
                     2 * a.n_split * a.group * sizeof(float), stream, a);
  e = hipGetLastError();
  if (ev) (void)hipEventRecord(ev[2], stream);
  return e;
}

template <typename T, int D>
hipError_t launch_group(const DecodeArgs &a, hipStream_t stream, hipEvent_t *ev) {
  switch (a.group) {
    case 1: return launch_typed<T, D, 1>(a, stream, ev);
    case 2: return launch_typed<T, D, 2>(a, stream, ev);
    case 3: return launch_typed<T, D, 3>(a, stream, ev);
    case 4: return launch_typed<T, D, 4>(a, stream, ev);
    case 5: return launch_typed<T, D, 5>(a, stream, ev);
    case 6: return launch_typed<T, D, 6>(a, stream, ev);
    case 7: return launch_typed<T, D, 7>(a, stream, ev);
    case 8: return launch_typed<T, D, 8>(a, stream, ev);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

int decode_chunk_max() { return kChunkMax; }
int decode_split_max() { return kSplitMaxLds; }
int decode_slice_max() { return kSliceMax; }

hipError_t launch_decode(const DecodeArgs &a, hipStream_t stream, hipEvent_t *ev) {
  if (a.variant == 4 || a.variant == 6) return launch_decode_fused(a, stream, ev);
  if (a.chunk <= 0 || a.chunk > kChunkMax || a.n_split > kSplitMaxLds ||
      a.n_split > a.n_split_max || static_cast<long long>(a.n_split) * a.chunk < a.n_old + 1)
    return hipErrorInvalidValue;
  if (a.dtype == 0) {
    if (a.head_dim == 64) return launch_group<float, 64>(a, stream, ev);
    if (a.head_dim == 128) return launch_group<float, 128>(a, stream, ev);
  } else {
    if (a.head_dim == 64) return launch_group<bf16_t, 64>(a, stream, ev);
    if (a.head_dim == 128) return launch_group<bf16_t, 128>(a, stream, ev);
  }
  return hipErrorInvalidValue;
}

}  // namespace lazyev
