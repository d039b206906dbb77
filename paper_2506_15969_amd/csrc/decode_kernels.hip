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
constexpr int kSplitMaxLds = 1024; // split partials the combine kernel can weight in LDS

typedef unsigned short bf16_t;

__device__ __forceinline__ float bf16_to_float(bf16_t x) {
  return __uint_as_float(static_cast<unsigned>(x) << 16);
}
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
                     (static_cast<size_t>(seq) * a.n_q_heads + static_cast<size_t>(kvh) * G) * a.capacity;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float e = (tid < n_loc) ? expf(sv[g] - m_loc[g]) : 0.f;
      if (tid < n_loc) {
        s_lds[g][tid] = e;
        p_tilde[static_cast<size_t>(g) * a.capacity + tok0 + tid] = e;
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
template <typename T, int D, int G>
__global__ __launch_bounds__(kBlock) void decode_combine_kernel(const DecodeArgs a) {
  __shared__ float m_s[8], invl_s[8];
  __shared__ float w_lds[kSplitMaxLds][G];
  __shared__ unsigned cnt_lds[kWaves];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int unit = blockIdx.y, slice = blockIdx.x, n_slice = gridDim.x;
  const int seq = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const int n1 = a.n_old + 1;
  const float *ml = a.ws.part_ml + static_cast<size_t>(unit) * a.n_split_max * (2 * G);

  if (wave == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float m = -INFINITY;
      for (int j = lane; j < a.n_split; j += 64) m = fmaxf(m, ml[j * (2 * G) + g]);
      m = wave_max(m);
      float l = 0.f;
      for (int j = lane; j < a.n_split; j += 64)
        l += ml[j * (2 * G) + G + g] * expf(ml[j * (2 * G) + g] - m);
      l = wave_sum(l);
      if (lane == 0) { m_s[g] = m; invl_s[g] = 1.0f / l; }
    }
  }
  __syncthreads();
  for (int i = tid; i < a.n_split * G; i += kBlock) {
    const int j = i / G, g = i % G;
    w_lds[j][g] = expf(ml[j * (2 * G) + g] - m_s[g]) * invl_s[g];
  }
  __syncthreads();

  // output row: out[g][dd] = sum_j w[j][g] * acc_j[g][dd]
  {
    const float *pa = a.ws.part_acc + static_cast<size_t>(unit) * a.n_split_max * (G * D);
    T *out = static_cast<T *>(a.out) +
             (static_cast<size_t>(seq) * a.n_q_heads + static_cast<size_t>(kvh) * G) * D;
    for (int e = slice * kBlock + tid; e < G * D; e += n_slice * kBlock) {
      const int g = e / D;
      float v = 0.f;
      for (int j = 0; j < a.n_split; ++j) v = fmaf(w_lds[j][g], pa[static_cast<size_t>(j) * (G * D) + e], v);
      Elem<T>::store(out + e, v);
    }
  }

  // probabilities, activation test (Alg. 1) and Eq. 1 for this block's entries
  const size_t row0 = (static_cast<size_t>(seq) * a.n_q_heads + static_cast<size_t>(kvh) * G) * a.capacity;
  const float *p_tilde = a.ws.p_tilde + row0;
  int32_t *ts = a.ts + static_cast<size_t>(unit) * a.capacity;
  int32_t *mri = a.mri + static_cast<size_t>(unit) * a.capacity;
  unsigned n_act = 0;
  for (int i = slice * kBlock + tid; i < n1; i += n_slice * kBlock) {
    const int j = i / a.chunk;
    bool act = false;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float p = p_tilde[static_cast<size_t>(g) * a.capacity + i] * w_lds[j][g];
      if (a.p_out) a.p_out[row0 + static_cast<size_t>(g) * a.capacity + i] = p;
      if (a.p_override) p = a.p_override[row0 + static_cast<size_t>(g) * a.capacity + i];
      act = act || (p >= a.alpha);
    }
    if (i == a.n_old) {                       // the appended entry starts here (Sec. 4)
      ts[i] = a.t;
      mri[i] = 0;
      a.pos[static_cast<size_t>(unit) * a.capacity + i] = a.prompt_len + a.t - 1;
    } else if (act) {
      const int32_t prev = ts[i];
      const int32_t gap = a.t - prev;
      if (gap > mri[i]) mri[i] = gap;         // Eq. 1
      ts[i] = a.t;                            // Alg. 1
    }
    n_act += act ? 1u : 0u;
  }
  // activation count of the layer
  for (int o = 32; o > 0; o >>= 1) n_act += __shfl_xor(n_act, o);
  if (lane == 0) cnt_lds[wave] = n_act;
  __syncthreads();
  if (tid == 0) {
    unsigned total = 0;
    for (int w = 0; w < kWaves; ++w) total += cnt_lds[w];
    if (total) atomicAdd(a.activation_counter, static_cast<unsigned long long>(total));
  }
}

template <typename T, int D, int G>
hipError_t launch_typed(const DecodeArgs &a, hipStream_t stream, hipEvent_t *ev) {
  const int units = a.batch * a.n_kv_heads;
  dim3 grid_s(a.n_split, units);
  if (ev) hipEventRecord(ev[0], stream);
  hipLaunchKernelGGL((decode_split_kernel<T, D, G>), grid_s, dim3(kBlock), 0, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (ev) hipEventRecord(ev[1], stream);
  const int n1 = a.n_old + 1;
  int n_slice = (n1 + kBlock - 1) / kBlock;
  const int min_slice = (G * D + kBlock - 1) / kBlock;
  if (n_slice < min_slice) n_slice = min_slice;
  if (n_slice > 64) n_slice = 64;
  dim3 grid_c(n_slice, units);
  hipLaunchKernelGGL((decode_combine_kernel<T, D, G>), grid_c, dim3(kBlock), 0, stream, a);
  e = hipGetLastError();
  if (ev) hipEventRecord(ev[2], stream);
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

hipError_t launch_decode(const DecodeArgs &a, hipStream_t stream, hipEvent_t *ev) {
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
