// Decode step of one layer with ONE block per unit (bf16, head_dim 128): append, attention
// (Eq. 4 of the paper), and the recurrence tracking of Alg. 1 / Eq. 1, in a single kernel.
//
// A unit's whole cache is streamed by the 16 waves of one 1024-thread block, so nothing has to
// be merged across blocks: the logits live in LDS ([G][C] fp32), the softmax statistics are
// block-wide reductions, the probabilities that the >= alpha test needs never leave the chip,
// and no second kernel is launched.  Used when there are enough units to occupy the machine
// (it runs on `units` compute units); otherwise the split kernels of decode_kernels.hip run.
//
// Work is handed out in 16-entry sub-tiles through an LDS counter: the memory pipeline serves
// the waves of a block unevenly (the oldest waves run ahead), and with a fixed assignment the
// block would wait at every barrier for its slowest wave.  The softmax denominator is kept as
// one partial sum per sub-tile and added up in a fixed order, so probabilities, activation
// decisions and all recurrence state are bitwise reproducible; only the fp32 summation order
// of the output row depends on which wave took which sub-tile.  Two passes, each a software
// pipeline whose loads are unconditional (indices past the end are clamped) so that the
// compiler's load counters stay exact:
//   pass 1  K sub-tile -> S^T = K Q^T by v_mfma_f32_16x16x32_bf16 -> scaled logits to LDS,
//           running max per head;
//   pass 2  V sub-tile, logits from LDS -> exp(s - max) (fp32 back to LDS, bf16 into the
//           product) -> O += P V by v_mfma_f32_16x16x16_bf16 after an in-lane 4x8 transpose.
// MFMA operand layouts (lane l, c = l % 16, g = l / 16):
//   16x16x32: A[row c][k = 8g..8g+7]  B[k = 8g..8g+7][col c]  C[row 4g+i][col c]
//   16x16x16: A[row c][k = 4g..4g+3]  B[k = 4g..4g+3][col c]  C[row 4g+i][col c]
// so a lane that owns head c and entries 4g..4g+3 of a sub-tile after pass 1 already holds the
// A operand of pass 2.
#include "kernels.h"

namespace lazyev {
namespace {

constexpr int kUnitBlock = 1024;
constexpr int kUnitWaves = kUnitBlock / 64;
constexpr int D = 128;
constexpr int KC = D / 32;

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

// Barrier for data exchanged through LDS only: waits for this wave's LDS operations, not for
// its global loads and stores (which __syncthreads would also drain).
__device__ __forceinline__ void lds_barrier() {
  __asm__ volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0), vmcnt and expcnt untouched
  __builtin_amdgcn_s_barrier();
  __asm__ volatile("" ::: "memory");
}

// Row loads of the two streaming passes are issued through inline assembly and waited for
// with explicit counters: inside a loop the compiler's own accounting of outstanding loads
// falls back to draining them all before the next group is issued, which serialises the
// pipeline.  A load's destination registers must not be touched before the matching
// wait_loads<N>() ("at most N younger loads still in flight"), which also ties the registers
// to the wait so that no use can be scheduled ahead of it.
__device__ __forceinline__ void load16_async(u32x4_t &dst, const void *ptr) {
  __asm__ volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(ptr) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads(u32x4_t (&r)[4]) {
  __asm__ volatile("s_waitcnt vmcnt(%4)"
                   : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3])
                   : "n"(N)
                   : "memory");
}

__global__ __launch_bounds__(kUnitBlock) void decode_unit_kernel(const DecodeArgs a) {
  extern __shared__ float dyn_lds[];   // logits [G][c_pad] + sub-tile sums [n_sub][G]; later 16 partial outputs
  __shared__ float red_lds[kUnitWaves][16];
  __shared__ float invl_sh[16];
  __shared__ int next_sub[2];
  __shared__ unsigned cnt_lds[kUnitWaves];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int unit = blockIdx.x;
  const int seq = unit / a.n_kv_heads, kvh = unit % a.n_kv_heads;
  const int G = a.group;
  const int hc = min(c, G - 1);
  const int n_old = a.n_old, n1 = a.n_old + 1;
  const int n_sub = (n1 + 15) >> 4;
  const int c_pad = a.lds_stride;
  const size_t head0 = static_cast<size_t>(seq) * a.n_q_heads + static_cast<size_t>(kvh) * G;

  const bf16_t *kc = static_cast<const bf16_t *>(a.k_cache) + static_cast<size_t>(unit) * a.capacity * D;
  const bf16_t *vc = static_cast<const bf16_t *>(a.v_cache) + static_cast<size_t>(unit) * a.capacity * D;
  const bf16_t *k_new = static_cast<const bf16_t *>(a.k_new) + static_cast<size_t>(unit) * D;
  const bf16_t *v_new = static_cast<const bf16_t *>(a.v_new) + static_cast<size_t>(unit) * D;
  float *s_row = dyn_lds + hc * c_pad + 4 * g;     // this lane's head, its 4 entries of a sub-tile
  float *l_sub = dyn_lds + G * c_pad;              // [n_sub][G]

  if (tid == 0) { next_sub[0] = 0; next_sub[1] = 0; }

  // B operand of the logits: Q^T, head c (zero rows beyond the group)
  u32x4_t qb[KC];
  {
    const bf16_t *q = static_cast<const bf16_t *>(a.q) + (head0 + hc) * D + g * 8;
#pragma unroll
    for (int kk = 0; kk < KC; ++kk) load16_async(qb[kk], q + kk * 32);
  }
  lds_barrier();
  auto fetch = [&](int pass) {
    int v = 0;
    if (lane == 0) v = atomicAdd(&next_sub[pass], 1);
    return __builtin_amdgcn_readfirstlane(v);
  };

  // ---------------------------------------------------------------- pass 1: logits
  float mx = -INFINITY;
  {
    auto load_k = [&](u32x4_t (&dst)[KC], int sub) {
      const int row = min(min(sub, n_sub - 1) * 16 + c, n_old);
      const bf16_t *src = (row == n_old) ? k_new : kc + static_cast<size_t>(row) * D;
#pragma unroll
      for (int kk = 0; kk < KC; ++kk) load16_async(dst[kk], src + kk * 32 + g * 8);
    };
    auto compute_k = [&](const u32x4_t (&buf)[KC], int sub) {
      f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < KC; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, buf[kk]),
                                                      __builtin_bit_cast(bf16x8_t, qb[kk]), acc, 0, 0, 0);
      float4 s4;
      float *sp = &s4.x;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float v = (sub * 16 + 4 * g + i) < n1 ? acc[i] * a.scale : -INFINITY;
        sp[i] = v;
        mx = fmaxf(mx, v);
      }
      if (c < G) *reinterpret_cast<float4 *>(s_row + sub * 16) = s4;
    };
    // software pipeline: the loads of the next sub-tile are in flight while this one is multiplied
    u32x4_t r0[KC], r1[KC];
    int cur = fetch(0);
    load_k(r0, cur);
    wait_loads<4>(qb);
    if (c >= G) {
#pragma unroll
      for (int kk = 0; kk < KC; ++kk) qb[kk] = u32x4_t{0, 0, 0, 0};
    }
    while (cur < n_sub) {
      int nxt = fetch(0);
      load_k(r1, nxt);
      wait_loads<4>(r0);
      compute_k(r0, cur);
      cur = nxt;
      if (cur >= n_sub) break;
      nxt = fetch(0);
      load_k(r0, nxt);
      wait_loads<4>(r1);
      compute_k(r1, cur);
      cur = nxt;
    }
    wait_loads<0>(r0);                             // nothing of this pass is left in flight
  }

  // ---------------------------------------------------------------- pass 2: exp and P V
  float m_glob;
  f32x4_t o[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  {
    auto load_v = [&](u32x4_t (&dst)[4], int sub) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = min(min(sub, n_sub - 1) * 16 + 4 * g + i, n_old);
        const bf16_t *src = (row == n_old) ? v_new : vc + static_cast<size_t>(row) * D;
        load16_async(dst[i], src + c * 8);
      }
    };
    auto compute_v = [&](const u32x4_t (&buf)[4], int sub) {
      float4 s4 = *reinterpret_cast<const float4 *>(s_row + sub * 16);
      s4.x = __expf(s4.x - m_glob); s4.y = __expf(s4.y - m_glob);
      s4.z = __expf(s4.z - m_glob); s4.w = __expf(s4.w - m_glob);
      float ls = (s4.x + s4.y) + (s4.z + s4.w);   // sub-tile share of the softmax denominator
      ls += __shfl_xor(ls, 16);
      ls += __shfl_xor(ls, 32);
      if (c < G) {
        *reinterpret_cast<float4 *>(s_row + sub * 16) = s4;             // kept for the tracking
        if (g == 0) l_sub[sub * G + c] = ls;
      }
      u32x2_t pw;
      pw[0] = static_cast<unsigned>(float_to_bf16(s4.x)) | (static_cast<unsigned>(float_to_bf16(s4.y)) << 16);
      pw[1] = static_cast<unsigned>(float_to_bf16(s4.z)) | (static_cast<unsigned>(float_to_bf16(s4.w)) << 16);
      const s16x4_t pa = __builtin_bit_cast(s16x4_t, pw);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const unsigned sel = (e & 1) ? 0x07060302u : 0x05040100u;
        u32x2_t vb;
        vb[0] = __builtin_amdgcn_perm(buf[1][e >> 1], buf[0][e >> 1], sel);
        vb[1] = __builtin_amdgcn_perm(buf[3][e >> 1], buf[2][e >> 1], sel);
        o[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, __builtin_bit_cast(s16x4_t, vb), o[e], 0, 0, 0);
      }
    };
    u32x4_t va[4], vb2[4];
    int cur = fetch(1);
    load_v(va, cur);                               // in flight across the max exchange below
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (g == 0) red_lds[wave][c] = mx;
    lds_barrier();
    m_glob = red_lds[0][hc];
#pragma unroll
    for (int w = 1; w < kUnitWaves; ++w) m_glob = fmaxf(m_glob, red_lds[w][hc]);
    while (cur < n_sub) {
      int nxt = fetch(1);
      load_v(vb2, nxt);
      wait_loads<4>(va);
      compute_v(va, cur);
      cur = nxt;
      if (cur >= n_sub) break;
      nxt = fetch(1);
      load_v(va, nxt);
      wait_loads<4>(vb2);
      compute_v(vb2, cur);
      cur = nxt;
    }
    wait_loads<0>(va);
  }

  // recurrence state of this thread's first two entries, requested before it is needed
  int32_t *ts = a.ts + static_cast<size_t>(unit) * a.capacity;
  int32_t *mri = a.mri + static_cast<size_t>(unit) * a.capacity;
  int32_t ts_pre[2] = {0, 0}, mri_pre[2] = {0, 0};
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int i = tid + b * kUnitBlock;
    if (i < n_old) { ts_pre[b] = ts[i]; mri_pre[b] = mri[i]; }
  }
  lds_barrier();
  for (int h = wave; h < G; h += kUnitWaves) {     // fixed order: lane-strided, then the lanes
    float l = 0.f;
    for (int sub = lane; sub < n_sub; sub += 64) l += l_sub[sub * G + h];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off);
    if (lane == 0) invl_sh[h] = 1.0f / l;
  }
  lds_barrier();

  // ---------------------------------------------------------------- tracking (Alg. 1, Eq. 1)
  unsigned n_act = 0;
  for (int i = tid, b = 0; i < n1; i += kUnitBlock, ++b) {
    int32_t ts0, mri0;
    if (b < 2) { ts0 = ts_pre[b]; mri0 = mri_pre[b]; }
    else { ts0 = 0; mri0 = 0; if (i < n_old) { ts0 = ts[i]; mri0 = mri[i]; } }
    bool act = false;
    for (int h = 0; h < G; ++h) {
      float p = dyn_lds[h * c_pad + i] * invl_sh[h];
      const size_t at = (head0 + h) * a.capacity + i;
      if (a.p_out) a.p_out[at] = p;
      if (a.p_override) p = a.p_override[at];
      act = act || (p >= a.alpha);
    }
    if (i == n_old) {                              // the appended entry starts here (Sec. 4)
      ts[i] = a.t;
      mri[i] = 0;
      a.pos[static_cast<size_t>(unit) * a.capacity + i] = a.prompt_len + a.t - 1;
    } else if (act) {
      const int32_t gap = a.t - ts0;
      if (gap > mri0) mri[i] = gap;                // Eq. 1
      ts[i] = a.t;                                 // Alg. 1
    }
    n_act += act ? 1u : 0u;
  }
  for (int off = 32; off > 0; off >>= 1) n_act += __shfl_xor(n_act, off);
  if (lane == 0) cnt_lds[wave] = n_act;
  lds_barrier();                                    // the logits in LDS are no longer needed

  // ---------------------------------------------------------------- output row
  // o[e][i] = O[head 4g+i][d = 8c+e] of this wave's share: add up the 16 waves, normalise
  {
    float *mine = dyn_lds + wave * (G * D);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int head = 4 * g + i;
      if (head < G) {
        float *dst = mine + head * D + 8 * c;
        *reinterpret_cast<float4 *>(dst) = make_float4(o[0][i], o[1][i], o[2][i], o[3][i]);
        *reinterpret_cast<float4 *>(dst + 4) = make_float4(o[4][i], o[5][i], o[6][i], o[7][i]);
      }
    }
  }
  lds_barrier();
  if (tid < G * D) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kUnitWaves; ++w) v += dyn_lds[w * (G * D) + tid];
    static_cast<bf16_t *>(a.out)[head0 * D + tid] = float_to_bf16(v * invl_sh[tid / D]);
  }
  if (tid == 0) {
    unsigned total = 0;
    for (int w = 0; w < kUnitWaves; ++w) total += cnt_lds[w];
    if (total) a.activation_counter[unit * 64] += total;
  }
  // the appended row goes to slot N (everybody read it from k_new / v_new)
  if (wave == 1) {
    if (lane < 16)
      reinterpret_cast<uint4 *>(const_cast<bf16_t *>(kc) + static_cast<size_t>(n_old) * D)[lane] =
          reinterpret_cast<const uint4 *>(k_new)[lane];
    else if (lane < 32)
      reinterpret_cast<uint4 *>(const_cast<bf16_t *>(vc) + static_cast<size_t>(n_old) * D)[lane - 16] =
          reinterpret_cast<const uint4 *>(v_new)[lane - 16];
  }
}

}  // namespace

// Dynamic LDS: logits [G][stride] and sub-tile sums [stride/16 + 1][G]; the partial outputs of
// the 16 waves later reuse the space.
size_t decode_unit_stage_offset(int group, int lds_stride) {
  const size_t floats = static_cast<size_t>(group) * lds_stride + static_cast<size_t>(group) * (lds_stride / 16 + 1);
  return (floats * sizeof(float) + 255) / 256 * 256;
}
size_t decode_unit_lds_bytes(int group, int lds_stride) {
  const size_t first = decode_unit_stage_offset(group, lds_stride);
  const size_t partial = static_cast<size_t>(kUnitWaves) * group * D * sizeof(float);
  return first > partial ? first : partial;
}

hipError_t decode_unit_prepare() {
  // one block may use most of the 160 KB of LDS of a compute unit
  return hipFuncSetAttribute(reinterpret_cast<const void *>(decode_unit_kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
}

hipError_t launch_decode_unit(const DecodeArgs &a, hipStream_t stream, hipEvent_t *ev) {
  const size_t lds = decode_unit_lds_bytes(a.group, a.lds_stride);
  if (a.dtype != 1 || a.head_dim != D || lds > 150 * 1024 || a.group * D > kUnitBlock)
    return hipErrorInvalidValue;
  const int units = a.batch * a.n_kv_heads;
  if (ev) (void)hipEventRecord(ev[0], stream);
  hipLaunchKernelGGL(decode_unit_kernel, dim3(units), dim3(kUnitBlock), lds, stream, a);
  const hipError_t e = hipGetLastError();
  if (ev) { (void)hipEventRecord(ev[1], stream); (void)hipEventRecord(ev[2], stream); }
  return e;
}

}  // namespace lazyev
