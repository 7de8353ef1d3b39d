// Causal attention of nq new tokens per series against that series' paged KV cache.
//
// The keys/values of the new tokens were written into the cache by the QKV epilogue, so query t
// (absolute position base + t) simply attends to cache positions 0 .. base + t.
// One wavefront per (series, head).  Queries are processed in chunks of QC; for a chunk the
// keys are read once (one key per lane, dot products against the chunk's queries held in LDS),
// the softmax runs across lanes in fp32, and P.V is accumulated with lanes over the head dim.
#include <type_traits>

#include "tsd_internal.h"

namespace tsd {

constexpr int QC = 8;

template <typename T>
struct Vec;
template <>
struct Vec<float> {
  static constexpr int N = 4;
  __device__ static void load(const float* p, float* o) {
    float4 v = *reinterpret_cast<const float4*>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
};
template <>
struct Vec<bf16> {
  static constexpr int N = 8;
  __device__ static void load(const bf16* p, float* o) {
    bf16x8 v = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (float)v[i];
  }
};

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

template <typename T, int HD>
__global__ __launch_bounds__(64) void attn_kernel(const AttnP p, int s_pad) {
  extern __shared__ float dyn[];
  float* qs = dyn;              // [QC][HD]
  float* ps = dyn + QC * HD;    // [QC][s_pad]
  const int lane = threadIdx.x;
  const int bl = blockIdx.x / p.Hh, h = blockIdx.x % p.Hh;
  const int b = p.s0 + bl;
  const int base = (p.base_pos ? p.base_pos[b] : 0) + p.pos_off;
  const T* pool = reinterpret_cast<const T*>(p.kv_pool);
  const int* pt = p.page_table + (long)b * p.pt_stride;
  const int PT = p.PT, Hh = p.Hh;
  const T* q = reinterpret_cast<const T*>(p.q);
  T* out = reinterpret_cast<T*>(p.out);
  constexpr int G = 64 / HD;  // key groups in the P.V stage
  const int d = lane % HD, sg = lane / HD;

  for (int q0 = 0; q0 < p.nq; q0 += QC) {
    const int nqc = min(QC, p.nq - q0);
    __syncthreads();
    for (int i = lane; i < nqc * HD; i += 64) {
      int j = i / HD, e = i % HD;
      qs[j * HD + e] = (float)q[((long)bl * p.nq + q0 + j) * p.D + h * HD + e] * p.scale;
    }
    __syncthreads();
    const int nkeys = base + q0 + nqc;  // the chunk's last query sees keys 0 .. nkeys-1
    // ---- scores: one key per lane ----
    for (int s = lane; s < nkeys; s += 64) {
      const int page = pt[s / PT];
      const T* kp = pool + ((((long)page * 2 + 0) * Hh + h) * PT + (s % PT)) * HD;
      float sc[QC];
#pragma unroll
      for (int j = 0; j < QC; ++j) sc[j] = 0.f;
#pragma unroll
      for (int v = 0; v < HD / Vec<T>::N; ++v) {
        float kf[Vec<T>::N];
        Vec<T>::load(kp + v * Vec<T>::N, kf);
#pragma unroll
        for (int j = 0; j < QC; ++j)
#pragma unroll
          for (int e = 0; e < Vec<T>::N; ++e) sc[j] = fmaf(kf[e], qs[j * HD + v * Vec<T>::N + e], sc[j]);
      }
#pragma unroll
      for (int j = 0; j < QC; ++j)
        if (j < nqc) ps[j * s_pad + s] = (s <= base + q0 + j) ? sc[j] : -INFINITY;
    }
    __syncthreads();
    // ---- softmax over keys, per query ----
    float inv_sum[QC];
#pragma unroll
    for (int j = 0; j < QC; ++j) {
      inv_sum[j] = 0.f;
      if (j < nqc) {
        float m = -INFINITY;
        for (int s = lane; s < nkeys; s += 64) m = fmaxf(m, ps[j * s_pad + s]);
        m = wave_max(m);
        float sum = 0.f;
        for (int s = lane; s < nkeys; s += 64) {
          float e = __expf(ps[j * s_pad + s] - m);
          ps[j * s_pad + s] = e;
          sum += e;
        }
        inv_sum[j] = 1.f / wave_sum(sum);
      }
    }
    __syncthreads();
    // ---- P.V: lanes over the head dim (G key groups when HD < 64) ----
    float acc[QC];
#pragma unroll
    for (int j = 0; j < QC; ++j) acc[j] = 0.f;
    for (int s = sg; s < nkeys; s += G) {
      const int page = pt[s / PT];
      const float vv = (float)pool[((((long)page * 2 + 1) * Hh + h) * PT + (s % PT)) * HD + d];
#pragma unroll
      for (int j = 0; j < QC; ++j)
        if (j < nqc) acc[j] = fmaf(ps[j * s_pad + s], vv, acc[j]);
    }
    if constexpr (G > 1) {
#pragma unroll
      for (int j = 0; j < QC; ++j)
#pragma unroll
        for (int o = HD; o < 64; o <<= 1) acc[j] += __shfl_xor(acc[j], o);
    }
    if (sg == 0) {
#pragma unroll
      for (int j = 0; j < QC; ++j)
        if (j < nqc) out[((long)bl * p.nq + q0 + j) * p.D + h * HD + d] = (T)(acc[j] * inv_sum[j]);
    }
  }
}

template <typename T>
static hipError_t launch_t(const AttnP& p, hipStream_t st, int s_pad) {
  dim3 grid((unsigned)(p.B * p.Hh)), block(64);
  size_t smem = (size_t)(QC * p.hd + QC * s_pad) * sizeof(float);
  switch (p.hd) {
    case 16: hipLaunchKernelGGL((attn_kernel<T, 16>), grid, block, smem, st, p, s_pad); break;
    case 32: hipLaunchKernelGGL((attn_kernel<T, 32>), grid, block, smem, st, p, s_pad); break;
    case 64: hipLaunchKernelGGL((attn_kernel<T, 64>), grid, block, smem, st, p, s_pad); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_attention(int dtype, const AttnP& p, int s_max, hipStream_t st) {
  if (p.B <= 0 || p.nq <= 0 || s_max <= 0) return hipErrorInvalidValue;
  int s_pad = (s_max + 3) & ~3;
  return dtype == TSD_BF16 ? launch_t<bf16>(p, st, s_pad) : launch_t<float>(p, st, s_pad);
}

}  // namespace tsd
