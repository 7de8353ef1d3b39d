// Causal attention of nq new tokens per series against that series' paged KV cache.
//
// The keys/values of the new tokens were written into the cache by the QKV epilogue, so query t
// (absolute position base + t) simply attends to cache positions 0 .. base + t.
//
// One wavefront per (series, head).  The head's K and V rows (at most a few hundred tokens) are
// staged into LDS once with 16-byte loads that are all in flight together (the pass is bound by
// HBM latency/bandwidth, not arithmetic); queries are then processed in chunks of QC:
// scores with one key per lane, fp32 softmax across lanes, P.V with lanes over the head dim.
#include <type_traits>

#include "tsd_internal.h"
#include "attn_mfma.h"

namespace tsd {

constexpr int QC = 8;

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

template <typename T>
__device__ __forceinline__ void unpack16(const uint4& r, float* o);
template <>
__device__ __forceinline__ void unpack16<float>(const uint4& r, float* o) {
  const float4 f = *reinterpret_cast<const float4*>(&r);
  o[0] = f.x; o[1] = f.y; o[2] = f.z; o[3] = f.w;
}
template <>
__device__ __forceinline__ void unpack16<bf16>(const uint4& r, float* o) {
  const bf16x8 v = *reinterpret_cast<const bf16x8*>(&r);
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (float)v[i];
}

// LDS bytes of one staged K (or V) row: the head's HD elements plus 16 bytes of padding so that
// consecutive rows start in different banks.
__host__ __device__ constexpr int row_bytes(int hd, int es) { return hd * es + 16; }

template <typename T, int HD>
__global__ __launch_bounds__(64) void attn_kernel(const AttnP p, int s_pad) {
  constexpr int ES = (int)sizeof(T);
  constexpr int RB = row_bytes(HD, ES);
  constexpr int CPR = HD * ES / 16;   // 16-byte chunks per row
  constexpr int EPC = 16 / ES;        // elements per chunk
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn[];
  unsigned char* Ks = dyn;                                   // [s_pad][RB]
  unsigned char* Vs = dyn + (size_t)s_pad * RB;              // [s_pad][RB]
  float* qs = reinterpret_cast<float*>(Vs + (size_t)s_pad * RB);  // [QC][HD]
  float* ps = qs + QC * HD;                                  // [QC][s_pad]

  const int lane = threadIdx.x;
  const int bl = blockIdx.x / p.Hh, h = blockIdx.x % p.Hh;
  const int b = p.act ? p.act[bl] : p.s0 + bl;  // (entries past the active count are stale but valid series)
  const int PT = p.PT, Hh = p.Hh, pts = p.pt_shift;
  const T* q = reinterpret_cast<const T*>(p.q);
  T* out = reinterpret_cast<T*>(p.out);

  // Independent loads first, all in flight together: this lane's page-table entry, the series'
  // base position, and the first chunk's queries.
  const int my_page = p.page_table[(long)b * p.pt_stride + min(lane, p.pt_stride - 1)];
  const int base = (p.base_pos ? p.base_pos[b] : 0) + p.pos_off;
  if (p.n_dev && bl >= *p.n_dev) return;  // replayed launch: this slot is past the active list
  constexpr int QR = QC * HD / 64;
  float qreg[QR];
  {
    const int n_first = min(QC, p.nq) * HD;
#pragma unroll
    for (int r = 0; r < QR; ++r) {
      const int i = min(lane + r * 64, n_first - 1);
      qreg[r] = (float)q[((long)bl * p.nq + i / HD) * p.D + h * HD + i % HD];
    }
  }
  const int total_keys = base + p.nq;

  // ---- stage this head's K and V rows (page ids come from other lanes' registers) ----
  {
    const unsigned char* pool = reinterpret_cast<const unsigned char*>(p.kv_pool);
    const int total = total_keys * CPR;
    constexpr int U = 4;
    // uniform trip count: every lane stays active, so the page-id shuffles see all lanes
    for (int base_c = 0; base_c < total; base_c += 64 * U) {
      const int c0 = base_c + lane;
      uint4 rk[U], rv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int c = min(c0 + u * 64, total - 1);  // clamped: always a valid row, stored only if in range
        const int s = c / CPR, kc = c % CPR;
        const int page = __shfl(my_page, s >> pts);
        const long rowk = ((((long)page * 2 + 0) * Hh + h) * PT + (s & (PT - 1))) * HD;
        const long rowv = rowk + (long)Hh * PT * HD;
        rk[u] = *reinterpret_cast<const uint4*>(pool + rowk * ES + kc * 16);
        rv[u] = *reinterpret_cast<const uint4*>(pool + rowv * ES + kc * 16);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int c = c0 + u * 64;
        if (c < total) {
          const int s = c / CPR, kc = c % CPR;
          *reinterpret_cast<uint4*>(Ks + (size_t)s * RB + kc * 16) = rk[u];
          *reinterpret_cast<uint4*>(Vs + (size_t)s * RB + kc * 16) = rv[u];
        }
      }
    }
  }

  constexpr int G = 64 / HD;  // key groups in the P.V stage
  const int d = lane % HD, sg = lane / HD;

  for (int q0 = 0; q0 < p.nq; q0 += QC) {
    const int nqc = min(QC, p.nq - q0);
    __syncthreads();  // staging done / previous chunk's ps and qs no longer read
    if (q0 == 0) {
#pragma unroll
      for (int r = 0; r < QR; ++r) qs[lane + r * 64] = qreg[r] * p.scale;
    } else {
      for (int i = lane; i < nqc * HD; i += 64) {
        const int j = i / HD, e = i % HD;
        qs[j * HD + e] = (float)q[((long)bl * p.nq + q0 + j) * p.D + h * HD + e] * p.scale;
      }
    }
    __syncthreads();
    const int nkeys = base + q0 + nqc;  // the chunk's last query sees keys 0 .. nkeys-1
    // ---- scores: one key per lane ----
    for (int s = lane; s < nkeys; s += 64) {
      float sc[QC];
#pragma unroll
      for (int j = 0; j < QC; ++j) sc[j] = 0.f;
#pragma unroll
      for (int v = 0; v < CPR; ++v) {
        float kf[EPC];
        unpack16<T>(*reinterpret_cast<const uint4*>(Ks + (size_t)s * RB + v * 16), kf);
#pragma unroll
        for (int j = 0; j < QC; ++j) {
          if (j < nqc) {
#pragma unroll
            for (int e4 = 0; e4 < EPC; e4 += 4) {
              const float4 qq = *reinterpret_cast<const float4*>(qs + j * HD + v * EPC + e4);
              sc[j] = fmaf(kf[e4 + 0], qq.x, sc[j]);
              sc[j] = fmaf(kf[e4 + 1], qq.y, sc[j]);
              sc[j] = fmaf(kf[e4 + 2], qq.z, sc[j]);
              sc[j] = fmaf(kf[e4 + 3], qq.w, sc[j]);
            }
          }
        }
      }
#pragma unroll
      for (int j = 0; j < QC; ++j)
        if (j < nqc) ps[j * s_pad + s] = (s <= base + q0 + j) ? sc[j] : -INFINITY;
    }
    // keys nkeys .. round-up-to-4 are read (as zeros) by the vectorised P.V loop
    const int nk4 = (nkeys + 3) & ~3;
    for (int i = lane; i < nqc * (nk4 - nkeys); i += 64) {
      const int j = i / (nk4 - nkeys), s = nkeys + i % (nk4 - nkeys);
      ps[j * s_pad + s] = -INFINITY;
    }
    __syncthreads();
    // ---- softmax over keys, per query ----
    float inv_sum[QC];
#pragma unroll
    for (int j = 0; j < QC; ++j) {
      inv_sum[j] = 0.f;
      if (j < nqc) {
        float m = -INFINITY;
        for (int s = lane; s < nk4; s += 64) m = fmaxf(m, ps[j * s_pad + s]);
        m = wave_max(m);
        float sum = 0.f;
        for (int s = lane; s < nk4; s += 64) {
          const float e = __expf(ps[j * s_pad + s] - m);
          ps[j * s_pad + s] = e;
          sum += e;
        }
        inv_sum[j] = 1.f / wave_sum(sum);
      }
    }
    __syncthreads();
    // ---- P.V: lanes over the head dim (G key groups when HD < 64), four keys per step ----
    float acc[QC];
#pragma unroll
    for (int j = 0; j < QC; ++j) acc[j] = 0.f;
    for (int s4 = sg * 4; s4 < nk4; s4 += 4 * G) {
      float vv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        vv[u] = (s4 + u < nkeys) ? (float)*reinterpret_cast<const T*>(Vs + (size_t)(s4 + u) * RB + d * ES) : 0.f;
#pragma unroll
      for (int j = 0; j < QC; ++j) {
        if (j < nqc) {
          const float4 pp = *reinterpret_cast<const float4*>(ps + j * s_pad + s4);
          acc[j] = fmaf(pp.x, vv[0], acc[j]);
          acc[j] = fmaf(pp.y, vv[1], acc[j]);
          acc[j] = fmaf(pp.z, vv[2], acc[j]);
          acc[j] = fmaf(pp.w, vv[3], acc[j]);
        }
      }
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

// ---- bf16, head_dim 64: attention on the matrix cores (core in attn_mfma.h) ---------------------
// MODEL (TSD_TARGET / TSD_DRAFT) changes nothing in the code: the two models' passes run under two kernel names so
// that a profiler's per-kernel statistics keep the target's large passes apart from the draft's small ones.
// Three wavefronts per SIMD asked for: the kernel needs 142 registers, which allows three, and told so the compiler
// schedules for it (66 against 69 us for 1024 series x 16 heads x 66 keys; four costs spills and 76 us).  Two 32-key
// steps per trip: three (one trip for 65 .. 96 keys instead of a full and an all but empty one) took 174 registers
// and 72 us.
template <int MODEL>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(3, 3))) void attn_mfma_kernel(const AttnP p) {
  constexpr int NST = 2;
  __shared__ __attribute__((aligned(16))) bf16 vt[NST * 32 * 64];  // the V rows of a trip's 32-key steps
  const int lane = threadIdx.x;
  const int bl = blockIdx.x / p.Hh, h = blockIdx.x % p.Hh;
  const int b = p.act ? p.act[bl] : p.s0 + bl;  // (entries past the active count are stale but valid series)
  const bf16* q = reinterpret_cast<const bf16*>(p.q);
  bf16* out = reinterpret_cast<bf16*>(p.out);
  const bf16* pool = reinterpret_cast<const bf16*>(p.kv_pool);
  const int my_page = p.page_table[(long)b * p.pt_stride + min(lane, p.pt_stride - 1)];
  const int base = (p.base_pos ? p.base_pos[b] : 0) + p.pos_off;
  if (p.n_dev && bl >= *p.n_dev) return;  // replayed launch: this slot is past the active list
  for (int q0 = 0; q0 < p.nq; q0 += 16) {
    const int nqt = min(16, p.nq - q0);
    const bf16* qt = q + ((long)bl * p.nq + q0) * p.D + h * 64;
    bf16* ot = out + ((long)bl * p.nq + q0) * p.D + h * 64;
    attn_tile_mfma<true, NST>(pool, h, p.Hh, p.PT, p.pt_shift, my_page, base + q0, nqt, p.scale,
                       [&](int r) { return qt + (long)r * p.D; }, [&](int r) { return ot + (long)r * p.D; }, vt);
  }
}

size_t attention_lds_bytes(int dtype, int hd, int s_max, int page_tokens) {
  const int es = dtype == TSD_BF16 ? 2 : 4;
  const int s_pad = (s_max + 3) & ~3;
  const int pages = (s_pad + page_tokens - 1) / page_tokens + 1;
  return (size_t)2 * s_pad * row_bytes(hd, es) + (size_t)(QC * hd + QC * s_pad) * 4 + (size_t)pages * 4;
}

template <typename T, int HD>
static hipError_t launch_hd(const AttnP& p, hipStream_t st, int s_pad, size_t smem) {
  hipLaunchKernelGGL((attn_kernel<T, HD>), dim3((unsigned)(p.B * p.Hh)), dim3(64), smem, st, p, s_pad);
  return hipGetLastError();
}

template <typename T, int HD>
static hipError_t raise_lds() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_kernel<T, HD>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

// More than 64 KB of dynamic LDS needs a one-time opt-in per kernel; done at handle creation so
// that no such call happens while a stream is being captured.
hipError_t prepare_attention(int dtype, int hd, int s_max, int page_tokens) {
  if (attention_lds_bytes(dtype, hd, s_max, page_tokens) <= 64 * 1024) return hipSuccess;
  const bool bf = dtype == TSD_BF16;
  switch (hd) {
    case 16: return bf ? raise_lds<bf16, 16>() : raise_lds<float, 16>();
    case 32: return bf ? raise_lds<bf16, 32>() : raise_lds<float, 32>();
    case 64: return bf ? raise_lds<bf16, 64>() : raise_lds<float, 64>();
    default: return hipErrorInvalidValue;
  }
}

template <typename T>
static hipError_t launch_t(const AttnP& p, hipStream_t st, int s_pad, size_t smem) {
  switch (p.hd) {
    case 16: return launch_hd<T, 16>(p, st, s_pad, smem);
    case 32: return launch_hd<T, 32>(p, st, s_pad, smem);
    case 64: return launch_hd<T, 64>(p, st, s_pad, smem);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_attention(int dtype, const AttnP& p, int s_max, hipStream_t st) {
  if (p.B <= 0 || p.nq <= 0 || s_max <= 0) return hipErrorInvalidValue;
  if (p.mfma) {
    if (dtype != TSD_BF16 || p.hd != 64 || p.PT < 8) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(p.B * p.Hh)), block(64);
    if (p.model == TSD_DRAFT) hipLaunchKernelGGL(attn_mfma_kernel<TSD_DRAFT>, grid, block, 0, st, p);
    else hipLaunchKernelGGL(attn_mfma_kernel<TSD_TARGET>, grid, block, 0, st, p);
    return hipGetLastError();
  }
  const int s_pad = (s_max + 3) & ~3;
  const size_t smem = attention_lds_bytes(dtype, p.hd, s_max, p.PT);
  if (smem > 160 * 1024) return hipErrorInvalidValue;
  return dtype == TSD_BF16 ? launch_t<bf16>(p, st, s_pad, smem) : launch_t<float>(p, st, s_pad, smem);
}

}  // namespace tsd
