// Fused GEMM family: C[M,N] = A[M,K] * Wt[N,K]^T with fp32 accumulation.
//
// One kernel template covers every dense contraction of the transformer pass (patch embedding,
// QKV, attention output, FFN up/down, output head).  What varies is where the A rows come from
// (AMode) and what happens to the product (Epi); the main loop is the same:
//   global -> registers -> LDS (double buffered) -> MFMA 32x32x16 bf16 (or fp32 FMAs) -> LDS -> epilogue.
// RMSNorm is never materialised: with the gain folded into the weights at load time,
//   RMSNorm(x) W = rsqrt(mean(x^2) + eps) * (x W'),
// so the kernel accumulates the row's sum of squares while it streams the row through and
// scales the product's row in the epilogue.
#include <type_traits>

#include "tsd_internal.h"

namespace tsd {

__device__ __forceinline__ float gelu_tanh(float z) {
  const float c = 0.7978845608028654f;  // sqrt(2/pi)
  return 0.5f * z * (1.0f + tanhf(c * (z + 0.044715f * z * z * z)));
}

template <typename T>
__device__ __forceinline__ void store4(T* dst, float4 v);
template <>
__device__ __forceinline__ void store4<float>(float* dst, float4 v) {
  *reinterpret_cast<float4*>(dst) = v;
}
template <>
__device__ __forceinline__ void store4<bf16>(bf16* dst, float4 v) {
  bf16x4 o;
  o[0] = (bf16)v.x;
  o[1] = (bf16)v.y;
  o[2] = (bf16)v.z;
  o[3] = (bf16)v.w;
  *reinterpret_cast<bf16x4*>(dst) = o;
}

template <typename T, int AM, int EP, int BM, int BN, int BK>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmP p) {
  constexpr bool kBf = !std::is_same<T, float>::value;
  constexpr int LDT = BK + (kBf ? 8 : 1);  // padded LDS row, in elements
  constexpr int LDC = BN + 4;
  constexpr int AB_BYTES = 2 * (BM + BN) * LDT * (int)sizeof(T);
  constexpr int C_BYTES = 64 * LDC * 4;
  constexpr int SMEM = AB_BYTES > C_BYTES ? AB_BYTES : C_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];
  __shared__ float row_scale[BM];
  T* As = reinterpret_cast<T*>(smem);  // [2][BM][LDT]
  T* Bs = As + 2 * BM * LDT;           // [2][BN][LDT]
  float* Cs = reinterpret_cast<float*>(smem);  // [64][LDC], reuses the tile buffers

  const int tid = threadIdx.x;
  const int tiles_n = (p.N + BN - 1) / BN;
  const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;
  const int M = p.M, N = p.N, K = p.K;

  // ---- A loader set-up ----------------------------------------------------------------------
  constexpr bool kASrcF32 = (AM != A_ACT) || !kBf;   // source rows are fp32
  constexpr int CHA = kASrcF32 ? 4 : 8;              // elements per 16-byte chunk
  constexpr int CPRA = BK / CHA;                     // chunks per tile row
  constexpr int NA = BM * CPRA / 256;
  static_assert(NA >= 1, "tile too small for 256 threads");
  const char* arow[NA];
  int a_r[NA], a_kc[NA];
  float ss[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    int id = tid + i * 256;
    a_r[i] = id / CPRA;
    a_kc[i] = id % CPRA;
    ss[i] = 0.f;
    int gm = m0 + a_r[i];
    arow[i] = nullptr;
    if (gm < M) {
      if constexpr (AM == A_TOK) {
        int b = gm / p.nq, t = gm % p.nq;
        const float* src = (t < p.n0) ? p.src0 + (long)b * p.stride0 + (long)t * K
                                      : p.src1 + (long)b * p.stride1 + (long)(t - p.n0) * K;
        arow[i] = reinterpret_cast<const char*>(src);
      } else if constexpr (kASrcF32) {
        arow[i] = reinterpret_cast<const char*>(reinterpret_cast<const float*>(p.A) + (long)gm * K);
      } else {
        arow[i] = reinterpret_cast<const char*>(reinterpret_cast<const T*>(p.A) + (long)gm * K);
      }
    }
  }
  // ---- B loader set-up ----------------------------------------------------------------------
  constexpr int CHB = kBf ? 8 : 4;
  constexpr int CPRB = BK / CHB;
  constexpr int NB = BN * CPRB / 256;
  static_assert(NB >= 1, "tile too small for 256 threads");
  const char* brow[NB];
  int b_r[NB], b_kc[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    int id = tid + i * 256;
    b_r[i] = id / CPRB;
    b_kc[i] = id % CPRB;
    int gn = n0 + b_r[i];
    brow[i] = gn < N ? reinterpret_cast<const char*>(reinterpret_cast<const T*>(p.W) + (long)gn * K) : nullptr;
  }

  // Two tiles are kept in flight in two register sets that alternate (no copies between them:
  // a copy would wait for the younger load), so the HBM latency of one tile overlaps the MFMA
  // work and LDS traffic of two others.
  uint4 ra0[NA], rb0[NB], ra1[NA], rb1[NB];
  auto load_global = [&](int kt, uint4* xa, uint4* xb) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      int k = kt * BK + a_kc[i] * CHA;
      xa[i] = make_uint4(0, 0, 0, 0);
      if (arow[i] && k < K) xa[i] = *reinterpret_cast<const uint4*>(arow[i] + (long)k * (kASrcF32 ? 4 : 2));
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      int k = kt * BK + b_kc[i] * CHB;
      xb[i] = make_uint4(0, 0, 0, 0);
      if (brow[i] && k < K) xb[i] = *reinterpret_cast<const uint4*>(brow[i] + (long)k * (int)sizeof(T));
    }
  };
  auto store_lds = [&](int buf, uint4* ra, uint4* rb) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      T* dst = As + (buf * BM + a_r[i]) * LDT + a_kc[i] * CHA;
      if constexpr (kASrcF32) {
        float4 f = *reinterpret_cast<float4*>(&ra[i]);
        if constexpr (AM == A_NORM) ss[i] += f.x * f.x + f.y * f.y + f.z * f.z + f.w * f.w;
        if constexpr (kBf) {
          store4<bf16>(reinterpret_cast<bf16*>(dst), f);
        } else {
          dst[0] = f.x;
          dst[1] = f.y;
          dst[2] = f.z;
          dst[3] = f.w;
        }
      } else {
        *reinterpret_cast<uint4*>(dst) = ra[i];
      }
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      T* dst = Bs + (buf * BN + b_r[i]) * LDT + b_kc[i] * CHB;
      if constexpr (kBf) {
        *reinterpret_cast<uint4*>(dst) = rb[i];
      } else {
        float4 f = *reinterpret_cast<float4*>(&rb[i]);
        dst[0] = f.x;
        dst[1] = f.y;
        dst[2] = f.z;
        dst[3] = f.w;
      }
    }
  };

  // ---- accumulators -------------------------------------------------------------------------
  const int lane = tid & 63, wid = tid >> 6;
  const int wm = wid >> 1, wn = wid & 1;
  constexpr int WTM = BM / 2, WTN = BN / 2;            // wave tile (bf16 path)
  constexpr int TM = kBf ? WTM / 32 : 1, TN = kBf ? WTN / 32 : 1;
  f32x16 acc[TM][TN];
  float accf[4][4];
  if constexpr (kBf) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  } else {
    static_assert(kBf || (BM == 64 && BN == 64), "fp32 path uses 64x64 tiles");
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) accf[i][j] = 0.f;
  }
  const int ty = tid >> 4, tx = tid & 15;  // fp32 path: 4x4 micro-tile at (ty*4, tx*4)

  // ---- main loop ----------------------------------------------------------------------------
  auto compute = [&](int buf) {
    const T* at = As + buf * BM * LDT;
    const T* bt = Bs + buf * BN * LDT;
    if constexpr (kBf) {
#pragma unroll
      for (int k16 = 0; k16 < BK / 16; ++k16) {
        bf16x8 af[TM], bfr[TN];
        const int ko = k16 * 16 + (lane >> 5) * 8;
#pragma unroll
        for (int i = 0; i < TM; ++i)
          af[i] = *reinterpret_cast<const bf16x8*>(at + (wm * WTM + i * 32 + (lane & 31)) * LDT + ko);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          bfr[j] = *reinterpret_cast<const bf16x8*>(bt + (wn * WTN + j * 32 + (lane & 31)) * LDT + ko);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int k = 0; k < BK; ++k) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = at[(ty * 4 + i) * LDT + k];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = bt[(tx * 4 + j) * LDT + k];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) accf[i][j] = fmaf(a[i], b[j], accf[i][j]);
      }
    }
  };
  const int nk = (K + BK - 1) / BK;
  load_global(0, ra0, rb0);
  if (nk > 1) load_global(1, ra1, rb1);
  store_lds(0, ra0, rb0);
  __syncthreads();
  for (int kt = 0; kt < nk; kt += 2) {
    // even tile: lives in LDS buffer 0; set 1 holds tile kt+1, set 0 is free for tile kt+2
    if (kt + 2 < nk) load_global(kt + 2, ra0, rb0);
    compute(0);
    if (kt + 1 < nk) store_lds(1, ra1, rb1);
    __syncthreads();
    if (kt + 1 >= nk) break;
    // odd tile: LDS buffer 1; set 0 holds tile kt+2, set 1 is free for tile kt+3
    if (kt + 3 < nk) load_global(kt + 3, ra1, rb1);
    compute(1);
    if (kt + 2 < nk) store_lds(0, ra0, rb0);
    __syncthreads();
  }

  // ---- RMSNorm row scale --------------------------------------------------------------------
  if constexpr (AM == A_NORM) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      float s = ss[i];
#pragma unroll
      for (int o = CPRA / 2; o >= 1; o >>= 1) s += __shfl_xor(s, o);
      if (a_kc[i] == 0) row_scale[a_r[i]] = rsqrtf(s / (float)K + kRmsEps);
    }
  }

  // ---- epilogue, 64 rows at a time through LDS ----------------------------------------------
  for (int pass = 0; pass < BM / 64; ++pass) {
    __syncthreads();  // tile buffers (or the previous pass's Cs) are no longer read
    if constexpr (kBf) {
      // accumulator element r of a 32x32 block: row (r/4)*8 + (lane/32)*4 + r%4, column lane%32
      if (BM == 64 || wm == pass) {
        const int rbase = (BM == 64) ? wm * WTM : 0;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              int row = rbase + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
              int col = wn * WTN + j * 32 + (lane & 31);
              Cs[row * LDC + col] = acc[i][j][r];
            }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) Cs[(ty * 4 + i) * LDC + tx * 4 + j] = accf[i][j];
    }
    __syncthreads();
    constexpr int GPR = BN / 4;  // 4-column groups per row
#pragma unroll
    for (int it = 0; it < 64 * GPR / 256; ++it) {
      const int g = tid + it * 256;
      const int row = g / GPR, col = (g % GPR) * 4;
      const int gm = m0 + pass * 64 + row, gn = n0 + col;
      if (gm >= M || gn >= N) continue;
      float4 v = *reinterpret_cast<const float4*>(Cs + row * LDC + col);
      float rs = 1.f;
      if constexpr (AM == A_NORM) {
        rs = row_scale[pass * 64 + row];
        v.x *= rs;
        v.y *= rs;
        v.z *= rs;
        v.w *= rs;
      }
      if constexpr (EP == EP_STORE) {
        *reinterpret_cast<float4*>(p.Cf + (long)gm * N + gn) = v;
      } else if constexpr (EP == EP_RESID) {
        float4* dst = reinterpret_cast<float4*>(p.Cf + (long)gm * N + gn);
        float4 o = *dst;
        o.x += v.x;
        o.y += v.y;
        o.z += v.z;
        o.w += v.w;
        *dst = o;
      } else if constexpr (EP == EP_GELU) {
        v.x = gelu_tanh(v.x);
        v.y = gelu_tanh(v.y);
        v.z = gelu_tanh(v.z);
        v.w = gelu_tanh(v.w);
        store4<T>(reinterpret_cast<T*>(p.Ct) + (long)gm * N + gn, v);
      } else if constexpr (EP == EP_HEAD) {
        const int b = gm / p.nq, t = gm % p.nq;
        if (t >= p.t_skip) *reinterpret_cast<float4*>(p.out + (long)b * p.out_stride_b + (long)(t - p.t_skip) * N + gn) = v;
      } else {  // EP_QKV
        const int D = p.D, hd = p.hd, half = hd >> 1;
        const int which = gn / D, c = gn - which * D;
        const int h = c / hd, d = c - h * hd;
        const int bl = gm / p.nq, t = gm - bl * p.nq;
        const int b = p.s0 + bl;
        const int pos = (p.base_pos ? p.base_pos[b] : 0) + p.pos_off + t;
        if (which < 2) {
          const bool lo = d < half;
          const int pcol = lo ? col + half : col - half;
          float4 pv = *reinterpret_cast<const float4*>(Cs + row * LDC + pcol);
          const int f = lo ? d : d - half;
          const float4 cs = *reinterpret_cast<const float4*>(p.rope_cos + (long)pos * half + f);
          const float4 sn = *reinterpret_cast<const float4*>(p.rope_sin + (long)pos * half + f);
          const float sg = lo ? -rs : rs;
          v.x = v.x * cs.x + sg * pv.x * sn.x;
          v.y = v.y * cs.y + sg * pv.y * sn.y;
          v.z = v.z * cs.z + sg * pv.z * sn.z;
          v.w = v.w * cs.w + sg * pv.w * sn.w;
        }
        if (which == 0) {
          store4<T>(reinterpret_cast<T*>(p.q_out) + (long)gm * D + c, v);
        } else {
          const int page = p.page_table[(long)b * p.pt_stride + (pos >> p.pt_shift)];
          const int tok = pos & (p.PT - 1);
          if (which == 2 && p.v_transposed) {
            // V block stored [head][dim][token]: four strided element stores
            T* vp = reinterpret_cast<T*>(p.kv_pool) + (((long)page * 2 + 1) * p.Hh + h) * p.PT * hd + (long)d * p.PT + tok;
            vp[0] = (T)v.x;
            vp[p.PT] = (T)v.y;
            vp[2 * p.PT] = (T)v.z;
            vp[3 * p.PT] = (T)v.w;
          } else {
            const long off = ((((long)page * 2 + (which - 1)) * p.Hh + h) * p.PT + tok) * hd + d;
            store4<T>(reinterpret_cast<T*>(p.kv_pool) + off, v);
          }
        }
      }
    }
  }
}

template <typename T, int AM, int EP>
static hipError_t launch_cfg(const GemmP& p, hipStream_t st) {
  constexpr bool kBf = !std::is_same<T, float>::value;
  if constexpr (kBf) {
    long t128 = (long)((p.M + 127) / 128) * ((p.N + 127) / 128);
    if (t128 >= 192) {
      hipLaunchKernelGGL((gemm_kernel<T, AM, EP, 128, 128, 32>), dim3((unsigned)t128), dim3(256), 0, st, p);
      return hipGetLastError();
    }
  }
  long t64 = (long)((p.M + 63) / 64) * ((p.N + 63) / 64);
  hipLaunchKernelGGL((gemm_kernel<T, AM, EP, 64, 64, (kBf ? 64 : 16)>), dim3((unsigned)t64), dim3(256), 0, st, p);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_t(int amode, int epi, const GemmP& p, hipStream_t st) {
  if (amode == A_TOK && epi == EP_STORE) return launch_cfg<T, A_TOK, EP_STORE>(p, st);
  if (amode == A_NORM && epi == EP_QKV) return launch_cfg<T, A_NORM, EP_QKV>(p, st);
  if (amode == A_ACT && epi == EP_RESID) return launch_cfg<T, A_ACT, EP_RESID>(p, st);
  if (amode == A_NORM && epi == EP_GELU) return launch_cfg<T, A_NORM, EP_GELU>(p, st);
  if (amode == A_NORM && epi == EP_HEAD) return launch_cfg<T, A_NORM, EP_HEAD>(p, st);
  if (amode == A_NORM && epi == EP_STORE) return launch_cfg<T, A_NORM, EP_STORE>(p, st);
  return hipErrorInvalidValue;
}

hipError_t launch_gemm(int dtype, int amode, int epi, const GemmP& p, hipStream_t st) {
  if (p.M <= 0 || p.N <= 0 || p.K <= 0) return hipErrorInvalidValue;
  return dtype == TSD_BF16 ? launch_t<bf16>(amode, epi, p, st) : launch_t<float>(amode, epi, p, st);
}

}  // namespace tsd
