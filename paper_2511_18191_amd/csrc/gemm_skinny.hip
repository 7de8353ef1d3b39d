// Skinny GEMM for passes of at most 32 rows (batch 1..few series: the latency regime):
//   C[M,N] = A[M,K] * Wt[N,K]^T,  M <= 32, bf16 operands, fp32 accumulation.
//
// With so few rows the product is a stream over the weights (every byte of Wt is needed once,
// there is nothing to reuse), so the kernel is built around HBM: a workgroup owns 16 output
// columns and ALL rows; its wavefronts split K among themselves and each streams its slab of Wt
// straight from global memory into MFMA B-operand registers (16 bytes per lane per load, many
// loads in flight, no LDS on the way); the per-wavefront partial products are summed in a fixed
// order through LDS, which keeps the result deterministic, and the same fused epilogues as the
// tiled kernel follow (RMSNorm row scale, RoPE + KV-cache scatter, GELU, residual, head).
// For the QKV product a workgroup's 16 columns are 8 + 8 rotary partners of one head.
#include <type_traits>

#include "tsd_internal.h"

namespace tsd {

namespace {

__device__ __forceinline__ void store4_bf16(bf16* dst, float4 v) {
  bf16x4 o;
  o[0] = (bf16)v.x;
  o[1] = (bf16)v.y;
  o[2] = (bf16)v.z;
  o[3] = (bf16)v.w;
  *reinterpret_cast<bf16x4*>(dst) = o;
}

__device__ __forceinline__ void split_hi_lo(const float* f, bf16x8& hi, bf16x8& lo) {
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    hi[e] = (bf16)f[e];
    lo[e] = (bf16)(f[e] - (float)hi[e]);
  }
}

constexpr int kRowsMax = 32;  // two 16-row MFMA tiles
constexpr int kU = 4;         // k-steps whose loads are issued together

template <int AM, int EP, int NW>
__global__ __launch_bounds__(NW * 64) void gemm_skinny_kernel(const GemmP p) {
  constexpr bool kNorm = (AM == A_NORM || AM == A_NORM32);
  constexpr bool kF32 = (AM == A_TOK || AM == A_NORM32);  // fp32 A rows, split into hi + lo bf16
  __shared__ float part[NW][kRowsMax][17];   // per-wavefront partial products
  __shared__ float ss_part[NW][kRowsMax];    // per-wavefront partial sums of squares
  __shared__ int row_pos[kRowsMax], row_page[kRowsMax];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int M = p.M, N = p.N, K = p.K;

  // ---- the 16 columns of this workgroup ----
  int col_of[2];  // first global column of LDS columns 0..7 and 8..15
  if constexpr (EP == EP_QKV) {
    const int per_head = p.hd / 16;                      // column groups per head (hd = 64 -> 4)
    const int hidx = blockIdx.x / per_head, j = blockIdx.x % per_head;
    const int base = hidx * p.hd;                        // heads of q, then k, then v, are consecutive
    col_of[0] = base + j * 8;
    col_of[1] = base + p.hd / 2 + j * 8;
  } else {
    col_of[0] = blockIdx.x * 16;
    col_of[1] = blockIdx.x * 16 + 8;
  }
  const int my_col = col_of[li >> 3] + (li & 7);
  const bf16* wrow = reinterpret_cast<const bf16*>(p.W) + (long)min(my_col, N - 1) * K;

  // ---- A rows of this lane (one per 16-row tile), clamped ----
  const char* arow[2];
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int gm = min(r * 16 + li, M - 1);
    if constexpr (AM == A_TOK) {
      int b = gm / p.nq;
      const int t = gm % p.nq;
      if (p.act) b = p.act[b];
      const float* src = (t < p.n0) ? p.src0 + (long)b * p.stride0 + (long)t * K
                                    : p.src1 + (long)b * p.stride1 + (long)(t - p.n0) * K;
      arow[r] = reinterpret_cast<const char*>(src);
    } else if constexpr (kF32) {
      arow[r] = reinterpret_cast<const char*>(reinterpret_cast<const float*>(p.A) + (long)gm * K);
    } else {
      arow[r] = reinterpret_cast<const char*>(reinterpret_cast<const bf16*>(p.A) + (long)gm * K);
    }
  }
  const bool two_tiles = M > 16;

  // epilogue inputs that do not depend on the product
  if constexpr (EP == EP_QKV) {
    if (tid < kRowsMax) {
      const int gm = min(tid, M - 1);
      const int bl = gm / p.nq, t = gm - bl * p.nq, b = p.act ? p.act[bl] : p.s0 + bl;
      const int pos = (p.base_pos ? p.base_pos[b] : 0) + p.pos_off + t;
      row_pos[tid] = pos;
      row_page[tid] = p.page_table[(long)b * p.pt_stride + (pos >> p.pt_shift)];
    }
  }

  // ---- this wavefront's share of K, in steps of 32 ----
  const int nks = (K + 31) / 32;
  const int per_w = (nks + NW - 1) / NW;
  const int ks0 = w * per_w, ks1 = min(ks0 + per_w, nks);
  f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
  float ss[2] = {0.f, 0.f};

  for (int ksb = ks0; ksb < ks1; ksb += kU) {
    bf16x8 bfr[kU];
    uint4 araw[kU][2][kF32 ? 2 : 1];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int k = min((ksb + u) * 32 + lg * 8, K - 8);  // clamped; zeroed below if out of range
      bfr[u] = *reinterpret_cast<const bf16x8*>(wrow + k);
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        if (r == 1 && !two_tiles) continue;
        if constexpr (kF32) {
          araw[u][r][0] = *reinterpret_cast<const uint4*>(arow[r] + (long)k * 4);
          araw[u][r][1] = *reinterpret_cast<const uint4*>(arow[r] + (long)k * 4 + 16);
        } else {
          araw[u][r][0] = *reinterpret_cast<const uint4*>(arow[r] + (long)k * 2);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const bool live = (ksb + u) < ks1 && ((ksb + u) * 32 + lg * 8) < K;
      bf16x8 bq = bfr[u];
      if (!live) {
#pragma unroll
        for (int e = 0; e < 8; ++e) bq[e] = (bf16)0.f;
      }
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        if (r == 1 && !two_tiles) continue;
        if constexpr (kF32) {
          float f[8];
          *reinterpret_cast<uint4*>(f) = araw[u][r][0];
          *reinterpret_cast<uint4*>(f + 4) = araw[u][r][1];
          if (!live) {
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = 0.f;
          }
          if constexpr (kNorm) {
#pragma unroll
            for (int e = 0; e < 8; ++e) ss[r] = fmaf(f[e], f[e], ss[r]);
          }
          bf16x8 hi, lo;
          split_hi_lo(f, hi, lo);
          acc[r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lo, bq, acc[r], 0, 0, 0);
          acc[r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi, bq, acc[r], 0, 0, 0);
        } else {
          bf16x8 a = *reinterpret_cast<const bf16x8*>(&araw[u][r][0]);
          if (!live) {
#pragma unroll
            for (int e = 0; e < 8; ++e) a[e] = (bf16)0.f;
          }
          if constexpr (kNorm) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const float f = (float)a[e];
              ss[r] = fmaf(f, f, ss[r]);
            }
          }
          acc[r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bq, acc[r], 0, 0, 0);
        }
      }
    }
  }

  // ---- partials to LDS: accumulator element i of tile r is row r*16 + 4*(lane/16) + i, column lane%16 ----
#pragma unroll
  for (int r = 0; r < 2; ++r)
#pragma unroll
    for (int i = 0; i < 4; ++i) part[w][r * 16 + lg * 4 + i][li] = acc[r][i];
  if constexpr (kNorm) {
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      float s = ss[r];
      s += __shfl_xor(s, 16);
      s += __shfl_xor(s, 32);
      if (lg == 0) ss_part[w][r * 16 + li] = s;
    }
  }
  __syncthreads();

  // ---- reduce over wavefronts in a fixed order, then the epilogue: one thread per (row, 4 columns) ----
  if (tid >= kRowsMax * 4) return;
  const int row = tid >> 2, c4 = (tid & 3) * 4;
  // a launch replayed from a graph stores only the rows of series that are still active
  if (row >= (p.n_dev ? min(M, *p.n_dev * p.nq) : M)) return;
  const int gm = row;
  const int gn = col_of[c4 >> 3] + (c4 & 7);
  if (gn >= N) return;
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f), pv = make_float4(0.f, 0.f, 0.f, 0.f);
  float sumsq = 0.f;
  const int pc4 = c4 ^ 8;  // rotary partner columns
#pragma unroll
  for (int ww = 0; ww < NW; ++ww) {
    v.x += part[ww][row][c4 + 0];
    v.y += part[ww][row][c4 + 1];
    v.z += part[ww][row][c4 + 2];
    v.w += part[ww][row][c4 + 3];
    if constexpr (EP == EP_QKV) {
      pv.x += part[ww][row][pc4 + 0];
      pv.y += part[ww][row][pc4 + 1];
      pv.z += part[ww][row][pc4 + 2];
      pv.w += part[ww][row][pc4 + 3];
    }
    if constexpr (kNorm) sumsq += ss_part[ww][row];
  }
  float rs = 1.f;
  if constexpr (kNorm) {
    rs = rsqrtf(sumsq / (float)K + kRmsEps);
    v.x *= rs;
    v.y *= rs;
    v.z *= rs;
    v.w *= rs;
  }
  if constexpr (EP == EP_STORE) {
    *reinterpret_cast<float4*>(p.Cf + (long)gm * N + gn) = v;
    if (p.Cb) store4_bf16(reinterpret_cast<bf16*>(p.Cb) + (long)gm * N + gn, v);
  } else if constexpr (EP == EP_RESID) {
    float4* dst = reinterpret_cast<float4*>(p.Cf + (long)gm * N + gn);
    float4 o = *dst;
    o.x += v.x;
    o.y += v.y;
    o.z += v.z;
    o.w += v.w;
    *dst = o;
    if (p.Cb) store4_bf16(reinterpret_cast<bf16*>(p.Cb) + (long)gm * N + gn, o);
  } else if constexpr (EP == EP_GELU) {
    v.x = gelu_tanh(v.x);
    v.y = gelu_tanh(v.y);
    v.z = gelu_tanh(v.z);
    v.w = gelu_tanh(v.w);
    store4_bf16(reinterpret_cast<bf16*>(p.Ct) + (long)gm * N + gn, v);
  } else if constexpr (EP == EP_HEAD) {
    const int bl = gm / p.nq, t = gm % p.nq;
    const int b = p.act ? p.act[bl] : bl;
    if (t >= p.t_skip) *reinterpret_cast<float4*>(p.out + (long)b * p.out_stride_b + (long)(t - p.t_skip) * N + gn) = v;
  } else {  // EP_QKV
    const int D = p.D, hd = p.hd, half = hd >> 1;
    const int which = gn / D, c = gn - which * D;
    const int h = c / hd, d = c - h * hd;
    const int pos = row_pos[row];
    if (which < 2) {
      const bool lo = d < half;
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
      store4_bf16(reinterpret_cast<bf16*>(p.q_out) + (long)gm * D + c, v);
    } else {
      const int page = row_page[row];
      const int tok = pos & (p.PT - 1);
      const long off = ((((long)page * 2 + (which - 1)) * p.Hh + h) * p.PT + tok) * hd + d;
      store4_bf16(reinterpret_cast<bf16*>(p.kv_pool) + off, v);
    }
  }
}

template <int AM, int EP>
hipError_t launch_nw(const GemmP& p, hipStream_t st) {
  const unsigned grid = (unsigned)(p.N / 16);
  if (p.K >= 512)
    hipLaunchKernelGGL((gemm_skinny_kernel<AM, EP, 16>), dim3(grid), dim3(16 * 64), 0, st, p);
  else
    hipLaunchKernelGGL((gemm_skinny_kernel<AM, EP, 4>), dim3(grid), dim3(4 * 64), 0, st, p);
  return hipGetLastError();
}

}  // namespace

// True when the skinny kernel can take this product (bf16, at most 32 rows, whole 16-column groups,
// dense, and for the QKV product head_dim 64 so that rotary partners pair up as 8 + 8 columns).
bool skinny_applicable(int dtype, int amode, int epi, const GemmP& p) {
  if (dtype != TSD_BF16 || p.M > kRowsMax || p.M < 1 || (p.N % 16) || (p.K % 8) || p.K < 8 || p.tile_map) return false;
  if (epi == EP_QKV && p.hd != 64) return false;
  return true;
}

hipError_t launch_gemm_skinny(int amode, int epi, const GemmP& p, hipStream_t st) {
  if (amode == A_TOK && epi == EP_STORE) return launch_nw<A_TOK, EP_STORE>(p, st);
  if (amode == A_NORM && epi == EP_QKV) return launch_nw<A_NORM, EP_QKV>(p, st);
  if (amode == A_ACT && epi == EP_RESID) return launch_nw<A_ACT, EP_RESID>(p, st);
  if (amode == A_NORM && epi == EP_GELU) return launch_nw<A_NORM, EP_GELU>(p, st);
  if (amode == A_NORM32 && epi == EP_HEAD) return launch_nw<A_NORM32, EP_HEAD>(p, st);
  if (amode == A_ACT && epi == EP_STORE) return launch_nw<A_ACT, EP_STORE>(p, st);
  if (amode == A_NORM && epi == EP_STORE) return launch_nw<A_NORM, EP_STORE>(p, st);
  return hipErrorInvalidValue;
}

}  // namespace tsd
