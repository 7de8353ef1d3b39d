// Epilogues of the fused GEMM family, shared by the tiled kernels: one pass over 64 rows of the product
// that sit in LDS (or wherever `read_c4` finds them).
#pragma once
#include <type_traits>

#include "tsd_internal.h"

namespace tsd {

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

// T: compute dtype; kNorm: scale row r by row_scale[r] (the fused RMSNorm); BN: tile width; NT: lanes taking part;
// kOld: the old residual values of this lane's items were fetched ahead into oldc[].
// read_c4(row, col): four consecutive elements of row `row` (0..63 of the pass) of the product tile.
// row_scale / row_pos / row_page are indexed by the row inside the tile (pass * 64 + row).
// kBatchQKV: the RoPE epilogue in batches of four groups per lane (below).
template <typename T, int EP, bool kNorm, int BN, int NT, bool kOld, bool kBatchQKV = (BN == 64), typename ReadC>
__device__ __forceinline__ void epilogue_pass(const GemmP& p, ReadC read_c4, const float* row_scale, const int* row_pos,
                                              const int* row_page, int m0, int n0, int pass, int m_lim, int N, int tid,
                                              const float4* oldc) {
  constexpr bool kBf = !std::is_same<T, float>::value;
  constexpr int GPR = BN / 4;  // 4-column groups per row
  if constexpr (EP == EP_QKV && kBatchQKV) {
    // RoPE + q / KV-cache write, four 4-column groups per lane at a time: first every read (accumulators and
    // rotary partners from LDS, positions and pages, cos / sin from global memory, clamped for groups outside
    // the product), then the arithmetic, then the stores.  Written as one read-compute-store body per group,
    // each group's global loads wait for the previous group's stores to issue and pay a full round trip.
    // (Not in the register-staged 128 x 128 kernel: there the extra live registers cost occupancy and 9 % of a
    //  verification pass at 7168 rows.  The wide-tile kernels, which hold no staging registers, take it.)
    constexpr int ITS = 64 * GPR / NT, BATCH = ITS < 4 ? ITS : 4;
    const int D = p.D, hd = p.hd, half = hd >> 1;
#pragma unroll
    for (int it0 = 0; it0 < ITS; it0 += BATCH) {
      float4 v[BATCH], pv[BATCH], cs[BATCH], sn[BATCH];
      int pos[BATCH], page[BATCH], gmv[BATCH], gnv[BATCH];
      bool ok[BATCH];
#pragma unroll
      for (int j = 0; j < BATCH; ++j) {
        const int g = tid + (it0 + j) * NT;
        const int row = g / GPR, col = (g % GPR) * 4;
        gmv[j] = m0 + pass * 64 + row;
        gnv[j] = n0 + col;
        ok[j] = gmv[j] < m_lim && gnv[j] < N;
        const int c = gnv[j] % D, d = c % hd;
        const bool lo = d < half;
        v[j] = read_c4(row, col);
        pv[j] = read_c4(row, lo ? col + half : col - half);
        pos[j] = ok[j] ? row_pos[pass * 64 + row] : 0;
        page[j] = ok[j] ? row_page[pass * 64 + row] : 0;
        const int f = lo ? d : d - half;
        cs[j] = *reinterpret_cast<const float4*>(p.rope_cos + (long)pos[j] * half + f);
        sn[j] = *reinterpret_cast<const float4*>(p.rope_sin + (long)pos[j] * half + f);
        if constexpr (kNorm) {
          const float rs = row_scale[pass * 64 + row];
          v[j].x *= rs;
          v[j].y *= rs;
          v[j].z *= rs;
          v[j].w *= rs;
          pv[j].x *= rs;
          pv[j].y *= rs;
          pv[j].z *= rs;
          pv[j].w *= rs;
        }
      }
#pragma unroll
      for (int j = 0; j < BATCH; ++j) {
        const int which = gnv[j] / D, c = gnv[j] - which * D;
        const int h = c / hd, d = c - h * hd;
        if (which < 2) {
          const float sg = d < half ? -1.f : 1.f;
          v[j].x = v[j].x * cs[j].x + sg * pv[j].x * sn[j].x;
          v[j].y = v[j].y * cs[j].y + sg * pv[j].y * sn[j].y;
          v[j].z = v[j].z * cs[j].z + sg * pv[j].z * sn[j].z;
          v[j].w = v[j].w * cs[j].w + sg * pv[j].w * sn[j].w;
        }
        if (!ok[j]) continue;
        if (which == 0) {
          store4<T>(reinterpret_cast<T*>(p.q_out) + (long)gmv[j] * D + c, v[j]);
        } else {
          const int tok = pos[j] & (p.PT - 1);
          const long off = ((((long)page[j] * 2 + (which - 1)) * p.Hh + h) * p.PT + tok) * hd + d;
          store4<T>(reinterpret_cast<T*>(p.kv_pool) + off, v[j]);
        }
      }
    }
    return;
  }
  if constexpr (EP == EP_GELU && kBf && BN % 8 == 0 && (64 * (BN / 8)) % NT == 0) {
    // eight columns per lane: one 16-byte store instead of two 8-byte ones (N is a multiple of 8 here: d_ff is)
    constexpr int G8 = BN / 8;
#pragma unroll
    for (int it = 0; it < 64 * G8 / NT; ++it) {
      const int g = tid + it * NT;
      const int row = g / G8, col = (g % G8) * 8;
      const int gm = m0 + pass * 64 + row, gn = n0 + col;
      if (gm >= m_lim || gn >= N) continue;
      const float4 v0 = read_c4(row, col), v1 = read_c4(row, col + 4);
      const float rs = kNorm ? row_scale[pass * 64 + row] : 1.f;
      bf16x8 o;
      o[0] = (bf16)gelu_tanh(v0.x * rs);
      o[1] = (bf16)gelu_tanh(v0.y * rs);
      o[2] = (bf16)gelu_tanh(v0.z * rs);
      o[3] = (bf16)gelu_tanh(v0.w * rs);
      o[4] = (bf16)gelu_tanh(v1.x * rs);
      o[5] = (bf16)gelu_tanh(v1.y * rs);
      o[6] = (bf16)gelu_tanh(v1.z * rs);
      o[7] = (bf16)gelu_tanh(v1.w * rs);
      *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16*>(p.Ct) + (long)gm * N + gn) = o;
    }
    return;
  }
#pragma unroll
  for (int it = 0; it < 64 * GPR / NT; ++it) {
    const int g = tid + it * NT;
    const int row = g / GPR, col = (g % GPR) * 4;
    const int gm = m0 + pass * 64 + row, gn = n0 + col;
    if (gm >= m_lim || gn >= N) continue;
    float4 v = read_c4(row, col);
    float rs = 1.f;
    if constexpr (kNorm) {
      rs = row_scale[pass * 64 + row];
      v.x *= rs;
      v.y *= rs;
      v.z *= rs;
      v.w *= rs;
    }
    if constexpr (EP == EP_STORE) {
      *reinterpret_cast<float4*>(p.Cf + (long)gm * N + gn) = v;
      if (kBf && p.Cb) store4<T>(reinterpret_cast<T*>(p.Cb) + (long)gm * N + gn, v);
    } else if constexpr (EP == EP_RESID) {
      float4* dst = reinterpret_cast<float4*>(p.Cf + (long)gm * N + gn);
      float4 o;
      if constexpr (kOld) o = oldc[it]; else o = *dst;
      o.x += v.x;
      o.y += v.y;
      o.z += v.z;
      o.w += v.w;
      *dst = o;
      if (kBf && p.Cb) store4<T>(reinterpret_cast<T*>(p.Cb) + (long)gm * N + gn, o);
    } else if constexpr (EP == EP_GELU) {
      v.x = gelu_tanh(v.x);
      v.y = gelu_tanh(v.y);
      v.z = gelu_tanh(v.z);
      v.w = gelu_tanh(v.w);
      store4<T>(reinterpret_cast<T*>(p.Ct) + (long)gm * N + gn, v);
    } else if constexpr (EP == EP_HEAD) {
      const int bl = gm / p.nq, t = gm % p.nq;
      const int b = p.act ? p.act[bl] : bl;
      if (t >= p.t_skip) *reinterpret_cast<float4*>(p.out + (long)b * p.out_stride_b + (long)(t - p.t_skip) * N + gn) = v;
    } else {  // EP_QKV
      const int D = p.D, hd = p.hd, half = hd >> 1;
      const int which = gn / D, c = gn - which * D;
      const int h = c / hd, d = c - h * hd;
      const int pos = row_pos[pass * 64 + row];
      if (which < 2) {
        const bool lo = d < half;
        const int pcol = lo ? col + half : col - half;
        float4 pv = read_c4(row, pcol);
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
        const int page = row_page[pass * 64 + row];
        const int tok = pos & (p.PT - 1);
        const long off = ((((long)page * 2 + (which - 1)) * p.Hh + h) * p.PT + tok) * hd + d;
        store4<T>(reinterpret_cast<T*>(p.kv_pool) + off, v);
      }
    }
  }
}

}  // namespace tsd
