// Core of the bf16, head_dim-64 attention on the matrix cores: one wavefront handles up to 16
// query rows of one (series, head) against that series' paged KV cache, without LDS.
//
// V is cached transposed inside a page ([head][dim][token]) so that both MFMA B-operands are
// single 16-byte loads.  Keys go in steps of 32:
//   S^T = K Q^T   two 16x16x32 MFMAs per 16 keys; key rows are permuted so that lane group g
//                 (lane / 16) ends up with scores of the 8 consecutive keys 8g .. 8g+7 of the step
//                 for query lane % 16 -- exactly the A-operand layout of the next product;
//   online softmax in fp32 (running max / sum per query, shared by its 4 lanes);
//   O += P V      four 16x16x32 MFMAs (one per 16 output dims), V^T chunks straight from memory.
// Every K and V byte of the head is read exactly once per tile.
#pragma once
#include "tsd_internal.h"

namespace tsd {

// pool: this layer's KV pool; my_page: this lane's entry of the series' page table (lane i holds
// page i); base: absolute position of the tile's first query; nqt: queries in the tile (1..16);
// q_row(r) / out_row(r): pointers to the 64 dims of query / output row r of the tile.
template <typename QRow, typename ORow>
__device__ __forceinline__ void attn_tile_mfma(const bf16* pool, int h, int Hh, int PT, int pts, int my_page, int base,
                                               int nqt, float scale, QRow q_row, ORow out_row) {
  const int lane = threadIdx.x & 63;
  const int qi = lane & 15, g = lane >> 4;
  const long page_elems = (long)2 * Hh * PT * 64;
  const long v_off = (long)Hh * PT * 64;
  const int qrow = min(qi, nqt - 1);  // rows past the tile clone its last row
  const int qpos = base + qrow;       // last key this query may see
  const int total = base + nqt;       // keys the tile's last query sees
  bf16x8 qf[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(q_row(qrow) + kk * 32 + g * 8);
  f32x4 o[4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) o[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  for (int s0 = 0; s0 < total; s0 += 64) {  // two 32-key steps per trip, loads issued together
    bf16x8 kf[2][2][2], vf[2][4];
#pragma unroll
    for (int st = 0; st < 2; ++st) {
      const int sb = s0 + st * 32;
#pragma unroll
      for (int bi = 0; bi < 2; ++bi) {
        // A-operand row qi of block bi holds key sb + 8*(qi/4) + 4*bi + qi%4
        const int key = min(sb + 8 * (qi >> 2) + 4 * bi + (qi & 3), total - 1);
        const int page = __shfl(my_page, key >> pts);
        const bf16* kp = pool + page * page_elems + ((long)h * PT + (key & (PT - 1))) * 64;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) kf[st][bi][kk] = *reinterpret_cast<const bf16x8*>(kp + kk * 32 + g * 8);
      }
      // B-operand of P.V: 8 consecutive tokens sb + 8g .. of one dim, from the transposed V block
      const int vkey = min(sb + 8 * g, ((total - 1) >> 3) << 3);
      const int vpage = __shfl(my_page, vkey >> pts);
      const bf16* vp = pool + vpage * page_elems + v_off + (long)h * 64 * PT + (vkey & (PT - 1));
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) vf[st][nb] = *reinterpret_cast<const bf16x8*>(vp + (long)(nb * 16 + qi) * PT);
    }
#pragma unroll
    for (int st = 0; st < 2; ++st) {
      const int sb = s0 + st * 32;
      if (sb >= total) break;  // uniform across the wavefront
      f32x4 sc[2];
#pragma unroll
      for (int bi = 0; bi < 2; ++bi) {
        sc[bi] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
          sc[bi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[st][bi][kk], qf[kk], sc[bi], 0, 0, 0);
      }
      // this lane now holds query qi's scores for keys sb + 8g + j, j = 4*bi + r
      float sv[8];
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int key = sb + 8 * g + j;
        sv[j] = (key <= qpos) ? sc[j >> 2][j & 3] * scale : -INFINITY;
        mx = fmaxf(mx, sv[j]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx);  // finite: key 0 is visible to every query
      const float alpha = __expf(m_run - m_new);
      bf16x8 pf;
      float psum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float e = __expf(sv[j] - m_new);
        psum += e;
        pf[j] = (bf16)e;
      }
      l_run = l_run * alpha + psum;
      m_run = m_new;
      // accumulator rows of O are queries 4g + r: fetch their rescale factors from those lanes
      float ar[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) ar[r] = __shfl(alpha, 4 * g + r);
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) {
#pragma unroll
        for (int r = 0; r < 4; ++r) o[nb][r] *= ar[r];
        // tokens past the cached length may hold anything (even NaN bit patterns): P is 0 there,
        // so zero V as well to keep 0 * x out of the accumulators
        bf16x8 vv = vf[st][nb];
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (sb + 8 * g + j >= total) vv[j] = (bf16)0.f;
        o[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf, vv, o[nb], 0, 0, 0);
      }
    }
  }
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  const float inv = 1.f / l_run;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const float ir = __shfl(inv, 4 * g + r);
    const int qq = 4 * g + r;
    if (qq < nqt) {
      bf16* orow = out_row(qq);
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) orow[nb * 16 + qi] = (bf16)(o[nb][r] * ir);
    }
  }
}

}  // namespace tsd
