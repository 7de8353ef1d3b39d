// Core of the bf16, head_dim-64 attention on the matrix cores: one wavefront handles up to 16
// query rows of one (series, head) against that series' paged KV cache.
//
// K and V pages are row-major ([head][token][dim]), so a new token's K and V are one contiguous
// 128-byte row each per head.  Keys go in steps of 32:
//   S^T = K Q^T   two 16x16x32 MFMAs per 16 keys; key rows are permuted so that lane group g
//                 (lane / 16) ends up with scores of the 8 consecutive keys 8g .. 8g+7 of the step
//                 for query lane % 16 -- exactly the A-operand layout of the next product;
//   online softmax in fp32 (running max / sum per query, shared by its 4 lanes);
//   O += P V      four 16x16x32 MFMAs (one per 16 output dims).  Their B operand wants, per lane,
//                 eight consecutive tokens of one dim: the 32 V rows of a step are fetched with
//                 coalesced 16-byte loads, parked in LDS (4 KB per wavefront and step) and
//                 picked up transposed with ds_read_b64_tr_b16.
// Every K and V byte of the head is read exactly once per tile.
// (A cache that keeps V transposed, [head][dim][token], makes that operand a plain 16-byte load, but
// every new token then costs 64 two-byte stores over 16 cache lines per head in the QKV epilogue:
// 5 % of a verification pass and 9 % of a one-token step at batch 1024, against nothing measurable
// for the transposing read.)
#pragma once
#include "tsd_internal.h"

namespace tsd {

// pool: this layer's KV pool; my_page: this lane's entry of the series' page table (lane i holds
// page i); base: absolute position of the tile's first query; nqt: queries in the tile (1..16);
// q_row(r) / out_row(r): pointers to the 64 dims of query / output row r of the tile.
// vt: LDS, bf16 [NST][32][64], private to the wavefront.  NST: 32-key steps per trip (the loads of a trip are issued
// together; a step past the tile's last key is skipped, loads included).  kOneWave: the workgroup is this one wavefront
// (then a workgroup barrier orders the tile's LDS traffic); otherwise the wavefront may be one of
// several that run different trip counts, and only its own LDS operations, which the hardware
// executes in issue order, are fenced.
template <bool kOneWave = true, int NST = 2, typename QRow, typename ORow>
__device__ __forceinline__ void attn_tile_mfma(const bf16* pool, int h, int Hh, int PT, int pts, int my_page, int base,
                                               int nqt, float scale, QRow q_row, ORow out_row, bf16* vt) {
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
  auto lds_order = [] {
    if constexpr (kOneWave) {
      __syncthreads();
    } else {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  };

  for (int s0 = 0; s0 < total; s0 += 32 * NST) {  // NST 32-key steps per trip, loads issued together
    bf16x8 kf[NST][2][2], vf[NST][4];
#pragma unroll
    for (int st = 0; st < NST; ++st) {
      const int sb = s0 + st * 32;
      if (sb >= total) break;  // (uniform across the wavefront) nothing is fetched for a step past the last key
#pragma unroll
      for (int bi = 0; bi < 2; ++bi) {
        // A-operand row qi of block bi holds key sb + 8*(qi/4) + 4*bi + qi%4
        const int key = min(sb + 8 * (qi >> 2) + 4 * bi + (qi & 3), total - 1);
        const int page = __shfl(my_page, key >> pts);
        const bf16* kp = pool + page * page_elems + ((long)h * PT + (key & (PT - 1))) * 64;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) kf[st][bi][kk] = *reinterpret_cast<const bf16x8*>(kp + kk * 32 + g * 8);
      }
      // V: 8 lanes fetch one 128-byte row; load i of the lane is row (lane / 8) + 8 i of the step
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = min(sb + (lane >> 3) + 8 * i, total - 1);
        const int page = __shfl(my_page, key >> pts);
        vf[st][i] = *reinterpret_cast<const bf16x8*>(pool + page * page_elems + v_off + ((long)h * PT + (key & (PT - 1))) * 64 +
                                                     (lane & 7) * 8);
      }
    }
    {
      // through LDS: row r of a step lands rotated by 16 (r / 8) dims, so that the four key groups of a
      // transposed read fall on different banks
      lds_order();  // the previous trip's reads before these writes
#pragma unroll
      for (int st = 0; st < NST; ++st) {
        if (s0 + st * 32 >= total) break;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          *reinterpret_cast<bf16x8*>(vt + (st * 32 + (lane >> 3) + 8 * i) * 64 + (((lane & 7) * 8 + 16 * i) & 63)) = vf[st][i];
      }
      lds_order();
      // LDS transpose read (ds_read_b64_tr_b16): within 16 lanes, lane i receives element i % 4 of the
      // 8-byte chunks addressed by lanes i / 4, i / 4 + 4, i / 4 + 8, i / 4 + 12.  Lane L of key group g
      // therefore points at row 8g + 4 half + L / 4, dims 16 nb + 4 (L % 4) .., and lane qi gets the four
      // tokens 8g + 4 half .. of dim 16 nb + qi: one half of its B operand per read.
      typedef short short4v __attribute__((ext_vector_type(4)));
      typedef short short8v __attribute__((ext_vector_type(8)));
#pragma unroll
      for (int st = 0; st < NST; ++st) {
        if (s0 + st * 32 >= total) break;
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
          short4v hv[2];
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const bf16* src = vt + (st * 32 + 8 * g + 4 * half + (qi >> 2)) * 64 + ((nb * 16 + 4 * (qi & 3) + 16 * g) & 63);
            hv[half] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)src);
          }
          const short8v both = __builtin_shufflevector(hv[0], hv[1], 0, 1, 2, 3, 4, 5, 6, 7);
          vf[st][nb] = __builtin_bit_cast(bf16x8, both);
        }
      }
    }
#pragma unroll
    for (int st = 0; st < NST; ++st) {
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
