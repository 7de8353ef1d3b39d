// Routed FFN (softmax router, top-k experts, renormalised gates) around the grouped GEMMs:
//   router_kernel   per token: RMSNorm scale, router logits in fp32, softmax, top-k by probability
//                   (ties to the lower expert index), gates renormalised to sum to one;
//   permute_kernel  stable counting sort of the (token, choice) assignments by expert: slot lists,
//                   the inverse map, and the tile map the grouped GEMMs walk;
//   combine_kernel  x[token] += sum_j gate_j * Y[slot_j(token)]  (fixed order, deterministic).
#include "tsd_internal.h"

namespace tsd {

constexpr int kMaxExperts = 16;
constexpr int kMaxTopK = 4;

// One wavefront per token.  x: fp32 residual rows [M][D]; Wr: fp32 [E][D] with the norm gain folded.
__global__ __launch_bounds__(64) void router_kernel(const float* x, const float* Wr, int M, int D, int E, int topk,
                                                    int* ids, float* gates) {
  const int row = blockIdx.x, lane = threadIdx.x;
  const float* xr = x + (long)row * D;
  float ss = 0.f, dot[kMaxExperts];
#pragma unroll
  for (int e = 0; e < kMaxExperts; ++e) dot[e] = 0.f;
  for (int k = lane * 4; k < D; k += 256) {
    const float4 v = *reinterpret_cast<const float4*>(xr + k);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
#pragma unroll
    for (int e = 0; e < kMaxExperts; ++e) {
      if (e < E) {
        const float4 w = *reinterpret_cast<const float4*>(Wr + (long)e * D + k);
        dot[e] += v.x * w.x + v.y * w.y + v.z * w.z + v.w * w.w;
      }
    }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    ss += __shfl_xor(ss, o);
#pragma unroll
    for (int e = 0; e < kMaxExperts; ++e) dot[e] += __shfl_xor(dot[e], o);
  }
  if (lane == 0) {
    const float rs = rsqrtf(ss / (float)D + kRmsEps);
    float pr[kMaxExperts], mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < kMaxExperts; ++e) {
      pr[e] = e < E ? dot[e] * rs : -INFINITY;
      mx = fmaxf(mx, pr[e]);
    }
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < kMaxExperts; ++e) {
      pr[e] = e < E ? expf(pr[e] - mx) : 0.f;
      sum += pr[e];
    }
    int chosen[kMaxTopK];
    float g[kMaxTopK], gsum = 0.f;
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) {
      if (j < topk) {
        int best = 0;
        float bv = -1.f;
#pragma unroll
        for (int e = 0; e < kMaxExperts; ++e)
          if (e < E && pr[e] > bv) {  // strict: the first (lowest) index wins ties
            bv = pr[e];
            best = e;
          }
        chosen[j] = best;
        g[j] = bv / sum;
        gsum += g[j];
#pragma unroll
        for (int e = 0; e < kMaxExperts; ++e)
          if (e == best) pr[e] = -1.f;  // remove from later picks (probabilities are >= 0)
      }
    }
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j)
      if (j < topk) {
        ids[(long)row * topk + j] = chosen[j];
        gates[(long)row * topk + j] = g[j] / gsum;
      }
  }
}

// One block of 1024 lanes: a stable counting sort of the assignments a = token * topk + choice by
// expert.  Lane t owns the contiguous run of assignments [t * per, (t + 1) * per), so "earlier lane,
// then earlier position" is assignment order and the sort is stable.  Per expert: counts per lane,
// an exclusive scan over the lanes of a wavefront (shuffles) and over the wavefronts (LDS), then
// every lane places its own run.  The expert ids are first staged in LDS (one byte each) by
// coalesced loads, eight in flight per lane: read straight from memory, a lane's run would be a
// chain of dependent-latency loads.  The tile map of the grouped GEMMs (one entry per BM-row tile
// of an expert's run of slots) is written by one lane per tile.
__global__ __launch_bounds__(1024) void permute_kernel(const int* ids, int n_assign, int topk, int E, int BM, int n_mtiles,
                                                       int* src_row, int* slot_of, int4* tile_map) {
  extern __shared__ unsigned char lds_id[];   // [n_assign]
  __shared__ int wave_tot[16][kMaxExperts];   // assignments of expert e in wavefront w
  __shared__ int wave_base[16][kMaxExperts];  // ... in the wavefronts before w
  __shared__ int tot[kMaxExperts];
  __shared__ int beg[kMaxExperts + 1];       // first slot of expert e
  __shared__ int tile_beg[kMaxExperts + 1];  // first tile of expert e
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  for (int a = t; a < n_assign; a += 8 * 1024) {
    int v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = ids[min(a + u * 1024, n_assign - 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (a + u * 1024 < n_assign) lds_id[a + u * 1024] = (unsigned char)v[u];
  }
  __syncthreads();
  const int per = (n_assign + 1023) / 1024;
  const int a0 = min(t * per, n_assign), a1 = min(a0 + per, n_assign);
  int cnt[kMaxExperts];
#pragma unroll
  for (int e = 0; e < kMaxExperts; ++e) cnt[e] = 0;
  for (int a = a0; a < a1; ++a) {
    const int id = lds_id[a];
#pragma unroll
    for (int e = 0; e < kMaxExperts; ++e) cnt[e] += (id == e) ? 1 : 0;
  }
  // exclusive prefix of cnt[e] over the lanes of this wavefront, and the wavefront's total
  int start[kMaxExperts];
#pragma unroll
  for (int e = 0; e < kMaxExperts; ++e) {
    int incl = cnt[e];
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    start[e] = incl - cnt[e];
    if (lane == 63) wave_tot[w][e] = incl;
  }
  __syncthreads();
  // Scans over the 16 wavefronts (per expert) and over the 16 experts, by lanes rather than by one
  // lane walking LDS: 256 lanes hold (expert, wavefront) pairs, 16 consecutive lanes per expert.
  if (t < 256) {
    const int e = t >> 4, i = t & 15;
    const int v = wave_tot[i][e];
    int incl = v;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
      const int up = __shfl_up(incl, o, 16);
      if (i >= o) incl += up;
    }
    wave_base[i][e] = incl - v;
    if (i == 15) tot[e] = incl;
  }
  __syncthreads();
  if (t < 64) {
    const int c = t < kMaxExperts ? tot[t] : 0;
    const int tl = (c + BM - 1) / BM;
    int ic = c, it = tl;
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
      const int uc = __shfl_up(ic, o, 16), ut = __shfl_up(it, o, 16);
      if ((t & 15) >= o) {
        ic += uc;
        it += ut;
      }
    }
    if (t < kMaxExperts) {
      beg[t] = ic - c;
      tile_beg[t] = it - tl;
      if (t == kMaxExperts - 1) {
        beg[kMaxExperts] = ic;
        tile_beg[kMaxExperts] = it;
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < kMaxExperts; ++e) start[e] += beg[e] + wave_base[w][e];
  for (int a = a0; a < a1; ++a) {
    const int id = lds_id[a];
    int slot = 0;
#pragma unroll
    for (int e = 0; e < kMaxExperts; ++e)
      if (id == e) {
        slot = start[e];
        start[e] += 1;
      }
    src_row[slot] = a / topk;
    slot_of[a] = slot;
  }
  // tile map: tile j belongs to the expert e with tile_beg[e] <= j < tile_beg[e + 1]
  for (int j = t; j < n_mtiles; j += 1024) {
    int4 entry = make_int4(-1, 0, 0, 0);
#pragma unroll
    for (int e = 0; e < kMaxExperts; ++e)
      if (e < E && j >= tile_beg[e] && j < tile_beg[e + 1])
        entry = make_int4(e, beg[e] + (j - tile_beg[e]) * BM, beg[e + 1], 0);
    tile_map[j] = entry;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(const float* Y, const int* slot_of, const float* gates, float* x,
                                                      T* xb, int M, int D, int topk) {
  const long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= (long)M * D) return;
  const int row = (int)(i / D), col = (int)(i % D);
  float4 o = *reinterpret_cast<const float4*>(x + i);
  for (int j = 0; j < topk; ++j) {
    const float g = gates[(long)row * topk + j];
    const float4 y = *reinterpret_cast<const float4*>(Y + (long)slot_of[(long)row * topk + j] * D + col);
    o.x = fmaf(g, y.x, o.x);
    o.y = fmaf(g, y.y, o.y);
    o.z = fmaf(g, y.z, o.z);
    o.w = fmaf(g, y.w, o.w);
  }
  *reinterpret_cast<float4*>(x + i) = o;
  if (xb) {
    xb[i] = (T)o.x;
    xb[i + 1] = (T)o.y;
    xb[i + 2] = (T)o.z;
    xb[i + 3] = (T)o.w;
  }
}

constexpr size_t kPermuteLdsMax = 144 * 1024;  // one byte per assignment
// More than 64 KB of dynamic LDS needs a one-time opt-in (done at handle creation).
hipError_t prepare_moe() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&permute_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)kPermuteLdsMax);
}

hipError_t launch_router(const float* x, const float* Wr, int M, int D, int E, int topk, int* ids, float* gates,
                         hipStream_t st) {
  if (E > kMaxExperts || topk > kMaxTopK || topk > E || D % 4) return hipErrorInvalidValue;
  hipLaunchKernelGGL(router_kernel, dim3(M), dim3(64), 0, st, x, Wr, M, D, E, topk, ids, gates);
  return hipGetLastError();
}

hipError_t launch_permute(const int* ids, int n_assign, int topk, int E, int BM, int n_mtiles, int* src_row,
                          int* slot_of, void* tile_map, hipStream_t st) {
  if (E > kMaxExperts || n_assign < 1 || (size_t)n_assign > kPermuteLdsMax) return hipErrorInvalidValue;
  hipLaunchKernelGGL(permute_kernel, dim3(1), dim3(1024), (size_t)((n_assign + 15) & ~15), st, ids, n_assign, topk, E, BM, n_mtiles, src_row, slot_of,
                     reinterpret_cast<int4*>(tile_map));
  return hipGetLastError();
}

hipError_t launch_combine(int dtype, const float* Y, const int* slot_of, const float* gates, float* x, void* xb, int M,
                          int D, int topk, hipStream_t st) {
  const unsigned grid = (unsigned)(((long)M * D / 4 + 255) / 256);
  if (dtype == TSD_BF16)
    hipLaunchKernelGGL(combine_kernel<bf16>, dim3(grid), dim3(256), 0, st, Y, slot_of, gates, x, reinterpret_cast<bf16*>(xb), M, D, topk);
  else
    hipLaunchKernelGGL(combine_kernel<float>, dim3(grid), dim3(256), 0, st, Y, slot_of, gates, x, (float*)nullptr, M, D, topk);
  return hipGetLastError();
}

}  // namespace tsd
