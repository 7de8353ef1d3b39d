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
// EMAX (8 or 16) bounds the expert count at compile time so that the loads of one k-step carry no
// branch and are all in flight together: rows past E re-read row E - 1 and their sums are ignored.
template <int EMAX>
__global__ __launch_bounds__(64) void router_kernel(const float* x, const float* Wr, int M, int D, int E, int topk,
                                                    int* ids, float* gates) {
  const int row = blockIdx.x, lane = threadIdx.x;
  const float* xr = x + (long)row * D;
  float ss = 0.f, dot[EMAX];
  const float* wr[EMAX];
#pragma unroll
  for (int e = 0; e < EMAX; ++e) {
    dot[e] = 0.f;
    wr[e] = Wr + (long)min(e, E - 1) * D;
  }
  for (int k = lane * 4; k < D; k += 256) {
    const float4 v = *reinterpret_cast<const float4*>(xr + k);
    float4 w[EMAX];
#pragma unroll
    for (int e = 0; e < EMAX; ++e) w[e] = *reinterpret_cast<const float4*>(wr[e] + k);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
#pragma unroll
    for (int e = 0; e < EMAX; ++e) dot[e] += v.x * w[e].x + v.y * w[e].y + v.z * w[e].z + v.w * w[e].w;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    ss += __shfl_xor(ss, o);
#pragma unroll
    for (int e = 0; e < EMAX; ++e) dot[e] += __shfl_xor(dot[e], o);
  }
  if (lane == 0) {
    const float rs = rsqrtf(ss / (float)D + kRmsEps);
    float pr[EMAX], mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < EMAX; ++e) {
      pr[e] = e < E ? dot[e] * rs : -INFINITY;
      mx = fmaxf(mx, pr[e]);
    }
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < EMAX; ++e) {
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
        for (int e = 0; e < EMAX; ++e)
          if (e < E && pr[e] > bv) {  // strict: the first (lowest) index wins ties
            bv = pr[e];
            best = e;
          }
        chosen[j] = best;
        g[j] = bv / sum;
        gsum += g[j];
#pragma unroll
        for (int e = 0; e < EMAX; ++e)
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

// Of the 64 assignments of one step (lane l holds expert id `id`, `valid` says whether there is
// one), the lanes whose id equals THIS lane's number modulo 2^NB, as a bit mask: one ballot per bit
// of the id and one for validity, combined per lane.  flip[b] is all ones where bit b of the lane
// number is clear.  Lane e < 2^NB so learns where expert e's assignments sit.
template <int NB>
__device__ __forceinline__ unsigned long long lanes_of_my_expert(int id, bool valid, const unsigned long long (&flip)[NB]) {
  unsigned long long m = __ballot(valid);
#pragma unroll
  for (int b = 0; b < NB; ++b) m &= __ballot((id >> b) & 1) ^ flip[b];
  return m;
}

// One block of 1024 lanes: a stable counting sort of the assignments a = token * topk + choice by
// expert.  Wavefront w owns the contiguous run of assignments [w * chunk, (w + 1) * chunk) and walks
// it 64 at a time, lane l holding assignment base + l, so "earlier wavefront, earlier step, lower
// lane" is assignment order and the sort is stable.  In a step, lane e finds the mask of the lanes
// that chose expert e (see above); its population is what the step adds to the wavefront's count of
// expert e, and an assignment's rank among the step's assignments of its expert is the number of
// set bits of that expert's mask below its own lane.  So the only scans left are the two small
// ones over wavefronts and over experts.  The first pass counts and keeps the expert ids in LDS
// (one byte each); the second pass places.  The tile map of the grouped GEMMs (one entry per
// BM-row tile of an expert's run of slots) is written by one lane per tile.  EMAX (8 or 16) is the
// compile-time bound of the expert count.
template <int EMAX>
__global__ __launch_bounds__(1024) void permute_kernel(const int* ids, int n_assign, int topk, int E, int BM, int n_mtiles,
                                                       int* src_row, int* slot_of, int4* tile_map) {
  extern __shared__ unsigned char lds_id[];  // [n_assign]
  __shared__ int wave_tot[16][EMAX];         // assignments of expert e in wavefront w
  __shared__ int wave_base[16][EMAX];        // ... in the wavefronts before w
  __shared__ int tot[EMAX];
  __shared__ int beg[EMAX + 1];       // first slot of expert e
  __shared__ int tile_beg[EMAX + 1];  // first tile of expert e
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int chunk = ((n_assign + 15) / 16 + 63) & ~63;
  const int a0 = w * chunk, a1 = min(a0 + chunk, n_assign);
  constexpr int NB = EMAX == 8 ? 3 : 4;
  static_assert(EMAX == 8 || EMAX == 16, "expert bound");
  unsigned long long flip[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) flip[b] = ((lane >> b) & 1) ? 0ull : ~0ull;
  int cnt = 0;  // lane e: this wavefront's assignments of expert e
  for (int base = a0; base < a1; base += 8 * 64) {  // eight loads in flight per lane
    int v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = ids[min(base + u * 64 + lane, n_assign - 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (base + u * 64 < a1) {  // the same for the whole wavefront
        const int a = base + u * 64 + lane;
        if (a < a1) lds_id[a] = (unsigned char)v[u];
        cnt += (int)__popcll(lanes_of_my_expert<NB>(v[u], a < a1, flip));
      }
    }
  }
  if (lane < EMAX) wave_tot[w][lane] = cnt;
  __syncthreads();
  // Scans over the 16 wavefronts (per expert) and over the experts, by lanes rather than by one
  // lane walking LDS: 16 * EMAX lanes hold (expert, wavefront) pairs, 16 consecutive lanes per expert.
  if (t < 16 * EMAX) {
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
    const int c = t < EMAX ? tot[t] : 0;
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
    if (t < EMAX) {
      beg[t] = ic - c;
      tile_beg[t] = it - tl;
      if (t == EMAX - 1) {
        beg[EMAX] = ic;
        tile_beg[EMAX] = it;
      }
    }
  }
  __syncthreads();
  int run = lane < EMAX ? beg[lane] + wave_base[w][lane] : 0;  // lane e: next slot of expert e for this wavefront
  for (int base = a0; base < a1; base += 64) {
    const int a = base + lane;
    const bool valid = a < a1;
    const int id = valid ? (int)lds_id[a] : 0;
    const unsigned long long m = lanes_of_my_expert<NB>(id, valid, flip);
    // the mask and the running slot of the expert this lane's assignment chose sit in lane `id`
    const unsigned lo = (unsigned)__shfl((int)(unsigned)m, id), hi = (unsigned)__shfl((int)(unsigned)(m >> 32), id);
    const int slot = __shfl(run, id) + (int)__builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u));
    run += (int)__popcll(m);
    if (valid) {
      src_row[slot] = topk == 2 ? a >> 1 : a / topk;
      slot_of[a] = slot;
    }
  }
  // tile map: tile j belongs to the expert e with tile_beg[e] <= j < tile_beg[e + 1]
  for (int j = t; j < n_mtiles; j += 1024) {
    int4 entry = make_int4(-1, 0, 0, 0);
#pragma unroll
    for (int e = 0; e < EMAX; ++e)
      if (e < E && j >= tile_beg[e] && j < tile_beg[e + 1])
        entry = make_int4(e, beg[e] + (j - tile_beg[e]) * BM, beg[e + 1], 0);
    tile_map[j] = entry;
  }
}

// TOPK > 0: the number of choices per token at compile time, so that the slots and gates of all
// choices, and then their Y rows, are fetched together (two memory latencies, not two per choice).
// The sums are taken in choice order either way.
template <typename T, int TOPK>
__global__ __launch_bounds__(256) void combine_kernel(const float* Y, const int* slot_of, const float* gates, float* x,
                                                      T* xb, int M, int D, int topk) {
  const long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= (long)M * D) return;
  const int row = (int)(i / D), col = (int)(i % D);
  float4 o = *reinterpret_cast<const float4*>(x + i);
  if constexpr (TOPK > 0) {
    int slot[TOPK];
    float g[TOPK];
    float4 y[TOPK];
#pragma unroll
    for (int j = 0; j < TOPK; ++j) {
      slot[j] = slot_of[(long)row * TOPK + j];
      g[j] = gates[(long)row * TOPK + j];
    }
#pragma unroll
    for (int j = 0; j < TOPK; ++j) y[j] = *reinterpret_cast<const float4*>(Y + (long)slot[j] * D + col);
#pragma unroll
    for (int j = 0; j < TOPK; ++j) {
      o.x = fmaf(g[j], y[j].x, o.x);
      o.y = fmaf(g[j], y[j].y, o.y);
      o.z = fmaf(g[j], y[j].z, o.z);
      o.w = fmaf(g[j], y[j].w, o.w);
    }
  } else {
    for (int j = 0; j < topk; ++j) {
      const float g = gates[(long)row * topk + j];
      const float4 y = *reinterpret_cast<const float4*>(Y + (long)slot_of[(long)row * topk + j] * D + col);
      o.x = fmaf(g, y.x, o.x);
      o.y = fmaf(g, y.y, o.y);
      o.z = fmaf(g, y.z, o.z);
      o.w = fmaf(g, y.w, o.w);
    }
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
// Parity tap (off unless the caller installed a buffer): the experts the router chose for every row of a pass,
// filed under the row's (layer, series, absolute position) so that another implementation can be evaluated with
// the same discrete choices.  tap: int32 [layers][max_batch][max_tokens][topk].
__global__ __launch_bounds__(256) void route_tap_kernel(const int* ids, int* tap, int layer, int M, int nq, const int* act,
                                                        int s0, const int* base_pos, int pos_off, int max_batch,
                                                        int max_tokens, int topk) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= M * topk) return;
  const int row = i / topk, j = i - row * topk;
  const int bl = row / nq, t = row - bl * nq;
  const int b = act ? act[bl] : s0 + bl;
  const int pos = (base_pos ? base_pos[b] : 0) + pos_off + t;
  if (b < 0 || b >= max_batch || pos < 0 || pos >= max_tokens) return;
  tap[(((long)layer * max_batch + b) * max_tokens + pos) * topk + j] = ids[i];
}
hipError_t launch_route_tap(const int* ids, int* tap, int layer, int M, int nq, const int* act, int s0, const int* base_pos,
                            int pos_off, int max_batch, int max_tokens, int topk, hipStream_t st) {
  hipLaunchKernelGGL(route_tap_kernel, dim3((unsigned)((M * topk + 255) / 256)), dim3(256), 0, st, ids, tap, layer, M, nq, act, s0,
                     base_pos, pos_off, max_batch, max_tokens, topk);
  return hipGetLastError();
}

hipError_t prepare_moe() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&permute_kernel<8>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPermuteLdsMax);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&permute_kernel<16>), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)kPermuteLdsMax);
}

hipError_t launch_router(const float* x, const float* Wr, int M, int D, int E, int topk, int* ids, float* gates,
                         hipStream_t st) {
  if (E < 1 || E > kMaxExperts || topk < 1 || topk > kMaxTopK || topk > E || D % 4 || M < 1) return hipErrorInvalidValue;
  if (E <= 8)
    hipLaunchKernelGGL(router_kernel<8>, dim3(M), dim3(64), 0, st, x, Wr, M, D, E, topk, ids, gates);
  else
    hipLaunchKernelGGL(router_kernel<16>, dim3(M), dim3(64), 0, st, x, Wr, M, D, E, topk, ids, gates);
  return hipGetLastError();
}

hipError_t launch_permute(const int* ids, int n_assign, int topk, int E, int BM, int n_mtiles, int* src_row,
                          int* slot_of, void* tile_map, hipStream_t st) {
  if (E < 1 || E > kMaxExperts || topk < 1 || n_assign < 1 || (size_t)n_assign > kPermuteLdsMax) return hipErrorInvalidValue;
  const size_t lds = (size_t)((n_assign + 15) & ~15);
  if (E <= 8)
    hipLaunchKernelGGL(permute_kernel<8>, dim3(1), dim3(1024), lds, st, ids, n_assign, topk, E, BM, n_mtiles, src_row, slot_of,
                       reinterpret_cast<int4*>(tile_map));
  else
    hipLaunchKernelGGL(permute_kernel<16>, dim3(1), dim3(1024), lds, st, ids, n_assign, topk, E, BM, n_mtiles, src_row, slot_of,
                       reinterpret_cast<int4*>(tile_map));
  return hipGetLastError();
}

template <typename T>
static void combine_dispatch(unsigned grid, hipStream_t st, const float* Y, const int* slot_of, const float* gates, float* x,
                             T* xb, int M, int D, int topk) {
  if (topk == 1)
    hipLaunchKernelGGL((combine_kernel<T, 1>), dim3(grid), dim3(256), 0, st, Y, slot_of, gates, x, xb, M, D, topk);
  else if (topk == 2)
    hipLaunchKernelGGL((combine_kernel<T, 2>), dim3(grid), dim3(256), 0, st, Y, slot_of, gates, x, xb, M, D, topk);
  else
    hipLaunchKernelGGL((combine_kernel<T, 0>), dim3(grid), dim3(256), 0, st, Y, slot_of, gates, x, xb, M, D, topk);
}

hipError_t launch_combine(int dtype, const float* Y, const int* slot_of, const float* gates, float* x, void* xb, int M,
                          int D, int topk, hipStream_t st) {
  const unsigned grid = (unsigned)(((long)M * D / 4 + 255) / 256);
  if (dtype == TSD_BF16)
    combine_dispatch<bf16>(grid, st, Y, slot_of, gates, x, reinterpret_cast<bf16*>(xb), M, D, topk);
  else
    combine_dispatch<float>(grid, st, Y, slot_of, gates, x, (float*)nullptr, M, D, topk);
  return hipGetLastError();
}

}  // namespace tsd
