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
constexpr size_t kPermuteLdsMax = 150 * 1024;  // expert ids of one pass staged in LDS

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

// One block, one wavefront per expert.  Assignment a = token * topk + choice.  The expert ids are
// first copied into LDS with every load in flight; the two scans (count, then place) run from LDS.
__global__ __launch_bounds__(1024) void permute_kernel(const int* ids, int n_assign, int topk, int E, int BM, int n_mtiles,
                                                       int* src_row, int* slot_of, int4* tile_map) {
  extern __shared__ int lds_ids[];  // [n_assign]
  __shared__ int cnt[kMaxExperts], beg[kMaxExperts + 1];
  for (int a = threadIdx.x; a < n_assign; a += blockDim.x) lds_ids[a] = ids[a];
  __syncthreads();
  const int e = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int c = 0;
  for (int a0 = 0; a0 < n_assign; a0 += 64) {
    const int a = a0 + lane;
    c += __popcll(__ballot(a < n_assign && lds_ids[a] == e));
  }
  if (lane == 0) cnt[e] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0, t = 0;
    for (int i = 0; i < E; ++i) {
      beg[i] = run;
      for (int r0 = 0; r0 < cnt[i]; r0 += BM) tile_map[t++] = make_int4(i, run + r0, run + cnt[i], 0);
      run += cnt[i];
    }
    beg[E] = run;
    for (; t < n_mtiles; ++t) tile_map[t] = make_int4(-1, 0, 0, 0);
  }
  __syncthreads();
  int pos = beg[e];
  for (int a0 = 0; a0 < n_assign; a0 += 64) {
    const int a = a0 + lane;
    const bool mine = a < n_assign && lds_ids[a] == e;
    const unsigned long long m = __ballot(mine);
    if (mine) {
      const int slot = pos + __popcll(m & ((1ull << lane) - 1ull));
      src_row[slot] = a / topk;
      slot_of[a] = slot;
    }
    pos += __popcll(m);
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
  if (E > kMaxExperts || (size_t)n_assign * 4 > kPermuteLdsMax) return hipErrorInvalidValue;
  hipLaunchKernelGGL(permute_kernel, dim3(1), dim3(64 * E), (size_t)n_assign * 4, st, ids, n_assign, topk, E, BM, n_mtiles, src_row, slot_of,
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
