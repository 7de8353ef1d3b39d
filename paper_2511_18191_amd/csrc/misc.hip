// Small kernels around the transformer pass: weight packing, prefill statistics, the fused
// acceptance / correction / commit / rollback kernel, and read-out helpers.
#include <algorithm>
#include <type_traits>

#include "philox.h"
#include "tsd_internal.h"

namespace tsd {

// ---- weight packing: out[n][k] = T(gain[k] * W[k][n]) ---------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void pack_kernel(const PackP p) {
  __shared__ float tile[32][33];
  const int k0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int r = ty; r < 32; r += 8) {
    int k = k0 + r, n = n0 + tx;
    float v = 0.f;
    if (k < p.K && n < p.N) v = p.W[(long)k * p.N + n] * (p.gain ? p.gain[k] : 1.f);
    tile[r][tx] = v;
  }
  __syncthreads();
  T* out = reinterpret_cast<T*>(p.out);
  for (int r = ty; r < 32; r += 8) {
    int n = n0 + r, k = k0 + tx;
    if (k < p.K && n < p.N) out[(long)n * p.K + k] = (T)tile[tx][r];
  }
}

hipError_t launch_pack(int dtype, const PackP& p, hipStream_t st) {
  dim3 grid((p.N + 31) / 32, (p.K + 31) / 32), block(256);
  if (dtype == TSD_BF16)
    hipLaunchKernelGGL(pack_kernel<bf16>, grid, block, 0, st, p);
  else
    hipLaunchKernelGGL(pack_kernel<float>, grid, block, 0, st, p);
  return hipGetLastError();
}

// ---- prefill: frozen instance statistics, normalised context, initial per-series state ------
__device__ __forceinline__ double block_sum(double v, double* sh) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = 0;
  for (int i = 0; i < (int)(blockDim.x >> 6); ++i) t += sh[i];
  return t;
}

// Every series decodes again: the active list is the identity, its count the batch, and the
// largest number of patches still needed is T.
__device__ __forceinline__ void reset_active_list(const PrefillP& p, int b) {
  if (!p.act_list) return;
  p.act_list[b] = b;
  if (b == 0) {
    p.act_count[0] = p.batch;
    p.act_count[1] = p.T;
  }
}

__device__ __forceinline__ void init_state(const PrefillP& p, int b) {
  p.len[b] = p.N - 1;  // context patches 0..N-2 are cached; patch N-1 is pending at position N-1
  p.committed[b] = 0;
  p.round[b] = 0;
  p.active[b] = 1;
  for (int i = 0; i < 5; ++i) p.stat[(long)b * 5 + i] = 0;
  reset_active_list(p, b);
}

__global__ __launch_bounds__(256) void prefill_stats_kernel(const PrefillP p) {
  __shared__ double sh[4];
  const int n = p.N * p.P;
  const int b = p.slots ? p.slots[blockIdx.x] : (int)blockIdx.x;
  const float* x = p.series + (long)blockIdx.x * n;
  double s = 0;
  for (int i = threadIdx.x; i < n; i += 256) s += x[i];
  const double mean = block_sum(s, sh) / n;
  double v = 0;
  for (int i = threadIdx.x; i < n; i += 256) {
    double dlt = x[i] - mean;
    v += dlt * dlt;
  }
  const double var = block_sum(v, sh) / n;  // population variance of the context only
  const float mf = (float)mean, sf = (float)sqrt(var + (double)kNormEps);
  float* z = p.znorm + (long)b * n;
  for (int i = threadIdx.x; i < n; i += 256) z[i] = (x[i] - mf) / sf;
  __syncthreads();
  for (int i = threadIdx.x; i < p.P; i += 256) {
    p.pending[(long)b * p.P + i] = z[(long)(p.N - 1) * p.P + i];
    p.prev[(long)b * p.P + i] = z[(long)(p.N - 2) * p.P + i];
  }
  if (threadIdx.x == 0) {
    p.mean[b] = mf;
    p.sdev[b] = sf;
    if (p.keep_counters) {  // a new series in a used slot: its draws continue the slot's round counter
      p.len[b] = p.N - 1;
      p.committed[b] = 0;
      p.active[b] = 1;
    } else {
      init_state(p, b);
    }
  }
}

__global__ __launch_bounds__(256) void reset_kernel(const PrefillP p) {
  const int b = blockIdx.x, n = p.N * p.P;
  const float* z = p.znorm + (long)b * n;
  for (int i = threadIdx.x; i < p.P; i += 256) {
    p.pending[(long)b * p.P + i] = z[(long)(p.N - 1) * p.P + i];
    p.prev[(long)b * p.P + i] = z[(long)(p.N - 2) * p.P + i];
  }
  if (threadIdx.x == 0) init_state(p, b);
}

hipError_t launch_prefill_stats(const PrefillP& p, hipStream_t st) {
  hipLaunchKernelGGL(prefill_stats_kernel, dim3(p.B), dim3(256), 0, st, p);
  return hipGetLastError();
}
hipError_t launch_reset(const PrefillP& p, hipStream_t st) {
  hipLaunchKernelGGL(reset_kernel, dim3(p.B), dim3(256), 0, st, p);
  return hipGetLastError();
}

// ---- acceptance + correction + commit + rollback ---------------------------------------------
// Sampled proposals: X[b, i-1, :] = mu_q[b, i-1, :] + sigma_q * eps for the covered series, with
// each series' own round counter.  One 64-thread block per series.
__global__ __launch_bounds__(64) void sample_kernel(const SampleP p) {
  if (p.n_dev && (int)blockIdx.x >= *p.n_dev) return;
  const int b = p.act ? p.act[blockIdx.x] : (int)blockIdx.x;
  const unsigned r = (unsigned)p.round[b];
  const long off = ((long)b * p.K + (p.i - 1)) * p.P;
  for (int e = threadIdx.x; e < p.P; e += 64)
    p.X[off + e] = p.mu_q[off + e] + (p.sigma_q_vec ? p.sigma_q_vec[e] : p.sigma_q) * normal_draw((unsigned)b, r, (unsigned)p.i, kStreamProposal, e, p.key0, p.key1);
}
hipError_t launch_sample(const SampleP& p, hipStream_t st) {
  if (p.n <= 0) return hipSuccess;
  hipLaunchKernelGGL(sample_kernel, dim3(p.n), dim3(64), 0, st, p);
  return hipGetLastError();
}

// One wavefront per series.  Energies are reduced across lanes per proposal, then lane i owns
// proposal i+1: statistic, uniform, test; a ballot over the reject flags gives the first
// rejection.  The same wavefront then writes the committed patches, the new pending / previous
// tokens and the cache lengths (rollback is metadata only: speculative KV entries past the
// accepted length are simply overwritten by the next round).
__global__ __launch_bounds__(64) void accept_kernel(const AcceptP p) {
  if (p.n_dev && (int)blockIdx.x >= *p.n_dev) return;
  const int b = p.act ? p.act[blockIdx.x] : (int)blockIdx.x, lane = threadIdx.x;
  const int K = p.K, P = p.P;
  const int KE = K > 0 ? K : 1;
  if (!p.active[b]) {
    if (lane == 0) p.n_acc[b] = -1;
    if (lane < K) {
      p.ell[(long)b * KE + lane] = NAN;
      p.logu[(long)b * KE + lane] = NAN;
    }
    return;
  }
  const int r = p.round[b];
  const int c0 = p.committed[b];
  // a series with fewer than K patches left proposes and tests only as many positions as it
  // still needs: later ones could never be committed
  const int Kb = min(K, p.T - c0);
  const float* X = p.X + (long)b * K * P;
  const float* MQ = p.mu_q + (long)b * K * P;
  const float* MP = p.mu_p + (long)b * (K + 1) * P;
  float my_ep = 0.f, my_eq = 0.f;
  // four positions at a time: all their loads are issued before the first is used and the eight butterfly
  // reductions interleave (one position after the other, every position paid its own memory round trip and
  // twelve dependent cross-lane steps); positions past Kb re-read the last one and are dropped
  for (int i0 = 0; i0 < Kb; i0 += 4) {
    float ep[4] = {0.f, 0.f, 0.f, 0.f}, eq[4] = {0.f, 0.f, 0.f, 0.f};
    for (int e = lane; e < P; e += 64) {
      float x[4], mp[4], mq[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int ii = min(i0 + j, Kb - 1);
        x[j] = X[ii * P + e];
        mp[j] = MP[ii * P + e];
        mq[j] = MQ[ii * P + e];
      }
      float wp = 1.f, wq = 1.f;
      if (p.inv2sp2_vec) {  // Mahalanobis energies of the diagonal surrogate, already halved
        wp = p.inv2sp2_vec[e];
        wq = p.inv2sq2_vec[e];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float dp = x[j] - mp[j], dq = x[j] - mq[j];
        if (p.inv2sp2_vec) {
          ep[j] = fmaf(dp * dp, wp, ep[j]);
          eq[j] = fmaf(dq * dq, wq, eq[j]);
        } else {
          ep[j] = fmaf(dp, dp, ep[j]);
          eq[j] = fmaf(dq, dq, eq[j]);
        }
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        ep[j] += __shfl_xor(ep[j], o);
        eq[j] += __shfl_xor(eq[j], o);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (i0 + j < Kb && lane == i0 + j) {
        my_ep = ep[j];
        my_eq = eq[j];
      }
    }
  }
  bool reject = false;
  float ell = NAN, logu = NAN, thr = 0.f;
  if (lane < Kb) {
    // Eq. 5 with per-dimension energies ||.||^2 / P
    if (p.threshold) {
      // threshold rule: ||x - mu_p||_d^2 <= sigma_p^2, written as ell >= -1/2 so that the recorded
      // pair (ell, log u) shows how close to the boundary the decision was
      ell = p.temper * (p.inv2sp2_vec ? -(my_ep / (float)P) : -(my_ep / (float)P) * p.inv2sp2);
      logu = -0.5f;
    } else {
      if (p.inv2sp2_vec)
        ell = p.temper * (-(my_ep / (float)P) + (my_eq / (float)P) + p.logdet_dev[0]);
      else
        ell = p.temper * (-(my_ep / (float)P) * p.inv2sp2 + (my_eq / (float)P) * p.inv2sq2 + p.logdet);
      unsigned w = philox_word0((unsigned)b, (unsigned)r, (unsigned)(lane + 1), 0u, p.key0, p.key1);
      float u = word_uniform(w);
      logu = logf(u);
    }
    thr = (p.log_alpha_override <= 0.f) ? p.log_alpha_override : fminf(0.f, ell);
    reject = !(logu <= thr);
  }
  const unsigned long long rej = __ballot(reject);
  const int n_free = rej ? (int)__builtin_ctzll(rej) : Kb;  // leading accepts
  const int tested = n_free + (n_free < Kb ? 1 : 0);
  const bool is_tested = lane < tested;
  const unsigned long long near = __ballot(is_tested && fabsf(thr - logu) < 1e-4f);
  int n = n_free;
  if (p.forced) {
    int f = p.forced[b];
    if (f >= 0 && f <= Kb) n = f;
  }
  if (p.mode == 1) {  // synchronised round, first launch: only the minimum over the series
    if (lane == 0) atomicMin(p.sync, n);
    return;
  }
  if (p.mode == 2) n = min(n, *p.sync);
  if (lane < K) {
    p.ell[(long)b * KE + lane] = is_tested ? ell : NAN;
    p.logu[(long)b * KE + lane] = is_tested ? logu : NAN;
  }
  const int L = n + 1;
  const int Lc = min(L, p.T - c0);
  float* fc = p.forecast + ((long)b * p.T + c0) * P;
  for (int j = 0; j < min(Lc, n); ++j)
    for (int e = lane; e < P; e += 64) fc[j * P + e] = X[j * P + e];
  // corrected (n < K) or bonus (n = K) patch: the target mean, plus r * eps when fallback noise is on
  for (int e = lane; e < P; e += 64) {
    float t = MP[n * P + e];
    if (p.fallback_r > 0.f)
      t += p.fallback_r * normal_draw((unsigned)b, (unsigned)r, (unsigned)(n + 1), kStreamFallback, e, p.key0, p.key1);
    if (n < Lc) fc[n * P + e] = t;
    float old_pending = p.pending[(long)b * P + e];
    p.prev[(long)b * P + e] = (n >= 1) ? X[(n - 1) * P + e] : old_pending;
    p.pending[(long)b * P + e] = t;
  }
  if (lane == 0) {
    p.n_acc[b] = n_free;
    p.len[b] += Lc;
    p.committed[b] = c0 + Lc;
    p.round[b] = r + 1;
    p.active[b] = (c0 + Lc < p.T) ? 1 : 0;
    long long* st = p.stat + (long)b * 5;
    st[0] += 1;
    st[1] += tested;
    st[2] += n_free;
    st[3] += Lc;
    st[4] += __popcll(near);
  }
}

hipError_t launch_accept(const AcceptP& p, hipStream_t st) {
  hipLaunchKernelGGL(accept_kernel, dim3(p.B), dim3(64), 0, st, p);
  return hipGetLastError();
}

__global__ void fill_int_kernel(int* p, int value, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = value;
}
hipError_t launch_fill_int(int* p, int value, int n, hipStream_t st) {
  hipLaunchKernelGGL(fill_int_kernel, dim3((unsigned)((n + 63) / 64)), dim3(64), 0, st, p, value, n);
  return hipGetLastError();
}

// ---- read-out helpers ------------------------------------------------------------------------
__global__ void forecast_out_kernel(const float* forecast, const float* mean, const float* sdev, const int* committed,
                                    float* out, int P, int T, int H) {
  const int b = blockIdx.x;
  const int have = committed[b] * P;
  for (int t = threadIdx.x; t < H; t += blockDim.x)
    out[(long)b * H + t] = t < have ? forecast[(long)b * T * P + t] * sdev[b] + mean[b] : 0.f;
}
hipError_t launch_forecast_out(const float* forecast, const float* mean, const float* sdev, const int* committed,
                               float* out, int B, int P, int T, int H, hipStream_t st) {
  hipLaunchKernelGGL(forecast_out_kernel, dim3(B), dim3(256), 0, st, forecast, mean, sdev, committed, out, P, T, H);
  return hipGetLastError();
}

// One block: stable compaction of the active series (ascending series index) and their count.
// count[0] = number of active series, count[1] = the largest number of patches any of them still
// needs (T - committed).
__global__ __launch_bounds__(1024) void compact_active_kernel(const int* active, const int* committed, int T, int B,
                                                              int* list, int* count, int* host) {
  __shared__ int wave_cnt[16];
  __shared__ int base_s, max_rem;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (threadIdx.x == 0) {
    base_s = 0;
    max_rem = 0;
  }
  __syncthreads();
  for (int b0 = 0; b0 < B; b0 += 1024) {
    const int b = b0 + threadIdx.x;
    const bool on = b < B && active[b] != 0;
    const unsigned long long m = __ballot(on);
    if (lane == 0) wave_cnt[w] = __popcll(m);
    __syncthreads();
    int off = base_s;
    for (int i = 0; i < w; ++i) off += wave_cnt[i];
    if (on) {
      list[off + __popcll(m & ((1ull << lane) - 1ull))] = b;
      atomicMax(&max_rem, T - committed[b]);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int t = 0;
      for (int i = 0; i < 16; ++i) t += wave_cnt[i];
      base_s += t;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    count[0] = base_s;
    count[1] = max_rem;
    if (host) {
      // straight into pinned host memory, so the caller needs neither a copy nor a stream wait: it watches
      // host[2] for this launch's number, which is stored last
      const int seq = count[4] + 1;
      count[4] = seq;
      host[0] = base_s;
      host[1] = max_rem;
      __hip_atomic_store(&host[2], seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
  }
}
hipError_t launch_compact_active(const int* active, const int* committed, int T, int B, int* list, int* count,
                                 int* host, hipStream_t st) {
  hipLaunchKernelGGL(compact_active_kernel, dim3(1), dim3(1024), 0, st, active, committed, T, B, list, count, host);
  return hipGetLastError();
}

__global__ void sum_stats_kernel(const long long* stat, int B, long long* out5) {
  long long c[5] = {0, 0, 0, 0, 0};
  for (int i = threadIdx.x; i < B; i += 64)
    for (int j = 0; j < 5; ++j) c[j] += stat[(long)i * 5 + j];
  for (int j = 0; j < 5; ++j) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) c[j] += __shfl_xor(c[j], o);
    if (threadIdx.x == 0) out5[j] = c[j];
  }
}
__global__ void identity_list_kernel(int* list, int* count, int B, int T) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) list[b] = b;
  if (b == 0) {
    count[0] = B;
    count[1] = T;
  }
}
hipError_t launch_identity_list(int* list, int* count, int B, int T, hipStream_t st) {
  hipLaunchKernelGGL(identity_list_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, st, list, count, B, T);
  return hipGetLastError();
}

hipError_t launch_sum_stats(const long long* stat, int B, long long* out5, hipStream_t st) {
  hipLaunchKernelGGL(sum_stats_kernel, dim3(1), dim3(64), 0, st, stat, B, out5);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void copy_kernel(uint4* dst, const uint4* src, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t st) {
  const size_t n16 = bytes / 16;
  const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 32);
  hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, st, (uint4*)dst, (const uint4*)src, n16);
  return hipGetLastError();
}

// Matrix-core tap: four independent accumulation chains per wavefront keep the MFMA pipe full; the
// operands stay in registers, so nothing but the matrix cores is measured.
__global__ __launch_bounds__(256) void mfma_peak_kernel(int iters, float* sink) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (bf16)(0.015625f * (float)(1 + ((threadIdx.x + e) & 3)));
    b[e] = (bf16)(0.015625f * (float)(1 + ((threadIdx.x >> 2) & 3)));
  }
  f32x16 c0, c1, c2, c3;
#pragma unroll
  for (int r = 0; r < 16; ++r) c0[r] = c1[r] = c2[r] = c3[r] = 0.f;
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}
hipError_t launch_mfma_peak(int blocks, int iters, float* sink, hipStream_t st) {
  hipLaunchKernelGGL(mfma_peak_kernel, dim3(blocks), dim3(256), 0, st, iters, sink);
  return hipGetLastError();
}

__global__ void fill_nan_kernel(float* p, long n) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = NAN;
}
hipError_t launch_fill_nan(float* p, long n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_nan_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n);
  return hipGetLastError();
}

}  // namespace tsd
