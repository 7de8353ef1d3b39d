// tsd_accept_commit_static: the acceptance / correction / commit step of one round on caller tensors, for
// callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
// that forbid it).  It runs the same accept_kernel as tsd_accept_commit; the per-series state that kernel
// keeps between its steps (round counter, committed count, cache length, active flag, pending / previous
// token, counters, the synchronised round's minimum, and the statistic / draw taps when the caller does not
// want them) lives in one file-scope device array instead of a caller-provided arena.
#include <climits>
#include <cmath>
#include <cstring>
#include <string>

#include "tsd_internal.h"

namespace tsd {
// implemented in tsd_api.hip: records the message tsd_last_error(NULL) returns
int fail_no_handle(int code, const std::string& msg);
}  // namespace tsd

using namespace tsd;

namespace {

// Limits of the static variant (the scratch array is sized for them and is held on every GPU the library runs
// on until the process ends).
constexpr int kMaxB = 4096;             // series per call
constexpr int kMaxK = 16;               // proposals per round
constexpr long kMaxBP = 256 * 1024;     // B * P: e.g. 1024 series of 256-step patches, or 4096 of 64

// Layout of the scratch array, in bytes from its start (every part 256-byte aligned).
constexpr size_t kOffPending = 0;                                     // float [B][P]
constexpr size_t kOffPrev = kOffPending + (size_t)kMaxBP * 4;         // float [B][P]
constexpr size_t kOffEll = kOffPrev + (size_t)kMaxBP * 4;             // float [B][K]
constexpr size_t kOffLogu = kOffEll + (size_t)kMaxB * kMaxK * 4;      // float [B][K]
constexpr size_t kOffStat = kOffLogu + (size_t)kMaxB * kMaxK * 4;     // int64 [B][5]
constexpr size_t kOffLen = kOffStat + (size_t)kMaxB * 5 * 8;          // int [B]
constexpr size_t kOffCommitted = kOffLen + (size_t)kMaxB * 4;         // int [B]
constexpr size_t kOffRound = kOffCommitted + (size_t)kMaxB * 4;       // int [B]
constexpr size_t kOffActive = kOffRound + (size_t)kMaxB * 4;          // int [B]
constexpr size_t kOffSync = kOffActive + (size_t)kMaxB * 4;           // int [64]
constexpr size_t kScratchBytes = kOffSync + 256;                      // about 2.8 MB

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Address of this device's copy of `scratch` (each GPU holds its own), looked up once per device.
constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Everything the accept kernel reads before it writes must start from a defined state: the series are all
// active with nothing committed, their round counters are the caller's, counters are zero, the pending token
// (which becomes the "previous token" when nothing is accepted) is zero, and the synchronised round's minimum
// starts at INT_MAX.  (A fill kernel, not a memset: the call may be captured into a graph.)
__global__ __launch_bounds__(256) void static_init_kernel(unsigned char* s, const int* round_in, int B, int P) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  float* pending = reinterpret_cast<float*>(s + kOffPending);
  float* prev = reinterpret_cast<float*>(s + kOffPrev);
  if (i < (long)B * P) {
    pending[i] = 0.f;
    prev[i] = 0.f;
  }
  if (i < B) {
    reinterpret_cast<int*>(s + kOffLen)[i] = 0;
    reinterpret_cast<int*>(s + kOffCommitted)[i] = 0;
    reinterpret_cast<int*>(s + kOffRound)[i] = round_in ? round_in[i] : 0;
    reinterpret_cast<int*>(s + kOffActive)[i] = 1;
    long long* st = reinterpret_cast<long long*>(s + kOffStat) + i * 5;
    for (int j = 0; j < 5; ++j) st[j] = 0;
  }
  if (i == 0) reinterpret_cast<int*>(s + kOffSync)[0] = INT_MAX;
}

}  // namespace

extern "C" int tsd_accept_commit_static(const float* X_dev, const float* mu_q_dev, const float* mu_p_dev,
                                        const int32_t* round_dev, int32_t B, int32_t K, int32_t P, float sigma_p,
                                        float sigma_q, float fallback_r, uint64_t seed, uint32_t flags,
                                        int32_t* n_acc_dev, float* commit_dev, float* ell_dev, float* logu_dev,
                                        void* stream) {
  if (!X_dev || !mu_q_dev || !mu_p_dev || !n_acc_dev || !commit_dev)
    return fail_no_handle(TSD_E_INVALID_ARG, "X_dev, mu_q_dev, mu_p_dev, n_acc_dev and commit_dev must not be NULL");
  if (B < 1 || K < 1 || P < 1) return fail_no_handle(TSD_E_INVALID_ARG, "need B >= 1, K >= 1, P >= 1");
  if (B > kMaxB || K > kMaxK || (long)B * P > kMaxBP)
    return fail_no_handle(TSD_E_OUT_OF_RANGE,
                          "tsd_accept_commit_static holds its state in a fixed device array: at most 4096 series, K <= 16 "
                          "and B * P <= 262144 (use a handle and tsd_accept_commit beyond that)");
  if (!(sigma_p > 0.f) || !(sigma_q > 0.f) || !std::isfinite(sigma_p) || !std::isfinite(sigma_q))
    return fail_no_handle(TSD_E_INVALID_ARG, "sigma_p and sigma_q must be positive and finite");
  if (!(fallback_r >= 0.f) || fallback_r > sigma_p) return fail_no_handle(TSD_E_INVALID_ARG, "fallback_r must lie in [0, sigma_p]");
  if (flags & ~(TSD_FLAG_NO_TEMPERING | TSD_FLAG_THRESHOLD_RULE | TSD_FLAG_BATCH_SYNC))
    return fail_no_handle(TSD_E_INVALID_ARG, "flags: only TSD_FLAG_NO_TEMPERING, TSD_FLAG_THRESHOLD_RULE and TSD_FLAG_BATCH_SYNC apply here");
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_no_handle(TSD_E_HIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail_no_handle(TSD_E_OUT_OF_RANGE, "device index beyond 63");
  if (!g_scratch_ptr[dev]) {
    // the array's name is only a host-side stand-in: the device address has to be asked for, with this device current
    unsigned char* ptr = nullptr;
    e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail_no_handle(TSD_E_HIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  unsigned char* s = g_scratch_ptr[dev];
  hipStream_t st = (hipStream_t)stream;
  const long cells = std::max((long)B * P, (long)B);
  hipLaunchKernelGGL(static_init_kernel, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, st, s, round_dev, B, P);
  if ((e = hipGetLastError()) != hipSuccess) return fail_no_handle(TSD_E_HIP, std::string("state set-up launch: ") + hipGetErrorString(e));

  AcceptP a;
  std::memset(&a, 0, sizeof(a));
  a.X = X_dev;
  a.mu_q = mu_q_dev;
  a.mu_p = mu_p_dev;
  a.pending = reinterpret_cast<float*>(s + kOffPending);
  a.prev = reinterpret_cast<float*>(s + kOffPrev);
  a.forecast = commit_dev;  // with T = K + 1 and nothing committed before, the round's patches land at [b][0 .. n]
  a.len = reinterpret_cast<int*>(s + kOffLen);
  a.committed = reinterpret_cast<int*>(s + kOffCommitted);
  a.round = reinterpret_cast<int*>(s + kOffRound);
  a.active = reinterpret_cast<int*>(s + kOffActive);
  a.n_acc = n_acc_dev;
  a.ell = ell_dev ? ell_dev : reinterpret_cast<float*>(s + kOffEll);
  a.logu = logu_dev ? logu_dev : reinterpret_cast<float*>(s + kOffLogu);
  a.stat = reinterpret_cast<long long*>(s + kOffStat);
  a.B = B;
  a.K = K;
  a.P = P;
  a.T = K + 1;
  a.inv2sp2 = 1.0f / (2.0f * sigma_p * sigma_p);
  a.inv2sq2 = 1.0f / (2.0f * sigma_q * sigma_q);
  a.logdet = 0.5f * std::log((sigma_q * sigma_q) / (sigma_p * sigma_p));
  a.temper = (flags & TSD_FLAG_NO_TEMPERING) ? (float)P : 1.0f;
  a.log_alpha_override = 1.0f;
  a.fallback_r = fallback_r;
  a.key0 = (unsigned)(seed & 0xFFFFFFFFull);
  a.key1 = (unsigned)(seed >> 32);
  a.threshold = (flags & TSD_FLAG_THRESHOLD_RULE) ? 1 : 0;
  if (flags & TSD_FLAG_BATCH_SYNC) {
    a.sync = reinterpret_cast<int*>(s + kOffSync);
    a.mode = 1;
    if ((e = launch_accept(a, st)) != hipSuccess) return fail_no_handle(TSD_E_HIP, std::string("acceptance launch: ") + hipGetErrorString(e));
    a.mode = 2;
  }
  if ((e = launch_accept(a, st)) != hipSuccess) return fail_no_handle(TSD_E_HIP, std::string("acceptance launch: ") + hipGetErrorString(e));
  return TSD_OK;
}
