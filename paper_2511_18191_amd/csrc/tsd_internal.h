// Internal declarations shared by the libtsd translation units (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "tsd.h"

namespace tsd {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kRmsEps = 1e-6f;   // inside the root of RMSNorm
constexpr float kNormEps = 1e-5f;  // inside the root of the instance normalisation
constexpr double kRopeBase = 10000.0;

#if defined(__HIPCC__)
// tanh-GELU, 0.5 z (1 + tanh(u)) with u = sqrt(2/pi) (z + 0.044715 z^3), evaluated as z / (1 + exp(-2u)) with the
// exponent formed directly in base 2: -2 u log2(e) = z (a + b z^2).  Three multiplications, one fused multiply-add,
// one addition, one hardware exponential and one reciprocal: every output element of the FFN-up GEMM pays it in the
// epilogue, where the matrix cores wait, so it is written out to the instruction (a library tanh costs ten times that).
__device__ __forceinline__ float gelu_tanh(float z) {
  constexpr float a = -2.0f * 0.7978845608028654f * 1.4426950408889634f;  // -2 sqrt(2/pi) log2(e)
  constexpr float b = a * 0.044715f;
  const float q = z * fmaf(z * z, b, a);
  return z * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(q));
}
#endif

// ---- A-operand sources and epilogues of the fused GEMM family ------------------------------
enum AMode {
  A_TOK = 0,   // fp32 patches gathered from two per-series segments (patch embedding)
  A_NORM = 1,  // fp32 residual stream; RMSNorm applied as a per-row scale of the product
  A_ACT = 2,   // activations already in the compute dtype
  A_NORM32 = 3 // like A_NORM but reads the fp32 residual itself (output head; split hi+lo in bf16 mode)
};
enum Epi {
  EP_STORE = 0,  // x = C                       (fp32)
  EP_RESID = 1,  // x += C                      (fp32 residual stream)
  EP_GELU = 2,   // h = GELU_tanh(C)            (compute dtype)
  EP_QKV = 3,    // RoPE on q,k; q -> buffer, k,v -> paged KV cache
  EP_HEAD = 4    // mu = C, fp32, scattered to [series][token - t_skip]
};

struct GemmP {
  int M, N, K;
  // A operand
  const void* A;  // A_NORM: const float* [M][K]; A_ACT: const T* [M][K]
  const float* src0;
  const float* src1;  // A_TOK: token t of series b comes from src0 + b*stride0 + t*K (t < n0)
  long stride0, stride1;  //        else from src1 + b*stride1 + (t - n0)*K
  int n0;
  int nq;        // tokens per series in this pass: row r = (series r / nq, token r % nq)
  const void* W;  // T [N][K]: transposed weights
  // outputs
  float* Cf;      // EP_STORE / EP_RESID: [M][N]
  void* Cb;       // EP_STORE / EP_RESID, bf16 mode: shadow copy of the result in bf16 (nullable)
  void* Ct;       // EP_GELU: T [M][N]
  // EP_QKV
  void* q_out;    // T [M][D]
  void* kv_pool;  // this layer's pool: T [n_pages][2 (K, V)][Hh][PT][hd]
  const int* page_table;
  int pt_stride;
  const int* base_pos;  // per-series position of token 0 minus pos_off (NULL = 0)
  int pos_off;
  int s0;  // first series of this pass (chunked prefill)
  const int* act;
  // compacted pass: row block i belongs to series act[i] (NULL: series s0 + i)
  const int* n_dev;  // device-side series count for launches replayed from a graph: rows = min(M, *n_dev * nq) (NULL: M)
  const float* rope_cos;
  const float* rope_sin;  // [max_tokens][hd/2]
  int D, Hh, hd, PT;
  int pt_shift;  // log2(PT)
  // grouped (routed-FFN) mode: the row tiles come from a device-side map, one expert per tile
  const void* tile_map;  // int4 per row tile: (expert or -1, first slot, end slot of the expert, 0); NULL = dense
  const int* src_row;    // A row of slot s is src_row[s] (NULL: the slot itself)
  long w_stride;         // elements between consecutive experts' matrices in W
  int n_mtiles;          // entries of tile_map
  int force_bm;          // row-tile size the map was built for (0 = pick by problem size)
  int allow_skinny;      // the handle runs its <= 32-row passes through the skinny kernel
  int no_wide;           // never pick the direct-to-LDS wide-tile kernels (gemm_wide.hip)
  // EP_HEAD
  float* out;
  long out_stride_b;
  int t_skip;
};

struct AttnP {
  const void* q;       // T [rows][D]
  void* out;           // T [rows][D]
  const void* kv_pool; // this layer's pool
  const int* page_table;
  int pt_stride;
  const int* base_pos;
  int pos_off;
  int s0;
  const int* act;  // compacted pass: block i handles series act[i] (NULL: series s0 + i)
  const int* n_dev;  // device-side series count (NULL: B): blocks of series >= *n_dev exit
  int nq, B, Hh, hd, D, PT;
  int pt_shift;  // log2(PT)
  int mfma;          // bf16, head_dim 64, pages of at least 8 tokens: the matrix-core kernel
  int model;         // TSD_TARGET / TSD_DRAFT: selects the kernel's name only (profilers then keep the two models apart)
  float scale;
};

// ---- launchers (each returns the hipError_t of the launch) ---------------------------------
hipError_t launch_gemm(int dtype, int amode, int epi, const GemmP& p, hipStream_t st);
hipError_t prepare_gemm(int dtype);
// bf16 products of activations with K >= kQuarterK are summed in four runs of k-steps (see gemm.hip)
constexpr int kQuarterK = 1024;
// skinny path (at most 32 rows): see gemm_skinny.hip
bool skinny_applicable(int dtype, int amode, int epi, const GemmP& p);
hipError_t launch_gemm_skinny(int amode, int epi, const GemmP& p, hipStream_t st);
int gemm_row_tile(int dtype, int M, int N, int force_bm);
// wide-tile kernels (gemm_wide.hip): row-tile size for this product (256 or 128), or 0 for the register-staged kernels
int gemm_wide_bm(int dtype, int amode, int epi, const GemmP& p);
hipError_t launch_gemm_wide(int amode, int epi, int bm, const GemmP& p, hipStream_t st);
hipError_t prepare_gemm_wide();
// which kernel launch_gemm picks for this product: 16 = skinny, 64 / 128 = tile size, 464 = 64 x 64 tiles with K split over four wavefront groups,
// 2256 / 2128 = the wide-tile kernels with 256 / 128-row tiles
int gemm_variant(int dtype, int amode, int epi, const GemmP& p);
// s_max: upper bound on (position of the pass's last token) + 1 over all series; sizes the score buffer.
hipError_t launch_attention(int dtype, const AttnP& p, int s_max, hipStream_t st);
// dynamic LDS the attention kernel needs for up to s_max cached tokens (must stay <= 160 KB)
size_t attention_lds_bytes(int dtype, int hd, int s_max, int page_tokens);
hipError_t prepare_attention(int dtype, int hd, int s_max, int page_tokens);

// ---- the draft phase in one launch (dense bf16 draft, head_dim 64): see draft_fused.hip ----
constexpr int kDraftFusedSeries = 8;     // most series per workgroup
constexpr int kDraftFusedMaxLayers = 8;
struct DraftFusedP {
  // the draft's weights in fragment order (launch_repack_fragments)
  const bf16* W_e;  // of [D][P]
  const bf16* W_h;  // of [P][D]
  const bf16* Wqkv[kDraftFusedMaxLayers];  // of [3D][D], columns in rotary-pair order
  const bf16* Wo[kDraftFusedMaxLayers];    // of [D][D]
  const bf16* W1[kDraftFusedMaxLayers];    // of [F][D]
  const bf16* W2[kDraftFusedMaxLayers];    // of [D][F]
  bf16* kv_pool;           // the draft's pools, layer after layer
  size_t layer_pool_elems;
  const float* rope_cos;
  const float* rope_sin;   // [max_tokens][32]
  const int* page_table;
  int pt_stride;           // pages per series (at most 64)
  const int* len;          // committed tokens per series: the pending patch sits at position len
  const int* act;          // slot j is series act[j] (NULL: series j)
  const int* n_dev;        // device-side count of listed series (NULL: n)
  int n;                   // listed series (the grid covers them)
  int spw;                 // series per workgroup: 1, 2, 4 or 8
  const float* prev;       // [B][P] token before the pending one
  const float* pending;    // [B][P]
  float* X;                // proposals: x_i of series b at X + b * x_stride + (i - 1) * P
  // sampled proposals (mu_q NULL: x_i is the mean): means to mu_q (laid out like X), x_i = mu_q^(i) + sigma_q eps
  float* mu_q;
  const int* round;        // per-series round counter (second word of the draw's counter)
  float sigma_q;
  const float* sigma_q_vec;  // per-dimension scales (NULL: sigma_q)
  unsigned key0, key1;
  long x_stride;
  int Kr;                  // steps (proposals) of this round
  int L, D, F, Hh, P, PT, pt_shift;
  float scale;             // 1 / sqrt(head_dim)
  int chunk;               // k-steps per streamed chunk the fragment copy was padded for: 4 or 8
  long long* trace;        // measurement tap (NULL: off): wall-clock ticks after every stage barrier of workgroup 0
  int trace_max;
};
size_t draft_fused_lds_bytes(int D, int F, int P);
// k-steps per streamed chunk for a draft of these widths (the fragment copy pads every block's k to whole chunks)
int draft_fused_chunk(int D, int F);
// elements of the fragment-order copy of a bf16 [N][K] matrix
size_t draft_fused_packed_elems(int N, int K, int chunk);
// dst <- src [N][K] in fragment order; qkv_heads > 0: N = 3 D and the columns take the QKV block order
hipError_t launch_repack_fragments(const void* src, void* dst, int N, int K, int chunk, int qkv_heads, int D, hipStream_t st);
hipError_t prepare_draft_fused();
hipError_t launch_draft_fused(const DraftFusedP& p, hipStream_t st);

struct PackP {
  const float* W;     // [K][N] row-major source (y = x W)
  const float* gain;  // [K] or NULL: folded as W'[n][k] = gain[k] * W[k][n]
  void* out;          // T [N][K]
  int K, N;
};
hipError_t launch_pack(int dtype, const PackP& p, hipStream_t st);

struct PrefillP {
  const float* series;  // [B][N*P]
  float* znorm;         // [B][N*P] normalised
  float* mean;
  float* sdev;          // [B]
  float* pending;
  float* prev;          // [B][P]
  int* len;
  int* committed;
  int* round;
  int* active;
  long long* stat;      // [B][5]
  int B, N, P;
  const int* slots;     // refill: row j of `series` goes to slot slots[j] (NULL: slot j)
  int keep_counters;    // refill: the slot's round counter and statistics run on
  int* act_list;        // prefill / reset: the active list becomes the identity ...
  int* act_count;       // ... with count[0] = batch, count[1] = T (NULL: leave both alone)
  int batch, T;
};
hipError_t launch_prefill_stats(const PrefillP& p, hipStream_t st);
hipError_t launch_reset(const PrefillP& p, hipStream_t st);

struct AcceptP {
  const float* X;
  const float* mu_q;  // [B][K][P]
  const float* mu_p;  // [B][K+1][P]
  const int* forced;  // nullable
  const int* act;     // compacted round: block i handles series act[i] (NULL: series i)
  const int* n_dev;   // device-side series count (NULL: B)
  float* pending;
  float* prev;
  float* forecast;    // [B][T*P] normalised
  int* len;
  int* committed;
  int* round;
  int* active;
  int* n_acc;         // [B]
  float* ell;
  float* logu;        // [B][max(K,1)]
  long long* stat;    // [B][5]: rounds, tested, accepted, committed, near_ties
  int B, K, P, T;
  float inv2sp2, inv2sq2, logdet, temper;  // temper = 1 (Eq. 5) or P (ablation without 1/d)
  float log_alpha_override;                // > 0 means "no override"
  float fallback_r;                        // noise scale of the corrected / bonus patch (0: target mean)
  // diagonal-covariance surrogate (NULL: isotropic): 1 / (2 s_p[e]^2), 1 / (2 s_q[e]^2) per dimension and
  // the scalar (1 / 2P) sum_e log(s_q[e]^2 / s_p[e]^2)
  const float *inv2sp2_vec, *inv2sq2_vec, *logdet_dev;
  unsigned key0, key1;
  int threshold;  // deterministic rule: -||x - mu_p||_d^2 / (2 sigma_p^2) against log u = -1/2, no draw
  // batch-synchronised acceptance runs the kernel twice: mode 1 only folds every series' own count
  // into *sync (atomic minimum; the word starts at INT_MAX), mode 2 commits with n = *sync;
  // mode 0 is the unsynchronised round in one launch
  int mode;
  int* sync;
};
hipError_t launch_accept(const AcceptP& p, hipStream_t st);
hipError_t launch_fill_int(int* p, int value, int n, hipStream_t st);

struct SampleP {  // X[b, i-1] = mu_q[b, i-1] + sigma_q * eps(b, round[b], i)
  const float* mu_q;
  float* X;
  const int* act;    // block j handles series act[j] (NULL: series j)
  const int* n_dev;  // device-side series count (NULL: n)
  const int* round;
  int n, K, P, i;
  float sigma_q;
  const float* sigma_q_vec;  // per-dimension scales (NULL: sigma_q)
  unsigned key0, key1;
};
hipError_t launch_sample(const SampleP& p, hipStream_t st);

hipError_t prepare_moe();
hipError_t launch_router(const float* x, const float* Wr, int M, int D, int E, int topk, int* ids, float* gates,
                         hipStream_t st);
hipError_t launch_permute(const int* ids, int n_assign, int topk, int E, int BM, int n_mtiles, int* src_row,
                          int* slot_of, void* tile_map, hipStream_t st);
hipError_t launch_route_tap(const int* ids, int* tap, int layer, int M, int nq, const int* act, int s0, const int* base_pos,
                            int pos_off, int max_batch, int max_tokens, int topk, hipStream_t st);
hipError_t launch_combine(int dtype, const float* Y, const int* slot_of, const float* gates, float* x, void* xb, int M,
                          int D, int topk, hipStream_t st);

hipError_t launch_forecast_out(const float* forecast, const float* mean, const float* sdev, const int* committed,
                               float* out, int B, int P, int T, int H, hipStream_t st);
// stable list of the series with active != 0; count[0] = how many, count[1] = max over them of T - committed.
// host (nullable): pinned host words; the kernel also bumps its launch counter count[4] and delivers
// host[0] = count[0], host[1] = count[1], then host[2] = the new counter value (system-scope release).
hipError_t launch_compact_active(const int* active, const int* committed, int T, int B, int* list, int* count,
                                 int* host, hipStream_t st);
// active list = identity, count[0] = B, count[1] = T
hipError_t launch_identity_list(int* list, int* count, int B, int T, hipStream_t st);
hipError_t launch_sum_stats(const long long* stat, int B, long long* out5, hipStream_t st);
hipError_t launch_fill_nan(float* p, long n, hipStream_t st);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t st);
hipError_t launch_mfma_peak(int blocks, int iters, float* sink, hipStream_t st);

}  // namespace tsd
