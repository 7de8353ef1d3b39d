// The whole draft phase of a speculation round in one launch (Sec. "Speculative Decoding for
// Patch-Autoregressive Models": the draft proposes x_1 .. x_K autoregressively, each step feeding
// its own mean back in).
//
// A draft step of a small model over a few hundred series is a chain of a dozen dependent kernels
// that each run for a few microseconds: the chain, not the arithmetic, sets its duration.  But the
// steps of different series never meet -- a series' proposals depend on its own history and on the
// weights only -- so a workgroup can own a few series (1 to 8) for the whole phase: all K steps, all layers,
// with the residual stream, the activations and the proposals kept in LDS, and nothing but
// workgroup barriers between the stages.  Every workgroup then streams the full set of draft
// weights once per step (from L2, which they fit) straight into MFMA B-operand registers, 16 bytes
// per lane with several loads in flight; that stream through one CU's vector-memory path is what
// bounds the kernel.  The stream reads a second copy of the draft weights kept in fragment order
// (per 16-column block and 32-wide k-step the 64 lanes' 16-byte pieces back to back, k zero-padded
// to whole steps, the QKV columns already in rotary-pair order), so each load instruction of a
// wavefront covers one contiguous kilobyte.
//
// Rows of the 16-row MFMA tile: step 1 ingests two tokens per series (row 2s + t: the token before
// the pending one, and the pending one), later steps one (row s); the other rows idle.  The arithmetic
// per row is that of the kernel-per-stage path: bf16 operands, fp32 accumulation, fp32 residual
// with a bf16 shadow as the next A operand, RMSNorm as a row scale of the product, RoPE and the
// KV-cache write in the QKV epilogue, fp32 inputs (patches, the head's residual) split hi + lo.
#include <algorithm>

#include "attn_mfma.h"
#include "philox.h"
#include "tsd_internal.h"

namespace tsd {

namespace {

constexpr int kRows = 16;  // one MFMA row tile
constexpr int kSerMax = kDraftFusedSeries;  // most series a workgroup keeps (16 rows in step 1)

struct Lds {  // element offsets of the regions carved from dynamic LDS
  int ldx, ldb, ldh, ldp;
  size_t xs, pin, xb, qb, ab, hb, misc, total;
};

__host__ __device__ inline Lds carve(int D, int F, int P) {
  Lds l;
  l.ldx = D + 4;                    // fp32 residual rows
  l.ldb = D + 8;                    // bf16 rows of width D
  l.ldh = F + 8;                    // bf16 hidden rows
  l.ldp = ((P + 31) & ~31) + 4;     // fp32 patch rows, zero-padded to whole k-steps
  size_t o = 0;
  l.xs = o;
  o += (size_t)kRows * l.ldx * 4;
  l.pin = o;
  o += (size_t)kRows * l.ldp * 4;
  l.xb = o;
  o += (size_t)kRows * l.ldb * 2;
  l.qb = o;
  o += (size_t)kRows * l.ldb * 2;
  l.ab = o;
  o += (size_t)kRows * l.ldb * 2;
  l.hb = o;  // hidden activations; the attention stage parks its V tiles here (8 KB per wavefront, 8 wavefronts)
  const size_t hid = (size_t)kRows * l.ldh * 2, vt = (size_t)8 * 2 * 32 * 64 * 2;
  o += hid > vt ? hid : vt;
  l.misc = o;  // kvrow[16] long, pos[16] int, page[16] int, ser[8] int, lens[8] int, spt[8][64] int, rope cos / sin [16][32] float
  o += (size_t)(2 * 16 + 16 + 16 + 8 + 8 + 8 * 64 + 2 * 16 * 32) * 4;
  l.total = (o + 15) & ~(size_t)15;
  return l;
}

__device__ __forceinline__ void split_hi_lo8(const float* f, bf16x8& hi, bf16x8& lo) {
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    hi[e] = (bf16)f[e];
    lo[e] = (bf16)(f[e] - (float)hi[e]);
  }
}

// Column of the [3D][D] QKV matrix that lane-column l16 of 16-column block blk stands for:
// block -> (q | k | v, head, j), columns head*64 + 8 j + 0..7 and their rotary partners 32 further on.
__host__ __device__ inline int qkv_col(int blk, int l16, int Hh, int D) {
  const int which = blk / (4 * Hh), rem = blk - which * 4 * Hh;
  return which * D + (rem >> 2) * 64 + (rem & 3) * 8 + (l16 & 7) + (l16 >> 3) * 32;
}

// One streamed product: W in fragment order, its 16-column blocks, its 32-wide k-steps, and the k-steps per
// block of the fragment copy (padded with zero fragments to whole chunks).
struct Wsrc {
  const bf16* Wp;
  int nblk, nks, nksp;
};

// The four register buffers a wavefront streams weights through (CH k-steps, one kilobyte each, per buffer).
template <int CH>
struct Wbuf {
  bf16x8 b0[CH], b1[CH], b2[CH], b3[CH];
};

// Chunk `item` of this wavefront's share of `w` (its blocks wave, wave + NW, ..., each in nksp / CH
// chunks) -> registers: CH consecutive kilobytes.  The caller keeps item in range.
template <int NW, int CH>
__device__ __forceinline__ void fetch_chunk(const Wsrc& w, int item, int wave, int lane, bf16x8 (&dst)[CH]) {
  const int nch = w.nksp / CH;
  const int j = item / nch, c = item - j * nch;
  const bf16* base = w.Wp + lane * 8 + ((long)(wave + j * NW) * w.nksp + c * CH) * 512;
#pragma unroll
  for (int u = 0; u < CH; ++u) dst[u] = *reinterpret_cast<const bf16x8*>(base + u * 512);
}

template <int NW, int CH>
__device__ __forceinline__ int my_items(const Wsrc& w, int wave) {
  return wave < w.nblk ? ((w.nblk - wave + NW - 1) / NW) * (w.nksp / CH) : 0;
}

// Starts the loads of the first three chunks of `w`: called ahead of the barriers and small stages
// that precede the product, so that its first operands are on their way while those run.
template <int NW, int CH>
__device__ __forceinline__ void prime(const Wsrc& w, int wave, int lane, Wbuf<CH>& B) {
  // every buffer is dead here: say so (an output-only empty asm defines the registers at no cost), or the
  // conditionally written ones would count as live across the whole kernel
#pragma unroll
  for (int u = 0; u < CH; ++u) {
    asm volatile("" : "=v"(B.b0[u]));
    asm volatile("" : "=v"(B.b1[u]));
    asm volatile("" : "=v"(B.b2[u]));
    asm volatile("" : "=v"(B.b3[u]));
  }
  const int total = my_items<NW, CH>(w, wave);
  if (total > 0) fetch_chunk<NW, CH>(w, 0, wave, lane, B.b0);
  if (total > 1) fetch_chunk<NW, CH>(w, 1, wave, lane, B.b1);
  if (total > 2) fetch_chunk<NW, CH>(w, 2, wave, lane, B.b2);
}

// One wavefront's share of C[16, N] = A[16, K] W[N, K]^T, `w` primed beforehand.  A sits in LDS (bf16, or
// fp32 split into hi + lo).  While one chunk feeds the MFMAs, the loads of the next three are in flight;
// nothing is fetched past the wavefront's last chunk, and once that is consumed `next` is primed.
// epi(block, acc): acc[i] is row 4 (lane / 16) + i, column lane % 16 of the block.
template <int NW, int CH, bool kSplit, typename Epi>
__device__ __forceinline__ void wave_gemm(const Wsrc& w, const Wsrc& next, const void* a_lds, int lda, int wave, int lane,
                                          Wbuf<CH>& B, Epi epi) {
  // (an opaque copy of the lane id: keeps the address arithmetic below inside this call instead of
  //  hoisted, with one live register per value, to the top of the kernel's step loop)
  asm volatile("" : "+v"(lane));
  const int total = my_items<NW, CH>(w, wave);
  const int li = lane & 15, koff = (lane >> 4) * 8;
  const int nks = w.nks, nch = w.nksp / CH;
  f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
  // (k-steps past nks meet zero fragments of W: their A operand is re-read from the last real step, no branch)
  int cj = 0, cc = 0;  // block and chunk of the chunk consumed next (counted along: no division per chunk)
  auto consume = [&](const bf16x8 (&use)[CH]) {
    const int j = cj, c = cc;
    if (++cc == nch) {
      cc = 0;
      ++cj;
    }
    if constexpr (kSplit) {
#pragma unroll
      for (int u = 0; u < CH; ++u) {
        if (c * CH + u >= nks) break;  // (the few fp32-split products are short: a branch per k-step is fine here)
        const float* ap = reinterpret_cast<const float*>(a_lds) + li * lda + (c * CH + u) * 32 + koff;
        float f[8];
        *reinterpret_cast<float4*>(f) = *reinterpret_cast<const float4*>(ap);
        *reinterpret_cast<float4*>(f + 4) = *reinterpret_cast<const float4*>(ap + 4);
        bf16x8 hi, lo;
        split_hi_lo8(f, hi, lo);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lo, use[u], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi, use[u], acc, 0, 0, 0);
      }
    } else {
      bf16x8 a[CH];
#pragma unroll
      for (int u = 0; u < CH; ++u)
        a[u] = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const bf16*>(a_lds) + li * lda + min(c * CH + u, nks - 1) * 32 + koff);
#pragma unroll
      for (int u = 0; u < CH; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u], use[u], acc, 0, 0, 0);
    }
    if (c == nch - 1) {
      epi(wave + j * NW, acc);
      acc = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  };
  // chunk 3 is the next to fetch: its address, then a walk by pointer (chunks of a block are contiguous, the
  // wavefront's next block lies NW blocks further on)
  const long chunk_elems = (long)CH * 512, block_skip = (long)(NW - 1) * w.nksp * 512;
  int fc = 3 % nch;
  const bf16* fptr = w.Wp + lane * 8 + ((long)(wave + (3 / nch) * NW) * w.nksp + fc * CH) * 512;
  auto fetch = [&](int item, bf16x8 (&dst)[CH]) {
    if (item < total) {
#pragma unroll
      for (int u = 0; u < CH; ++u) dst[u] = *reinterpret_cast<const bf16x8*>(fptr + u * 512);
    }
    fptr += chunk_elems;
    if (++fc == nch) {
      fc = 0;
      fptr += block_skip;
    }
  };
  for (int it = 0; it < total; it += 4) {
    fetch(it + 3, B.b3);
    consume(B.b0);
    if (it + 1 >= total) break;
    fetch(it + 4, B.b0);
    consume(B.b1);
    if (it + 2 >= total) break;
    fetch(it + 5, B.b1);
    consume(B.b2);
    if (it + 3 >= total) break;
    fetch(it + 6, B.b2);
    consume(B.b3);
  }
  prime<NW, CH>(next, wave, lane, B);
}

// Workgroup barrier that orders LDS traffic only: weight loads primed ahead stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// RMSNorm scales 1 / sqrt(mean_k a[r][k]^2 + eps) of the 16 rows, computed by every wavefront for itself
// (four lanes per row, K a multiple of 32) so that no barrier separates them from the product that applies
// them: out[i] is the scale of row 4 (lane / 16) + i, the rows of this lane's accumulator.
template <typename T>
__device__ __forceinline__ void row_scales(const T* a, int lda, int K, int lane, float (&out)[4]) {
  asm volatile("" : "+v"(lane));
  const int r = lane >> 2, q = lane & 3;
  float s = 0.f;
  for (int k = q * 8; k < K; k += 32) {
    float f[8];
    if constexpr (sizeof(T) == 2) {
      const bf16x8 v = *reinterpret_cast<const bf16x8*>(a + r * lda + k);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = (float)v[e];
    } else {
      *reinterpret_cast<float4*>(f) = *reinterpret_cast<const float4*>(a + r * lda + k);
      *reinterpret_cast<float4*>(f + 4) = *reinterpret_cast<const float4*>(a + r * lda + k + 4);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) s = fmaf(f[e], f[e], s);
  }
  s += __shfl_xor(s, 1);
  s += __shfl_xor(s, 2);
  const float rsv = rsqrtf(s / (float)K + kRmsEps);
#pragma unroll
  for (int i = 0; i < 4; ++i) out[i] = __shfl(rsv, (4 * (lane >> 4) + i) * 4);
}

// kTrace: the measurement build (tsd_trace_draft) that stamps the wall clock after every stage barrier; the
// production instantiation (kTrace = false) contains none of it.
template <int NW, int CH, bool kTrace>
__global__ __launch_bounds__(NW * 64) void draft_fused_kernel(const DraftFusedP p) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), li = lane & 15, lg = lane >> 4;
  // measurement build only: workgroup 0 notes the 100 MHz wall clock after every stage barrier
  long long* const trace = kTrace && blockIdx.x == 0 && threadIdx.x == 0 ? p.trace : nullptr;
  int n_stamps = 0;
#define STAGE_STAMP()                                                                     \
  do {                                                                                    \
    if constexpr (kTrace) {                                                               \
      if (trace && n_stamps < p.trace_max) trace[n_stamps++] = wall_clock64();            \
    }                                                                                     \
  } while (0)
  const int n = p.n_dev ? min(*p.n_dev, p.n) : p.n;
  const int kSer = p.spw;  // series of this workgroup: 1, 2, 4 or 8
  const int j0 = blockIdx.x * kSer;
  if (j0 >= n) return;  // (uniform: the whole workgroup leaves)
  const int D = p.D, F = p.F, P = p.P, Hh = p.Hh;
  const Lds L = carve(D, F, P);
  float* xs = reinterpret_cast<float*>(smem + L.xs);
  float* pin = reinterpret_cast<float*>(smem + L.pin);
  bf16* xb = reinterpret_cast<bf16*>(smem + L.xb);
  bf16* qb = reinterpret_cast<bf16*>(smem + L.qb);
  bf16* ab = reinterpret_cast<bf16*>(smem + L.ab);
  bf16* hb = reinterpret_cast<bf16*>(smem + L.hb);
  long* kvrow = reinterpret_cast<long*>(smem + L.misc);  // [16]: element offset of the row's token in a K plane of head 0
  int* pos = reinterpret_cast<int*>(kvrow + 16);
  int* page = pos + 16;
  int* ser = page + 16;
  int* lens = ser + 8;  // [8]: committed tokens of the series (position of the pending patch)
  int* spt = lens + 8;  // [8][64]: the series' page tables
  float* rcos = reinterpret_cast<float*>(spt + 8 * 64);  // [16][32]: the rows' rotary factors
  float* rsin = rcos + 16 * 32;
  const int ldx = L.ldx, ldb = L.ldb, ldh = L.ldh, ldp = L.ldp;

  // ---- set-up: series of this workgroup, their page tables, zeroed patch rows (the k padding stays 0) ----
  if (tid < kSerMax) ser[tid] = p.act ? p.act[min(j0 + tid, n - 1)] : min(j0 + tid, n - 1);  // slots past n clone the last series
  for (int i = tid; i < kRows * ldp; i += NW * 64) pin[i] = 0.f;
  __syncthreads();
  STAGE_STAMP();
  for (int i = tid; i < kSerMax * 64; i += NW * 64) {
    const int s = i >> 6, pg = i & 63;
    spt[i] = p.page_table[(long)ser[s] * p.pt_stride + min(pg, p.pt_stride - 1)];
  }
  if (tid < kSerMax) lens[tid] = p.len[ser[tid]];
  // the two tokens step 1 ingests (in the same round trip as the page tables)
  for (int i = tid; i < kRows * P; i += NW * 64) {
    const int r = i / P, e = i - r * P;
    const float* src = (r & 1) ? p.pending : p.prev;
    pin[r * ldp + e] = src[(long)ser[r >> 1] * P + e];
  }
  __syncthreads();
  STAGE_STAMP();

  // the products of a step, in the order the weights are streamed
  const Wsrc none{nullptr, 0, 0, 0};
  auto padded = [](int nks) { return (nks + CH - 1) / CH * CH; };
  const int ksP = (P + 31) >> 5, ksD = D >> 5, ksF = F >> 5;
  const Wsrc w_e{p.W_e, D / 16, ksP, padded(ksP)}, w_h{p.W_h, P / 16, ksD, padded(ksD)};
  auto w_qkv = [&](int l) { return Wsrc{p.Wqkv[l], 3 * D / 16, ksD, padded(ksD)}; };
  auto w_o = [&](int l) { return Wsrc{p.Wo[l], D / 16, ksD, padded(ksD)}; };
  auto w_1 = [&](int l) { return Wsrc{p.W1[l], F / 16, ksD, padded(ksD)}; };
  auto w_2 = [&](int l) { return Wsrc{p.W2[l], D / 16, ksF, padded(ksF)}; };
  Wbuf<CH> B;
  prime<NW, CH>(w_e, wave, lane, B);

  for (int step = 1; step <= p.Kr; ++step) {
    const int nq = step == 1 ? 2 : 1;
    const int nrows = kSer * nq;
    // ---- positions and rotary factors of the step's rows (its input patches are in place: loaded at set-up
    //      for step 1, left there by the previous step's head afterwards) ----
    for (int i = tid; i < kRows * 32; i += NW * 64) {
      const int r = i >> 5, f = i & 31;
      const int s = step == 1 ? r >> 1 : min(r, kSer - 1);
      const int ps = lens[s] + (step == 1 ? (r & 1) - 1 : step - 1);
      rcos[i] = p.rope_cos[(long)ps * 32 + f];
      rsin[i] = p.rope_sin[(long)ps * 32 + f];
      if (f == 0) {
        pos[r] = ps;
        page[r] = spt[s * 64 + (ps >> p.pt_shift)];
        kvrow[r] = ((long)page[r] * 2 * Hh * p.PT + (ps & (p.PT - 1))) * 64;
      }
    }
    lds_barrier();
    STAGE_STAMP();
    auto row_live = [&](int r) { return r < nrows && j0 + (step == 1 ? r >> 1 : r) < n; };
    // (the epilogues below read everything they need first, compute, then store: written with `if`s per
    //  element they cost 1300 cycles per QKV block, mostly LDS round trips waited for one at a time)
    bool live4[4];  // rows 4 lg + i of this lane's accumulators
#pragma unroll
    for (int i = 0; i < 4; ++i) live4[i] = row_live(4 * lg + i);

    // ---- patch embedding: x = W_e patch ----
    wave_gemm<NW, CH, true>(
        w_e, w_qkv(0), pin, ldp, wave, lane, B,
        [&](int blk, f32x4 acc) {
          const int c = blk * 16 + li;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int r = 4 * lg + i;
            xs[r * ldx + c] = acc[i];
            xb[r * ldb + c] = (bf16)acc[i];
          }
        });
    lds_barrier();
    STAGE_STAMP();

    for (int l = 0; l < p.L; ++l) {
      bf16* pool = p.kv_pool + (size_t)l * p.layer_pool_elems;
      // ---- RMSNorm + QKV + RoPE; k, v to the paged cache, q stays here ----
      float rs[4];
      row_scales(xb, ldb, D, lane, rs);
      // (with 4-step chunks the next product's first operands can stay in registers through the attention stage)
      constexpr bool kPrimeOverAttn = CH <= 4;
      wave_gemm<NW, CH, false>(w_qkv(l), kPrimeOverAttn ? w_o(l) : none, xb, ldb, wave, lane, B, [&](int blk, f32x4 acc) {
        const int which = blk / (4 * Hh), rem = blk - which * 4 * Hh;  // (uniform over the wavefront)
        const int h = rem >> 2, f = (rem & 3) * 8 + (li & 7), d = f + (li >> 3) * 32;
        float v[4], pv[4], cs[4], sn[4];
        long kvo[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          cs[i] = rcos[(4 * lg + i) * 32 + f];
          sn[i] = rsin[(4 * lg + i) * 32 + f];
          kvo[i] = kvrow[4 * lg + i];
          v[i] = acc[i] * rs[i];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) pv[i] = __shfl_xor(v[i], 8);
        if (which < 2) {
          const float sg = li < 8 ? -1.f : 1.f;
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = v[i] * cs[i] + sg * pv[i] * sn[i];
        }
        if (which == 0) {
#pragma unroll
          for (int i = 0; i < 4; ++i) qb[(4 * lg + i) * ldb + h * 64 + d] = (bf16)v[i];
        } else {
          const long plane = ((long)((which - 1) * Hh + h) * p.PT) * 64 + d;
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (live4[i]) pool[kvo[i] + plane] = (bf16)v[i];
        }
      });
      __syncthreads();  // (also makes the cache rows written above visible to the workgroup's loads)
      STAGE_STAMP();

      // ---- causal attention of the new tokens over the series' cache: one (series, head) per wavefront turn ----
      if (wave < 8) {
        bf16* vt = hb + wave * (2 * 32 * 64);
        for (int pr = wave; pr < kSer * Hh; pr += 8) {
          const int s = pr / Hh, h = pr - s * Hh;
          if (j0 + s >= n) continue;
          const int r0 = s * nq;
          const int my_page = spt[s * 64 + lane];
          const bf16* qt = qb + r0 * ldb + h * 64;
          bf16* ot = ab + r0 * ldb + h * 64;
          attn_tile_mfma<false>(pool, h, Hh, p.PT, p.pt_shift, my_page, pos[r0], nq, p.scale,
                                [&](int r) { return qt + r * ldb; }, [&](int r) { return ot + r * ldb; }, vt);
        }
      }
      if constexpr (!kPrimeOverAttn) prime<NW, CH>(w_o(l), wave, lane, B);
      lds_barrier();
      STAGE_STAMP();

      // ---- attention output projection + residual ----
      auto resid_epi = [&](int blk, f32x4 acc) {
        const int c = blk * 16 + li;
        float o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = xs[(4 * lg + i) * ldx + c];
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] += acc[i];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          xs[(4 * lg + i) * ldx + c] = o[i];
          xb[(4 * lg + i) * ldb + c] = (bf16)o[i];
        }
      };
      wave_gemm<NW, CH, false>(w_o(l), w_1(l), ab, ldb, wave, lane, B, resid_epi);
      lds_barrier();
      STAGE_STAMP();

      // ---- RMSNorm + FFN up + GELU ----
      row_scales(xb, ldb, D, lane, rs);
      wave_gemm<NW, CH, false>(w_1(l), w_2(l), xb, ldb, wave, lane, B, [&](int blk, f32x4 acc) {
        const int c = blk * 16 + li;
        float g[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) g[i] = gelu_tanh(acc[i] * rs[i]);
#pragma unroll
        for (int i = 0; i < 4; ++i) hb[(4 * lg + i) * ldh + c] = (bf16)g[i];
      });
      lds_barrier();
      STAGE_STAMP();

      // ---- FFN down + residual ----
      wave_gemm<NW, CH, false>(w_2(l), l + 1 < p.L ? w_qkv(l + 1) : w_h, hb, ldh, wave, lane, B, resid_epi);
      lds_barrier();
      STAGE_STAMP();
    }

    // ---- RMSNorm (of the fp32 residual) + head: the step's proposal, also the next step's input ----
    float rs[4];
    row_scales(xs, ldx, D, lane, rs);
    wave_gemm<NW, CH, true>(w_h, step < p.Kr ? w_e : none, xs, ldx, wave, lane, B,
                            [&](int blk, f32x4 acc) {
                              const int c = blk * 16 + li;
#pragma unroll
                              for (int i = 0; i < 4; ++i) {
                                const int r = 4 * lg + i;
                                if (r >= nrows || (step == 1 && !(r & 1))) continue;  // step 1 emits from the pending token only
                                const int s = step == 1 ? r >> 1 : r;
                                float v = acc[i] * rs[i];
                                const long xo = (long)ser[s] * p.x_stride + (long)(step - 1) * P + c;
                                if (p.mu_q) {
                                  // sampled proposals: the mean goes to its own buffer, the draw x_i = mu_q + sigma_q eps
                                  // (the series' own round counter, position `step`) is what everyone downstream consumes
                                  if (j0 + s < n) p.mu_q[xo] = v;
                                  v += (p.sigma_q_vec ? p.sigma_q_vec[c] : p.sigma_q) *
                                       normal_draw((unsigned)ser[s], (unsigned)p.round[ser[s]], (unsigned)step, kStreamProposal, c, p.key0, p.key1);
                                }
                                if (j0 + s < n) p.X[xo] = v;
                                pin[s * ldp + c] = v;
                              }
                            });
    lds_barrier();
    STAGE_STAMP();
  }
}

#undef STAGE_STAMP

// dst (fragment order, nksp k-steps per block: k zero-padded to whole chunks of 32-wide steps) <- src [N][K];
// Hh > 0: the QKV column order
__global__ __launch_bounds__(256) void repack_kernel(const bf16* src, bf16* dst, int N, int K, int nksp, int Hh, int D) {
  const long total = (long)N * nksp * 32;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
    const int e = (int)(i & 7), lane = (int)((i >> 3) & 63);
    const long fr = i >> 9;
    const int ks = (int)(fr % nksp), blk = (int)(fr / nksp);
    const int l16 = lane & 15, k = ks * 32 + (lane >> 4) * 8 + e;
    const int col = Hh > 0 ? qkv_col(blk, l16, Hh, D) : blk * 16 + l16;
    dst[i] = k < K ? src[(long)col * K + k] : (bf16)0.f;
  }
}

template <int NW, int CH>
hipError_t launch_cfg(const DraftFusedP& p, size_t smem, hipStream_t st) {
  const dim3 grid((unsigned)((p.n + p.spw - 1) / p.spw)), block(NW * 64);
  if (p.trace)
    hipLaunchKernelGGL((draft_fused_kernel<NW, CH, true>), grid, block, smem, st, p);
  else
    hipLaunchKernelGGL((draft_fused_kernel<NW, CH, false>), grid, block, smem, st, p);
  return hipGetLastError();
}

}  // namespace

size_t draft_fused_lds_bytes(int D, int F, int P) { return carve(D, F, P).total; }

int draft_fused_chunk(int D, int F) { return (D % 256 == 0 && F % 256 == 0) ? 8 : 4; }

static int padded_ksteps(int K, int chunk) { return (((K + 31) >> 5) + chunk - 1) / chunk * chunk; }

size_t draft_fused_packed_elems(int N, int K, int chunk) { return (size_t)N * padded_ksteps(K, chunk) * 32; }

hipError_t launch_repack_fragments(const void* src, void* dst, int N, int K, int chunk, int qkv_heads, int D, hipStream_t st) {
  if (N % 16 || K < 8 || (chunk != 4 && chunk != 8)) return hipErrorInvalidValue;
  const size_t total = draft_fused_packed_elems(N, K, chunk);
  const unsigned grid = (unsigned)std::min<size_t>((total + 255) / 256, 4096);
  hipLaunchKernelGGL(repack_kernel, dim3(grid), dim3(256), 0, st, reinterpret_cast<const bf16*>(src), reinterpret_cast<bf16*>(dst), N,
                     K, padded_ksteps(K, chunk), qkv_heads, D);
  return hipGetLastError();
}

hipError_t prepare_draft_fused() {
  const void* fns[4] = {reinterpret_cast<const void*>(&draft_fused_kernel<8, 8, false>),
                        reinterpret_cast<const void*>(&draft_fused_kernel<8, 4, false>),
                        reinterpret_cast<const void*>(&draft_fused_kernel<8, 8, true>),
                        reinterpret_cast<const void*>(&draft_fused_kernel<8, 4, true>)};
  for (const void* f : fns) {
    hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_draft_fused(const DraftFusedP& p, hipStream_t st) {
  const size_t smem = carve(p.D, p.F, p.P).total;
  if (smem > 160 * 1024 || p.n < 1 || p.Kr < 1 || p.L < 1 || p.L > kDraftFusedMaxLayers) return hipErrorInvalidValue;
  if (p.spw != 1 && p.spw != 2 && p.spw != 4 && p.spw != 8) return hipErrorInvalidValue;
  if (p.chunk == 4) return launch_cfg<8, 4>(p, smem, st);
  if (p.chunk == 8) return launch_cfg<8, 8>(p, smem, st);
  return hipErrorInvalidValue;
}

}  // namespace tsd
