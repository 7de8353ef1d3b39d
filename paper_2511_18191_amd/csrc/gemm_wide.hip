// Wide-tile bf16 GEMM for products that fill the chip: C[M,N] = A[M,K] * Wt[N,K]^T with the fused epilogues of the
// tiled family (gemm_epilogue.h).  Both operands go from global memory straight into LDS (global_load_lds_dwordx4:
// no staging registers, no LDS writes by the lanes) through a small ring of stages of one k-tile each.
//
// What bounds a GEMM on this chip is the number of requests its compute units send to L2 (counters: at 64 bytes per
// request the 128 L2 channels saturate near one request per clock each, ~12 TB/s, long before the matrix cores do).
// So a k-tile is 64 wide (a row of it is one whole 128-byte cache line: one request instead of two) and the tile is
// as large as the product's tile count allows (256 x 128 where that still fills the chip, else 128 x 128).
//
//   * A stage is its rows back to back (A rows, then B rows), 128 bytes per row; the eight 16-byte chunks of a row
//     sit at chunk ^ ((row >> 1) & 7), which makes the fragment reads (32 consecutive rows, one chunk) conflict-free
//     without padding.  A load instruction fills 1 KB = 8 rows; lane l fetches the chunk that belongs at l.
//   * A wavefront owns one contiguous run of every stage and addresses its loads through the instruction's immediate
//     offset around one base, so M0 (the LDS base of such a load) is written once per k-tile.
//   * The k loop is software-pipelined by k16 sub-steps: while the MFMAs of one sub-step run, the fragments of the next
//     are on their way from LDS, also across k-tiles.  One barrier per k-tile, before its LAST sub-step: by then every
//     wavefront holds all of the k-tile's fragments in registers, so the k-tile's own slot is refilled at once (with two
//     stages a k-tile has a whole k-tile's time to arrive, with three two).
//   * The RMSNorm row sums come from the A fragments on their way to the matrix cores (A never sits in registers
//     otherwise), in the summation order of the register-staged kernel (gemm.hip): per row eight partial sums, one per
//     16-byte chunk position of a 64-wide k-run, each a chain of packed bf16 dot products, combined as
//     ((P0 + P4) + (P2 + P6)) + ((P1 + P5) + (P3 + P7)).  The products accumulate k in the same order with the
//     same instruction, so both kernels give the same bits and the launcher may pick either by the product's shape.
#include <cstdlib>

#include "gemm_epilogue.h"
#include "tsd_internal.h"

// Timing experiments (never defined in the library build): bits of TSD_WIDE_PROBE switch pieces of the k loop off
// to price them (1 loads, 2 fragment reads, 4 MFMAs, 8 barrier, 16 epilogue arithmetic and stores, 32 the whole epilogue);
// the results are then garbage, every access stays in bounds and every wavefront meets the same barriers.
#ifndef TSD_WIDE_PROBE
#define TSD_WIDE_PROBE 0
#endif

namespace tsd {

#define TSD_GLOBAL_PTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define TSD_LDS_PTR(p) ((void __attribute__((address_space(3)))*)(p))

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// BM x BN x BK tiles, WGM x WGN wavefronts, NS stages
template <int BM_, int BN_, int BK_, int WGM_, int WGN_, int NS_>
struct WideShape {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_, NS = NS_;
  static constexpr int NW = WGM * WGN, NT = NW * 64;
  static constexpr int ROWB = BK * 2;               // bytes of a stage row: 64 or 128
  static constexpr int CPR = ROWB / 16;             // 16-byte chunks per row
  static constexpr int RPL = 1024 / ROWB;           // rows a load instruction covers
  static constexpr int ROWS = BM + BN;              // rows of a stage
  static constexpr int STAGE = ROWS * ROWB;
  static constexpr int NL = STAGE / 1024 / NW;      // load instructions of a wavefront per stage
  static constexpr int REGION = NL * 1024;          // a wavefront's bytes of a stage
  static constexpr int BIAS = REGION / 2 / 1024 * 1024;  // M0 points here inside the region: immediates stay small
  static constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;  // 32 x 32 blocks per wavefront
  static constexpr int NSUB = BK / 16;              // k16 sub-steps per k-tile
  static constexpr int NPAR = 64 / BK;              // k-tiles per 64-wide k-run
  static constexpr int LDC = BN + 4;
  static constexpr int CS_BYTES = 64 * LDC * 4;
  static constexpr size_t SMEM = (size_t)NS * STAGE + BM * 12;  // stages, then row_scale / row_pos / row_page
  static_assert(BK == 32 || BK == 64, "k-tiles of 32 or 64");
  static_assert(STAGE % (1024 * NW) == 0 && BM % RPL == 0, "every wavefront loads whole instructions, each all A or all B");
  static_assert(CS_BYTES <= NS * STAGE, "the epilogue's buffer reuses the stages");
  static_assert(REGION - BIAS <= 4096 && BIAS <= 4096, "immediate offsets are 13 bits, signed");
};

// The NL loads of one wavefront for one stage: load J goes to base + J * 1024 - BIAS (the immediate must be a
// compile-time constant, hence the recursion instead of a loop).
template <int J, int NL, int BIAS>
__device__ __forceinline__ void issue_stage_loads(const bf16* const* gp, long koff, void __attribute__((address_space(3)))* base) {
  if constexpr (J < NL) {
    __builtin_amdgcn_global_load_lds(TSD_GLOBAL_PTR(gp[J] + koff), base, 16, J * 1024 - BIAS, 0);
    issue_stage_loads<J + 1, NL, BIAS>(gp, koff, base);
  }
}

template <int N>
struct IC : std::integral_constant<int, N> {};

template <int AM, int EP, typename S>
__global__ __launch_bounds__(S::NT, 2) void gemm_wide_kernel(const GemmP p) {
  constexpr bool kNorm = (AM == A_NORM);
  constexpr int BM = S::BM, BN = S::BN, BK = S::BK, NS = S::NS, TM = S::TM, TN = S::TN, NL = S::NL, REGION = S::REGION,
                STAGE = S::STAGE, LDC = S::LDC, BIAS = S::BIAS, ROWB = S::ROWB, CPR = S::CPR, RPL = S::RPL, NSUB = S::NSUB,
                NPAR = S::NPAR, WGN = S::WGN;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  float* Cs = reinterpret_cast<float*>(smem);                            // [64][LDC], after the main loop
  float* row_scale = reinterpret_cast<float*>(smem + NS * STAGE);        // [BM]
  int* row_pos = reinterpret_cast<int*>(smem + NS * STAGE + BM * 4);     // [BM] EP_QKV
  int* row_page = row_pos + BM;                                          // [BM] EP_QKV

  const int tid = threadIdx.x, lane = tid & 63, wid = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wid / WGN, wn = wid % WGN;
  // rows of the product: fixed at launch, or capped by a device-side series count (workgroups past the cap leave)
  const int M = p.n_dev ? min(p.M, *p.n_dev * p.nq) : p.M;
  const int N = p.N, K = p.K;
  // tile order: every XCD walks one contiguous run of the tile list, the list ordered in groups of 8 tile columns
  // walked row by row (see gemm.hip)
  const int tiles_m = p.tile_map ? p.n_mtiles : (M + BM - 1) / BM, tiles_n = N / BN;
  const int n_tiles = tiles_m * tiles_n;
  const int per_xcd = (n_tiles + 7) >> 3;
  if ((int)(blockIdx.x >> 3) >= per_xcd) return;
  const int lin = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (lin >= n_tiles) return;
  constexpr int GW = 8;
  const int gc = lin / (GW * tiles_m), rem = lin - gc * (GW * tiles_m);
  const int gw = min(GW, tiles_n - gc * GW);
  const int tm = rem / gw, tn = gc * GW + rem - tm * gw;
  int m0 = tm * BM, m_lim = M;
  const int n0 = tn * BN;
  const bf16* Wp = reinterpret_cast<const bf16*>(p.W);
  if (p.tile_map) {  // routed FFN: this row tile belongs to one expert's run of slots
    const int4 tmap = reinterpret_cast<const int4*>(p.tile_map)[tm];
    if (tmap.x < 0) return;
    m0 = tmap.y;
    m_lim = tmap.z;
    Wp += (long)tmap.x * p.w_stride;
  }

  if constexpr (EP == EP_QKV) {
    for (int r = tid; r < BM; r += S::NT) {
      const int gm = min(m0 + r, m_lim - 1);
      const int bl = gm / p.nq, t = gm - bl * p.nq, b = p.act ? p.act[bl] : p.s0 + bl;
      const int pos = (p.base_pos ? p.base_pos[b] : 0) + p.pos_off + t;
      row_pos[r] = pos;
      row_page[r] = p.page_table[(long)b * p.pt_stride + (pos >> p.pt_shift)];
    }
  }

  // ---- loads: wavefront w fills the stage rows [NL * RPL * w, NL * RPL * (w + 1)); stage row R is A row R (R < BM) or B
  // row R - BM.  Lane l of load j covers row (w NL + j) RPL + l / CPR and the physical chunk l % CPR of it, i.e. the
  // logical chunk (l % CPR) ^ swizzle(row).  The immediate of load j (j * 1024 - BIAS) is added to BOTH addresses by the
  // instruction, so it is taken off the global pointer here.
  auto swizzle = [](int R) { return BK == 64 ? (R >> 1) & 7 : (R >> 2) & 3; };
  const bf16* Ap = reinterpret_cast<const bf16*>(p.A);
  const bf16* gp[NL];
#pragma unroll
  for (int j = 0; j < NL; ++j) {
    const int R = (wid * NL + j) * RPL + lane / CPR;
    const int chunk = (lane % CPR) ^ swizzle(R);
    const bf16* row;
    if ((wid * NL + j) * RPL < BM) {  // (uniform per instruction: BM is a multiple of the rows it covers)
      int gm = min(m0 + R, m_lim - 1);  // rows past M are clamped to the last row: their products are never stored
      if (p.src_row) gm = p.src_row[gm];
      row = Ap + (long)gm * K;
    } else {
      row = Wp + (long)(n0 + R - BM) * K;
    }
    gp[j] = row + chunk * 8 - (j * 1024 - BIAS) / 2;
  }
  auto issue_loads = [&](int slot, int kt) {
    if constexpr (TSD_WIDE_PROBE & 1) return;  // probe: no operand loads
    void __attribute__((address_space(3)))* base = TSD_LDS_PTR(smem + slot * STAGE + wid * REGION + BIAS);
    issue_stage_loads<0, NL, BIAS>(gp, (long)kt * BK, base);
  };

  // ---- fragments: lane l reads row l % 32 of a 32-row block, chunk 2 s + l / 32 of k16 sub-step s
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  // Long contractions of activations are summed in four runs of ceil(nk / 4) k-tiles, each from zero, the runs added in
  // order (the order of the split workgroups of gemm.hip, which every kernel that can take such a product keeps to)
  constexpr bool kQuarters = (AM == A_ACT) && BK == 64;
  f32x16 tot[kQuarters ? TM : 1][kQuarters ? TN : 1];
  float ss[TM][4];  // row-sum chains of this lane: chunk positions hi, 2 + hi, 4 + hi, 6 + hi of a 64-wide k-run
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int c = 0; c < 4; ++c) ss[i][c] = 0.f;
  const int r31 = lane & 31, hi = lane >> 5;
  int offA[TM], offB[TN], swA[TM], swB[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int R = wm * (TM * 32) + i * 32 + r31;
    offA[i] = R * ROWB;
    swA[i] = swizzle(R);
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int R = BM + wn * (TN * 32) + j * 32 + r31;
    offB[j] = R * ROWB;
    swB[j] = swizzle(R);
  }

  // The k loop by k16 sub-steps (TM + TN fragment reads, TM x TN MFMAs each), two fragment sets F[0], F[1] in turn:
  //   sub-step s of k-tile kt:   read F[(s + 1) & 1] <- the next sub-step;   MFMAs on F[s & 1]
  // and before the read of the LAST sub-step's successor (sub-step 0 of k-tile kt + 1) the barrier of k-tile kt:
  //   this wavefront's loads of k-tile kt + 1 are done (only those of later k-tiles may still be in flight) and its
  //   fragments of k-tile kt all sit in registers (LDS counter at zero: they were requested a sub-step's MFMAs ago);
  //   after the barrier that holds for everybody, so k-tile kt + 1 can be read and the slot of k-tile kt itself refilled
  //   with k-tile kt + NS.
  // (a bare s_barrier: __syncthreads() would also wait for every load in flight)
  bf16x8 fa[2][TM], fb[2][TN];
  auto read_frags = [&](int kt, int s, bf16x8* af, bf16x8* bfr) {
    if constexpr (TSD_WIDE_PROBE & 2) return;  // probe: no fragment reads (the MFMAs run on whatever the registers hold)
    const unsigned char* st = smem + (kt % NS) * STAGE;
#pragma unroll
    for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const bf16x8*>(st + offA[i] + (((2 * s + hi) ^ swA[i]) << 4));
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(st + offB[j] + (((2 * s + hi) ^ swB[j]) << 4));
  };
  auto mfmas = [&](auto cpos, const bf16x8* af, const bf16x8* bfr) {
    constexpr int C = decltype(cpos)::value;  // which row-sum chain this sub-step feeds
    if constexpr (kNorm) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bf16x2 pr = {af[i][2 * e], af[i][2 * e + 1]};
          ss[i][C] = __builtin_amdgcn_fdot2_f32_bf16(pr, pr, ss[i][C], false);
        }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if constexpr (TSD_WIDE_PROBE & 4) {  // probe: no MFMAs (the fragments are still consumed)
          asm volatile("" ::"v"(af[i]), "v"(bfr[j]));
        } else {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
      }
  };
  // `arrived`: an empty statement that uses a fragment set, placed BEFORE the next set's reads are issued.  The compiler
  // waits for LDS data right before its first use and cannot tell the two sets' reads apart by count here, so without it
  // the wait would land after the next set's reads were issued and cover those too (a full LDS round trip exposed per
  // sub-step); with it the wait covers only reads issued a sub-step ago, which have long landed.
  auto arrived = [&](bf16x8* af, bf16x8* bfr) {
#pragma unroll
    for (int i = 0; i < TM; ++i) asm volatile("" : "+v"(af[i]));
#pragma unroll
    for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(bfr[j]));
  };
  // One k-tile.  PAR: its position inside the 64-wide k-run (always 0 for 64-wide k-tiles); PEND: the loads this
  // wavefront may leave in flight at the barrier (those of the k-tiles after kt + 1), or -1 for the last k-tile (no
  // barrier, nothing left to read); REFILL: k-tile kt + NS exists.
  auto tile = [&](auto par, int kt, auto pend, auto refill) {
    constexpr int PAR = decltype(par)::value, PEND = decltype(pend)::value;
    constexpr bool REFILL = decltype(refill)::value != 0;
    const auto sub = [&](auto sc) {
      constexpr int s = decltype(sc)::value;
      arrived(fa[s & 1], fb[s & 1]);
      if constexpr (s + 1 < NSUB) {
        read_frags(kt, s + 1, fa[(s + 1) & 1], fb[(s + 1) & 1]);
      } else if constexpr (PEND >= 0) {
        if constexpr (TSD_WIDE_PROBE & 8)  // probe: no barrier
          asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        else
          asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(PEND) : "memory");
        if constexpr (REFILL) issue_loads(kt % NS, kt + NS);
        read_frags(kt + 1, 0, fa[(s + 1) & 1], fb[(s + 1) & 1]);
      }
      __builtin_amdgcn_sched_barrier(0);
      mfmas(IC<PAR * NSUB + s>{}, fa[s & 1], fb[s & 1]);
      __builtin_amdgcn_sched_barrier(0);
    };
    sub(IC<0>{});
    sub(IC<1>{});
    if constexpr (NSUB == 4) {
      sub(IC<2>{});
      sub(IC<3>{});
    }
  };

  // ---- main loop (K is a multiple of 64, at least NS 64-wide runs) ------------------------------------------------------
  const int nk = K / BK;
  // (nothing older may be in flight when the counted waits begin: the counts assume only the stages' loads)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
  for (int s = 0; s < NS; ++s) issue_loads(s, s);
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NS - 1) * NL) : "memory");  // k-tile 0 has landed for everybody
  read_frags(0, 0, fa[0], fb[0]);
  // steady state: k-tiles 0 .. nk - NS - 1 (each refills its slot); then the last NS k-tiles
  constexpr int STEADY_PEND = (NS - 2) * NL;
  const int n_steady = nk - NS;
  const bool quarters = kQuarters && K >= kQuarterK;
  const int run = (nk + 3) / 4;
  auto fold = [&](int done) {  // `done` k-tiles are in acc: at a run's end move them into the running sum
    if constexpr (kQuarters) {
      if (!quarters || done % run != 0 || done >= nk) return;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            tot[i][j][r] = done == run ? acc[i][j][r] : tot[i][j][r] + acc[i][j][r];
            acc[i][j][r] = 0.f;
          }
    }
  };
  int kt = 0;
  if constexpr (NPAR == 1) {
    for (; kt < n_steady; ++kt) {
      tile(IC<0>{}, kt, IC<STEADY_PEND>{}, IC<1>{});
      fold(kt + 1);
    }
    // tail: k-tile nk - NS + t leaves NS - 2 - t stages in flight at its barrier; the last one has no barrier
    if constexpr (NS == 2) {
      tile(IC<0>{}, kt, IC<0>{}, IC<0>{});
      fold(kt + 1);
      tile(IC<0>{}, kt + 1, IC<-1>{}, IC<0>{});
    } else {
      tile(IC<0>{}, kt, IC<NL>{}, IC<0>{});
      fold(kt + 1);
      tile(IC<0>{}, kt + 1, IC<0>{}, IC<0>{});
      fold(kt + 2);
      tile(IC<0>{}, kt + 2, IC<-1>{}, IC<0>{});
    }
    if constexpr (kQuarters) {
      if (quarters) {  // the last run joins the sum of the first three
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = tot[i][j][r] + acc[i][j][r];
      }
    }
  } else {
    static_assert(NPAR == 1 || NS == 3, "32-wide k-tiles run with three stages");
    // nk is even, so nk - 3 is odd: pairs, then one more steady k-tile of parity 0, then the tail (parities 1, 0, 1)
    for (; kt + 1 < n_steady; kt += 2) {
      tile(IC<0>{}, kt, IC<STEADY_PEND>{}, IC<1>{});
      tile(IC<1>{}, kt + 1, IC<STEADY_PEND>{}, IC<1>{});
    }
    tile(IC<0>{}, kt, IC<STEADY_PEND>{}, IC<1>{});
    tile(IC<1>{}, kt + 1, IC<NL>{}, IC<0>{});
    tile(IC<0>{}, kt + 2, IC<0>{}, IC<0>{});
    tile(IC<1>{}, kt + 3, IC<-1>{}, IC<0>{});
  }

  // ---- RMSNorm row scale: this lane's chains are the chunk positions hi, 2 + hi, 4 + hi, 6 + hi ---------------------------
  if constexpr (kNorm) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const float b = (ss[i][0] + ss[i][2]) + (ss[i][1] + ss[i][3]);  // (P[hi] + P[4 + hi]) + (P[2 + hi] + P[6 + hi])
      const float tot = b + __shfl_xor(b, 32);
      if (wn == 0 && hi == 0) row_scale[wm * (TM * 32) + i * 32 + r31] = rsqrtf(tot / (float)K + kRmsEps);
    }
  }

  // ---- epilogue, 64 rows at a time through LDS ------------------------------------------------------------------
  // EP_RESID: the old residual values of a pass are requested one pass ahead (those of pass 0 before the accumulators'
  // trip through LDS), so that their latency hides behind LDS traffic and the previous pass's stores instead of being
  // paid once per item (a read that follows a store to the same array cannot be moved up by the compiler).
  auto read_c4 = [&](int row, int col) { return *reinterpret_cast<const float4*>(Cs + row * LDC + col); };
  constexpr int NPRE = (EP == EP_RESID) ? 64 * (BN / 4) / S::NT : 1;
  float4 oldc[2][NPRE];
  auto fetch_old = [&](int pass, float4* dst) {
    if constexpr (EP == EP_RESID) {
#pragma unroll
      for (int it = 0; it < NPRE; ++it) {
        const int g = tid + it * S::NT;
        const int gm = min(m0 + pass * 64 + g / (BN / 4), m_lim - 1), gn = n0 + (g % (BN / 4)) * 4;  // (N is a multiple of BN)
        dst[it] = *reinterpret_cast<const float4*>(p.Cf + (long)gm * N + gn);
      }
    }
  };
  if constexpr (TSD_WIDE_PROBE & 32) {  // probe: no epilogue at all (the accumulators are still produced)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) asm volatile("" ::"v"(acc[i][j][r]));
    return;
  }
  fetch_old(0, oldc[0]);
#pragma unroll
  for (int pass = 0; pass < BM / 64; ++pass) {
    __syncthreads();  // the stages (or the previous pass's rows) are no longer read
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int rbase = wm * (TM * 32) + i * 32 - pass * 64;  // first row of this block inside the pass
      if (rbase >= 0 && rbase < 64) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int row = rbase + (r >> 2) * 8 + hi * 4 + (r & 3);
            const int col = wn * (TN * 32) + j * 32 + r31;
            Cs[row * LDC + col] = acc[i][j][r];
          }
      }
    }
    if (pass + 1 < BM / 64) fetch_old(pass + 1, oldc[(pass + 1) & 1]);
    __syncthreads();
    if constexpr (TSD_WIDE_PROBE & 16) continue;  // probe: the accumulators' trip through LDS, but no epilogue arithmetic or stores
    epilogue_pass<bf16, EP, kNorm, BN, S::NT, EP == EP_RESID, true>(p, read_c4, row_scale, row_pos, row_page, m0, n0, pass, m_lim, N,
                                                                    tid, oldc[pass & 1]);
  }
}

// ---- host side -------------------------------------------------------------------------------------------------
#ifndef TSD_WIDE_SHAPE_256
#define TSD_WIDE_SHAPE_256 WideShape<256, 128, 64, 4, 2, 2>  // eight wavefronts of 64 x 64, one workgroup per compute unit
#endif
#ifndef TSD_WIDE_SHAPE_128
#define TSD_WIDE_SHAPE_128 WideShape<128, 128, 64, 2, 2, 2>  // four wavefronts of 64 x 64, two workgroups per compute unit
#endif
using Wide256 = TSD_WIDE_SHAPE_256;
using Wide128 = TSD_WIDE_SHAPE_128;

// Which row-tile size, if any, this product should take (0: the register-staged kernels of gemm.hip).
int gemm_wide_bm(int dtype, int amode, int epi, const GemmP& p) {
  if (dtype != TSD_BF16 || p.no_wide) return 0;
  const bool combo = (amode == A_ACT && (epi == EP_STORE || epi == EP_RESID)) ||
                     (amode == A_NORM && (epi == EP_STORE || epi == EP_GELU || epi == EP_QKV));
  if (!combo || (p.K % 64) || p.K < 192 || (p.N % 128)) return 0;
  // grouped products of the routed FFN: their tile map was built for force_bm-row tiles, and the 128-row map exists
  // only where the product already has 1.5 tiles per compute unit
  if (p.tile_map) return p.force_bm == 128 ? 128 : 0;
  if (p.src_row || p.force_bm) return 0;
  static const int forced = [] { const char* e = getenv("TSD_WIDE_FORCE"); return e ? atoi(e) : 0; }();  // A/B timing aid
  if (forced == 256 || forced == 128) return forced;
  const long cols = p.N / 128;
  const long t256 = (long)((p.M + 255) / 256) * cols, t128 = (long)((p.M + 127) / 128) * cols;
  // Measured over the products of the configurations (narrow / 128 / 256 timed side by side, same bits): two
  // workgroups of 128 x 128 per compute unit hide one's epilogue behind the other's k loop and win wherever there are
  // plenty of tiles; the 256-row tiles (one workgroup per unit, fewest operand requests) win the long-K products
  // with few tile columns; below about one tile per unit the 64 x 64 register-staged tiles keep more units busy.
  if (t128 >= 512) return 128;
  if (t128 >= 400 && t256 >= 200) return 256;
  if (p.K >= 2048) return t256 >= 140 ? 256 : t128 >= 200 ? 128 : 0;
  if (cols >= 12 && t128 >= 240) return 128;
  return 0;
}

template <int AM, int EP, typename S>
static hipError_t launch_wide_t(const GemmP& p, hipStream_t st) {
  const long tiles = (long)(p.tile_map ? p.n_mtiles : (p.M + S::BM - 1) / S::BM) * (p.N / S::BN);
  const unsigned grid = (unsigned)(((tiles + 7) / 8) * 8);
  constexpr size_t smem = S::SMEM;
  hipLaunchKernelGGL((gemm_wide_kernel<AM, EP, S>), dim3(grid), dim3(S::NT), smem, st, p);
  return hipGetLastError();
}

template <int AM, int EP>
static hipError_t launch_wide_bm(int bm, const GemmP& p, hipStream_t st) {
  return bm == 256 ? launch_wide_t<AM, EP, Wide256>(p, st) : launch_wide_t<AM, EP, Wide128>(p, st);
}

hipError_t launch_gemm_wide(int amode, int epi, int bm, const GemmP& p, hipStream_t st) {
  if (amode == A_ACT && epi == EP_STORE) return launch_wide_bm<A_ACT, EP_STORE>(bm, p, st);
  if (amode == A_ACT && epi == EP_RESID) return launch_wide_bm<A_ACT, EP_RESID>(bm, p, st);
  if (amode == A_NORM && epi == EP_STORE) return launch_wide_bm<A_NORM, EP_STORE>(bm, p, st);
  if (amode == A_NORM && epi == EP_GELU) return launch_wide_bm<A_NORM, EP_GELU>(bm, p, st);
  if (amode == A_NORM && epi == EP_QKV) return launch_wide_bm<A_NORM, EP_QKV>(bm, p, st);
  return hipErrorInvalidValue;
}

template <int AM, int EP>
static hipError_t raise_wide() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_wide_kernel<AM, EP, Wide256>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)Wide256::SMEM);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_wide_kernel<AM, EP, Wide128>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)Wide128::SMEM);
}

// More than 64 KB of dynamic LDS needs a one-time opt-in per kernel, outside any stream capture.
hipError_t prepare_gemm_wide() {
  hipError_t e;
  if ((e = raise_wide<A_ACT, EP_STORE>()) != hipSuccess) return e;
  if ((e = raise_wide<A_ACT, EP_RESID>()) != hipSuccess) return e;
  if ((e = raise_wide<A_NORM, EP_STORE>()) != hipSuccess) return e;
  if ((e = raise_wide<A_NORM, EP_GELU>()) != hipSuccess) return e;
  return raise_wide<A_NORM, EP_QKV>();
}

}  // namespace tsd
