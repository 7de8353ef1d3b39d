// Fused GEMM family: C[M,N] = A[M,K] * Wt[N,K]^T with fp32 accumulation.
//
// One kernel template covers every dense contraction of the transformer pass (patch embedding,
// QKV, attention output, FFN up/down, output head).  What varies is where the A rows come from
// (AMode) and what happens to the product (Epi); the main loop is the same:
//   global -> registers -> LDS (double buffered) -> MFMA 32x32x16 bf16 (or fp32 FMAs) -> LDS -> epilogue.
// RMSNorm is never materialised: with the gain folded into the weights at load time,
//   RMSNorm(x) W = rsqrt(mean(x^2) + eps) * (x W'),
// so the kernel accumulates the row's sum of squares while it streams the row through and
// scales the product's row in the epilogue.
#include <type_traits>

#include "tsd_internal.h"
#include "gemm_epilogue.h"

namespace tsd {

template <typename T, int AM, int EP, int BM, int BN, int BK, int G = 1>
__global__ __launch_bounds__(256 * G) void gemm_kernel(const GemmP p) {
  constexpr int NT = 256 * G;
  constexpr bool kBf = !std::is_same<T, float>::value;
  constexpr bool kNorm = (AM == A_NORM || AM == A_NORM32);  // RMSNorm fused as a row scale
  // fp32 A rows in bf16 mode (patches, and the residual feeding the output head) are split into
  // hi + lo bf16 parts, each multiplied by the same B fragment: the small GEMMs at the two ends of
  // the model then carry ~16 mantissa bits of their input instead of 8.
  constexpr bool kSplit = kBf && (AM == A_TOK || AM == A_NORM32);
  constexpr int NAS = kSplit ? 2 : 1;  // A tiles kept in LDS per buffer
  constexpr int LDT = BK + (kBf ? 8 : 1);  // padded LDS row, in elements
  constexpr int LDC = BN + 4;
  static_assert(G == 1 || (kBf && BM == 64 && !kNorm), "split workgroups: bf16, 64-row tiles, no fused norm");
  constexpr int GROUP_ELEMS = 2 * (NAS * BM + BN) * LDT;  // one group's pair of tile buffers
  constexpr int AB_BYTES = G * GROUP_ELEMS * (int)sizeof(T);
  constexpr int C_BYTES = G * 64 * LDC * 4;
  constexpr int SMEM = AB_BYTES > C_BYTES ? AB_BYTES : C_BYTES;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // SMEM + BM * 12 bytes
  const int tid = threadIdx.x;
  const int grp = G > 1 ? tid >> 8 : 0, gt = tid & 255;  // group of 4 wavefronts, lane index inside it
  T* As = reinterpret_cast<T*>(smem) + grp * GROUP_ELEMS;  // [2][NAS][BM][LDT] per group
  T* Bs = As + 2 * NAS * BM * LDT;     // [2][BN][LDT]
  float* Cs = reinterpret_cast<float*>(smem);  // [G][64][LDC], reuses the tile buffers
  float* row_scale = reinterpret_cast<float*>(smem + SMEM);  // [BM]
  int* row_pos = reinterpret_cast<int*>(smem + SMEM + BM * 4);   // [BM] EP_QKV: absolute position of the row's token
  int* row_page = row_pos + BM;                                   // [BM] EP_QKV: its physical KV page

  // rows of the product: fixed at launch, or capped by a device-side series count when the launch
  // is replayed from a graph while series finish (workgroups past the cap leave at once)
  const int M = p.n_dev ? min(p.M, *p.n_dev * p.nq) : p.M;
  const int N = p.N, K = p.K;
  // Tile order.  Workgroups go round-robin to the 8 XCDs (each with its own L2), so workgroup
  // w lands on XCD w % 8.  Give every XCD one contiguous run of the tile list, and order the
  // list in groups of 8 tile columns walked row by row: the ~32 tiles an XCD runs at a time then
  // form a 4 x 8 rectangle that shares 4 row panels and 8 column panels through that L2.
  const int tiles_m = p.tile_map ? p.n_mtiles : (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const int n_tiles = tiles_m * tiles_n;
  const int per_xcd = (n_tiles + 7) >> 3;
  // (a replayed launch may be larger than the tile list: workgroups past an XCD's run must not
  // wander into the next XCD's)
  if ((int)(blockIdx.x >> 3) >= per_xcd) return;
  const int lin = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (lin >= n_tiles) return;
  constexpr int GW = 8;
  const int gc = lin / (GW * tiles_m), rem = lin - gc * (GW * tiles_m);
  const int gw = min(GW, tiles_n - gc * GW);
  const int tm = rem / gw, tn = gc * GW + rem - tm * gw;
  int m0 = tm * BM, m_lim = M;
  const int n0 = tn * BN;
  const T* Wbase = reinterpret_cast<const T*>(p.W);
  if (p.tile_map) {  // routed FFN: this row tile belongs to one expert's run of slots
    const int4 tmap = reinterpret_cast<const int4*>(p.tile_map)[tm];
    if (tmap.x < 0) return;
    m0 = tmap.y;
    m_lim = tmap.z;
    Wbase += (long)tmap.x * p.w_stride;
  }

  // ---- A loader set-up ----------------------------------------------------------------------
  constexpr bool kASrcF32 = (AM == A_TOK) || (AM == A_NORM32) || !kBf;   // source rows are fp32 (bf16 mode reads the bf16 shadow of the residual)
  constexpr int CHA = kASrcF32 ? 4 : 8;              // elements per 16-byte chunk
  constexpr int CPRA = BK / CHA;                     // chunks per tile row
  constexpr int NA = BM * CPRA / 256;
  static_assert(NA >= 1, "tile too small for 256 threads");
  const char* arow[NA];
  int a_r[NA], a_kc[NA];
  float ss[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    int id = gt + i * 256;
    a_r[i] = id / CPRA;
    a_kc[i] = id % CPRA;
    ss[i] = 0.f;
    // rows past M are clamped to the last row: their products land in rows that are never stored
    int gm = min(m0 + a_r[i], m_lim - 1);
    if (p.src_row) gm = p.src_row[gm];
    arow[i] = nullptr;
    {
      if constexpr (AM == A_TOK) {
        int b = gm / p.nq, t = gm % p.nq;
        if (p.act) b = p.act[b];
        const float* src = (t < p.n0) ? p.src0 + (long)b * p.stride0 + (long)t * K
                                      : p.src1 + (long)b * p.stride1 + (long)(t - p.n0) * K;
        arow[i] = reinterpret_cast<const char*>(src);
      } else if constexpr (kASrcF32) {
        arow[i] = reinterpret_cast<const char*>(reinterpret_cast<const float*>(p.A) + (long)gm * K);
      } else {
        arow[i] = reinterpret_cast<const char*>(reinterpret_cast<const T*>(p.A) + (long)gm * K);
      }
    }
  }
  // ---- B loader set-up ----------------------------------------------------------------------
  constexpr int CHB = kBf ? 8 : 4;
  constexpr int CPRB = BK / CHB;
  constexpr int NB = BN * CPRB / 256;
  static_assert(NB >= 1, "tile too small for 256 threads");
  const char* brow[NB];
  int b_r[NB], b_kc[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    int id = gt + i * 256;
    b_r[i] = id / CPRB;
    b_kc[i] = id % CPRB;
    int gn = min(n0 + b_r[i], N - 1);  // clamped like the rows of A
    brow[i] = reinterpret_cast<const char*>(Wbase + (long)gn * K);
  }

  // Two tiles are kept in flight in two register sets that alternate (no copies between them:
  // a copy would wait for the younger load), so the HBM latency of one tile overlaps the MFMA
  // work and LDS traffic of two others.
  uint4 ra0[NA], rb0[NB], ra1[NA], rb1[NB];
  // Loads are unconditional (addresses clamped into range) so that the number of loads in flight
  // is the same on every path and the compiler can wait for exactly the older tile; the K tail
  // is zeroed when the registers are written to LDS.
  auto load_global = [&](int kt, uint4* xa, uint4* xb) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      const int k = min(kt * BK + a_kc[i] * CHA, K - CHA);
      xa[i] = *reinterpret_cast<const uint4*>(arow[i] + (long)k * (kASrcF32 ? 4 : 2));
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int k = min(kt * BK + b_kc[i] * CHB, K - CHB);
      xb[i] = *reinterpret_cast<const uint4*>(brow[i] + (long)k * (int)sizeof(T));
    }
  };
  auto store_lds = [&](int kt, int buf, uint4* ra, uint4* rb) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      T* dst = As + ((buf * NAS) * BM + a_r[i]) * LDT + a_kc[i] * CHA;
      if (kt * BK + a_kc[i] * CHA >= K) ra[i] = make_uint4(0, 0, 0, 0);
      if constexpr (kASrcF32) {
        float4 f = *reinterpret_cast<float4*>(&ra[i]);
        if constexpr (kNorm) ss[i] += f.x * f.x + f.y * f.y + f.z * f.z + f.w * f.w;
        if constexpr (kSplit) {
          const float4 hi = make_float4((float)(bf16)f.x, (float)(bf16)f.y, (float)(bf16)f.z, (float)(bf16)f.w);
          store4<bf16>(reinterpret_cast<bf16*>(dst), hi);
          store4<bf16>(reinterpret_cast<bf16*>(dst + BM * LDT), make_float4(f.x - hi.x, f.y - hi.y, f.z - hi.z, f.w - hi.w));
        } else if constexpr (kBf) {
          store4<bf16>(reinterpret_cast<bf16*>(dst), f);
        } else {
          dst[0] = f.x;
          dst[1] = f.y;
          dst[2] = f.z;
          dst[3] = f.w;
        }
      } else {
        if constexpr (kNorm) {
          // a chain of packed bf16 dot products per 16-byte chunk position: the wide-tile kernel (gemm_wide.hip)
          // forms the same chains from its MFMA fragments, so either kernel gives a row the same scale
          typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
          const bf16x8 v = *reinterpret_cast<const bf16x8*>(&ra[i]);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const bf16x2 pr = {v[2 * e], v[2 * e + 1]};
            ss[i] = __builtin_amdgcn_fdot2_f32_bf16(pr, pr, ss[i], false);
          }
        }
        *reinterpret_cast<uint4*>(dst) = ra[i];
      }
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      T* dst = Bs + (buf * BN + b_r[i]) * LDT + b_kc[i] * CHB;
      if (kt * BK + b_kc[i] * CHB >= K) rb[i] = make_uint4(0, 0, 0, 0);
      if constexpr (kBf) {
        *reinterpret_cast<uint4*>(dst) = rb[i];
      } else {
        float4 f = *reinterpret_cast<float4*>(&rb[i]);
        dst[0] = f.x;
        dst[1] = f.y;
        dst[2] = f.z;
        dst[3] = f.w;
      }
    }
  };

  // ---- accumulators -------------------------------------------------------------------------
  const int lane = tid & 63, wid = (tid >> 6) & 3;
  const int wm = wid >> 1, wn = wid & 1;
  constexpr int WTM = BM / 2, WTN = BN / 2;            // wave tile (bf16 path)
  constexpr int TM = kBf ? WTM / 32 : 1, TN = kBf ? WTN / 32 : 1;
  f32x16 acc[TM][TN];
  float accf[4][4];
  if constexpr (kBf) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  } else {
    static_assert(kBf || (BM == 64 && BN == 64), "fp32 path uses 64x64 tiles");
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) accf[i][j] = 0.f;
  }
  const int ty = gt >> 4, tx = gt & 15;  // fp32 path: 4x4 micro-tile at (ty*4, tx*4)
  // Long contractions of activations (K >= kQuarterK) are summed in four runs of ceil(nk / 4) k-steps, each from
  // zero, the runs added in order: the order the split workgroups (G = 4) produce by construction.  Every bf16
  // kernel that can take such a product (this one, the split one, the wide-tile ones) keeps to it, so which of them
  // the launcher picks, which follows the rows still active, changes no bit.
  constexpr bool kQuarters = kBf && AM == A_ACT && G == 1 && BM == 64;
  f32x16 tot[kQuarters ? TM : 1][kQuarters ? TN : 1];
  const bool quarters = kQuarters && p.K >= kQuarterK;
  auto fold = [&](int done) {  // `done` k-steps are in acc: at a run's end move them into the running sum
    if constexpr (kQuarters) {
      const int nk_all = (p.K + BK - 1) / BK, run = (nk_all + 3) / 4;
      if (!quarters || done % run != 0 || done >= nk_all) return;
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

  // ---- main loop ----------------------------------------------------------------------------
  auto compute = [&](int buf) {
    const T* at = As + buf * NAS * BM * LDT;
    const T* bt = Bs + buf * BN * LDT;
    if constexpr (kBf) {
#pragma unroll
      for (int k16 = 0; k16 < BK / 16; ++k16) {
        bf16x8 af[NAS][TM], bfr[TN];
        const int ko = k16 * 16 + (lane >> 5) * 8;
#pragma unroll
        for (int h = 0; h < NAS; ++h)
#pragma unroll
          for (int i = 0; i < TM; ++i)
            af[h][i] = *reinterpret_cast<const bf16x8*>(at + (h * BM + wm * WTM + i * 32 + (lane & 31)) * LDT + ko);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          bfr[j] = *reinterpret_cast<const bf16x8*>(bt + (wn * WTN + j * 32 + (lane & 31)) * LDT + ko);
#pragma unroll
        for (int h = NAS - 1; h >= 0; --h)  // low part first, then the high part
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[h][i], bfr[j], acc[i][j], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int k = 0; k < BK; ++k) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = at[(ty * 4 + i) * LDT + k];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = bt[(tx * 4 + j) * LDT + k];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) accf[i][j] = fmaf(a[i], b[j], accf[i][j]);
      }
    }
  };
  const int nk = (K + BK - 1) / BK;
  // Split workgroup: group g walks the g-th run of ceil(nk / G) k-steps with its own tile buffers and
  // accumulators (steps past K multiply zeros, so every group meets the same barriers); the epilogue
  // adds the G partial products in group order.
  const int nkl = G > 1 ? (nk + G - 1) / G : nk;  // k-steps this group walks
  const int kt0 = G > 1 ? grp * nkl : 0;
  load_global(kt0, ra0, rb0);
  load_global(kt0 + 1, ra1, rb1);
  // Epilogue inputs that do not depend on the product are requested now, so their latency hides
  // behind the main loop: the KV position/page of each row (QKV), the old residual values (RESID).
  int my_pos = 0, my_page = 0;
  if constexpr (EP == EP_QKV) {
    if (tid < BM) {
      const int gm = min(m0 + tid, m_lim - 1);
      const int bl = gm / p.nq, t = gm - bl * p.nq, b = p.act ? p.act[bl] : p.s0 + bl;
      my_pos = (p.base_pos ? p.base_pos[b] : 0) + p.pos_off + t;
      my_page = p.page_table[(long)b * p.pt_stride + (my_pos >> p.pt_shift)];
    }
  }
  constexpr bool kPrefetchC = (EP == EP_RESID) && BM == 64;
  constexpr int NPRE = kPrefetchC ? 64 * (BN / 4) / NT : 1;
  float4 oldc[NPRE];
  if constexpr (kPrefetchC) {
#pragma unroll
    for (int it = 0; it < NPRE; ++it) {
      const int g = tid + it * NT;
      const int gm = min(m0 + g / (BN / 4), m_lim - 1), gn = min(n0 + (g % (BN / 4)) * 4, N - 4);
      oldc[it] = *reinterpret_cast<const float4*>(p.Cf + (long)gm * N + gn);
    }
  }
  store_lds(kt0, 0, ra0, rb0);
  __syncthreads();
  int kt = 0;  // k-steps done, counted from kt0
  // Steady state, two tiles per trip and no branches inside: tile kt sits in LDS buffer 0, register
  // set 1 holds tile kt+1 (in flight), set 0 is free.  The scheduling barriers keep each prefetch
  // ahead of the MFMA work it is meant to overlap.
  for (; kt + 2 < nkl; kt += 2) {
    load_global(kt0 + kt + 2, ra0, rb0);
    __builtin_amdgcn_sched_barrier(0);
    compute(0);
    fold(kt + 1);
    store_lds(kt0 + kt + 1, 1, ra1, rb1);
    __syncthreads();
    load_global(kt0 + kt + 3, ra1, rb1);
    __builtin_amdgcn_sched_barrier(0);
    compute(1);
    fold(kt + 2);
    store_lds(kt0 + kt + 2, 0, ra0, rb0);
    __syncthreads();
  }
  compute(0);
  fold(kt + 1);
  if (kt + 1 < nkl) {
    store_lds(kt0 + kt + 1, 1, ra1, rb1);
    __syncthreads();
    compute(1);
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

  if constexpr (EP == EP_QKV) {
    if (tid < BM) {
      row_pos[tid] = my_pos;
      row_page[tid] = my_page;
    }
  }
  // ---- RMSNorm row scale --------------------------------------------------------------------
  if constexpr (kNorm) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      float s = ss[i];
#pragma unroll
      for (int o = CPRA / 2; o >= 1; o >>= 1) s += __shfl_xor(s, o);
      if (a_kc[i] == 0) row_scale[a_r[i]] = rsqrtf(s / (float)K + kRmsEps);
    }
  }

  // ---- epilogue, 64 rows at a time through LDS ----------------------------------------------
  auto read_c1 = [&](int row, int col) {  // one element / four consecutive elements of the product
    float v = Cs[row * LDC + col];
#pragma unroll
    for (int g = 1; g < G; ++g) v += Cs[(g * 64 + row) * LDC + col];
    return v;
  };
  auto read_c4 = [&](int row, int col) {
    float4 v = *reinterpret_cast<const float4*>(Cs + row * LDC + col);
#pragma unroll
    for (int g = 1; g < G; ++g) {
      const float4 w = *reinterpret_cast<const float4*>(Cs + (g * 64 + row) * LDC + col);
      v.x += w.x;
      v.y += w.y;
      v.z += w.z;
      v.w += w.w;
    }
    return v;
  };
  for (int pass = 0; pass < BM / 64; ++pass) {
    __syncthreads();  // tile buffers (or the previous pass's Cs) are no longer read
    if constexpr (kBf) {
      // accumulator element r of a 32x32 block: row (r/4)*8 + (lane/32)*4 + r%4, column lane%32
      if (BM == 64 || wm == pass) {
        const int rbase = (BM == 64) ? wm * WTM : 0;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              int row = rbase + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
              int col = wn * WTN + j * 32 + (lane & 31);
              Cs[(grp * 64 + row) * LDC + col] = acc[i][j][r];
            }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) Cs[(ty * 4 + i) * LDC + tx * 4 + j] = accf[i][j];
    }
    __syncthreads();
    epilogue_pass<T, EP, kNorm, BN, NT, kPrefetchC>(p, read_c4, row_scale, row_pos, row_page, m0, n0, pass, m_lim, N, tid, oldc);
  }
}

template <typename T, int AM, int BM, int BN, int BK, int G = 1>
constexpr size_t gemm_smem_bytes() {
  constexpr bool kBf = !std::is_same<T, float>::value;
  constexpr int LDT = BK + (kBf ? 8 : 1);
  constexpr int nas = (kBf && (AM == A_TOK || AM == A_NORM32)) ? 2 : 1;
  constexpr size_t ab = (size_t)G * 2 * (nas * BM + BN) * LDT * sizeof(T), c = (size_t)G * 64 * (BN + 4) * 4;
  return (ab > c ? ab : c) + BM * 12;
}

template <typename T, int AM, int EP, int BM, int BN, int BK, int G = 1>
static hipError_t launch_tile(const GemmP& p, hipStream_t st) {
  constexpr size_t smem = gemm_smem_bytes<T, AM, BM, BN, BK, G>();
  const long tiles = (long)(p.tile_map ? p.n_mtiles : (p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
  const unsigned grid = (unsigned)(((tiles + 7) / 8) * 8);  // padded so that every XCD gets a full run
  hipLaunchKernelGGL((gemm_kernel<T, AM, EP, BM, BN, BK, G>), dim3(grid), dim3(256 * G), smem, st, p);
  return hipGetLastError();
}

// Row-tile size the launcher will use for an M x N product (the routed FFN builds its tile map for it).
int gemm_row_tile(int dtype, int M, int N, int force_bm) {
  if (dtype != TSD_BF16) return 64;
  if (force_bm) return force_bm;
  const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
  // 128 x 128 tiles once there are at least 1.5 of them per CU; below that the 64 x 64 tiles, four times as many,
  // keep more of the chip busy (threshold found by timing whole passes: 192 .. 1024 tried)
  return t128 >= 384 ? 128 : 64;
}

// A long contraction with too few 64 x 64 tiles to cover the chip is bound by how fast the few busy
// compute units can pull their operand panels: such a product runs with 1024-lane workgroups whose
// four groups of wavefronts each stream a quarter of K (four times the loads in flight per unit, a
// quarter of the serial k-steps).  The partial sums are added in a fixed order, so the result does
// not depend on timing; it differs in the last bits from the single-group kernel's, which is why
// the choice depends on the shape of the product alone.
static bool gemm_split(const GemmP& p) {
  const long t64 = (long)(p.tile_map ? p.n_mtiles : (p.M + 63) / 64) * ((p.N + 63) / 64);
  return p.K >= kQuarterK && t64 <= 256;
}

template <typename T, int AM, int EP>
static hipError_t launch_cfg(const GemmP& p, hipStream_t st) {
  constexpr bool kBf = !std::is_same<T, float>::value;
  if constexpr (kBf) {
    // (the 128-row register-staged tiles have no room for the running sum of a long contraction's four runs: such
    //  products of activations go to the wide-tile kernels or stay on 64-row tiles)
    const bool long_act = AM == A_ACT && p.K >= kQuarterK;
    if (long_act && p.tile_map && p.force_bm == 128) return hipErrorInvalidValue;  // (the caller builds 64-row maps for these)
    if (!long_act && gemm_row_tile(TSD_BF16, p.M, p.N, p.force_bm) == 128) return launch_tile<T, AM, EP, 128, 128, 64>(p, st);
    if constexpr (AM == A_ACT) {
      if (gemm_split(p)) return launch_tile<T, AM, EP, 64, 64, 64, 4>(p, st);
    }
    return launch_tile<T, AM, EP, 64, 64, 64>(p, st);
  } else {
    return launch_tile<T, AM, EP, 64, 64, 16>(p, st);
  }
}

template <typename T, int AM, int EP>
static hipError_t raise_cfg() {
  if constexpr (!std::is_same<T, float>::value) {
    if constexpr (AM == A_ACT) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<T, AM, EP, 64, 64, 64, 4>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_smem_bytes<T, AM, 64, 64, 64, 4>());
      if (e != hipSuccess) return e;
    }
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<T, AM, EP, 128, 128, 64>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_smem_bytes<T, AM, 128, 128, 64>());
  }
  return hipSuccess;
}

// The 128x128x64 tiles use more than 64 KB of dynamic LDS: opt in once, outside any stream capture.
hipError_t prepare_gemm(int dtype) {
  if (dtype != TSD_BF16) return hipSuccess;
  hipError_t e;
  if ((e = prepare_gemm_wide()) != hipSuccess) return e;
  if ((e = raise_cfg<bf16, A_TOK, EP_STORE>()) != hipSuccess) return e;
  if ((e = raise_cfg<bf16, A_NORM, EP_QKV>()) != hipSuccess) return e;
  if ((e = raise_cfg<bf16, A_ACT, EP_RESID>()) != hipSuccess) return e;
  if ((e = raise_cfg<bf16, A_NORM, EP_GELU>()) != hipSuccess) return e;
  if ((e = raise_cfg<bf16, A_NORM32, EP_HEAD>()) != hipSuccess) return e;
  if ((e = raise_cfg<bf16, A_ACT, EP_STORE>()) != hipSuccess) return e;
  return raise_cfg<bf16, A_NORM, EP_STORE>();
}

template <typename T>
static hipError_t launch_t(int amode, int epi, const GemmP& p, hipStream_t st) {
  if (amode == A_TOK && epi == EP_STORE) return launch_cfg<T, A_TOK, EP_STORE>(p, st);
  if (amode == A_NORM && epi == EP_QKV) return launch_cfg<T, A_NORM, EP_QKV>(p, st);
  if (amode == A_ACT && epi == EP_RESID) return launch_cfg<T, A_ACT, EP_RESID>(p, st);
  if (amode == A_NORM && epi == EP_GELU) return launch_cfg<T, A_NORM, EP_GELU>(p, st);
  if (amode == A_NORM32 && epi == EP_HEAD) return launch_cfg<T, A_NORM32, EP_HEAD>(p, st);
  if (amode == A_NORM && epi == EP_STORE) return launch_cfg<T, A_NORM, EP_STORE>(p, st);
  if (amode == A_ACT && epi == EP_STORE) return launch_cfg<T, A_ACT, EP_STORE>(p, st);
  return hipErrorInvalidValue;
}

int gemm_variant(int dtype, int amode, int epi, const GemmP& p) {
  if (p.allow_skinny && skinny_applicable(dtype, amode, epi, p)) return 16;
  if (dtype != TSD_BF16) return 64;
  if (const int bm = gemm_wide_bm(dtype, amode, epi, p)) return 2000 + bm;
  if (!(amode == A_ACT && p.K >= kQuarterK) && gemm_row_tile(TSD_BF16, p.M, p.N, p.force_bm) == 128) return 128;
  return (amode == A_ACT && gemm_split(p)) ? 464 : 64;
}

hipError_t launch_gemm(int dtype, int amode, int epi, const GemmP& p, hipStream_t st) {
  if (p.M <= 0 || p.N <= 0 || p.K <= 0) return hipErrorInvalidValue;
  if (p.allow_skinny && skinny_applicable(dtype, amode, epi, p)) return launch_gemm_skinny(amode, epi, p, st);
  if (const int bm = gemm_wide_bm(dtype, amode, epi, p)) return launch_gemm_wide(amode, epi, bm, p, st);
  return dtype == TSD_BF16 ? launch_t<bf16>(amode, epi, p, st) : launch_t<float>(amode, epi, p, st);
}

}  // namespace tsd
