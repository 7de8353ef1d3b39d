// Counter-based random numbers of the method: Philox4x32-10 words, the lattice uniform of the acceptance test
// and the Box-Muller normals of the sampled variants.  Shared by the kernels that draw (acceptance, proposal
// sampling, the one-launch draft) so that every path produces the same bits from the same counter.
#pragma once
#include <hip/hip_runtime.h>

namespace tsd {

// Philox4x32-10 (Salmon et al., SC'11): counter (c0..c3), key (k0, k1) -> four output words.
__device__ __forceinline__ void philox4(unsigned c0, unsigned c1, unsigned c2, unsigned c3, unsigned k0, unsigned k1,
                                        unsigned (&w)[4]) {
  const unsigned M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    unsigned hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    unsigned hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    unsigned n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0;
    c1 = lo1;
    c2 = n2;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  w[0] = c0;
  w[1] = c1;
  w[2] = c2;
  w[3] = c3;
}
__device__ __forceinline__ unsigned philox_word0(unsigned c0, unsigned c1, unsigned c2, unsigned c3, unsigned k0,
                                                 unsigned k1) {
  unsigned w[4];
  philox4(c0, c1, c2, c3, k0, k1, w);
  return w[0];
}
// 23-bit mid-point lattice uniform of a Philox word: exact in fp32, strictly inside (0, 1).
__device__ __forceinline__ float word_uniform(unsigned w) { return ((float)(w >> 9) + 0.5f) * 1.1920928955078125e-07f; }

// Standard normal draw for element e of the patch of (series b, round r, position i) in `stream`
// (1 = proposals, 2 = fallback / bonus patch; Sec. "Fallback Correction and Sampled Variants"):
// Philox block (b, r, i, stream * 2^16 + e / 4) gives uniforms u0..u3 and the Box-Muller pairs
// sqrt(-2 ln u0) (cos, sin)(2 pi u1), sqrt(-2 ln u2) (cos, sin)(2 pi u3); element e takes
// number e % 4.  sincospi keeps the angle exact (2 u is representable).
constexpr unsigned kStreamProposal = 1u, kStreamFallback = 2u;
__device__ __forceinline__ float normal_draw(unsigned b, unsigned r, unsigned i, unsigned stream, int e, unsigned k0,
                                             unsigned k1) {
  unsigned w[4];
  philox4(b, r, i, (stream << 16) + (unsigned)(e >> 2), k0, k1, w);
  const int pair = (e >> 1) & 1;
  const float rad = sqrtf(-2.0f * logf(word_uniform(w[2 * pair])));
  float sn, cs;
  sincospif(2.0f * word_uniform(w[2 * pair + 1]), &sn, &cs);
  return rad * ((e & 1) ? sn : cs);
}

}  // namespace tsd
