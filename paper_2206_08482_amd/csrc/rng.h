// Device-side counter-based random numbers: Philox4x32-10 (Salmon et al., SC'11) and the
// bit-reproducible Box-Muller map used for all Gaussian draws of the hot path.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gmi {

enum : uint32_t { kStreamAction = 0, kStreamEnv = 1, kStreamDone = 2, kStreamReset = 3, kStreamShuffle = 4 };

struct Words4 { uint32_t w[4]; };

// counter = (c0,c1,c2,c3), key = (k0,k1); ten rounds, key advanced by the Weyl constants.
__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // one 32 x 32 -> 64 bit multiply per product (integer multiplies run at a quarter of the vector rate, and the
    // separate high / low forms take one such instruction each)
    const uint64_t p0 = (uint64_t)M0 * c0, p1 = (uint64_t)M1 * c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  Words4 o;
  o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
  return o;
}

// Two words -> two standard normals.  Every floating-point step is one correctly rounded
// add / multiply / divide / sqrt in the order written: contraction into FMA is switched off so that
// a CPU implementation of the same recipe reproduces the bits.
//   u1 = (2 (wa >> 9) + 1) / 2^24 written as m * 2^e, m folded to [sqrt(1/2), sqrt(2));
//   ln m = 2 atanh((m-1)/(m+1)), 6-term series; ln u1 = (e-24) ln2 + ln m, ln2 in two words;
//   r = sqrt(-2 ln u1);  quadrant = wb >> 30; x = (pi/2) (2 ((wb>>7) & 0x7FFFFF) + 1) / 2^24;
//   sin x / cos x by Taylor polynomials of degree 13 / 14, rotated by the quadrant.
__device__ __forceinline__ void normal_pair(uint32_t wa, uint32_t wb, float& z0, float& z1) {
#pragma clang fp contract(off)
  const uint32_t j = ((wa >> 9) << 1) | 1u;
  const float fj = (float)j;
  const uint32_t bits = __float_as_uint(fj);
  int e = (int)(bits >> 23) - 127;
  float m = __uint_as_float((bits & 0x7FFFFFu) | 0x3F800000u);
  if (m > 0x1.6a09e6p+0f) { m = m * 0.5f; e += 1; }
  const float t = __fdiv_rn(m - 1.0f, m + 1.0f);
  const float t2 = t * t;
  float p = 0x1.745d18p-4f;
  p = p * t2 + 0x1.c71c72p-4f;
  p = p * t2 + 0x1.24924ap-3f;
  p = p * t2 + 0x1.99999ap-3f;
  p = p * t2 + 0x1.555556p-2f;
  p = p * t2 + 1.0f;
  const float q = t * p;
  const float lnm = q + q;
  const float k = (float)(e - 24);
  const float lnu = k * 0x1.62e4p-1f + (k * 0x1.7f7d1cp-20f + lnm);
  const float r = __builtin_sqrtf(lnu * -2.0f);  // correctly rounded (the _rn intrinsic is not)

  const uint32_t quad = wb >> 30;
  const uint32_t jf = (((wb >> 7) & 0x7FFFFFu) << 1) | 1u;
  const float f = (float)jf * 0x1p-24f;
  const float x = f * 0x1.921fb6p+0f;
  const float x2 = x * x;
  float ps = 0x1.612462p-33f;
  ps = ps * x2 + -0x1.ae6456p-26f;
  ps = ps * x2 + 0x1.71de3ap-19f;
  ps = ps * x2 + -0x1.a01a02p-13f;
  ps = ps * x2 + 0x1.111112p-7f;
  ps = ps * x2 + -0x1.555556p-3f;
  const float s = x * (ps * x2 + 1.0f);
  float pc = -0x1.93974ap-37f;
  pc = pc * x2 + 0x1.1eed8ep-29f;
  pc = pc * x2 + -0x1.27e4fcp-22f;
  pc = pc * x2 + 0x1.a01a02p-16f;
  pc = pc * x2 + -0x1.6c16c2p-10f;
  pc = pc * x2 + 0x1.555556p-5f;
  pc = pc * x2 + -0x1p-1f;
  const float c = pc * x2 + 1.0f;
  const float ct = quad == 0 ? c : (quad == 1 ? -s : (quad == 2 ? -c : s));
  const float st = quad == 0 ? s : (quad == 1 ? c : (quad == 2 ? -s : -c));
  z0 = r * ct;
  z1 = r * st;
}

// Four normals of one block: elements 4*block .. 4*block+3 of env `env` at (stream, step).
__device__ __forceinline__ void normal_block(uint32_t env, uint32_t step, uint32_t stream,
                                             uint32_t block, uint32_t k0, uint32_t k1, float z[4]) {
  const Words4 w = philox4x32_10(env, step, stream, block, k0, k1);
  normal_pair(w.w[0], w.w[1], z[0], z[1]);
  normal_pair(w.w[2], w.w[3], z[2], z[3]);
}

// Alternating unbalanced Feistel network on `bits` bits with cycle walking: a bijection of [0,n).
// Round function = word 0 of Philox(counter = (R, iteration, 4, epoch*256 + round)).
__device__ __forceinline__ uint32_t feistel_perm(uint32_t i, uint32_t n, int bits, uint32_t iteration,
                                                 uint32_t epoch, uint32_t k0, uint32_t k1) {
  if (n <= 1) return 0;
  uint32_t y = i;
  do {
    int wl = bits / 2, wr = bits - bits / 2;
#pragma unroll 1
    for (int r = 0; r < 6; ++r) {
      const uint32_t left = y >> wr;
      const uint32_t right = y & ((1u << wr) - 1u);
      const Words4 f = philox4x32_10(right, iteration, kStreamShuffle, (epoch << 8) + (uint32_t)r, k0, k1);
      y = (right << wl) | (left ^ (f.w[0] & ((1u << wl) - 1u)));
      const int tmp = wl; wl = wr; wr = tmp;
    }
  } while (y >= n);
  return y;
}

}  // namespace gmi
