// Device-side building blocks for the gfx950 kernels: counter-based random words, the
// binary32 Gaussian transform, bf16 packing, tanh and wavefront reductions.
//
// The whole library is compiled with floating-point contraction off; every fused
// multiply-add below is explicit, so the bit-defined sequences (Gaussian transform,
// perturbation, reset) round exactly as written.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace es {

struct Words4 { uint32_t x, y, z, w; };

// Philox4x32 with 10 rounds (Salmon et al., SC'11).  Counter (c0..c3), key (k0,k1).
__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;      // one 32x32->64 multiply each
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Words4{c0, c1, c2, c3};
}

// Two 32-bit words -> two standard normal variates (cosine branch, sine branch).
// Box-Muller with u1 = k1 2^-24, k1 = (xa >> 8) + 1, angle = 2 pi (xb >> 8) 2^-24.
//   -ln u1 = n ln 2 - ln m with u1 = m 2^-n, m in (sqrt(1/2), sqrt(2)],
//   ln m = 2 atanh(s), s = (m - 1)/(m + 1), odd series through s^11;
//   sine / cosine by Taylor polynomials on [0, pi/4] and octant symmetry.
// Every operation is an IEEE binary32 operation in this order (division and square root
// correctly rounded), so the result is bit-reproducible on any conforming machine.
__device__ __forceinline__ void gauss_pair(uint32_t xa, uint32_t xb, float& zc, float& zs) {
  const uint32_t k1 = (xa >> 8) + 1u;
  const uint32_t k2 = xb >> 8;
  const uint32_t fb = __float_as_uint((float)k1);
  int e = (int)(fb >> 23) - 127;
  float m = __uint_as_float((fb & 0x007FFFFFu) | 0x3F800000u);
  if (m > 1.41421354f) { m = m * 0.5f; e += 1; }
  const int n = 24 - e;
  const float s = (m - 1.0f) / (m + 1.0f);          // correctly rounded division
  const float t = s * s;
  float p = 0x1.745d18p-4f;                    // 1/11
  p = __fmaf_rn(t, p, 0x1.c71c72p-4f);         // 1/9
  p = __fmaf_rn(t, p, 0x1.24924ap-3f);         // 1/7
  p = __fmaf_rn(t, p, 0x1.99999ap-3f);         // 1/5
  p = __fmaf_rn(t, p, 0x1.555556p-2f);         // 1/3
  p = __fmaf_rn(t, p, 1.0f);
  float lnm = s * p;
  lnm = lnm + lnm;
  const float nlu = __fmaf_rn((float)n, 0.693147182f, -lnm);
  const float rad = __builtin_sqrtf(nlu + nlu);    // correctly rounded (not the native approximation)

  const uint32_t oct = k2 >> 21;
  uint32_t f = k2 & 0x1FFFFFu;
  if (oct & 1u) f = 0x200000u - f;
  const float x = ((float)f * 0.785398185f) * 0x1p-21f;
  const float y = x * x;
  float sp = 0x1.71de3ap-19f;                  //  1/362880
  sp = __fmaf_rn(y, sp, -0x1.a01a02p-13f);     // -1/5040
  sp = __fmaf_rn(y, sp, 0x1.111112p-7f);       //  1/120
  sp = __fmaf_rn(y, sp, -0x1.555556p-3f);      // -1/6
  sp = __fmaf_rn(y, sp, 1.0f);
  sp = x * sp;
  float cp = -0x1.27e4fcp-22f;                 // -1/3628800
  cp = __fmaf_rn(y, cp, 0x1.a01a02p-16f);      //  1/40320
  cp = __fmaf_rn(y, cp, -0x1.6c16c2p-10f);     // -1/720
  cp = __fmaf_rn(y, cp, 0x1.555556p-5f);       //  1/24
  cp = __fmaf_rn(y, cp, -0.5f);
  cp = __fmaf_rn(y, cp, 1.0f);

  // octant -> (cos, sin): 0 (c,s) 1 (s,c) 2 (-s,c) 3 (-c,s) 4 (-c,-s) 5 (-s,-c) 6 (s,-c) 7 (c,-s)
  const bool swap = ((oct + 1u) & 2u) != 0u;           // octants 1,2,5,6
  float c = swap ? sp : cp;
  float sn = swap ? cp : sp;
  const bool negc = ((oct + 2u) & 4u) != 0u;           // octants 2,3,4,5
  const bool negs = (oct & 4u) != 0u;                  // octants 4,5,6,7
  c = negc ? -c : c;
  sn = negs ? -sn : sn;
  zc = rad * c;
  zs = rad * sn;
}

// binary32 -> bf16 bit pattern, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t bf16_bits(float x) {
  uint32_t b = __float_as_uint(x);
  b += 0x7FFFu + ((b >> 16) & 1u);
  return b >> 16;
}
__device__ __forceinline__ float bf16_round(float x) { return __uint_as_float(bf16_bits(x) << 16); }
__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// Noise values recomputed from the counter stream instead of being read back (paper Sec. 5.1:
// perturbations generated on the fly; nothing is stored when the caller asks for that).
// Columns d0..d0+3 (d0 a multiple of 4) of noise row `row`: one Philox block, two transforms.
// `round` reproduces the value a bf16-stored matrix would hold.
__device__ __forceinline__ void noise_regen4(uint32_t row, uint32_t d0, uint32_t gen, uint32_t k0, uint32_t k1,
                                             bool round, float (&z)[4]) {
  const Words4 w = philox4x32_10(d0 >> 2, row, gen, 1u, k0, k1);     // stream 1 = noise
  gauss_pair(w.x, w.y, z[0], z[1]);
  gauss_pair(w.z, w.w, z[2], z[3]);
  if (round) {
#pragma unroll
    for (int k = 0; k < 4; ++k) z[k] = bf16_round(z[k]);
  }
}
// A single column (one transform; used where a thread's columns are not aligned groups of four).
__device__ __forceinline__ float noise_regen1(uint32_t row, uint32_t d, uint32_t gen, uint32_t k0, uint32_t k1, bool round) {
  const Words4 w = philox4x32_10(d >> 2, row, gen, 1u, k0, k1);
  const uint32_t xa = (d & 2u) ? w.z : w.x, xb = (d & 2u) ? w.w : w.y;
  float za, zb;
  gauss_pair(xa, xb, za, zb);
  const float z = (d & 1u) ? zb : za;
  return round ? bf16_round(z) : z;
}
// Noise element (row, d) under any of the four storage modes of es_config.noise_dtype.
__device__ __forceinline__ float noise_value(uint32_t mode, const void* base, uint32_t ld, uint32_t row, uint32_t d,
                                             uint32_t gen, uint32_t k0, uint32_t k1) {
  if (mode >= 2u) return noise_regen1(row, d, gen, k0, k1, mode == 3u);
  if (mode == 1u) return bf16_to_f32(static_cast<const uint16_t*>(base)[(size_t)row * ld + d]);
  return static_cast<const float*>(base)[(size_t)row * ld + d];
}

// With a shared noise table, row `row` starts at base + offs[row] elements; returns that row's base
// (to be indexed as row 0) for the stored element type of `mode` (0 binary32, 1 bf16).
__device__ __forceinline__ const void* table_row_base(uint32_t mode, const void* base, const uint32_t* offs, uint32_t row) {
  const uint32_t o = offs[row];
  return mode == 1u ? static_cast<const void*>(static_cast<const uint16_t*>(base) + o)
                    : static_cast<const void*>(static_cast<const float*>(base) + o);
}

// Initial state element k of environment copy e: uniform on [-0.1, 0.1).
__device__ __forceinline__ float reset_value(uint32_t k, uint32_t e, uint32_t gen, uint32_t k0, uint32_t k1) {
  const Words4 w = philox4x32_10(k >> 2, e, gen, 2u, k0, k1);
  const uint32_t q = k & 3u;
  const uint32_t word = q == 0 ? w.x : q == 1 ? w.y : q == 2 ? w.z : w.w;
  const float u = (float)(word >> 8) * 0x1p-24f;
  return __fmaf_rn(u, 0.2f, -0.1f);
}

// tanh with absolute error of a few 1e-7: odd series near zero, 1 - 2/(e^{2|x|} + 1) elsewhere.
__device__ __forceinline__ float tanh_accurate(float x) {
  const float ax = fabsf(x);
  const float x2 = x * x;
  float p = -0x1.226e36p-7f;                   // -1382/155925
  p = __fmaf_rn(x2, p, 0x1.664f48p-6f);        //  62/2835
  p = __fmaf_rn(x2, p, -0x1.ba1ba2p-5f);       // -17/315
  p = __fmaf_rn(x2, p, 0x1.111112p-3f);        //  2/15
  p = __fmaf_rn(x2, p, -0x1.555556p-2f);       // -1/3
  const float small = __fmaf_rn(x * x2, p, x);
  const float ex = __expf(ax + ax);
  const float big = copysignf(1.0f - __fdividef(2.0f, ex + 1.0f), x);
  return ax < 0.3f ? small : big;
}

// tanh as 1 - 2/(2^{c x} + 1), two transcendental issues: absolute error ~1e-7 everywhere (relative
// ~1e-6 for |x| > 1e-2; near zero the result has the absolute accuracy of 1 - (1 - 2x), which is
// what the sums it feeds need).  Used by the register-resident kernels, binary32 and bf16.
__device__ __forceinline__ float tanh_fast(float x) {
  const float ex = __builtin_amdgcn_exp2f(x * 2.88539008f);     // 2 log2(e)
  const float r = __builtin_amdgcn_rcpf(ex + 1.0f);
  return __fmaf_rn(-2.0f, r, 1.0f);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

}  // namespace es
