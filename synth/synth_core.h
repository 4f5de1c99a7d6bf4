/* Seeded synthetic-input generator: the arithmetic core.
 *
 * This header is the single definition of the counter-based generator that
 * produces every synthetic tensor (weights, KV prefill, token ids).  It is
 * compiled twice -- by gcc for the host fill (synth_host.c) and by hipcc for the
 * device fill (synth_device.hip) -- and must give bit-identical values in both.
 * To make that hold it uses only operations that IEEE-754 fixes exactly:
 * integer arithmetic, and fp64 add/mul/div/sqrt/fma written out explicitly
 * (contraction is switched off, no libm transcendental is called).
 *
 * It contains none of the decoder's arithmetic; it only makes inputs.
 *
 * Element i of stream (seed, stream_id):
 *   pair p = i >> 1,  key = mix(mix(seed) ^ (stream_id * GOLDEN))
 *   h1 = mix(key + 2p), h2 = mix(key + 2p + 1)
 *   u1 = ((h1 >> 11) + 1) * 2^-53  in (0,1],  u2 = (h2 >> 11) * 2^-53 in [0,1)
 *   r = sqrt(-2 ln u1);  z = r cos(2 pi u2) for even i,  r sin(2 pi u2) for odd i
 * (Box-Muller).  value = (float)(sigma * z), optionally rounded to bf16 (RNE) or to an FP8 E4M3
 * byte or an FP4 E2M1 nibble (both RNE, saturating; two nibbles per byte, even element low), or to
 * block-scaled FP4: nibbles of value / 2^e with one exponent e per 32 elements of a row.
 */
#ifndef PI_SYNTH_CORE_H
#define PI_SYNTH_CORE_H

#include <stdint.h>

#ifdef __HIPCC__
#define SYNTH_FN __host__ __device__ static inline
#else
#define SYNTH_FN static inline
#endif

#ifdef __clang__
#pragma clang fp contract(off)
#else
#pragma STDC FP_CONTRACT OFF
#endif

#define SYNTH_FMA(a, b, c) __builtin_fma((a), (b), (c))
#define SYNTH_SQRT(a) __builtin_sqrt((a))

SYNTH_FN uint64_t synth_mix(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

SYNTH_FN uint64_t synth_key(uint64_t seed, uint64_t stream_id) {
  return synth_mix(synth_mix(seed) ^ (stream_id * 0x9E3779B97F4A7C15ull));
}

SYNTH_FN double synth_bits_to_double(uint64_t b) {
  union { uint64_t u; double d; } c;
  c.u = b;
  return c.d;
}

/* ln(u) for u in (0,1], u a multiple of 2^-53: exponent split + atanh series. */
SYNTH_FN double synth_log(double u) {
  union { uint64_t b; double d; } c;
  c.d = u;
  int e = (int)((c.b >> 52) & 0x7ff) - 1023;
  c.b = (c.b & 0x000fffffffffffffull) | 0x3ff0000000000000ull; /* m in [1,2) */
  double m = c.d;
  if (m > 1.4142135623730951) { m = m * 0.5; e += 1; }
  double f = m - 1.0;           /* exact */
  double s = f / (2.0 + f);
  double z = s * s;
  /* 2*atanh(s) = 2s (1 + z/3 + z^2/5 + ...), |s| <= 0.1716 */
  double p = 1.0 / 23.0;
  p = SYNTH_FMA(p, z, 1.0 / 21.0);
  p = SYNTH_FMA(p, z, 1.0 / 19.0);
  p = SYNTH_FMA(p, z, 1.0 / 17.0);
  p = SYNTH_FMA(p, z, 1.0 / 15.0);
  p = SYNTH_FMA(p, z, 1.0 / 13.0);
  p = SYNTH_FMA(p, z, 1.0 / 11.0);
  p = SYNTH_FMA(p, z, 1.0 / 9.0);
  p = SYNTH_FMA(p, z, 1.0 / 7.0);
  p = SYNTH_FMA(p, z, 1.0 / 5.0);
  p = SYNTH_FMA(p, z, 1.0 / 3.0);
  p = SYNTH_FMA(p, z, 1.0);
  double lm = 2.0 * s * p;
  return SYNTH_FMA((double)e, 0.6931471805599453, lm);
}

/* cos and sin of 2*pi*u, u in [0,1) a multiple of 2^-53: octant reduction is
 * exact (scaling by 8), then Taylor series on [-pi/4, pi/4]. */
SYNTH_FN void synth_sincos2pi(double u, double* cs, double* sn) {
  double a = u * 8.0;              /* exact */
  int o = (int)a;                  /* 0..7 */
  int j = (o + 1) >> 1;            /* 0..4 */
  double t = a - (double)(2 * j);  /* exact, in [-1,1) */
  double x = t * 0.78539816339744831; /* pi/4 * t */
  double x2 = x * x;
  double sp = 1.0 / 355687428096000.0;             /*  1/17! */
  sp = SYNTH_FMA(sp, x2, -1.0 / 1307674368000.0);  /* -1/15! */
  sp = SYNTH_FMA(sp, x2, 1.0 / 6227020800.0);      /*  1/13! */
  sp = SYNTH_FMA(sp, x2, -1.0 / 39916800.0);       /* -1/11! */
  sp = SYNTH_FMA(sp, x2, 1.0 / 362880.0);          /*  1/9!  */
  sp = SYNTH_FMA(sp, x2, -1.0 / 5040.0);           /* -1/7!  */
  sp = SYNTH_FMA(sp, x2, 1.0 / 120.0);             /*  1/5!  */
  sp = SYNTH_FMA(sp, x2, -1.0 / 6.0);              /* -1/3!  */
  sp = SYNTH_FMA(sp, x2, 1.0);
  sp = sp * x;
  double cp = 1.0 / 20922789888000.0;              /*  1/16! */
  cp = SYNTH_FMA(cp, x2, -1.0 / 87178291200.0);    /* -1/14! */
  cp = SYNTH_FMA(cp, x2, 1.0 / 479001600.0);       /*  1/12! */
  cp = SYNTH_FMA(cp, x2, -1.0 / 3628800.0);        /* -1/10! */
  cp = SYNTH_FMA(cp, x2, 1.0 / 40320.0);           /*  1/8!  */
  cp = SYNTH_FMA(cp, x2, -1.0 / 720.0);            /* -1/6!  */
  cp = SYNTH_FMA(cp, x2, 1.0 / 24.0);              /*  1/4!  */
  cp = SYNTH_FMA(cp, x2, -0.5);
  cp = SYNTH_FMA(cp, x2, 1.0);
  switch (j & 3) {
    case 0: *cs = cp;  *sn = sp;  break;
    case 1: *cs = -sp; *sn = cp;  break;
    case 2: *cs = -cp; *sn = -sp; break;
    default: *cs = sp; *sn = -cp; break;
  }
}

/* Standard-normal pair number `pair` of the stream with key `key`. */
SYNTH_FN void synth_normal_pair(uint64_t key, uint64_t pair, double* z0, double* z1) {
  uint64_t h1 = synth_mix(key + 2 * pair);
  uint64_t h2 = synth_mix(key + 2 * pair + 1);
  double u1 = (double)((h1 >> 11) + 1) * 1.1102230246251565e-16; /* 2^-53 */
  double u2 = (double)(h2 >> 11) * 1.1102230246251565e-16;
  double r = SYNTH_SQRT(-2.0 * synth_log(u1));
  double c, s;
  synth_sincos2pi(u2, &c, &s);
  *z0 = r * c;
  *z1 = r * s;
}

/* fp32 -> bf16 bits, round to nearest even (finite inputs only here). */
SYNTH_FN uint16_t synth_f32_to_bf16(float f) {
  union { float f; uint32_t u; } c;
  c.f = f;
  uint32_t u = c.u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

/* fp32 -> FP8 E4M3 byte (4 exponent bits with bias 7, 3 mantissa bits, subnormals, no infinity;
 * the OCP 8-bit format): round to nearest even, magnitudes beyond the largest finite value
 * (448) saturate to it.  Finite inputs only.  Integer arithmetic except one exact rounding of a
 * value below 8 to an integer, so host and device agree bit for bit. */
SYNTH_FN uint8_t synth_f32_to_e4m3(float f) {
  union { float f; uint32_t u; } c;
  c.f = f;
  const uint32_t sign = (c.u >> 24) & 0x80u;
  const uint32_t a = c.u & 0x7fffffffu;
  uint32_t b;
  if (a < 0x3c800000u) {             /* |f| < 2^-6: subnormal range, steps of 2^-9 */
    c.u = a;
    b = (uint32_t)__builtin_rintf(c.f * 512.0f); /* 0..8; 8 is the smallest normal, bit pattern 0x08 */
  } else {
    const uint32_t r = a + 0x7ffffu + ((a >> 20) & 1u); /* RNE at three mantissa bits */
    b = (r >> 20) - (120u << 3);     /* rebias 127 -> 7 */
    if (b > 0x7eu) b = 0x7eu;        /* 448 */
  }
  return (uint8_t)(sign | b);
}

/* fp32 -> FP4 E2M1 nibble (sign, 2 exponent bits with bias 1, 1 mantissa bit: magnitudes 0, 0.5,
 * 1, 1.5, 2, 3, 4, 6; the OCP 4-bit format): round to nearest, ties to the code with mantissa
 * bit 0, magnitudes beyond 6 saturate.  Finite inputs only; comparisons with exactly
 * representable constants, so host and device agree. */
SYNTH_FN uint8_t synth_f32_to_e2m1(float f) {
  union { float f; uint32_t u; } c;
  c.f = f;
  const uint8_t sign = (uint8_t)((c.u >> 28) & 0x8u);
  c.u &= 0x7fffffffu;
  const float a = c.f;
  const int code = (a > 0.25f) + (a >= 0.75f) + (a > 1.25f) + (a >= 1.75f) + (a > 2.5f) + (a >= 3.5f) + (a > 5.0f);
  return (uint8_t)(sign | (uint8_t)code);
}

/* One block of a block-scaled 4-bit row: `count` (even, <= 32) consecutive elements starting at the
 * even element `first` of stream `key` share a power-of-two scale 2^e, stored as the byte e + 127.
 * e = floor(log2(largest magnitude)) - 2, so the largest element lands in [4, 8) before rounding
 * (magnitudes above 6 saturate at 6); a block of zeros gets e = 0.  Each element is then rounded
 * to an FP4 E2M1 nibble of value / 2^e.  codes: count / 2 bytes, even element in the low nibble.
 * Integer exponent arithmetic and exact power-of-two scaling only: host and device agree. */
SYNTH_FN uint8_t synth_fp4_block(uint64_t key, uint64_t first, int count, double sigma, uint8_t* codes) {
  float v[32];
  uint32_t amax_bits = 0;
  for (int p = 0; p < count / 2; ++p) {
    double z0, z1;
    synth_normal_pair(key, first / 2 + (uint64_t)p, &z0, &z1);
    v[2 * p] = (float)(sigma * z0);
    v[2 * p + 1] = (float)(sigma * z1);
  }
  for (int j = 0; j < count; ++j) {
    union { float f; uint32_t u; } c;
    c.f = v[j];
    const uint32_t a = c.u & 0x7fffffffu;
    if (a > amax_bits) amax_bits = a;   /* magnitudes of finite floats order like their bit patterns */
  }
  int e = 0;
  if (amax_bits >= 0x00800000u) {       /* a normal number: its exponent field is floor(log2) + 127 */
    e = (int)(amax_bits >> 23) - 127 - 2;
    if (e < -120) e = -120;
    if (e > 120) e = 120;
  }
  union { float f; uint32_t u; } inv;
  inv.u = (uint32_t)(127 - e) << 23;    /* 2^-e */
  for (int p = 0; p < count / 2; ++p)
    codes[p] = (uint8_t)(synth_f32_to_e2m1(v[2 * p] * inv.f) | (synth_f32_to_e2m1(v[2 * p + 1] * inv.f) << 4));
  return (uint8_t)(e + 127);
}

/* Uniform integer in [0, range) for element i. */
SYNTH_FN int32_t synth_uniform_int(uint64_t key, uint64_t i, uint32_t range) {
  uint64_t h = synth_mix(key + i);
  return (int32_t)(((h >> 32) * (uint64_t)range) >> 32);
}

#endif /* PI_SYNTH_CORE_H */
