/* Host fills of the seeded synthetic-input generator (see synth_core.h).
 * Plain C, OpenMP over elements; no decoder arithmetic lives here. */
#include "synth_core.h"
#include <stddef.h>

/* dtype: 0 = fp32 (float), 1 = bf16 (uint16 bit patterns), 2 = FP8 E4M3 (bytes),
 * 3 = FP4 E2M1 (two per byte, element 2p in the low nibble; n must be even) */
int synth_fill_normal_host(void* dst, int64_t n, uint64_t seed, uint64_t stream_id,
                           double sigma, int dtype) {
  if (!dst || n < 0 || dtype < 0 || dtype > 3 || (dtype == 3 && (n & 1))) return -1;
  const uint64_t key = synth_key(seed, stream_id);
  const int64_t pairs = (n + 1) / 2;
#pragma omp parallel for schedule(static)
  for (int64_t p = 0; p < pairs; ++p) {
    double z0, z1;
    synth_normal_pair(key, (uint64_t)p, &z0, &z1);
    float f0 = (float)(sigma * z0), f1 = (float)(sigma * z1);
    int64_t i = 2 * p;
    if (dtype == 0) {
      ((float*)dst)[i] = f0;
      if (i + 1 < n) ((float*)dst)[i + 1] = f1;
    } else if (dtype == 1) {
      ((uint16_t*)dst)[i] = synth_f32_to_bf16(f0);
      if (i + 1 < n) ((uint16_t*)dst)[i + 1] = synth_f32_to_bf16(f1);
    } else if (dtype == 2) {
      ((uint8_t*)dst)[i] = synth_f32_to_e4m3(f0);
      if (i + 1 < n) ((uint8_t*)dst)[i + 1] = synth_f32_to_e4m3(f1);
    } else {
      ((uint8_t*)dst)[p] = (uint8_t)(synth_f32_to_e2m1(f0) | (synth_f32_to_e2m1(f1) << 4));
    }
  }
  return 0;
}

/* Block-scaled 4-bit matrix [rows][cols] (cols even): codes[rows][cols / 2] and
 * scales[rows][ceil(cols / 32)]; a row's last block may be shorter than 32. */
int synth_fill_normal_fp4b_host(uint8_t* codes, uint8_t* scales, int64_t rows, int64_t cols, uint64_t seed,
                                uint64_t stream_id, double sigma) {
  if (!codes || !scales || rows < 0 || cols < 0 || (cols & 1)) return -1;
  const uint64_t key = synth_key(seed, stream_id);
  const int64_t bpr = (cols + 31) / 32;
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < rows * bpr; ++b) {
    const int64_t r = b / bpr, j = b % bpr;
    const int count = (int)(cols - 32 * j < 32 ? cols - 32 * j : 32);
    scales[b] = synth_fp4_block(key, (uint64_t)(r * cols + 32 * j), count, sigma, codes + (r * cols + 32 * j) / 2);
  }
  return 0;
}

int synth_fill_uniform_int_host(int32_t* dst, int64_t n, uint64_t seed, uint64_t stream_id,
                                uint32_t range) {
  if (!dst || n < 0 || range == 0) return -1;
  const uint64_t key = synth_key(seed, stream_id);
  for (int64_t i = 0; i < n; ++i) dst[i] = synth_uniform_int(key, (uint64_t)i, range);
  return 0;
}

/* Exposed for pin tests: the FP8 rounding of arbitrary floats. */
int synth_debug_e4m3_host(const float* src, uint8_t* dst, int64_t n) {
  for (int64_t i = 0; i < n; ++i) dst[i] = synth_f32_to_e4m3(src[i]);
  return 0;
}

int synth_debug_e2m1_host(const float* src, uint8_t* dst, int64_t n) {
  for (int64_t i = 0; i < n; ++i) dst[i] = synth_f32_to_e2m1(src[i]);
  return 0;
}

/* Exposed for the generator's own pin tests: raw uniforms and normals in fp64. */
int synth_debug_pair_host(uint64_t seed, uint64_t stream_id, uint64_t pair, double* out4) {
  const uint64_t key = synth_key(seed, stream_id);
  uint64_t h1 = synth_mix(key + 2 * pair), h2 = synth_mix(key + 2 * pair + 1);
  out4[0] = (double)((h1 >> 11) + 1) * 1.1102230246251565e-16;
  out4[1] = (double)(h2 >> 11) * 1.1102230246251565e-16;
  synth_normal_pair(key, pair, &out4[2], &out4[3]);
  return 0;
}
