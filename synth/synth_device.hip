// Device fills of the seeded synthetic-input generator (see synth_core.h).
// Same arithmetic core as the host fill, so a tensor filled here is bit-identical
// to the one the host fill produces for the same (seed, stream_id).
#include <hip/hip_runtime.h>
#include "synth_core.h"

namespace {

template <int DTYPE>
__global__ void __launch_bounds__(256) fill_normal_kernel(void* dst, int64_t n, uint64_t key,
                                                          double sigma) {
  const int64_t pairs = (n + 1) / 2;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < pairs;
       p += (int64_t)gridDim.x * blockDim.x) {
    double z0, z1;
    synth_normal_pair(key, (uint64_t)p, &z0, &z1);
    float f0 = (float)(sigma * z0), f1 = (float)(sigma * z1);
    int64_t i = 2 * p;
    if (DTYPE == 0) {
      float* d = (float*)dst;
      if (i + 1 < n) {
        *(float2*)(d + i) = make_float2(f0, f1);
      } else {
        d[i] = f0;
      }
    } else if (DTYPE == 1) {
      uint16_t* d = (uint16_t*)dst;
      uint32_t lo = synth_f32_to_bf16(f0), hi = synth_f32_to_bf16(f1);
      if (i + 1 < n) {
        *(uint32_t*)(d + i) = lo | (hi << 16);
      } else {
        d[i] = (uint16_t)lo;
      }
    } else if (DTYPE == 2) {
      uint8_t* d = (uint8_t*)dst;
      const uint8_t lo = synth_f32_to_e4m3(f0), hi = synth_f32_to_e4m3(f1);
      if (i + 1 < n) {
        *(uint16_t*)(d + i) = (uint16_t)(lo | ((uint16_t)hi << 8));
      } else {
        d[i] = lo;
      }
    } else {
      ((uint8_t*)dst)[p] = (uint8_t)(synth_f32_to_e2m1(f0) | (synth_f32_to_e2m1(f1) << 4));
    }
  }
}

// one thread per 32-column block of a block-scaled 4-bit matrix
__global__ void __launch_bounds__(256) fill_fp4b_kernel(uint8_t* codes, uint8_t* scales, int64_t rows, int64_t cols,
                                                        uint64_t key, double sigma) {
  const int64_t bpr = (cols + 31) / 32;
  for (int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; b < rows * bpr; b += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = b / bpr, j = b % bpr;
    const int count = (int)(cols - 32 * j < 32 ? cols - 32 * j : 32);
    uint8_t c[16];
    const uint8_t sc = synth_fp4_block(key, (uint64_t)(r * cols + 32 * j), count, sigma, c);
    uint8_t* d = codes + (r * cols + 32 * j) / 2;
    for (int p = 0; p < count / 2; ++p) d[p] = c[p];
    scales[b] = sc;
  }
}

__global__ void __launch_bounds__(256) fill_uniform_int_kernel(int32_t* dst, int64_t n,
                                                               uint64_t key, uint32_t range) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = synth_uniform_int(key, (uint64_t)i, range);
}

}  // namespace

// dst: device pointer, 4-byte aligned. dtype: 0 = fp32, 1 = bf16, 2 = FP8 E4M3 bytes, 3 = FP4 E2M1 (two per byte, n even). Asynchronous on `stream`.
extern "C" int synth_fill_normal_device(void* dst, int64_t n, uint64_t seed, uint64_t stream_id,
                                        double sigma, int dtype, void* stream) {
  if (!dst || n < 0 || dtype < 0 || dtype > 3 || (dtype == 3 && (n & 1))) return -1;
  if (n == 0) return 0;
  const uint64_t key = synth_key(seed, stream_id);
  const int64_t pairs = (n + 1) / 2;
  int64_t blocks = (pairs + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipStream_t s = (hipStream_t)stream;
  if (dtype == 0)
    fill_normal_kernel<0><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(dst, n, key, sigma);
  else if (dtype == 1)
    fill_normal_kernel<1><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(dst, n, key, sigma);
  else if (dtype == 2)
    fill_normal_kernel<2><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(dst, n, key, sigma);
  else
    fill_normal_kernel<3><<<dim3((unsigned)blocks), dim3(256), 0, s>>>(dst, n, key, sigma);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}

// codes[rows][cols / 2] and scales[rows][ceil(cols / 32)] on the device. Asynchronous on `stream`.
extern "C" int synth_fill_normal_fp4b_device(uint8_t* codes, uint8_t* scales, int64_t rows, int64_t cols, uint64_t seed,
                                             uint64_t stream_id, double sigma, void* stream) {
  if (!codes || !scales || rows < 0 || cols < 0 || (cols & 1)) return -1;
  const int64_t blocks_total = rows * ((cols + 31) / 32);
  if (blocks_total == 0) return 0;
  int64_t blocks = (blocks_total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  fill_fp4b_kernel<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>(codes, scales, rows, cols,
                                                                                   synth_key(seed, stream_id), sigma);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}

extern "C" int synth_fill_uniform_int_device(int32_t* dst, int64_t n, uint64_t seed,
                                             uint64_t stream_id, uint32_t range, void* stream) {
  if (!dst || n < 0 || range == 0) return -1;
  if (n == 0) return 0;
  const uint64_t key = synth_key(seed, stream_id);
  int64_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  fill_uniform_int_kernel<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>(
      dst, n, key, range);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}
