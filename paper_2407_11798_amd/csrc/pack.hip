// Weight repacking: logical row-major tensor -> the tiled streaming layout (PackedMat).
#include "pi_internal.h"

namespace pi {
namespace {

__device__ __forceinline__ float load_src(const void* src, int src_dtype, size_t idx) {
  if (src_dtype == PI_DTYPE_F32) return ((const float*)src)[idx];
  return bf16_to_f32(((const uint16_t*)src)[idx]);
}

// One thread per (source row, chunk of 16 bytes of the destination row).
__global__ void __launch_bounds__(256) repack_kernel(const void* src, int src_dtype, int rows,
                                                     int cols, char* dst, int KT, int dst_dtype,
                                                     int row_mul, int row_add) {
  const int per_chunk = dst_dtype == PI_DTYPE_BF16 ? 8 : 4;
  const int chunks_per_row = KT * kKTile / per_chunk;
  const size_t total = (size_t)rows * chunks_per_row;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (size_t)gridDim.x * blockDim.x) {
    const int r = (int)(i / chunks_per_row);
    const int c = (int)(i % chunks_per_row);
    const int pr = r * row_mul + row_add;
    const int rb = pr / kRowBlock, lr = pr % kRowBlock;
    const int k0 = c * per_chunk;
    float v[8];
    for (int j = 0; j < per_chunk; ++j)
      v[j] = (k0 + j < cols) ? load_src(src, src_dtype, (size_t)r * cols + k0 + j) : 0.0f;
    if (dst_dtype == PI_DTYPE_BF16) {
      const int t = c / 4, g = c % 4;
      const size_t off = ((size_t)rb * KT + t) * 1024 + (size_t)(g * 16 + lr) * 16;
      uint32_t w[4];
      for (int j = 0; j < 4; ++j)
        w[j] = (uint32_t)f32_to_bf16_rne(v[2 * j]) | ((uint32_t)f32_to_bf16_rne(v[2 * j + 1]) << 16);
      *(uint4*)(dst + off) = make_uint4(w[0], w[1], w[2], w[3]);
    } else {
      const int t = c / 8, q = c % 8, g = q / 2, h = q % 2;
      const size_t off = ((size_t)rb * KT + t) * 2048 + (size_t)h * 1024 + (size_t)(g * 16 + lr) * 16;
      *(float4*)(dst + off) = make_float4(v[0], v[1], v[2], v[3]);
    }
  }
}

// 8-bit weights: one thread per (source row, 8 bytes of the row); bytes are copied, not converted.
__global__ void __launch_bounds__(256) repack_fp8_kernel(const uint8_t* src, int rows, int cols, char* dst, int KT,
                                                         int row_mul, int row_add) {
  const int chunks_per_row = KT * 8;  // 64 columns per tile
  const size_t total = (size_t)rows * chunks_per_row;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (size_t)gridDim.x * blockDim.x) {
    const int r = (int)(i / chunks_per_row);
    const int c = (int)(i % chunks_per_row);
    const int pr = r * row_mul + row_add;
    const int rb = pr / kRowBlock, lr = pr % kRowBlock;
    const int k0 = c * 8;
    uint32_t w[2] = {0u, 0u};
    for (int j = 0; j < 8; ++j)
      if (k0 + j < cols) w[j >> 2] |= (uint32_t)src[(size_t)r * cols + k0 + j] << (8 * (j & 3));
    const int t = c / 8, q = c % 8, half = q / 4, g = q % 4;  // 32-column half of the tile, 8-column group
    const size_t off = ((size_t)rb * KT + t) * 1024 + (size_t)(g * 16 + lr) * 16 + (size_t)half * 8;
    *(uint2*)(dst + off) = make_uint2(w[0], w[1]);
  }
}

// 4-bit weights: one thread per (source row, 4 bytes = 8 weights of the row); nibbles are copied.
__global__ void __launch_bounds__(256) repack_fp4_kernel(const uint8_t* src, int rows, int cols, char* dst, int KT,
                                                         int row_mul, int row_add) {
  const int chunks_per_row = KT * 16;  // 128 columns per tile
  const size_t total = (size_t)rows * chunks_per_row;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (size_t)gridDim.x * blockDim.x) {
    const int r = (int)(i / chunks_per_row);
    const int c = (int)(i % chunks_per_row);
    const int pr = r * row_mul + row_add;
    const int rb = pr / kRowBlock, lr = pr % kRowBlock;
    const int k0 = c * 8;
    uint32_t w = 0u;
    for (int j = 0; j < 4; ++j)  // cols is even: a byte is inside the row or outside it as a whole
      if (k0 + 2 * j < cols) w |= (uint32_t)src[((size_t)r * cols + k0) / 2 + j] << (8 * j);
    const int t = c / 16, q = c % 16, h = q / 4, g = q % 4;  // 32-column quarter of the tile, 8-column group
    const size_t off = ((size_t)rb * KT + t) * 1024 + (size_t)(g * 16 + lr) * 16 + (size_t)h * 4;
    *(uint32_t*)(dst + off) = w;
  }
}

// Scale plane of a block-scaled 4-bit matrix: one thread per (source row, 128-column tile) writes the
// four scale bytes of the row's 32-column blocks in that tile (2^0 where the row has no such block).
__global__ void __launch_bounds__(256) repack_fp4_scales_kernel(const uint8_t* scales, int rows, int cols, char* dst, int KT,
                                                                int row_mul, int row_add) {
  const int bpr = (cols + 31) / 32;
  const size_t total = (size_t)rows * KT;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int r = (int)(i / KT), t = (int)(i % KT);
    const int pr = r * row_mul + row_add;
    const int rb = pr / kRowBlock, lr = pr % kRowBlock;
    uint32_t w = 0u;
    for (int h = 0; h < 4; ++h) {
      const int b = 4 * t + h;
      w |= (uint32_t)(b < bpr ? scales[(size_t)r * bpr + b] : 127u) << (8 * h);
    }
    *(uint32_t*)(dst + (((size_t)rb * KT + t) * 16 + lr) * 4) = w;
  }
}

__global__ void __launch_bounds__(256) convert_kernel(const void* src, int src_dtype, void* dst,
                                                      int dst_dtype, size_t count) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
       i += (size_t)gridDim.x * blockDim.x) {
    const float f = load_src(src, src_dtype, i);
    if (dst_dtype == PI_DTYPE_BF16) ((uint16_t*)dst)[i] = f32_to_bf16_rne(f);
    else ((float*)dst)[i] = f;
  }
}

}  // namespace

hipError_t launch_convert(const void* src, int src_dtype, void* dst, int dst_dtype, size_t count,
                          hipStream_t s) {
  size_t blocks = (count + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  if (blocks == 0) return hipSuccess;
  convert_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(src, src_dtype, dst, dst_dtype, count);
  return hipGetLastError();
}

hipError_t launch_repack(const void* src, int src_dtype, int rows, int cols, PackedMat dst,
                         int dst_dtype, int row_mul, int row_add, hipStream_t s) {
  if (dst_dtype == kWeightFP8) {
    const size_t total8 = (size_t)rows * dst.KT * 8;
    size_t blocks8 = (total8 + 255) / 256;
    if (blocks8 > 16384) blocks8 = 16384;
    if (blocks8 == 0) return hipSuccess;
    repack_fp8_kernel<<<dim3((unsigned)blocks8), dim3(256), 0, s>>>((const uint8_t*)src, rows, cols, (char*)dst.data,
                                                                    dst.KT, row_mul, row_add);
    return hipGetLastError();
  }
  if (dst_dtype == kWeightFP4B) {  // the scale bytes follow the code bytes in the source buffer
    const uint8_t* sc = (const uint8_t*)src + (size_t)rows * cols / 2;
    const size_t totals = (size_t)rows * dst.KT;
    size_t blockss = (totals + 255) / 256;
    if (blockss > 16384) blockss = 16384;
    if (blockss) {
      repack_fp4_scales_kernel<<<dim3((unsigned)blockss), dim3(256), 0, s>>>(sc, rows, cols, (char*)dst.scales, dst.KT,
                                                                             row_mul, row_add);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  }
  if (weight_is_fp4(dst_dtype)) {
    const size_t total4 = (size_t)rows * dst.KT * 16;
    size_t blocks4 = (total4 + 255) / 256;
    if (blocks4 > 16384) blocks4 = 16384;
    if (blocks4 == 0) return hipSuccess;
    repack_fp4_kernel<<<dim3((unsigned)blocks4), dim3(256), 0, s>>>((const uint8_t*)src, rows, cols, (char*)dst.data,
                                                                    dst.KT, row_mul, row_add);
    return hipGetLastError();
  }
  const int per_chunk = dst_dtype == PI_DTYPE_BF16 ? 8 : 4;
  const size_t total = (size_t)rows * (dst.KT * kKTile / per_chunk);
  size_t blocks = (total + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  if (blocks == 0) return hipSuccess;
  repack_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(src, src_dtype, rows, cols,
                                                             (char*)dst.data, dst.KT, dst_dtype,
                                                             row_mul, row_add);
  return hipGetLastError();
}

}  // namespace pi
