// Weight-streaming skinny projection: y[n][N] = act(x)[n][K] . W[N][K]^T for n <= 16 tokens.
//
// The weights are streamed once from HBM with 128-bit non-temporal loads straight into MFMA
// A operands (the tile layout of PackedMat); the n activations are the B operand, staged in
// LDS in operand order.  With <= 16 tokens one MFMA per 1 KiB weight tile keeps the matrix
// cores a few percent busy, so the kernel is bound by the weight stream alone.
//
// Precision: bf16 weights are used exactly; fp32 activations are split into two bf16 terms
// (hi + lo, ~16 significant bits) and both are multiplied, accumulating in fp32.  fp32
// weights use the fp32 MFMA (16x16x4) with unsplit activations.
//
// Work decomposition: the matrix is cut into S_k column slices and row chunks of RBU row
// blocks; a workgroup takes (slice, chunk) units round-robin, stages its slice of x once,
// and its 4 waves walk the chunk's row blocks.  For S_k > 1 the partial tiles go to a
// scratch array and the last wave to arrive at a row block (an arrival counter) adds them
// in slice order -- a fixed order, so results do not depend on timing -- and runs the
// epilogue: RMSNorm scale, RoPE + KV-cache write, residual add, SwiGLU, or logits.
#include "pi_internal.h"

namespace pi {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 ld_stream(const u32x4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ f32x4 ld_stream(const f32x4* p) { return __builtin_nontemporal_load(p); }

// ---- activation staging ------------------------------------------------------------------
// LDS slot (tt, g, i) holds the 8 activations x[i][32(t0+tt) + 8g + 0..7] (times the gain):
// bf16 model: 16 B of hi parts at slot index, 16 B of lo parts at slot index + n_slots;
// fp32 model: 32 B of floats at 2*slot index.
template <int DT>
__device__ void stage_x(const ProjArgs& a, int t0, int nt, char* lds) {
  const int n = a.n;
  const int n_cblocks = nt;  // one cblock = the 4 chunks (g = 0..3) of one k tile
  const int items = n_cblocks * n * 4;
  const int n_slots = nt * 4 * n;
  for (int id = threadIdx.x; id < items; id += blockDim.x) {
    const int cl = id & 3;
    const int i = (id >> 2) % n;
    const int tt = (id >> 2) / n;
    const int k0 = (t0 + tt) * kKTile + cl * 8;
    float v[8];
    if (k0 < a.K) {
      const float4 p0 = *(const float4*)(a.xin + (size_t)i * a.K + k0);
      const float4 p1 = *(const float4*)(a.xin + (size_t)i * a.K + k0 + 4);
      v[0] = p0.x; v[1] = p0.y; v[2] = p0.z; v[3] = p0.w;
      v[4] = p1.x; v[5] = p1.y; v[6] = p1.z; v[7] = p1.w;
      if (a.gain) {
        const float4 g0 = *(const float4*)(a.gain + k0);
        const float4 g1 = *(const float4*)(a.gain + k0 + 4);
        v[0] *= g0.x; v[1] *= g0.y; v[2] *= g0.z; v[3] *= g0.w;
        v[4] *= g1.x; v[5] *= g1.y; v[6] *= g1.z; v[7] *= g1.w;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = 0.0f;
    }
    const int slot = (tt * 4 + cl) * n + i;
    if (DT == PI_DTYPE_BF16) {
      uint32_t hi[4], lo[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint16_t h0 = f32_to_bf16_rne(v[2 * j]), h1 = f32_to_bf16_rne(v[2 * j + 1]);
        const uint16_t l0 = f32_to_bf16_rne(v[2 * j] - bf16_to_f32(h0));
        const uint16_t l1 = f32_to_bf16_rne(v[2 * j + 1] - bf16_to_f32(h1));
        hi[j] = (uint32_t)h0 | ((uint32_t)h1 << 16);
        lo[j] = (uint32_t)l0 | ((uint32_t)l1 << 16);
      }
      ((uint4*)lds)[slot] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
      ((uint4*)lds)[slot + n_slots] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    } else {
      ((float4*)lds)[2 * slot] = make_float4(v[0], v[1], v[2], v[3]);
      ((float4*)lds)[2 * slot + 1] = make_float4(v[4], v[5], v[6], v[7]);
    }
  }
}

// 1/sqrt(mean x^2 + eps) per token from the per-row-block partial sums of squares; the sum
// runs in a fixed order.  red: 256 floats of LDS, rscale: 16 floats of LDS.
__device__ void compute_rscale(const ProjArgs& a, float* red, float* rscale) {
  const int i = threadIdx.x & 15, b0 = threadIdx.x >> 4;
  float s = 0.0f;
  for (int b = b0; b < a.n_ssq_blocks; b += 16) s += a.ssq_in[b * 16 + i];
  red[b0 * 16 + i] = s;
  __syncthreads();
  if (threadIdx.x < 16) {
    float t = 0.0f;
    for (int b = 0; b < 16; ++b) t += red[b * 16 + threadIdx.x];
    rscale[threadIdx.x] = 1.0f / sqrtf(t / (float)a.K + a.eps);
  }
}

// ---- the weight stream of one row block over k tiles [t0, t0+nt) ------------------------------
template <int DT>
__device__ __forceinline__ f32x4 stream_rowblock(const char* wtile, int nt, const char* lds, int n,
                                                 int lane);

template <>
__device__ __forceinline__ f32x4 stream_rowblock<PI_DTYPE_BF16>(const char* wtile, int nt,
                                                                const char* lds, int n, int lane) {
  constexpr int U = 8;
  const u32x4* wp = (const u32x4*)wtile + lane;
  const int g = lane >> 4, ln = min(lane & 15, n - 1);
  const u32x4* bh = (const u32x4*)lds + g * n + ln;
  const u32x4* bl = bh + nt * 4 * n;
  const int bstride = 4 * n;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  u32x4 w[U];
#pragma unroll
  for (int j = 0; j < U; ++j)
    if (j < nt) w[j] = ld_stream(wp + j * 64);
  int tb = 0;
  for (; tb + 2 * U <= nt; tb += U) {  // full chunk with a full chunk behind it: no guards
    u32x4 c[U];
#pragma unroll
    for (int j = 0; j < U; ++j) c[j] = w[j];
#pragma unroll
    for (int j = 0; j < U; ++j) w[j] = ld_stream(wp + (tb + U + j) * 64);
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const bf16x8 av = __builtin_bit_cast(bf16x8, c[j]);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bh[(tb + j) * bstride]), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bl[(tb + j) * bstride]), acc, 0, 0, 0);
    }
  }
  for (; tb < nt; tb += U) {
    u32x4 c[U];
#pragma unroll
    for (int j = 0; j < U; ++j) c[j] = w[j];
#pragma unroll
    for (int j = 0; j < U; ++j)
      if (tb + U + j < nt) w[j] = ld_stream(wp + (tb + U + j) * 64);
#pragma unroll
    for (int j = 0; j < U; ++j) {
      if (tb + j < nt) {
        const bf16x8 av = __builtin_bit_cast(bf16x8, c[j]);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bh[(tb + j) * bstride]), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bl[(tb + j) * bstride]), acc, 0, 0, 0);
      }
    }
  }
  return acc;
}

template <>
__device__ __forceinline__ f32x4 stream_rowblock<PI_DTYPE_F32>(const char* wtile, int nt,
                                                               const char* lds, int n, int lane) {
  const f32x4* wp = (const f32x4*)wtile + lane;
  const int g = lane >> 4, ln = min(lane & 15, n - 1);
  const f32x4* bx = (const f32x4*)lds + 2 * (g * n + ln);
  const int bstride = 8 * n;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int t = 0; t < nt; ++t) {
    const f32x4 w0 = ld_stream(wp + t * 128);
    const f32x4 w1 = ld_stream(wp + t * 128 + 64);
    const f32x4 x0 = bx[t * bstride], x1 = bx[t * bstride + 1];
#pragma unroll
    for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(w0[j], x0[j], acc, 0, 0, 0);
#pragma unroll
    for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(w1[j], x1[j], acc, 0, 0, 0);
  }
  return acc;
}

// ---- epilogues ---------------------------------------------------------------------------
// The accumulator tile of a wave: lane l holds rows 16rb + 4(l>>4) + 0..3 for token l & 15.

__device__ __forceinline__ void store_kv4(void* cache, int kv_dtype, size_t elem_idx, const float* v) {
  if (kv_dtype == PI_DTYPE_BF16) {
    uint2 p;
    p.x = (uint32_t)f32_to_bf16_rne(v[0]) | ((uint32_t)f32_to_bf16_rne(v[1]) << 16);
    p.y = (uint32_t)f32_to_bf16_rne(v[2]) | ((uint32_t)f32_to_bf16_rne(v[3]) << 16);
    *(uint2*)((uint16_t*)cache + elem_idx) = p;
  } else {
    *(float4*)((float*)cache + elem_idx) = make_float4(v[0], v[1], v[2], v[3]);
  }
}

template <int EPI>
__device__ __forceinline__ void epilogue(const ProjArgs& a, int rb, f32x4 acc, int lane,
                                         const float* rscale) {
  const int i = lane & 15, g = lane >> 4;
  const int row = rb * kRowBlock + g * 4;
  const bool live = i < a.n;
  if (EPI == EPI_QKV) {
    if (!live) return;
    const float r = rscale[i];
    float v[4] = {acc[0] * r, acc[1] * r, acc[2] * r, acc[3] * r};
    const int hd = a.head_dim;
    if (row < a.n_q_rows + a.n_kv_rows) {  // q or k: rotary embedding on adjacent pairs
      const int dim = row % hd;
      const float2* cs = a.rope + (size_t)a.positions[i] * (hd / 2) + dim / 2;
      const float2 c0 = cs[0], c1 = cs[1];
      const float a0 = v[0] * c0.x - v[1] * c0.y, a1 = v[0] * c0.y + v[1] * c0.x;
      const float a2 = v[2] * c1.x - v[3] * c1.y, a3 = v[2] * c1.y + v[3] * c1.x;
      v[0] = a0; v[1] = a1; v[2] = a2; v[3] = a3;
    }
    if (row < a.n_q_rows) {
      *(float4*)(a.out + (size_t)i * a.n_q_rows + row) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
      const bool is_k = row < a.n_q_rows + a.n_kv_rows;
      const int kr = row - a.n_q_rows - (is_k ? 0 : a.n_kv_rows);
      const int head = kr / hd, dim = kr % hd;
      const size_t idx = ((size_t)head * a.n_cells + a.slots[i]) * hd + dim;
      store_kv4(is_k ? a.kcache : a.vcache, a.kv_dtype, idx, v);
    }
  } else if (EPI == EPI_RESID) {
    float s = 0.0f;
    if (live && row < a.N) {
      float4* px = (float4*)(a.out + (size_t)i * a.N + row);
      float4 x = *px;
      x.x += acc[0]; x.y += acc[1]; x.z += acc[2]; x.w += acc[3];
      *px = x;
      s = x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
    }
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 32);
    if (g == 0) a.ssq_out[rb * 16 + i] = live ? s : 0.0f;
  } else if (EPI == EPI_SWIGLU) {
    if (!live || row >= a.N) return;
    const float r = rscale[i];
    const float g0 = acc[0] * r, u0 = acc[1] * r, g1 = acc[2] * r, u1 = acc[3] * r;
    float2 o;
    o.x = g0 / (1.0f + expf(-g0)) * u0;
    o.y = g1 / (1.0f + expf(-g1)) * u1;
    *(float2*)(a.out + (size_t)i * (a.N / 2) + row / 2) = o;
  } else {  // EPI_LOGITS
    if (!live || row >= a.N) return;
    const float r = rscale[i];
    *(float4*)(a.out + (size_t)i * a.N + row) = make_float4(acc[0] * r, acc[1] * r, acc[2] * r, acc[3] * r);
  }
}

template <int DT, int EPI>
__global__ void __launch_bounds__(kProjThreads) proj_kernel(ProjArgs a) {
  if (a.rs->dead) return;
  extern __shared__ __align__(16) char lds[];
  constexpr int kTileBytes = DT == PI_DTYPE_BF16 ? 1024 : 2048;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_chunks = (a.NRB + a.RBU - 1) / a.RBU;
  const int n_units = n_chunks * a.S_k;
  const int max_nt = (a.KT + a.S_k - 1) / a.S_k;
  float* red = (float*)(lds + (size_t)max_nt * 128 * a.n);
  float* rscale = red + 256;
  constexpr bool kScaled = EPI == EPI_QKV || EPI == EPI_SWIGLU || EPI == EPI_LOGITS;
  if (kScaled) {
    if (a.ssq_in) {
      compute_rscale(a, red, rscale);
    } else if (threadIdx.x < 16) {
      rscale[threadIdx.x] = 1.0f;
    }
  }
  for (int u = blockIdx.x; u < n_units; u += gridDim.x) {
    const int s = u % a.S_k, c = u / a.S_k;
    const int t0 = (int)((long)s * a.KT / a.S_k), t1 = (int)((long)(s + 1) * a.KT / a.S_k);
    const int nt = t1 - t0;
    __syncthreads();  // previous unit's readers are done with the staged slice
    stage_x<DT>(a, t0, nt, lds);
    __syncthreads();
    const int rb_end = min((c + 1) * a.RBU, a.NRB);
    for (int rb = c * a.RBU + wave; rb < rb_end; rb += kProjThreads / 64) {
      const char* wtile = (const char*)a.W + ((size_t)rb * a.KT + t0) * kTileBytes;
      f32x4 acc = stream_rowblock<DT>(wtile, nt, lds, a.n, lane);
      bool finish = true;
      if (a.S_k > 1) {
        f32x4* part = (f32x4*)a.part;
        part[((size_t)s * a.NRB + rb) * 64 + lane] = acc;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        int old = 0;
        if (lane == 0)
          old = __hip_atomic_fetch_add(a.cnt + rb, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        old = __shfl(old, 0);
        finish = old == a.S_k - 1;
        if (finish) {
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
          acc = f32x4{0.f, 0.f, 0.f, 0.f};
          for (int s2 = 0; s2 < a.S_k; ++s2) {
            const f32x4 p = __builtin_nontemporal_load(part + ((size_t)s2 * a.NRB + rb) * 64 + lane);
            acc += p;
          }
          if (lane == 0) a.cnt[rb] = 0;
        }
      }
      if (finish) {
        epilogue<EPI>(a, rb, acc, lane, rscale);
        if (EPI == EPI_RESID && a.rs_mut) {
          // Layer boundary: the wave that completes the last row block of the layer's last
          // projection records progress and probes the cancel flag for the next layer.
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
          int done = 0;
          if (lane == 0)
            done = __hip_atomic_fetch_add(a.done_cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          done = __shfl(done, 0);
          if (done == a.NRB - 1 && lane == 0) {
            *a.done_cnt = 0;
            a.rs_mut->layers_done = a.next_layer;
            if (a.probe && a.cancel_flag &&
                __hip_atomic_load(a.cancel_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != 0) {
              a.rs_mut->status = PI_CANCELLED;
              a.rs_mut->dead = 1;
            }
          }
        }
      }
    }
  }
}

template <int DT>
hipError_t launch_dt(const ProjArgs& a, int epi, int grid, size_t lds, hipStream_t s) {
  dim3 g((unsigned)grid), b(kProjThreads);
  switch (epi) {
    case EPI_QKV: proj_kernel<DT, EPI_QKV><<<g, b, lds, s>>>(a); break;
    case EPI_RESID: proj_kernel<DT, EPI_RESID><<<g, b, lds, s>>>(a); break;
    case EPI_SWIGLU: proj_kernel<DT, EPI_SWIGLU><<<g, b, lds, s>>>(a); break;
    default: proj_kernel<DT, EPI_LOGITS><<<g, b, lds, s>>>(a); break;
  }
  return hipGetLastError();
}

}  // namespace

size_t proj_lds_bytes(int n, int k_tiles_per_split) {
  return (size_t)k_tiles_per_split * 128 * n + (256 + 16) * sizeof(float);
}

hipError_t launch_proj(const ProjArgs& a, int epi, int dtype, int grid, hipStream_t s) {
  const size_t lds = proj_lds_bytes(a.n, (a.KT + a.S_k - 1) / a.S_k);
  if (dtype == PI_DTYPE_BF16) return launch_dt<PI_DTYPE_BF16>(a, epi, grid, lds, s);
  return launch_dt<PI_DTYPE_F32>(a, epi, grid, lds, s);
}

}  // namespace pi
