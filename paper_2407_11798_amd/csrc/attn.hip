// Masked attention of the speculated tokens over the KV cache (split over cells + combine).
//
// Token i attends to the canonical prefix cells [0, prefix_len) and to the window cells
// selected by its 64-bit mask word (its own cell, its tree ancestors, earlier runs' cells).
// Work unit = (kv head, range of cells): all G*n query rows that share the kv head make one
// pass over that range's K/V, staged through LDS in sub-chunks of 32 cells with a running
// (max, sum) softmax; a second kernel merges the units of each query row.
#include "pi_internal.h"

namespace pi {
namespace {

constexpr int kSC = 32;  // cells per sub-chunk
constexpr int kRT = 32;  // query rows per row tile
constexpr int kAttnThreads = 256;

__device__ __forceinline__ float ld_cache(const void* p, int dt, size_t idx) {
  return dt == PI_DTYPE_BF16 ? bf16_to_f32(((const uint16_t*)p)[idx]) : ((const float*)p)[idx];
}

template <int HD>
__global__ void __launch_bounds__(kAttnThreads) attn_partial_kernel(AttnArgs a) {
  if (a.rs->dead) return;
  constexpr int KS = HD + 4;              // padded K row stride (floats)
  constexpr int PAIRS = HD / 2;           // threads across the head dim in the PV step
  constexpr int PV_GROUPS = kAttnThreads / PAIRS;
  constexpr int PV_RPT = kRT / PV_GROUPS;  // rows per thread in the PV step
  constexpr int SC_GROUPS = kAttnThreads / kSC;  // 8
  constexpr int SC_RPT = kRT / SC_GROUPS;        // 4
  static_assert(PV_RPT >= 1, "head_dim too small for this thread mapping");

  __shared__ __align__(16) float Qs[kRT * HD];
  __shared__ __align__(16) float Ks[kSC * KS];
  __shared__ __align__(16) float Vs[kSC * HD];
  __shared__ __align__(16) float Ps[kRT * kSC];
  __shared__ float m_s[kRT], l_s[kRT], alpha_s[kRT];

  const int units_per_head = a.n_prefix_units + 1;
  const int h = blockIdx.x / units_per_head, u = blockIdx.x % units_per_head;
  const int G = a.n_q_heads / a.n_kv_heads;
  const int R = G * a.n;
  const bool window = u == a.n_prefix_units;
  const int cell_begin = window ? a.window_base : u * a.chunk_cells;
  const int cell_end = window ? min(a.window_base + PI_WINDOW, a.n_cells)
                              : min(a.prefix_len, cell_begin + a.chunk_cells);
  const float scale = 1.0f / sqrtf((float)HD);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t head_base = (size_t)h * a.n_cells * HD;

  for (int r0 = 0; r0 < R; r0 += kRT) {
    const int rows = min(kRT, R - r0);
    __syncthreads();
    // stage the query tile (scaled) and reset the running softmax state
    for (int e = tid; e < kRT * (HD / 4); e += kAttnThreads) {
      const int rr = e / (HD / 4), d4 = e % (HD / 4);
      float4 qv = make_float4(0.f, 0.f, 0.f, 0.f);
      if (rr < rows) {
        const int r = r0 + rr, gq = r / a.n, i = r % a.n;
        qv = *(const float4*)(a.q + ((size_t)i * a.n_q_heads + h * G + gq) * HD + d4 * 4);
        qv.x *= scale; qv.y *= scale; qv.z *= scale; qv.w *= scale;
      }
      *(float4*)(Qs + rr * HD + d4 * 4) = qv;
    }
    if (tid < kRT) { m_s[tid] = -INFINITY; l_s[tid] = 0.0f; }
    float acc[PV_RPT][2];
#pragma unroll
    for (int j = 0; j < PV_RPT; ++j) acc[j][0] = acc[j][1] = 0.0f;

    for (int c0 = cell_begin; c0 < cell_end; c0 += kSC) {
      const int ncell = min(kSC, cell_end - c0);
      __syncthreads();
      // stage K and V of the sub-chunk as fp32
      for (int e = tid; e < kSC * (HD / 4); e += kAttnThreads) {
        const int cc = e / (HD / 4), d4 = (e % (HD / 4)) * 4;
        float kv[4] = {0.f, 0.f, 0.f, 0.f}, vv[4] = {0.f, 0.f, 0.f, 0.f};
        if (cc < ncell) {
          const size_t idx = head_base + (size_t)(c0 + cc) * HD + d4;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            kv[j] = ld_cache(a.kcache, a.kv_dtype, idx + j);
            vv[j] = ld_cache(a.vcache, a.kv_dtype, idx + j);
          }
        }
        *(float4*)(Ks + cc * KS + d4) = make_float4(kv[0], kv[1], kv[2], kv[3]);
        *(float4*)(Vs + cc * HD + d4) = make_float4(vv[0], vv[1], vv[2], vv[3]);
      }
      __syncthreads();
      // scores: thread = (cell, row group); SC_RPT rows each
      {
        const int cc = tid % kSC, rg = tid / kSC;
        float s[SC_RPT];
#pragma unroll
        for (int j = 0; j < SC_RPT; ++j) s[j] = 0.0f;
        for (int d = 0; d < HD; d += 4) {
          const float4 kk = *(const float4*)(Ks + cc * KS + d);
#pragma unroll
          for (int j = 0; j < SC_RPT; ++j) {
            const float4 qq = *(const float4*)(Qs + (rg + SC_GROUPS * j) * HD + d);
            s[j] += qq.x * kk.x + qq.y * kk.y + qq.z * kk.z + qq.w * kk.w;
          }
        }
#pragma unroll
        for (int j = 0; j < SC_RPT; ++j) {
          const int rr = rg + SC_GROUPS * j;
          bool vis = cc < ncell && rr < rows;
          if (vis && window) {
            const int i = (r0 + rr) % a.n;
            vis = (a.mask[i] >> (c0 + cc - a.window_base)) & 1ull;
          }
          Ps[rr * kSC + cc] = vis ? s[j] : -INFINITY;
        }
      }
      __syncthreads();
      // running softmax: each wave owns rows wave, wave+4, ...; lanes 0..31 are the cells
      for (int rr = wave; rr < kRT; rr += kAttnThreads / 64) {
        const float sv = lane < kSC ? Ps[rr * kSC + lane] : -INFINITY;
        float mx = sv;
#pragma unroll
        for (int o = 16; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        const float m_old = m_s[rr];
        const float m_new = fmaxf(m_old, mx);
        const float p = (sv == -INFINITY) ? 0.0f : expf(sv - m_new);
        float sum = p;
#pragma unroll
        for (int o = 16; o >= 1; o >>= 1) sum += __shfl_xor(sum, o);
        const float alpha = (m_old == -INFINITY) ? 0.0f : expf(m_old - m_new);
        if (lane < kSC) Ps[rr * kSC + lane] = p;
        if (lane == 0) {
          m_s[rr] = m_new;
          l_s[rr] = l_s[rr] * alpha + sum;
          alpha_s[rr] = alpha;
        }
      }
      __syncthreads();
      // O += P V : thread = (pair of head dims, row group)
      {
        const int dp = tid % PAIRS, rg = tid / PAIRS;
#pragma unroll
        for (int j = 0; j < PV_RPT; ++j) {
          const float al = alpha_s[rg + PV_GROUPS * j];
          acc[j][0] *= al;
          acc[j][1] *= al;
        }
        for (int cc = 0; cc < kSC; cc += 4) {
          float2 v[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] = *(const float2*)(Vs + (cc + q) * HD + 2 * dp);
#pragma unroll
          for (int j = 0; j < PV_RPT; ++j) {
            const float4 p = *(const float4*)(Ps + (rg + PV_GROUPS * j) * kSC + cc);
            acc[j][0] += p.x * v[0].x + p.y * v[1].x + p.z * v[2].x + p.w * v[3].x;
            acc[j][1] += p.x * v[0].y + p.y * v[1].y + p.z * v[2].y + p.w * v[3].y;
          }
        }
      }
    }
    __syncthreads();
    // write this unit's partial result for the row tile
    {
      const int dp = tid % PAIRS, rg = tid / PAIRS;
      const size_t ubase = ((size_t)h * units_per_head + u) * R;
#pragma unroll
      for (int j = 0; j < PV_RPT; ++j) {
        const int rr = rg + PV_GROUPS * j;
        if (rr < rows)
          *(float2*)(a.part_o + (ubase + r0 + rr) * HD + 2 * dp) = make_float2(acc[j][0], acc[j][1]);
      }
      if (tid < rows) {
        a.part_ml[(ubase + r0 + tid) * 2] = m_s[tid];
        a.part_ml[(ubase + r0 + tid) * 2 + 1] = l_s[tid];
      }
    }
  }
}

// One block per (token, query head): merge the units in unit order.
template <int HD>
__global__ void __launch_bounds__(HD) attn_combine_kernel(AttnArgs a) {
  if (a.rs->dead) return;
  const int units_per_head = a.n_prefix_units + 1;
  const int G = a.n_q_heads / a.n_kv_heads;
  const int R = G * a.n;
  const int i = blockIdx.x / a.n_q_heads, qh = blockIdx.x % a.n_q_heads;
  const int h = qh / G, gq = qh % G, r = gq * a.n + i;
  const int d = threadIdx.x;
  const size_t ubase = (size_t)h * units_per_head;
  float M = -INFINITY;
  for (int u = 0; u < units_per_head; ++u) M = fmaxf(M, a.part_ml[((ubase + u) * R + r) * 2]);
  float L = 0.0f, o = 0.0f;
  for (int u = 0; u < units_per_head; ++u) {
    const float m = a.part_ml[((ubase + u) * R + r) * 2];
    if (m == -INFINITY) continue;
    const float w = expf(m - M);
    L += w * a.part_ml[((ubase + u) * R + r) * 2 + 1];
    o += w * a.part_o[((ubase + u) * R + r) * HD + d];
  }
  a.out[((size_t)i * a.n_q_heads + qh) * HD + d] = o / L;
}

template <int HD>
hipError_t launch_hd(const AttnArgs& a, hipStream_t s) {
  const int units = a.n_kv_heads * (a.n_prefix_units + 1);
  attn_partial_kernel<HD><<<dim3((unsigned)units), dim3(kAttnThreads), 0, s>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  attn_combine_kernel<HD><<<dim3((unsigned)(a.n * a.n_q_heads)), dim3(HD), 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace

int attn_sub_chunk(int) { return kSC; }

hipError_t launch_attention(const AttnArgs& a, hipStream_t s) {
  switch (a.head_dim) {
    case 32: return launch_hd<32>(a, s);
    case 64: return launch_hd<64>(a, s);
    case 128: return launch_hd<128>(a, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace pi
