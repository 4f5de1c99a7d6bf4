// The stage kernel: one persistent launch evaluates a whole slice of decoder layers.
//
// One workgroup of 8 waves per compute unit stays resident for the whole stage and walks the
// phases of every layer (QKV projection, attention, output projection, gate/up, down), with a
// grid-wide barrier between phases.  Weights never wait for activations: each wave owns a
// fixed, contiguous range of weight tiles in every phase and keeps a ring of 16 outstanding
// 128-bit non-temporal loads, which it refills for the NEXT phase before it arrives at the
// barrier, so HBM stays busy while the grid synchronises.
//
// Early Inference Cancellation: the last workgroup to arrive at a layer-boundary barrier
// probes the device-visible cancel flag and publishes the decision with the barrier release,
// so every workgroup takes the same decision and a cancelled run stops within one layer.
//
// Cross-workgroup data (activations, split-k partial tiles, counters) is written and read
// with agent-scope accesses that bypass the per-XCD L2, which is not coherent across XCDs;
// full-cache writeback/invalidate fences are never used.
#include "pi_internal.h"

namespace pi {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// Pointers read from device-resident tables are generic to the compiler; weight loads must be
// global-memory instructions (a flat load also ticks the LDS counter and would serialise the
// ring behind every LDS wait), so the address space is stated.
typedef const __attribute__((address_space(1))) u32x4* gptr_u32x4;
typedef const __attribute__((address_space(1))) f32x4* gptr_f32x4;

constexpr int kThreads = kStageThreads;
constexpr int kWaves = kThreads / 64;

// ---- agent-scope accessors ------------------------------------------------------------------
__device__ __forceinline__ float ld_ag(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_ag(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t ld_ag_u32(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_ag_u32(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_ag4(float* p, float a, float b, float c, float d) {
  st_ag(p, a); st_ag(p + 1, b); st_ag(p + 2, c); st_ag(p + 3, d);
}
// 128/64-bit agent-scope accesses through a raw buffer (cache policy sc1: coherent across XCDs)
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
constexpr int kAgent = 16;  // sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc_of(const void* base) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, 0x7fffffff, 0x00020000);
}
__device__ __forceinline__ f32x4 ld_ag4(__amdgpu_buffer_rsrc_t r, int byte_off) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, kAgent));
}
__device__ __forceinline__ void st_ag4(__amdgpu_buffer_rsrc_t r, int byte_off, f32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, byte_off, 0, kAgent);
}
__device__ __forceinline__ void st_ag2(__amdgpu_buffer_rsrc_t r, int byte_off, float a, float b) {
  u32x2 v = {__float_as_uint(a), __float_as_uint(b)};
  __builtin_amdgcn_raw_buffer_store_b64(v, r, byte_off, 0, kAgent);
}
// all earlier memory operations of this wave have completed (stores are visible at agent scope
// because they were issued with agent scope)
__device__ __forceinline__ void wave_drain() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void wg_mark(const StageArgs& A, int l, int ev) {
  if (A.wgtrace && l == A.wgtrace_layer && threadIdx.x == 0) A.wgtrace[blockIdx.x * 8 + ev] = wall_clock64();
}

// ---- grid barrier ---------------------------------------------------------------------------
// Every workgroup calls it the same number of times.  Returns false when the grid must stop
// (a wait ran into its time limit somewhere): callers then leave the kernel at once.
// probe_layer >= 0: layer boundary; the last arriver records progress and probes the cancel flag.
struct BarrierCtx {
  unsigned epoch;  // absolute number of the last barrier passed
  int* sh;         // 2 ints of LDS: {ok, dead}
};

// Every workgroup calls it the same number of times.  Returns false when the grid must stop (a
// wait ran into its time limit): callers then leave the kernel at once.  layers_done >= 0 marks
// a layer boundary: workgroup 0 records progress, probes the cancel flag when `probe` is set
// and publishes the decision, which every workgroup reads before going on.
__device__ bool grid_barrier(const StageArgs& A, BarrierCtx& bc, int layers_done, bool probe) {
  __syncthreads();  // every wave of this workgroup has drained its stores
  bc.epoch += 1;
  StageSync* sy = A.sync;
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    if (lane == 0) __hip_atomic_store(&sy->flags[blockIdx.x], bc.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const __amdgpu_buffer_rsrc_t fr = rsrc_of(sy->flags);
    const int G = gridDim.x;
    const unsigned long long t0 = wall_clock64();
    int ok = 1;
    for (unsigned spin = 0;; ++spin) {
      bool all = true;
      for (int base = 0; base < G; base += 256) {
        const int idx = base + lane * 4;
        u32x4 f = {bc.epoch, bc.epoch, bc.epoch, bc.epoch};
        if (idx < G) f = __builtin_amdgcn_raw_buffer_load_b128(fr, idx * 4, 0, kAgent);
#pragma unroll
        for (int q = 0; q < 4; ++q) all = all && (idx + q >= G || (int)(f[q] - bc.epoch) >= 0);
      }
      if (__builtin_amdgcn_ballot_w64(!all) == 0) break;
      __builtin_amdgcn_s_sleep(1);
      if ((spin & 15) == 15 && wall_clock64() - t0 > A.timeout_ticks) {
        ok = 0;
        break;
      }
    }
    int dead = 0;
    if (ok && layers_done >= 0) {
      if (blockIdx.x == 0) {
        if (lane == 0) {
          __hip_atomic_store(&A.rs->layers_done, layers_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (probe && A.cancel_flag &&
              __hip_atomic_load(A.cancel_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != 0) {
            __hip_atomic_store(&A.rs->status, PI_CANCELLED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&A.rs->dead, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
        }
        wave_drain();
        if (lane == 0) __hip_atomic_store(&sy->decision, bc.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      } else {
        for (unsigned spin = 0;; ++spin) {
          const unsigned d = __hip_atomic_load(&sy->decision, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if ((int)(d - bc.epoch) >= 0) break;
          __builtin_amdgcn_s_sleep(1);
          if ((spin & 15) == 15 && wall_clock64() - t0 > A.timeout_ticks) {
            ok = 0;
            break;
          }
        }
      }
      if (ok) dead = __hip_atomic_load(&A.rs->dead, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (lane == 0) {
      if (!ok) __hip_atomic_store(&sy->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (A.trace && blockIdx.x == 0 && (int)(bc.epoch - A.epoch_base) <= A.trace_cap)
        A.trace[bc.epoch - A.epoch_base - 1] = wall_clock64();
      bc.sh[0] = ok;
      bc.sh[1] = dead;
    }
  }
  __syncthreads();
  return __builtin_amdgcn_readfirstlane(bc.sh[0]) != 0;
}

// ---- per-wave weight stream -----------------------------------------------------------------
// In a projection with S_k column slices, workgroup wg serves slice wg % S_k together with the
// other gridDim/S_k workgroups of its group.  The slice's tiles, ordered row-block-major, are
// cut into equal contiguous ranges, one per wave of the group: flat index f -> row block f / nt,
// k tile t0 + f % nt.
struct WaveStream {
  __amdgpu_buffer_rsrc_t rsrc;  // the whole matrix as a raw buffer
  int KT, nt, t0, NRB;
  int f0, f1, share;
  int slice, gw;  // slice index, wave index within the slice group
  // loader cursor
  int lf, lrb, lt;
};

// Wave-uniform values computed with vector instructions (integer division) are moved back to
// scalar registers so that the streaming loop is controlled by scalar branches.
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <typename T>
__device__ __forceinline__ T* uni_ptr(T* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (T*)(((uint64_t)hi << 32) | lo);
}
// The per-layer tables live in device memory and are reached through generic pointers, which
// the compiler must assume per-lane; their contents are the same for every lane.
__device__ __forceinline__ MatDev uni_mat(const MatDev& m) {
  MatDev r;
  r.w = uni_ptr(m.w);
  r.N = uni(m.N);
  r.K = uni(m.K);
  r.NRB = uni(m.NRB);
  r.KT = uni(m.KT);
  return r;
}
__device__ __forceinline__ LayerDev uni_layer(const LayerDev& l) {
  LayerDev r;
  r.qkv = uni_mat(l.qkv);
  r.o = uni_mat(l.o);
  r.gateup = uni_mat(l.gateup);
  r.down = uni_mat(l.down);
  r.attn_gain = uni_ptr(l.attn_gain);
  r.ffn_gain = uni_ptr(l.ffn_gain);
  return r;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}

template <int DT>
__device__ __forceinline__ void stream_init(WaveStream& S, const MatDev& M, int S_k, int wave) {
  const int wg = blockIdx.x, G = gridDim.x;
  constexpr int kTileBytes = DT == PI_DTYPE_BF16 ? 1024 : 2048;
  S.rsrc = make_rsrc(M.w, (uint32_t)M.NRB * (uint32_t)M.KT * kTileBytes);
  S.KT = M.KT;
  S.NRB = M.NRB;
  S.nt = uni(M.KT / S_k);
  S.slice = uni(wg % S_k);
  S.t0 = S.slice * S.nt;
  const int nwaves = uni((G / S_k) * kWaves);
  S.gw = uni((wg / S_k) * kWaves + wave);
  const int total = M.NRB * S.nt;
  S.share = uni((total + nwaves - 1) / nwaves);
  S.f0 = min(total, S.gw * S.share);
  S.f1 = min(total, S.f0 + S.share);
  S.lf = S.f0;
  S.lrb = uni(S.f0 / S.nt);
  S.lt = S.f0 - S.lrb * S.nt;
}

// The ring of outstanding weight tiles: UR tiles, each 1 KiB (bf16: one 16-byte load per lane)
// or 2 KiB (fp32: two loads per lane).  Slot indices are compile-time, so it lives in registers.
template <int DT, int UR>
struct Ring {
  static constexpr int U = UR;
  static constexpr int kTileBytes = DT == PI_DTYPE_BF16 ? 1024 : 2048;
  static constexpr int kRegs = DT == PI_DTYPE_BF16 ? UR : 2 * UR;
  u32x4 r[kRegs];
};

// Issue the load of the next tile of the wave's range into slot J.  Branch-free: past the end
// of the range every lane re-reads the first 16 bytes of the matrix (one cached line) and the
// consumer discards the slot, so the steady-state loop is a single basic block and the loads
// stay in flight (a branch around a load makes the compiler wait for it at the join).
template <int DT, int UR, int J>
__device__ __forceinline__ void ring_issue(Ring<DT, UR>& R, WaveStream& S, int lane) {
  const bool valid = S.lf < S.f1;
  const int soff = valid ? (S.lrb * S.KT + S.t0 + S.lt) * Ring<DT, UR>::kTileBytes : 0;
  const int voff = valid ? lane * 16 : 0;
  if constexpr (DT == PI_DTYPE_BF16) {
    R.r[J] = __builtin_amdgcn_raw_buffer_load_b128(S.rsrc, voff, soff, 2);
  } else {
    R.r[2 * J] = __builtin_amdgcn_raw_buffer_load_b128(S.rsrc, voff, soff, 2);
    R.r[2 * J + 1] = __builtin_amdgcn_raw_buffer_load_b128(S.rsrc, voff, soff + (valid ? 1024 : 0), 2);
  }
  S.lf += 1;
  const bool wrap = S.lt + 1 == S.nt;
  S.lt = wrap ? 0 : S.lt + 1;
  S.lrb += wrap ? 1 : 0;
}

template <int DT, int UR, int J = 0>
__device__ __forceinline__ void ring_prefetch(Ring<DT, UR>& R, WaveStream& S, int lane) {
  if constexpr (J < UR) {
    ring_issue<DT, UR, J>(R, S, lane);
    ring_prefetch<DT, UR, J + 1>(R, S, lane);
  }
}

// ---- activation staging (once per phase and workgroup) ---------------------------------------
// LDS slot (tt, g, i) holds x[i][32(t0+tt) + 8g + 0..7] (times the gain): bf16 model: 16 B of hi
// parts at the slot, 16 B of lo parts n_slots further; fp32 model: 32 B of floats.
template <int DT>
__device__ void stage_x(const float* xin, const float* gain, int K, int n, int t0, int nt, char* lds) {
  const int items = nt * n * 4;
  const int n_slots = nt * 4 * n;
  const __amdgpu_buffer_rsrc_t xr = rsrc_of(xin);
  for (int id = threadIdx.x; id < items; id += kThreads) {
    const int cl = id & 3;
    const int i = (id >> 2) % n;
    const int tt = (id >> 2) / n;
    const int k0 = (t0 + tt) * kKTile + cl * 8;
    float v[8];
    if (k0 < K) {
      const int off = (i * K + k0) * 4;
      const f32x4 p0 = ld_ag4(xr, off), p1 = ld_ag4(xr, off + 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) { v[j] = p0[j]; v[4 + j] = p1[j]; }
      if (gain) {
        const f32x4 g0 = *(gptr_f32x4)(gain + k0);
        const f32x4 g1 = *(gptr_f32x4)(gain + k0 + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) { v[j] *= g0[j]; v[4 + j] *= g1[j]; }
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

// 1/sqrt(mean x^2 + eps) per token from the per-16-column partial sums of squares, summed in a
// fixed order.  red: kThreads floats of LDS, rscale: 16 floats of LDS.  Ends with a barrier.
__device__ void compute_rscale(const float* ssq, int n_blocks, int K, float eps, float* red, float* rscale) {
  const int i = threadIdx.x & 15, b0 = threadIdx.x >> 4;
  constexpr int kGroups = kThreads / 16;
  float s = 0.0f;
  for (int b = b0; b < n_blocks; b += kGroups) s += ld_ag(ssq + b * 16 + i);
  red[b0 * 16 + i] = s;
  __syncthreads();
  if (threadIdx.x < 16) {
    float t = 0.0f;
    for (int b = 0; b < kGroups; ++b) t += red[b * 16 + threadIdx.x];
    rscale[threadIdx.x] = 1.0f / sqrtf(t / (float)K + eps);
  }
  __syncthreads();
}

// ---- epilogues --------------------------------------------------------------------------------
struct EpiCtx {
  int n;
  int N;               // logical rows of the matrix
  float* out;          // RESID: x[n][N] ; SWIGLU: a[n][N/2] ; LOGITS: logits[n][N] ; QKV: q[n][n_q_rows]
  float* ssq_out;      // RESID
  int n_q_rows, n_kv_rows, head_dim;
  char* kcache;        // this layer's K: [Hkv][cells][hd]
  char* vcache;
  int n_cells, kv_dtype;
  const int32_t* positions;
  const int32_t* slots;
  const float2* rope;
};

__device__ __forceinline__ void store_kv4(char* cache, int kv_dtype, size_t elem_idx, const float* v) {
  const __amdgpu_buffer_rsrc_t r = rsrc_of(cache);
  if (kv_dtype == PI_DTYPE_BF16) {
    u32x2 p = {(uint32_t)f32_to_bf16_rne(v[0]) | ((uint32_t)f32_to_bf16_rne(v[1]) << 16),
               (uint32_t)f32_to_bf16_rne(v[2]) | ((uint32_t)f32_to_bf16_rne(v[3]) << 16)};
    __builtin_amdgcn_raw_buffer_store_b64(p, r, (int)(elem_idx * 2), 0, kAgent);
  } else {
    st_ag4(r, (int)(elem_idx * 4), f32x4{v[0], v[1], v[2], v[3]});
  }
}

// The accumulator tile of a wave: lane l holds rows 16rb + 4(l>>4) + 0..3 for token l & 15.
template <int EPI>
__device__ __forceinline__ void epilogue(const EpiCtx& e, int rb, f32x4 acc, int lane, const float* rscale) {
  const int i = lane & 15, g = lane >> 4;
  const int row = rb * kRowBlock + g * 4;
  const bool live = i < e.n;
  if (EPI == EPI_QKV) {
    if (!live) return;
    const float r = rscale[i];
    float v[4] = {acc[0] * r, acc[1] * r, acc[2] * r, acc[3] * r};
    const int hd = e.head_dim;
    if (row < e.n_q_rows + e.n_kv_rows) {  // q or k: rotary embedding on adjacent pairs
      const int dim = row % hd;
      const float2* cs = e.rope + (size_t)e.positions[i] * (hd / 2) + dim / 2;
      const float2 c0 = cs[0], c1 = cs[1];
      const float a0 = v[0] * c0.x - v[1] * c0.y, a1 = v[0] * c0.y + v[1] * c0.x;
      const float a2 = v[2] * c1.x - v[3] * c1.y, a3 = v[2] * c1.y + v[3] * c1.x;
      v[0] = a0; v[1] = a1; v[2] = a2; v[3] = a3;
    }
    if (row < e.n_q_rows) {
      st_ag4(rsrc_of(e.out), (i * e.n_q_rows + row) * 4, f32x4{v[0], v[1], v[2], v[3]});
    } else if (row < e.n_q_rows + 2 * e.n_kv_rows) {
      const bool is_k = row < e.n_q_rows + e.n_kv_rows;
      const int kr = row - e.n_q_rows - (is_k ? 0 : e.n_kv_rows);
      const int head = kr / hd, dim = kr % hd;
      const size_t idx = ((size_t)head * e.n_cells + e.slots[i]) * hd + dim;
      store_kv4(is_k ? e.kcache : e.vcache, e.kv_dtype, idx, v);
    }
  } else if (EPI == EPI_RESID) {
    float s = 0.0f;
    if (live && row < e.N) {
      const __amdgpu_buffer_rsrc_t xr = rsrc_of(e.out);
      const int off = (i * e.N + row) * 4;
      const f32x4 x = ld_ag4(xr, off) + acc;
      st_ag4(xr, off, x);
      s = x[0] * x[0] + x[1] * x[1] + x[2] * x[2] + x[3] * x[3];
    }
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 32);
    if (g == 0) st_ag(e.ssq_out + rb * 16 + i, live ? s : 0.0f);
  } else if (EPI == EPI_SWIGLU) {
    if (!live || row >= e.N) return;
    const float r = rscale[i];
    const float g0 = acc[0] * r, u0 = acc[1] * r, g1 = acc[2] * r, u1 = acc[3] * r;
    st_ag2(rsrc_of(e.out), (i * (e.N / 2) + row / 2) * 4, g0 / (1.0f + expf(-g0)) * u0,
           g1 / (1.0f + expf(-g1)) * u1);
  } else {  // EPI_LOGITS: read by later kernels only
    if (!live || row >= e.N) return;
    const float r = rscale[i];
    *(float4*)(e.out + (size_t)i * e.N + row) = make_float4(acc[0] * r, acc[1] * r, acc[2] * r, acc[3] * r);
  }
}

// One wave has finished its part of row block rb (slice S.slice).  If other waves contribute to
// the row block, park the partial tile and count arrivals; the last arriver adds all partial
// tiles in a fixed order (slice-major, then wave order) and runs the epilogue.
template <int EPI>
__device__ __forceinline__ void flush_rowblock(const StageArgs& A, const WaveStream& S, int S_k, int rb,
                                               f32x4 acc, int lane, const EpiCtx& e, const float* rscale) {
  const int first = uni((rb * S.nt) / S.share);
  const int last = uni(((rb + 1) * S.nt - 1) / S.share);
  const int c = last - first + 1;  // contributors per slice (same for every slice)
  const int expected = c * S_k;
  if (expected > 1) {
    const int i = lane & 15;
    const int maxc = A.part_maxc;
    const __amdgpu_buffer_rsrc_t pr = rsrc_of(A.part);
    const int mine = (((S.slice * S.NRB + rb) * maxc + (S.gw - first)) * 64 + lane) * 16;
    if (i < e.n) st_ag4(pr, mine, acc);
    wave_drain();
    int old = 0;
    if (lane == 0)
      old = __hip_atomic_fetch_add(A.cnt + rb, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __shfl(old, 0);
    if (old != expected - 1) return;
    acc = f32x4{0.f, 0.f, 0.f, 0.f};
    if (i < e.n) {
      for (int s2 = 0; s2 < S_k; ++s2)
        for (int j = 0; j < c; ++j)
          acc += ld_ag4(pr, (((s2 * S.NRB + rb) * maxc + j) * 64 + lane) * 16);
    }
    if (lane == 0) __hip_atomic_store(A.cnt + rb, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  epilogue<EPI>(e, rb, acc, lane, rscale);
}

// ---- the MFMA inner step ----------------------------------------------------------------------
template <int DT, int UR, int J>
__device__ __forceinline__ void mma_tile(const Ring<DT, UR>& R, const char* lds, int n_slots, int bslot, f32x4& acc) {
  if constexpr (DT == PI_DTYPE_BF16) {
    const u32x4* b = (const u32x4*)lds + bslot;
    const bf16x8 av = __builtin_bit_cast(bf16x8, R.r[J]);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, b[0]), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, b[n_slots]), acc, 0, 0, 0);
  } else {
    const f32x4* b = (const f32x4*)lds + 2 * bslot;
    const f32x4 w0 = __builtin_bit_cast(f32x4, R.r[2 * J]), w1 = __builtin_bit_cast(f32x4, R.r[2 * J + 1]);
    const f32x4 x0 = b[0], x1 = b[1];
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(w0[q], x0[q], acc, 0, 0, 0);
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(w1[q], x1[q], acc, 0, 0, 0);
  }
}

struct ConsumeState {
  int f, rb, t;
  f32x4 acc;
  bool pending;
  int prb;
  f32x4 pacc;
};

// One pass over the ring, branch-free.  The host guarantees nt >= UR, so at most one row block
// ends inside a pass; its tile is set aside (pacc) and flushed after the pass.
template <int DT, int UR, int J>
__device__ __forceinline__ void consume_step(Ring<DT, UR>& R, WaveStream& S, ConsumeState& C, const char* lds,
                                             int n, int lane) {
  if constexpr (J < UR) {
    const bool valid = C.f < S.f1;
    const int g = lane >> 4, ln = min(lane & 15, n - 1);
    f32x4 acc2 = C.acc;
    mma_tile<DT, UR, J>(R, lds, S.nt * 4 * n, (C.t * 4 + g) * n + ln, acc2);
    ring_issue<DT, UR, J>(R, S, lane);
    const int t1 = C.t + 1;
    const bool end_rb = valid && t1 == S.nt;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float a = valid ? acc2[q] : C.acc[q];
      C.pacc[q] = end_rb ? a : C.pacc[q];
      C.acc[q] = end_rb ? 0.0f : a;
    }
    C.prb = end_rb ? C.rb : C.prb;
    C.pending = C.pending || end_rb;
    C.f += valid ? 1 : 0;
    C.t = end_rb ? 0 : (valid ? t1 : C.t);
    C.rb += end_rb ? 1 : 0;
    consume_step<DT, UR, J + 1>(R, S, C, lds, n, lane);
  }
}

// Stream this wave's range of the phase; the ring already holds its first tiles.
template <int DT, int UR, int EPI>
__device__ __forceinline__ void consume_phase(const StageArgs& A, Ring<DT, UR>& R, WaveStream& S, int S_k,
                                              const char* lds, int n, int lane, const EpiCtx& e,
                                              const float* rscale, const MatDev* next, int next_sk, int wave) {
  ConsumeState C;
  C.f = S.f0;
  C.rb = uni(S.f0 / S.nt);
  C.t = S.f0 - C.rb * S.nt;
  C.acc = f32x4{0.f, 0.f, 0.f, 0.f};
  C.pending = false;
  C.prb = 0;
  C.pacc = C.acc;
  while (C.f < S.f1) {
    do {  // hot loop: passes without a row-block end
      consume_step<DT, UR, 0>(R, S, C, lds, n, lane);
    } while (!C.pending && C.f < S.f1);
    if (C.pending) {
      flush_rowblock<EPI>(A, S, S_k, C.prb, C.pacc, lane, e, rscale);
      C.pending = false;
    }
  }
  // The ring is free: start the next phase's weight stream before the last (slow) flush, so HBM
  // stays busy while this wave waits on its reduction round trips and on the grid barrier.
  WaveStream Sn = S;
  if (next) {
    stream_init<DT>(Sn, *next, next_sk, wave);
    ring_prefetch<DT, UR>(R, Sn, lane);
  }
  if (C.t > 0) flush_rowblock<EPI>(A, S, S_k, C.rb, C.acc, lane, e, rscale);  // range ends inside a row block
  S = Sn;
}

// ---- attention phase ----------------------------------------------------------------------------
constexpr int kSC = 32;  // cells per sub-chunk
constexpr int kRT = 32;  // query rows per row tile

__device__ __forceinline__ void ld_cache8(const char* base, int dt, size_t elem, bool agent, float* out) {
  // 8 consecutive cache elements starting at `elem` (a multiple of 8)
  if (dt == PI_DTYPE_BF16) {
    uint32_t w[4];
    const uint32_t* p = (const uint32_t*)(base + elem * 2);
    if (agent) {
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = ld_ag_u32(p + j);
    } else {
      const uint4 q = *(const uint4*)p;
      w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      out[2 * j] = __uint_as_float(w[j] << 16);
      out[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
    }
  } else {
    const float* p = (const float*)base + elem;
    if (agent) {
#pragma unroll
      for (int j = 0; j < 8; ++j) out[j] = ld_ag(p + j);
    } else {
      const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
      out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
      out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
    }
  }
}

// One work unit = (kv head h, unit u): prefix cells [u*chunk, ...) and, for the last unit of a
// head, also the speculative window.  All G*n query rows of the kv head pass over the unit's
// cells in sub-chunks of 32 with a running (max, sum) softmax.
template <int HD>
__device__ void attn_unit(const StageArgs& A, const char* kl, const char* vl, int h, int u, char* lds_raw) {
  constexpr int KS = HD + 4;
  constexpr int PAIRS = HD / 2;
  constexpr int PV_GROUPS = kThreads / PAIRS;
  constexpr int PV_RPT = (kRT + PV_GROUPS - 1) / PV_GROUPS;
  constexpr int SC_GROUPS = kThreads / kSC;
  constexpr int SC_RPT = kRT / SC_GROUPS;
  float* Qs = (float*)lds_raw;        // [kRT][HD]
  float* Ks = Qs + kRT * HD;          // [kSC][KS]
  float* Vs = Ks + kSC * KS;          // [kSC][HD]
  float* Ps = Vs + kSC * HD;          // [kRT][kSC]
  float* m_s = Ps + kRT * kSC;        // [kRT]
  float* l_s = m_s + kRT;
  float* alpha_s = l_s + kRT;

  const int G = A.n_q_heads / A.n_kv_heads;
  const int R = G * A.n;
  const int upH = A.attn_units_per_head;
  const bool has_window = u == upH - 1;
  const int p_begin = min(A.prefix_len, u * A.attn_chunk);
  const int p_end = min(A.prefix_len, p_begin + A.attn_chunk);
  const int n_psub = (p_end - p_begin + kSC - 1) / kSC;
  const int w_end = min(A.window_base + PI_WINDOW, A.n_cells);
  const int n_wsub = has_window ? (w_end - A.window_base + kSC - 1) / kSC : 0;
  const float scale = 1.0f / sqrtf((float)HD);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t head_base = (size_t)h * A.n_cells * HD;

  for (int r0 = 0; r0 < R; r0 += kRT) {
    const int rows = min(kRT, R - r0);
    __syncthreads();
    for (int e = tid; e < kRT * (HD / 4); e += kThreads) {
      const int rr = e / (HD / 4), d4 = e % (HD / 4);
      float4 qv = make_float4(0.f, 0.f, 0.f, 0.f);
      if (rr < rows) {
        const int r = r0 + rr, gq = r / A.n, i = r % A.n;
        const float* pq = A.q + ((size_t)i * A.n_q_heads + h * G + gq) * HD + d4 * 4;
        qv = make_float4(ld_ag(pq) * scale, ld_ag(pq + 1) * scale, ld_ag(pq + 2) * scale, ld_ag(pq + 3) * scale);
      }
      *(float4*)(Qs + rr * HD + d4 * 4) = qv;
    }
    if (tid < kRT) { m_s[tid] = -INFINITY; l_s[tid] = 0.0f; }
    float acc[PV_RPT][2];
#pragma unroll
    for (int j = 0; j < PV_RPT; ++j) acc[j][0] = acc[j][1] = 0.0f;

    for (int sc = 0; sc < n_psub + n_wsub; ++sc) {
      const bool window = sc >= n_psub;
      const int c0 = window ? A.window_base + (sc - n_psub) * kSC : p_begin + sc * kSC;
      const int cend = window ? w_end : p_end;
      const int ncell = min(kSC, cend - c0);
      if (window) {  // skip window sub-chunks no query of this run can see
        uint64_t any = 0;
        for (int i = 0; i < A.n; ++i) any |= A.mask[i];
        const int sh = c0 - A.window_base;
        if (((any >> sh) & 0xffffffffull) == 0) continue;
      }
      __syncthreads();
      for (int e = tid; e < kSC * (HD / 8); e += kThreads) {
        const int cc = e / (HD / 8), d8 = (e % (HD / 8)) * 8;
        float kv[8], vv[8];
        if (cc < ncell) {
          const size_t idx = head_base + (size_t)(c0 + cc) * HD + d8;
          ld_cache8(kl, A.kv_dtype, idx, window, kv);
          ld_cache8(vl, A.kv_dtype, idx, window, vv);
        } else {
#pragma unroll
          for (int j = 0; j < 8; ++j) kv[j] = vv[j] = 0.0f;
        }
        *(float4*)(Ks + cc * KS + d8) = make_float4(kv[0], kv[1], kv[2], kv[3]);
        *(float4*)(Ks + cc * KS + d8 + 4) = make_float4(kv[4], kv[5], kv[6], kv[7]);
        *(float4*)(Vs + cc * HD + d8) = make_float4(vv[0], vv[1], vv[2], vv[3]);
        *(float4*)(Vs + cc * HD + d8 + 4) = make_float4(vv[4], vv[5], vv[6], vv[7]);
      }
      __syncthreads();
      {  // scores: thread = (cell, row group)
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
            const int i = (r0 + rr) % A.n;
            vis = (A.mask[i] >> (c0 + cc - A.window_base)) & 1ull;
          }
          Ps[rr * kSC + cc] = vis ? s[j] : -INFINITY;
        }
      }
      __syncthreads();
      for (int rr = wave; rr < kRT; rr += kWaves) {  // running softmax, one wave per row
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
      {  // O += P V : thread = (pair of head dims, row group)
        const int dp = tid % PAIRS, rg = tid / PAIRS;
#pragma unroll
        for (int j = 0; j < PV_RPT; ++j) {
          const int rr = rg + PV_GROUPS * j;
          const float al = rr < kRT ? alpha_s[rr] : 0.0f;
          acc[j][0] *= al;
          acc[j][1] *= al;
        }
        for (int cc = 0; cc < kSC; cc += 4) {
          float2 v[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] = *(const float2*)(Vs + (cc + q) * HD + 2 * dp);
#pragma unroll
          for (int j = 0; j < PV_RPT; ++j) {
            const int rr = rg + PV_GROUPS * j;
            if (rr < kRT) {
              const float4 p = *(const float4*)(Ps + rr * kSC + cc);
              acc[j][0] += p.x * v[0].x + p.y * v[1].x + p.z * v[2].x + p.w * v[3].x;
              acc[j][1] += p.x * v[0].y + p.y * v[1].y + p.z * v[2].y + p.w * v[3].y;
            }
          }
        }
      }
    }
    __syncthreads();
    {  // park this unit's partial result for the row tile
      const int dp = tid % PAIRS, rg = tid / PAIRS;
      const size_t ubase = ((size_t)h * upH + u) * R;
#pragma unroll
      for (int j = 0; j < PV_RPT; ++j) {
        const int rr = rg + PV_GROUPS * j;
        if (rr < rows) {
          float* po = A.attn_o + (ubase + r0 + rr) * HD + 2 * dp;
          st_ag(po, acc[j][0]);
          st_ag(po + 1, acc[j][1]);
        }
      }
      if (tid < rows) {
        st_ag(A.attn_ml + (ubase + r0 + tid) * 2, m_s[tid]);
        st_ag(A.attn_ml + (ubase + r0 + tid) * 2 + 1, l_s[tid]);
      }
    }
  }
  // arrival count of this kv head; the last unit merges all units of the head, in unit order
  wave_drain();
  __syncthreads();
  int* flag = (int*)(alpha_s + kRT);
  if (tid == 0) {
    const int old = __hip_atomic_fetch_add(A.attn_cnt + h, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *flag = old == upH - 1;
    if (old == upH - 1) __hip_atomic_store(A.attn_cnt + h, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (*flag) {
    for (int e = tid; e < R * HD; e += kThreads) {
      const int r = e / HD, d = e % HD;
      const size_t hb = (size_t)h * upH;
      float M = -INFINITY;
      for (int uu = 0; uu < upH; ++uu) M = fmaxf(M, ld_ag(A.attn_ml + ((hb + uu) * R + r) * 2));
      float L = 0.0f, o = 0.0f;
      for (int uu = 0; uu < upH; ++uu) {
        const float m = ld_ag(A.attn_ml + ((hb + uu) * R + r) * 2);
        if (m == -INFINITY) continue;
        const float w = expf(m - M);
        L += w * ld_ag(A.attn_ml + ((hb + uu) * R + r) * 2 + 1);
        o += w * ld_ag(A.attn_o + ((hb + uu) * R + r) * HD + d);
      }
      const int gq = r / A.n, i = r % A.n;
      st_ag(A.o + ((size_t)i * A.n_q_heads + h * G + gq) * HD + d, o / L);
    }
  }
}

__device__ void attention_phase(const StageArgs& A, const char* kl, const char* vl, char* lds) {
  const int units = A.n_kv_heads * A.attn_units_per_head;
  for (int w = blockIdx.x; w < units; w += gridDim.x) {
    const int h = w / A.attn_units_per_head, u = w % A.attn_units_per_head;
    switch (A.head_dim) {
      case 32: attn_unit<32>(A, kl, vl, h, u, lds); break;
      case 64: attn_unit<64>(A, kl, vl, h, u, lds); break;
      default: attn_unit<128>(A, kl, vl, h, u, lds); break;
    }
  }
}

// ---- stage input / output ---------------------------------------------------------------------
__device__ void embed_phase(const StageArgs& A) {
  const int per_row = A.d / 4;
  const int total = A.n * per_row;
  const int stride = gridDim.x * kThreads;
  for (int base = 0; base < total; base += stride) {
    const int idx = base + blockIdx.x * kThreads + threadIdx.x;
    const bool live = idx < total;
    const int i = live ? idx / per_row : 0, c = live ? (idx % per_row) * 4 : 0;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (live) {
      if (A.layer_begin > 0) {
        const float4 t = *(const float4*)(A.hidden_in + (size_t)i * A.d + c);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
      } else {
        int tok = A.tokens[i];
        tok = tok < 0 ? 0 : (tok >= A.vocab ? A.vocab - 1 : tok);
        if (A.dtype == PI_DTYPE_BF16) {
          const uint2 p = *(const uint2*)((const uint16_t*)A.embed + (size_t)tok * A.d + c);
          v[0] = __uint_as_float(p.x << 16); v[1] = __uint_as_float(p.x & 0xffff0000u);
          v[2] = __uint_as_float(p.y << 16); v[3] = __uint_as_float(p.y & 0xffff0000u);
        } else {
          const float4 t = *(const float4*)((const float*)A.embed + (size_t)tok * A.d + c);
          v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
        }
      }
      st_ag4(rsrc_of(A.x), (i * A.d + c) * 4, f32x4{v[0], v[1], v[2], v[3]});
    }
    float s = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    s += __shfl_xor(s, 1);
    s += __shfl_xor(s, 2);
    if (live && (threadIdx.x & 3) == 0) st_ag(A.ssq + (c / 16) * 16 + i, s);
  }
  wave_drain();
}

__device__ void hidden_out_phase(const StageArgs& A) {
  const int total = A.n * A.d;
  for (int idx = blockIdx.x * kThreads + threadIdx.x; idx < total; idx += gridDim.x * kThreads)
    A.hidden_out[idx] = ld_ag(A.x + idx);
}

// ---- one projection phase: stage activations, stream, flush ----------------------------------------
template <int DT, int UR, int EPI>
__device__ __forceinline__ void proj_phase(const StageArgs& A, Ring<DT, UR>& R, WaveStream& S, int S_k,
                                           const float* xin, const float* gain, bool scaled, int K,
                                           const EpiCtx& e, char* lds, int lane, const MatDev* next, int next_sk,
                                           int wave, int trace_layer = -1) {
  const size_t xbytes = (size_t)S.nt * 128 * A.n;
  float* red = (float*)(lds + xbytes);
  float* rscale = red + kThreads;
  stage_x<DT>(xin, gain, K, A.n, S.t0, S.nt, lds);
  if (scaled) {
    compute_rscale(A.ssq, A.d / 16, K, A.eps, red, rscale);
  } else {
    __syncthreads();
  }
  wg_mark(A, trace_layer, 1);
  consume_phase<DT, UR, EPI>(A, R, S, S_k, lds, A.n, lane, e, rscale, next, next_sk, wave);
  wg_mark(A, trace_layer, 2);
  wave_drain();
}

template <int DT, int UR>
__global__ void __launch_bounds__(kThreads, 1) stage_kernel(const StageArgs A) {
  extern __shared__ __align__(16) char lds[];
  __shared__ int bar_sh[2];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform: keep it scalar
  BarrierCtx bc;
  bc.epoch = A.epoch_base;
  bc.sh = bar_sh;
  const int L = A.n_layers;

  // run latch: validate the run's slots, probe the cancel flag once
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    int status = PI_OK, dead = 0;
    const int len = *A.kv_len;
    for (int i = 0; i < A.n; ++i) {
      const int s = A.slots[i];
      if (s < len || s < A.window_base || s >= A.window_base + PI_WINDOW || s >= A.n_cells) {
        status = PI_E_SLOT_LIVE;
        dead = 1;
      }
    }
    if (!dead && A.cancel_flag &&
        __hip_atomic_load(A.cancel_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != 0) {
      status = PI_CANCELLED;
      dead = 1;
    }
    __hip_atomic_store(&A.rs->status, status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&A.rs->dead, dead, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&A.rs->layers_done, A.layer_begin, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    wave_drain();
  }
  Ring<DT, UR> R;
  WaveStream S;
  bool ok = grid_barrier(A, bc, A.layer_begin, false);
  bool dead = __builtin_amdgcn_readfirstlane(bar_sh[1]) != 0;
  if (ok && !dead) {
    embed_phase(A);
    stream_init<DT>(S, uni_mat(A.layers[A.layer_begin].qkv), A.sk[0], wave);
    ring_prefetch<DT, UR>(R, S, lane);
    ok = grid_barrier(A, bc, -1, false);
  }
  for (int l = A.layer_begin; ok && !dead && l < A.layer_end; ++l) {
    const LayerDev W = uni_layer(A.layers[l]);
    EpiCtx e;
    e.n = A.n;
    e.n_q_rows = A.n_q_heads * A.head_dim;
    e.n_kv_rows = A.n_kv_heads * A.head_dim;
    e.head_dim = A.head_dim;
    e.kcache = A.kbase + (size_t)l * A.kv_layer_bytes;
    e.vcache = A.vbase + (size_t)l * A.kv_layer_bytes;
    e.n_cells = A.n_cells;
    e.kv_dtype = A.kv_dtype;
    e.positions = A.positions;
    e.slots = A.slots;
    e.rope = A.rope;
    e.ssq_out = A.ssq;
    // RMSNorm + QKV projection + RoPE + KV write
    e.N = W.qkv.N;
    e.out = A.q;
    proj_phase<DT, UR, EPI_QKV>(A, R, S, A.sk[0], A.x, W.attn_gain, true, A.d, e, lds, lane, nullptr, 0, wave);
    if (!(ok = grid_barrier(A, bc, -1, false))) break;
    // attention
    attention_phase(A, e.kcache, e.vcache, lds);
    stream_init<DT>(S, W.o, A.sk[1], wave);
    ring_prefetch<DT, UR>(R, S, lane);
    if (!(ok = grid_barrier(A, bc, -1, false))) break;
    // output projection + residual
    e.N = W.o.N;
    e.out = A.x;
    proj_phase<DT, UR, EPI_RESID>(A, R, S, A.sk[1], A.o, nullptr, false, W.o.K, e, lds, lane, &W.gateup, A.sk[2],
                                  wave);
    if (!(ok = grid_barrier(A, bc, -1, false))) break;
    // RMSNorm + gate/up + SwiGLU
    e.N = W.gateup.N;
    e.out = A.a;
    wg_mark(A, l, 0);
    proj_phase<DT, UR, EPI_SWIGLU>(A, R, S, A.sk[2], A.x, W.ffn_gain, true, A.d, e, lds, lane, &W.down, A.sk[3],
                                   wave, l);
    wg_mark(A, l, 3);
    wg_mark(A, l, 4);
    if (!(ok = grid_barrier(A, bc, -1, false))) break;
    wg_mark(A, l, 5);
    // down projection + residual
    e.N = W.down.N;
    e.out = A.x;
    {
      MatDev nxt = A.lm_head;
      int nsk = A.sk[4];
      bool has_next = A.layer_end == L;
      if (l + 1 < A.layer_end) {
        nxt = uni_mat(A.layers[l + 1].qkv);
        nsk = A.sk[0];
        has_next = true;
      }
      proj_phase<DT, UR, EPI_RESID>(A, R, S, A.sk[3], A.a, nullptr, false, W.down.K, e, lds, lane,
                                    has_next ? &nxt : nullptr, nsk, wave);
    }
    // layer boundary: record progress; probe the cancel flag unless the stage is complete
    if (!(ok = grid_barrier(A, bc, l + 1, l + 1 < A.layer_end))) break;
    dead = __builtin_amdgcn_readfirstlane(bar_sh[1]) != 0;
  }
  if (ok && !dead) {
    if (A.layer_end == L) {  // final RMSNorm + LM head
      EpiCtx e;
      e.n = A.n;
      e.N = A.lm_head.N;
      e.out = A.logits_out;
      proj_phase<DT, UR, EPI_LOGITS>(A, R, S, A.sk[4], A.x, A.final_gain, true, A.d, e, lds, lane, nullptr, 0, wave);
    } else {
      hidden_out_phase(A);
    }
  }
  // Exit: the last workgroup to leave re-arms the barrier for the next launch and reports.
  __syncthreads();
  if (threadIdx.x == 0) {
    StageSync* sy = A.sync;
    const unsigned old = __hip_atomic_fetch_add(&sy->exited, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == gridDim.x - 1) {
      const unsigned aborted = __hip_atomic_load(&sy->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (A.run_status) {
        A.run_status[0] = aborted ? PI_E_HIP
                                  : __hip_atomic_load(&A.rs->status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        A.run_status[1] = __hip_atomic_load(&A.rs->layers_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __hip_atomic_store(&sy->exited, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

}  // namespace

size_t attn_lds_bytes(int head_dim) {
  return ((size_t)kRT * head_dim + (size_t)kSC * (head_dim + 4) + (size_t)kSC * head_dim + (size_t)kRT * kSC +
          3 * kRT + 4) * sizeof(float);
}

size_t stage_proj_lds_bytes(int n, int nt) { return (size_t)nt * 128 * n + (kStageThreads + 16) * sizeof(float); }

namespace {
const void* stage_fn(int dtype, int ring) {
  if (dtype == PI_DTYPE_BF16) {
    if (ring == 16) return (const void*)stage_kernel<PI_DTYPE_BF16, 16>;
    if (ring == 8) return (const void*)stage_kernel<PI_DTYPE_BF16, 8>;
    return (const void*)stage_kernel<PI_DTYPE_BF16, 4>;
  }
  if (ring == 8) return (const void*)stage_kernel<PI_DTYPE_F32, 8>;
  return (const void*)stage_kernel<PI_DTYPE_F32, 4>;
}
}  // namespace

int stage_ring_size(int dtype, int min_nt) {
  if (dtype == PI_DTYPE_BF16 && min_nt >= 16) return 16;
  if (min_nt >= 8) return 8;
  return min_nt >= 4 ? 4 : 0;
}

hipError_t stage_configure(int dtype, int ring, size_t max_lds, int* max_blocks_per_cu) {
  const void* fn = stage_fn(dtype, ring);
  hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_lds);
  if (e != hipSuccess) return e;
  return hipOccupancyMaxActiveBlocksPerMultiprocessor(max_blocks_per_cu, fn, kStageThreads, max_lds);
}

hipError_t launch_stage(const StageArgs& a, int dtype, int ring, int grid, size_t lds, hipStream_t s) {
  StageArgs args = a;
  void* params[] = {(void*)&args};
  return hipLaunchKernel(stage_fn(dtype, ring), dim3((unsigned)grid), dim3(kStageThreads), params, lds, s);
}

}  // namespace pi
