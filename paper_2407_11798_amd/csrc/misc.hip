// Kernels beside the stage kernel: greedy verification (argmax + tree walk), KV
// commit/rollback, KV cell set/get.
#include <mutex>

#include "pi_internal.h"

namespace pi {
namespace {

// Scratch of the verification entry point that allocates nothing: per logits row the largest value
// and its index, and the counter by which the last block to finish is found.  One copy per GPU
// the library runs on, held until the process ends.
constexpr int kScratchBytes = 256;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
static_assert(PI_MAX_BATCH * (sizeof(float) + sizeof(int32_t)) + sizeof(int) <= kScratchBytes, "scratch too small");

__global__ void clear_counter_kernel(int* cnt) { *cnt = 0; }

// ---- greedy verification -------------------------------------------------------------------
// One block per logits row finds argmax (lowest id on ties); the last block to finish walks
// the tree.  Chained form: the expectation for the root comes from the result of the run this
// one builds on, and counts only if that run was accepted whole and this run's forward ran to
// its end; otherwise nothing is accepted and the bonus token is -1.
__global__ void __launch_bounds__(256) verify_kernel(const int32_t* draft, const int32_t* parent, int n,
                                                     const float* logits, int vocab, int root_expected,
                                                     const int32_t* prev_result, int prev_n, const int32_t* run_status,
                                                     int32_t* accepted, int32_t* result,
                                                     float* best_val, int32_t* best_idx, int* cnt) {
  __shared__ float sv[4];
  __shared__ int si[4];
  __shared__ int last;
  const int row = blockIdx.x;
  const float* lg = logits + (size_t)row * vocab;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  // 16 bytes per load, four loads in flight per thread (the scan is a chain of memory round trips
  // otherwise); rows start 16-byte aligned when the vocabulary is a multiple of four
  const auto take = [&](float f, int v) {
    if (f > bv || (f == bv && v < bi)) { bv = f; bi = v; }
  };
  int v0 = 0;
  if ((vocab & 3) == 0 && ((size_t)lg & 15) == 0) {
    const float4* lg4 = (const float4*)lg;
    const int quads = vocab >> 2, step = blockDim.x;
    int q = threadIdx.x;
    for (; q + 3 * step < quads; q += 4 * step) {
      float4 t[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) t[k] = lg4[q + k * step];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int v = (q + k * step) * 4;
        take(t[k].x, v); take(t[k].y, v + 1); take(t[k].z, v + 2); take(t[k].w, v + 3);
      }
    }
    for (; q < quads; q += step) {
      const float4 t = lg4[q];
      take(t.x, q * 4); take(t.y, q * 4 + 1); take(t.z, q * 4 + 2); take(t.w, q * 4 + 3);
    }
    v0 = vocab;
  }
  for (int v = v0 + threadIdx.x; v < vocab; v += blockDim.x) take(lg[v], v);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const float ov = __shfl_xor(bv, o);
    const int oi = __shfl_xor(bi, o);
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w)
      if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; }
    best_val[row] = bv;
    best_idx[row] = bi;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    const int old = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    last = old == n - 1;
    if (last) {
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      *cnt = 0;
      int u = -1, expected = root_expected, a = 0;
      bool none = run_status && run_status[0] != PI_OK;
      if (prev_result) {
        none = none || prev_result[0] != prev_n;
        expected = prev_result[1];
      }
      if (none) expected = -1;
      while (!none) {
        int nxt = -1;
        for (int c = 0; c < n; ++c) {
          const int p = parent ? parent[c] : c - 1;
          if (p == u && draft[c] == expected) { nxt = c; break; }
        }
        if (nxt < 0) break;
        accepted[a++] = nxt;
        u = nxt;
        expected = __hip_atomic_load(best_idx + nxt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      for (int j = a; j < n; ++j) accepted[j] = -1;
      result[0] = a;
      result[1] = expected;
    }
  }
}

// ---- KV commit / rollback ------------------------------------------------------------------
// One thread per (layer, kv head, 16-byte piece of a cell row), for K and V: gather the
// accepted path's pieces, zero every slot of the run, then write the path to cells
// kv_len .. kv_len+a-1.  All of a thread's reads precede its writes and threads touch
// disjoint columns, so overlapping source and destination cells are safe.
// The slots and the verification result are device data the host never saw, and this kernel may
// be queued right behind a forward that refused them: only cells of [kv_len, n_cells) are ever
// read as a source or zero-filled (a slot outside is skipped: it is a live canonical cell, or no
// cell at all), the accepted count is cut at the first entry that does not name a token of the run
// whose slot is such a cell, and at what still fits below n_cells.  Every thread takes these
// decisions from the same words, so all agree.
__global__ void __launch_bounds__(256) rollback_kernel(char* kbuf, char* vbuf, int elem_size,
                                                       int n_layers, int n_kv_heads, int n_cells,
                                                       int head_dim, const int32_t* slots, int n,
                                                       const int32_t* accepted, const int32_t* result,
                                                       int32_t* kv_len, int* cnt) {
  const int pieces = head_dim * elem_size / 16;
  const size_t total = (size_t)n_layers * n_kv_heads * pieces * 2;
  const int len = *kv_len;
  int a = result ? result[0] : 0;
  a = a < 0 ? 0 : (a > n ? n : a);
  if (a > n_cells - len) a = n_cells - len > 0 ? n_cells - len : 0;
  int src[PI_MAX_BATCH];
#pragma unroll
  for (int j = 0; j < PI_MAX_BATCH; ++j) {
    src[j] = -1;
    if (j < a) {
      const int node = accepted[j];
      const int s = node >= 0 && node < n ? slots[node] : -1;
      if (s >= len && s < n_cells) src[j] = s;
      else a = j;  // the path ends before the first entry that cannot be committed
    }
  }
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < total) {
    const int which = (int)(idx & 1);
    size_t r = idx >> 1;
    const int piece = (int)(r % pieces);
    r /= pieces;
    const size_t lh = r;  // layer * n_kv_heads + head
    char* base = (which ? vbuf : kbuf) + lh * (size_t)n_cells * head_dim * elem_size + (size_t)piece * 16;
    const size_t cell_stride = (size_t)head_dim * elem_size;
    uint4 keep[PI_MAX_BATCH];
#pragma unroll
    for (int j = 0; j < PI_MAX_BATCH; ++j)
      if (j < a) keep[j] = *(const uint4*)(base + (size_t)src[j] * cell_stride);
    for (int i = 0; i < n; ++i) {
      const int s = slots[i];
      if (s >= len && s < n_cells) *(uint4*)(base + (size_t)s * cell_stride) = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < PI_MAX_BATCH; ++j)
      if (j < a) *(uint4*)(base + (size_t)(len + j) * cell_stride) = keep[j];
  }
  // the last block to finish publishes the new canonical length
  __shared__ int last;
  __syncthreads();
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    last = old == (int)gridDim.x - 1;
    if (last) {
      *cnt = 0;
      *kv_len = len + a;
    }
  }
}

// ---- KV cell set / get (prefill and read-back; not on the hot path) -------------------------
__global__ void __launch_bounds__(256) kv_set_kernel(char* kbuf, char* vbuf, int kv_dtype, int n_kv_heads,
                                                     int n_cells, int head_dim, int layer, int cell_begin,
                                                     int n, const void* ksrc, const void* vsrc, int src_dtype) {
  const size_t total = (size_t)n * n_kv_heads * head_dim;
  const int es = kv_dtype == PI_DTYPE_BF16 ? 2 : 4;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
    const int d = (int)(e % head_dim);
    const int h = (int)((e / head_dim) % n_kv_heads);
    const int c = (int)(e / ((size_t)head_dim * n_kv_heads));
    const size_t dst = (((size_t)layer * n_kv_heads + h) * n_cells + cell_begin + c) * head_dim + d;
    for (int which = 0; which < 2; ++which) {
      const void* src = which ? vsrc : ksrc;
      char* buf = which ? vbuf : kbuf;
      const float f = src_dtype == PI_DTYPE_BF16 ? bf16_to_f32(((const uint16_t*)src)[e]) : ((const float*)src)[e];
      if (es == 2) ((uint16_t*)buf)[dst] = f32_to_bf16_rne(f);
      else ((float*)buf)[dst] = f;
    }
  }
}

__global__ void __launch_bounds__(256) kv_get_kernel(const char* kbuf, const char* vbuf, int kv_dtype,
                                                     int n_kv_heads, int n_cells, int head_dim, int layer,
                                                     int cell_begin, int n, float* kdst, float* vdst) {
  const size_t total = (size_t)n * n_kv_heads * head_dim;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
    const int d = (int)(e % head_dim);
    const int h = (int)((e / head_dim) % n_kv_heads);
    const int c = (int)(e / ((size_t)head_dim * n_kv_heads));
    const size_t src = (((size_t)layer * n_kv_heads + h) * n_cells + cell_begin + c) * head_dim + d;
    if (kv_dtype == PI_DTYPE_BF16) {
      kdst[e] = bf16_to_f32(((const uint16_t*)kbuf)[src]);
      vdst[e] = bf16_to_f32(((const uint16_t*)vbuf)[src]);
    } else {
      kdst[e] = ((const float*)kbuf)[src];
      vdst[e] = ((const float*)vbuf)[src];
    }
  }
}

}  // namespace

hipError_t launch_verify(const int32_t* draft, const int32_t* parent, int n, const float* logits,
                         int vocab, int root_expected, const int32_t* prev_result, int prev_n,
                         const int32_t* run_status, int32_t* accepted, int32_t* result,
                         float* best_val, int32_t* best_idx, int* cnt, hipStream_t s) {
  verify_kernel<<<dim3((unsigned)n), dim3(256), 0, s>>>(draft, parent, n, logits, vocab, root_expected, prev_result,
                                                        prev_n, run_status, accepted, result, best_val, best_idx, cnt);
  return hipGetLastError();
}

hipError_t launch_rollback(void* k, void* v, int kv_dtype, int n_layers, int n_kv_heads, int n_cells,
                           int head_dim, const int32_t* slots, int n, const int32_t* accepted,
                           const int32_t* result, int32_t* kv_len, int* cnt, hipStream_t s) {
  const int es = kv_dtype == PI_DTYPE_BF16 ? 2 : 4;
  const size_t total = (size_t)n_layers * n_kv_heads * (head_dim * es / 16) * 2;
  rollback_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(
      (char*)k, (char*)v, es, n_layers, n_kv_heads, n_cells, head_dim, slots, n, accepted, result, kv_len, cnt);
  return hipGetLastError();
}

hipError_t launch_kv_set(void* k, void* v, int kv_dtype, int n_kv_heads, int n_cells, int head_dim,
                         int layer, int cell_begin, int n, const void* ksrc, const void* vsrc,
                         int src_dtype, hipStream_t s) {
  const size_t total = (size_t)n * n_kv_heads * head_dim;
  size_t blocks = (total + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  kv_set_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>((char*)k, (char*)v, kv_dtype, n_kv_heads, n_cells,
                                                             head_dim, layer, cell_begin, n, ksrc, vsrc, src_dtype);
  return hipGetLastError();
}

hipError_t launch_kv_get(const void* k, const void* v, int kv_dtype, int n_kv_heads, int n_cells,
                         int head_dim, int layer, int cell_begin, int n, float* kdst, float* vdst,
                         hipStream_t s) {
  const size_t total = (size_t)n * n_kv_heads * head_dim;
  size_t blocks = (total + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  kv_get_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const char*)k, (const char*)v, kv_dtype, n_kv_heads,
                                                             n_cells, head_dim, layer, cell_begin, n, kdst, vdst);
  return hipGetLastError();
}

}  // namespace pi

// The scratch array's address on each device, looked up once per device with that device current.
// (In host code the array's name is only a handle for this lookup, never a device address.)
namespace {
constexpr int kMaxDevices = 16;
struct ScratchAddr {
  unsigned char* ptr = nullptr;
  hipError_t err = hipSuccess;
  bool looked_up = false;
};
ScratchAddr g_scratch[kMaxDevices];
std::mutex g_scratch_mutex;
}  // namespace

extern "C" int32_t pi_verify_greedy_noalloc(const int32_t* draft, const int32_t* parent, int32_t n, const float* logits,
                                            int32_t vocab, int32_t root_expected, int32_t* accepted_nodes,
                                            int32_t* result, void* stream) {
  using namespace pi;
  if (!draft || !logits || !accepted_nodes || !result) return PI_E_ARG;
  if (n < 1 || n > PI_MAX_BATCH || vocab < 1 || vocab > (1 << 24)) return PI_E_SHAPE;  // more rows than the scratch array holds
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return PI_E_HIP;
  if (dev < 0 || dev >= kMaxDevices) return PI_E_SHAPE;
  ScratchAddr& sa = g_scratch[dev];
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!sa.looked_up) {
      void* p = nullptr;
      sa.err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      sa.ptr = (unsigned char*)p;
      sa.looked_up = true;
    }
  }
  if (sa.err != hipSuccess || !sa.ptr) return PI_E_HIP;
  float* best_val = (float*)sa.ptr;
  int32_t* best_idx = (int32_t*)(sa.ptr + PI_MAX_BATCH * sizeof(float));
  int* cnt = (int*)(sa.ptr + PI_MAX_BATCH * (sizeof(float) + sizeof(int32_t)));
  // the array keeps what the last call left: the counter must start at zero (a fill kernel, not a
  // memset node, so that the call can be captured into a graph)
  clear_counter_kernel<<<dim3(1), dim3(1), 0, (hipStream_t)stream>>>(cnt);
  e = hipGetLastError();
  if (e != hipSuccess) return PI_E_HIP;
  e = launch_verify(draft, parent, n, logits, vocab, root_expected, nullptr, 0, nullptr, accepted_nodes, result, best_val,
                    best_idx, cnt, (hipStream_t)stream);
  return e == hipSuccess ? PI_OK : PI_E_HIP;
}
