// KV cell metadata and sequence partitions (Sections "KV Cache" and "Pipelined KV Cache
// Multibuffering"): a device-resident table of (position, sequence set) per cache cell, edited
// by small kernels in stream order, the attention-mask builder that reads it, and compaction.
// The queue of free sequence identifiers is the only host state.
#include <deque>
#include <new>
#include <vector>

#include "pi_internal.h"

using namespace pi;

struct pi_kvmeta {
  int n_cells = 0, n_seq = 0;
  uint32_t all = 0;          // every sequence of this table
  int32_t* pos = nullptr;    // [n_cells], -1 = free
  uint32_t* seq = nullptr;   // [n_cells], bit s = sequence s
  int32_t* plan = nullptr;   // compaction: [0] number of moves, [1 + k] source cell of move k
  int* work = nullptr;       // mask builder: [0] pairs counted so far, [1] workgroups done
  std::deque<int> free_ids;  // FIFO of free partition identifiers
  std::vector<char> held;
};

namespace {

constexpr int kThreads = 256;
constexpr int kMaskBlocks = 64;

int32_t hip_status(hipError_t e) {
  if (e == hipSuccess) return PI_OK;
  return e == hipErrorOutOfMemory ? PI_E_OOM : PI_E_HIP;
}

unsigned blocks_for(int n) { return (unsigned)((n + kThreads - 1) / kThreads); }

__global__ void __launch_bounds__(kThreads) meta_fill_kernel(int32_t* pos, uint32_t* seq, int cell0, int n,
                                                             int pos0, uint32_t mask) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i < n) {
    pos[cell0 + i] = mask ? pos0 + i : -1;
    seq[cell0 + i] = mask;
  }
}

// bit leaves every cell that is not canonical
__global__ void __launch_bounds__(kThreads) meta_release_kernel(int32_t* pos, uint32_t* seq, int n_cells,
                                                                uint32_t bit) {
  const int c = blockIdx.x * kThreads + threadIdx.x;
  if (c >= n_cells) return;
  const uint32_t s = seq[c];
  if ((s & bit) && !(s & 1u)) {
    const uint32_t t = s & ~bit;
    seq[c] = t;
    if (!t) pos[c] = -1;
  }
}

__global__ void __launch_bounds__(kThreads) meta_cp_kernel(const int32_t* pos, uint32_t* seq, int n_cells,
                                                           uint32_t src_bit, uint32_t dst_mask, int p0, int p1) {
  const int c = blockIdx.x * kThreads + threadIdx.x;
  if (c >= n_cells) return;
  const uint32_t s = seq[c];
  const int p = pos[c];
  if ((s & src_bit) && p >= p0 && p < p1) seq[c] = s | dst_mask;
}

__global__ void __launch_bounds__(kThreads) meta_rm_kernel(int32_t* pos, uint32_t* seq, int n_cells, uint32_t mask,
                                                           int p0, int p1) {
  const int c = blockIdx.x * kThreads + threadIdx.x;
  if (c >= n_cells) return;
  const int p = pos[c];
  if (p >= 0 && p >= p0 && p < p1) {
    const uint32_t t = seq[c] & ~mask;
    seq[c] = t;
    if (!t) pos[c] = -1;
  }
}

// The accepted count and path are device data, so source sequence and position bound are
// worked out here (by every thread alike) before the copy.
__global__ void __launch_bounds__(kThreads) meta_accept_kernel(const int32_t* pos, uint32_t* seq, int n_cells, int n,
                                                               const int32_t* positions, const uint32_t* tok_seq,
                                                               const int32_t* accepted, const int32_t* result,
                                                               uint32_t all) {
  const int c = blockIdx.x * kThreads + threadIdx.x;
  const int a = min(result[0], n);
  if (a <= 0 || c >= n_cells) return;
  const int last = accepted[a - 1];
  if (last < 0 || last >= n) return;
  const uint32_t ts = tok_seq[last] & all;
  if (!ts) return;
  const uint32_t src_bit = ts & (0u - ts);  // lowest sequence of the token
  const int p1 = positions[last];           // inclusive bound
  const uint32_t s = seq[c];
  const int p = pos[c];
  if ((s & src_bit) && p >= 0 && p <= p1) seq[c] = s | all;
}

// One wave: lane c looks at window cell window_base + c; the ballot of free lanes is the free
// map, and a free lane's rank in it is the token it receives.
__global__ void __launch_bounds__(kWave) meta_place_kernel(int32_t* pos, uint32_t* seq, int n_cells, int n,
                                                           const int32_t* positions, const uint32_t* tok_seq,
                                                           int window_base, uint32_t all, int32_t* slots_out,
                                                           int32_t* status) {
  const int lane = threadIdx.x;
  const int cell = window_base + lane;
  const bool is_free = cell < n_cells && pos[cell] < 0;
  const unsigned long long free_map = __builtin_amdgcn_ballot_w64(is_free);
  bool bad_tok = false;
  if (lane < n) bad_tok = positions[lane] < 0 || (tok_seq[lane] & all) == 0 || (tok_seq[lane] & ~all) != 0;
  const bool bad_arg = __builtin_amdgcn_ballot_w64(bad_tok) != 0;
  const bool ok = !bad_arg && __builtin_popcountll(free_map) >= n;
  const int rank = __builtin_popcountll(free_map & ((1ull << lane) - 1ull));
  if (ok) {
    if (is_free && rank < n) {
      pos[cell] = positions[rank];
      seq[cell] = tok_seq[rank];
      slots_out[rank] = cell;
    }
  } else if (lane < n) {
    slots_out[lane] = -1;
  }
  if (lane == 0) status[0] = ok ? PI_OK : (bad_arg ? PI_E_ARG : PI_E_FULL);
}

// Window words by ballot (wave 0 of workgroup 0: lane = window cell), and the count of pairs
// that "dense prefix + window word" cannot express, summed over workgroups in integers; the
// last workgroup to finish publishes the count and clears the counters for the next call.
__global__ void __launch_bounds__(kThreads) meta_mask_kernel(const int32_t* pos, const uint32_t* seq, int n_cells,
                                                             int n, const int32_t* positions, const uint32_t* tok_seq,
                                                             int prefix_len, int window_base, unsigned long long* mask_out,
                                                             int32_t* n_unexpressed, int* work) {
  __shared__ int tok_pos[PI_MAX_BATCH];
  __shared__ uint32_t tok_s[PI_MAX_BATCH];
  __shared__ int block_bad;
  if (threadIdx.x < n) {
    tok_pos[threadIdx.x] = positions[threadIdx.x];
    tok_s[threadIdx.x] = tok_seq[threadIdx.x];
  }
  if (threadIdx.x == 0) block_bad = 0;
  __syncthreads();
  if (blockIdx.x == 0 && threadIdx.x < kWave) {
    const int cell = window_base + (int)threadIdx.x;
    const bool in_range = cell >= prefix_len && cell < n_cells;
    const int p = in_range ? pos[cell] : -1;
    const uint32_t s = in_range ? seq[cell] : 0u;
    for (int i = 0; i < n; ++i) {
      const unsigned long long word = __builtin_amdgcn_ballot_w64((s & tok_s[i]) != 0 && p <= tok_pos[i]);
      if (threadIdx.x == 0) mask_out[i] = word;
    }
  }
  int bad = 0;
  for (int c = blockIdx.x * kThreads + threadIdx.x; c < n_cells; c += gridDim.x * kThreads) {
    const bool in_prefix = c < prefix_len;
    if (!in_prefix && c >= window_base && c < window_base + PI_WINDOW) continue;
    const int p = pos[c];
    const uint32_t s = seq[c];
    for (int i = 0; i < n; ++i) {
      const bool vis = (s & tok_s[i]) != 0 && p <= tok_pos[i];
      bad += (vis != in_prefix) ? 1 : 0;
    }
  }
  if (bad) atomicAdd(&block_bad, bad);
  __syncthreads();
  if (threadIdx.x == 0) {
    if (block_bad) __hip_atomic_fetch_add(work, block_bad, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // release: this workgroup's sum is out before its arrival counts
    const int done = __hip_atomic_fetch_add(work + 1, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (done == (int)gridDim.x - 1) {
      n_unexpressed[0] = __hip_atomic_load(work, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(work, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(work + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// Compaction, step 1 (one wave, lane = window cell): decide, rank the canonical cells by
// position, write the move list, rewrite the window's metadata.
__global__ void __launch_bounds__(kWave) meta_compact_plan_kernel(int32_t* pos, uint32_t* seq, int n_cells,
                                                                  int prefix_len, int32_t* plan, int32_t* result,
                                                                  int32_t* kv_len) {
  __shared__ int new_pos[PI_WINDOW];
  __shared__ uint32_t new_seq[PI_WINDOW];
  const int lane = threadIdx.x;
  const int cell = prefix_len + lane;
  const bool valid = cell < n_cells;
  const int p = valid ? pos[cell] : -1;
  const uint32_t s = valid ? seq[cell] : 0u;
  const bool live = p >= 0;
  const bool canon = live && (s & 1u);
  bool clash = live && !canon;
  int rank = 0;
  for (int j = 0; j < kWave; ++j) {
    const int pj = __shfl(p, j);
    const int cj = __shfl((int)canon, j);
    if (canon && cj && j != lane && pj == p) clash = true;
    rank += (cj && pj < p) ? 1 : 0;
  }
  const bool busy = __builtin_amdgcn_ballot_w64(clash) != 0;
  const int m = busy ? 0 : __builtin_popcountll(__builtin_amdgcn_ballot_w64(canon));
  if (!busy && canon) {
    plan[1 + rank] = cell;
    new_pos[rank] = p;
    new_seq[rank] = s;
  }
  __syncthreads();
  if (!busy && valid) {
    pos[cell] = lane < m ? new_pos[lane] : -1;
    seq[cell] = lane < m ? new_seq[lane] : 0u;
  }
  if (lane == 0) {
    plan[0] = m;
    result[0] = busy ? PI_E_BUSY : PI_OK;
    result[1] = prefix_len + m;
    if (!busy && kv_len) *kv_len = prefix_len + m;
  }
}

// Compaction, step 2: move k copies cell plan[1+k] to cell prefix_len + k in every layer, K and V.
// A thread owns one 4-byte column of one (layer, head, K|V) plane: it reads the column of every
// source cell before it writes any target, so overlapping sources and targets are safe, and
// threads never touch each other's columns.
__global__ void __launch_bounds__(kThreads) meta_compact_move_kernel(char* kbuf, char* vbuf, int elem_size, int n_layers,
                                                                     int n_kv_heads, int n_cells, int head_dim,
                                                                     int prefix_len, const int32_t* plan) {
  const int m = plan[0];
  if (m <= 0) return;
  const int pieces = head_dim * elem_size / 4;
  const size_t total = (size_t)n_layers * n_kv_heads * pieces * 2;
  const size_t idx = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= total) return;
  const int piece = (int)(idx % pieces);
  size_t r = idx / pieces;
  const int which = (int)(r & 1);
  const size_t lh = r >> 1;  // layer * n_kv_heads + head
  const size_t cell_stride = (size_t)head_dim * elem_size;
  char* base = (which ? vbuf : kbuf) + lh * (size_t)n_cells * cell_stride + (size_t)piece * 4;
  uint32_t keep[PI_WINDOW];
#pragma unroll
  for (int k = 0; k < PI_WINDOW; ++k)
    if (k < m) keep[k] = *(const uint32_t*)(base + (size_t)plan[1 + k] * cell_stride);
#pragma unroll
  for (int k = 0; k < PI_WINDOW; ++k)
    if (k < m) *(uint32_t*)(base + (size_t)(prefix_len + k) * cell_stride) = keep[k];
}

bool seq_ok(const pi_kvmeta* m, int s) { return s >= 0 && s < m->n_seq; }

}  // namespace

extern "C" {

int32_t pi_kvmeta_alloc(int32_t n_cells, int32_t n_seq, pi_kvmeta** out) {
  if (!out) return PI_E_ARG;
  *out = nullptr;
  if (n_cells < 1 || n_cells > (1 << 20) || n_seq < 2 || n_seq > PI_MAX_SEQ) return PI_E_SHAPE;
  pi_kvmeta* m = new (std::nothrow) pi_kvmeta();
  if (!m) return PI_E_OOM;
  m->n_cells = n_cells;
  m->n_seq = n_seq;
  m->all = n_seq == 32 ? 0xffffffffu : ((1u << n_seq) - 1u);
  m->held.assign(n_seq, 0);
  for (int s = 1; s < n_seq; ++s) m->free_ids.push_back(s);
  hipError_t e = hipMalloc((void**)&m->pos, (size_t)n_cells * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc((void**)&m->seq, (size_t)n_cells * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMalloc((void**)&m->plan, (1 + PI_WINDOW) * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc((void**)&m->work, 2 * sizeof(int));
  if (e == hipSuccess) e = hipMemset(m->pos, 0xFF, (size_t)n_cells * sizeof(int32_t));
  if (e == hipSuccess) e = hipMemset(m->seq, 0, (size_t)n_cells * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMemset(m->plan, 0, (1 + PI_WINDOW) * sizeof(int32_t));
  if (e == hipSuccess) e = hipMemset(m->work, 0, 2 * sizeof(int));
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    pi_kvmeta_free(m);
    return hip_status(e);
  }
  *out = m;
  return PI_OK;
}

int32_t pi_kvmeta_free(pi_kvmeta* m) {
  if (!m) return PI_E_ARG;
  (void)hipDeviceSynchronize();
  for (void* p : {(void*)m->pos, (void*)m->seq, (void*)m->plan, (void*)m->work})
    if (p) (void)hipFree(p);
  delete m;
  return PI_OK;
}

int32_t pi_kvmeta_seq_acquire(pi_kvmeta* m, int32_t* seq_out) {
  if (!m || !seq_out) return PI_E_ARG;
  if (m->free_ids.empty()) return PI_E_FULL;
  const int s = m->free_ids.front();
  m->free_ids.pop_front();
  m->held[s] = 1;
  *seq_out = s;
  return PI_OK;
}

int32_t pi_kvmeta_seq_release(pi_kvmeta* m, int32_t seq, void* stream) {
  if (!m || seq < 1 || !seq_ok(m, seq) || !m->held[seq]) return PI_E_ARG;
  meta_release_kernel<<<dim3(blocks_for(m->n_cells)), dim3(kThreads), 0, (hipStream_t)stream>>>(m->pos, m->seq, m->n_cells,
                                                                                                1u << seq);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_status(e);
  m->held[seq] = 0;
  m->free_ids.push_back(seq);
  return PI_OK;
}

int32_t pi_kvmeta_fill(pi_kvmeta* m, int32_t cell_begin, int32_t n, int32_t pos_begin, uint32_t seq_mask, void* stream) {
  if (!m || cell_begin < 0 || n < 0 || n > m->n_cells - cell_begin || pos_begin < 0 || (seq_mask & ~m->all)) return PI_E_ARG;
  if (pos_begin > PI_POS_MAX - n) return PI_E_ARG;
  if (n == 0) return PI_OK;
  meta_fill_kernel<<<dim3(blocks_for(n)), dim3(kThreads), 0, (hipStream_t)stream>>>(m->pos, m->seq, cell_begin, n, pos_begin,
                                                                                    seq_mask);
  return hip_status(hipGetLastError());
}

int32_t pi_kvmeta_place(pi_kvmeta* m, int32_t n, const int32_t* positions, const uint32_t* tok_seq, int32_t window_base,
                        int32_t* slots_out, int32_t* status, void* stream) {
  if (!m || !positions || !tok_seq || !slots_out || !status) return PI_E_ARG;
  if (n < 1 || n > PI_MAX_BATCH) return PI_E_SHAPE;
  if (window_base < 0 || window_base >= m->n_cells) return PI_E_ARG;
  meta_place_kernel<<<dim3(1), dim3(kWave), 0, (hipStream_t)stream>>>(m->pos, m->seq, m->n_cells, n, positions, tok_seq,
                                                                      window_base, m->all, slots_out, status);
  return hip_status(hipGetLastError());
}

int32_t pi_kvmeta_seq_cp(pi_kvmeta* m, int32_t src, uint32_t dst_mask, int32_t p0, int32_t p1, void* stream) {
  if (!m || !seq_ok(m, src) || (dst_mask & ~m->all) || p0 < 0) return PI_E_ARG;
  if (!dst_mask || p1 <= p0) return PI_OK;
  meta_cp_kernel<<<dim3(blocks_for(m->n_cells)), dim3(kThreads), 0, (hipStream_t)stream>>>(m->pos, m->seq, m->n_cells,
                                                                                           1u << src, dst_mask, p0, p1);
  return hip_status(hipGetLastError());
}

int32_t pi_kvmeta_seq_rm(pi_kvmeta* m, uint32_t seq_mask, int32_t p0, int32_t p1, void* stream) {
  if (!m || (seq_mask & ~m->all) || p0 < 0) return PI_E_ARG;
  if (!seq_mask || p1 <= p0) return PI_OK;
  meta_rm_kernel<<<dim3(blocks_for(m->n_cells)), dim3(kThreads), 0, (hipStream_t)stream>>>(m->pos, m->seq, m->n_cells,
                                                                                           seq_mask, p0, p1);
  return hip_status(hipGetLastError());
}

int32_t pi_kvmeta_accept(pi_kvmeta* m, int32_t n, const int32_t* positions, const uint32_t* tok_seq,
                         const int32_t* accepted_nodes, const int32_t* result, void* stream) {
  if (!m || !positions || !tok_seq || !accepted_nodes || !result) return PI_E_ARG;
  if (n < 1 || n > PI_MAX_BATCH) return PI_E_SHAPE;
  meta_accept_kernel<<<dim3(blocks_for(m->n_cells)), dim3(kThreads), 0, (hipStream_t)stream>>>(
      m->pos, m->seq, m->n_cells, n, positions, tok_seq, accepted_nodes, result, m->all);
  return hip_status(hipGetLastError());
}

int32_t pi_kvmeta_build_mask(pi_kvmeta* m, int32_t n, const int32_t* positions, const uint32_t* tok_seq,
                             int32_t prefix_len, int32_t window_base, uint64_t* mask_out, int32_t* n_unexpressed,
                             void* stream) {
  if (!m || !positions || !tok_seq || !mask_out || !n_unexpressed) return PI_E_ARG;
  if (n < 1 || n > PI_MAX_BATCH) return PI_E_SHAPE;
  if (prefix_len < 0 || prefix_len > m->n_cells || window_base < 0 || window_base >= m->n_cells) return PI_E_ARG;
  unsigned blocks = blocks_for(m->n_cells);
  if (blocks > (unsigned)kMaskBlocks) blocks = kMaskBlocks;
  meta_mask_kernel<<<dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream>>>(m->pos, m->seq, m->n_cells, n, positions, tok_seq,
                                                                             prefix_len, window_base,
                                                                             (unsigned long long*)mask_out, n_unexpressed,
                                                                             m->work);
  return hip_status(hipGetLastError());
}

int32_t pi_kvmeta_compact(pi_kvmeta* m, pi_kv* kv, int32_t prefix_len, int32_t* result, void* stream) {
  if (!m || !result || prefix_len < 0 || prefix_len > m->n_cells) return PI_E_ARG;
  KvView w{};
  if (kv) {
    w = kv_view(kv);
    if (w.n_cells != m->n_cells) return PI_E_SHAPE;
  }
  meta_compact_plan_kernel<<<dim3(1), dim3(kWave), 0, (hipStream_t)stream>>>(m->pos, m->seq, m->n_cells, prefix_len, m->plan,
                                                                             result, kv ? w.len_dev : nullptr);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !kv) return hip_status(e);
  const int es = w.dtype == PI_DTYPE_BF16 ? 2 : 4;
  const size_t total = (size_t)w.n_layers * w.n_kv_heads * (w.head_dim * es / 4) * 2;
  meta_compact_move_kernel<<<dim3((unsigned)((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, (hipStream_t)stream>>>(
      (char*)w.k, (char*)w.v, es, w.n_layers, w.n_kv_heads, w.n_cells, w.head_dim, prefix_len, m->plan);
  return hip_status(hipGetLastError());
}

int32_t pi_kvmeta_read(const pi_kvmeta* m, int32_t* pos_host, uint32_t* seq_host) {
  if (!m) return PI_E_ARG;
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess && pos_host) e = hipMemcpy(pos_host, m->pos, (size_t)m->n_cells * sizeof(int32_t), hipMemcpyDeviceToHost);
  if (e == hipSuccess && seq_host) e = hipMemcpy(seq_host, m->seq, (size_t)m->n_cells * sizeof(uint32_t), hipMemcpyDeviceToHost);
  return hip_status(e);
}

}  // extern "C"
