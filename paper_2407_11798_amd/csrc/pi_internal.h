// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pipeinfer.h"

namespace pi {

constexpr int kWave = 64;
constexpr int kProjThreads = 256;  // 4 waves per workgroup in the projection kernels
constexpr int kRowBlock = 16;      // weight rows per MFMA tile
constexpr int kKTile = 32;         // input features per MFMA tile

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// A weight matrix in the streaming layout.  Logical W[N][K] (row = output feature) is cut
// into tiles of 16 rows x 32 columns, stored row-block-major, k-tile-minor, so a wave that
// walks one row block reads one contiguous run of memory.
//   bf16 tile (1 KiB): lane l holds the 8 values W[16rb + (l&15)][32t + 8(l>>4) + 0..7]
//                      -- exactly the A operand of v_mfma_f32_16x16x32_bf16.
//   fp32 tile (2 KiB): two 1 KiB halves h=0,1; lane l holds W[..][32t + 8(l>>4) + 4h + 0..3].
// Rows >= N and columns >= K are zero.
struct PackedMat {
  void* data = nullptr;
  int N = 0, K = 0;    // logical
  int NRB = 0, KT = 0; // row blocks, k tiles
  size_t bytes = 0;
};

// Device-visible state of the run in flight on a model.
struct RunState {
  int32_t dead;         // non-zero: every later kernel of the run falls through
  int32_t status;       // PI_OK / PI_CANCELLED / PI_E_SLOT_LIVE
  int32_t layers_done;  // first layer not evaluated
  int32_t pad;
};

struct LayerWeights {
  PackedMat qkv, o, gateup, down;
  float* attn_gain = nullptr;
  float* ffn_gain = nullptr;
};

enum Epilogue { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

// Everything a projection launch needs.  Pointers are device pointers.
struct ProjArgs {
  const void* W;
  int N, K, NRB, KT;
  int S_k;  // k splits
  int RBU;  // row blocks per work unit
  int n;    // tokens
  int NP;   // token slots staged in LDS (>= n, <= 16)
  const float* xin;     // [n][K] fp32
  const float* gain;    // [K] or nullptr
  const float* ssq_in;  // [n_ssq_blocks][16] partial sums of squares of xin rows, or nullptr
  int n_ssq_blocks;
  float eps;
  float* part;  // [S_k][NRB][256] split-k partial tiles
  int* cnt;     // [NRB] arrival counters, zero between launches
  const RunState* rs;
  // --- epilogue outputs
  float* out;          // RESID: x[n][N] (+=) ; SWIGLU: a[n][N/2] ; LOGITS: logits[n][N] ; QKV: q[n][n_q_rows]
  float* ssq_out;      // RESID: [NRB][16]
  // QKV only
  int n_q_rows, n_kv_rows, head_dim;
  void* kcache;        // this layer's K: [Hkv][cells][hd]
  void* vcache;
  int n_cells;
  int kv_dtype;
  const int32_t* positions;
  const int32_t* slots;
  const float2* rope;  // [max_pos][hd/2] (cos, sin)
  // layer-boundary cancellation probe (RESID of the down projection only)
  RunState* rs_mut;          // nullptr: no probe
  int* done_cnt;             // counts finished row blocks of this launch
  const int32_t* cancel_flag;
  int next_layer;            // value for layers_done once this launch has finished
  int probe;                 // 1: probe cancel_flag when the launch completes
};

struct AttnArgs {
  const float* q;   // [n][Hq*hd]
  const void* kcache;  // [Hkv][cells][hd]
  const void* vcache;
  int kv_dtype, n_cells;
  int n, n_q_heads, n_kv_heads, head_dim;
  int prefix_len, window_base;
  const uint64_t* mask;
  int chunk_cells;   // prefix cells per work unit (multiple of the sub-chunk size)
  int n_prefix_units;
  float* part_o;     // [Hkv][units][R][hd]
  float* part_ml;    // [Hkv][units][R][2]
  float* out;        // [n][Hq*hd]
  const RunState* rs;
};

// ---- launch wrappers (each defined next to its kernels) ---------------------------------
hipError_t launch_repack(const void* src, int src_dtype, int rows, int cols, PackedMat dst,
                         int dst_dtype, int row_mul, int row_add, hipStream_t s);
hipError_t launch_convert(const void* src, int src_dtype, void* dst, int dst_dtype, size_t count,
                          hipStream_t s);
hipError_t launch_proj(const ProjArgs& a, int epi, int dtype, int grid, hipStream_t s);
size_t proj_lds_bytes(int NP, int k_tiles_per_split);
hipError_t launch_attention(const AttnArgs& a, hipStream_t s);
int attn_sub_chunk(int kv_dtype);
hipError_t launch_latch(RunState* rs, const int32_t* cancel_flag, const int32_t* slots, int n,
                        const int32_t* kv_len, int window_base, int n_cells, int layer_begin,
                        hipStream_t s);
hipError_t launch_embed(const void* embed, int dtype, const int32_t* tokens, const float* hidden_in,
                        int n, int d, int vocab, float* x, float* ssq, const RunState* rs,
                        hipStream_t s);
hipError_t launch_finish(const RunState* rs, int32_t* run_status, const float* x, float* hidden_out,
                         int n, int d, hipStream_t s);
hipError_t launch_verify(const int32_t* draft, const int32_t* parent, int n, const float* logits,
                         int vocab, int root_expected, int32_t* accepted, int32_t* result,
                         float* best_val, int32_t* best_idx, int* cnt, hipStream_t s);
hipError_t launch_rollback(void* k, void* v, int kv_dtype, int n_layers, int n_kv_heads, int n_cells,
                           int head_dim, const int32_t* slots, int n, const int32_t* accepted,
                           const int32_t* result, int32_t* kv_len, int* cnt, hipStream_t s);
hipError_t launch_kv_set(void* k, void* v, int kv_dtype, int n_kv_heads, int n_cells, int head_dim,
                         int layer, int cell_begin, int n, const void* ksrc, const void* vsrc,
                         int src_dtype, hipStream_t s);
hipError_t launch_kv_get(const void* k, const void* v, int kv_dtype, int n_kv_heads, int n_cells,
                         int head_dim, int layer, int cell_begin, int n, float* kdst, float* vdst,
                         hipStream_t s);

// ---- small device helpers ---------------------------------------------------------------
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

}  // namespace pi
