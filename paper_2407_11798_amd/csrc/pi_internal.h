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
//   fp8 tile  (1 KiB): 16 rows x 64 columns, one byte per weight; lane l holds, in bytes 0..7,
//                      W[16rb + (l&15)][64t + 8(l>>4) + 0..7] and, in bytes 8..15, the same for
//                      columns 64t + 32 + ...: two consecutive bf16-shaped tiles in one 16-byte piece.
//   fp4 tile  (1 KiB): 16 rows x 128 columns, two weights per byte; lane l holds, in bytes 4h..4h+3
//                      (h = 0..3), W[16rb + (l&15)][128t + 32h + 8(l>>4) + 0..7], lower column in the
//                      low nibble: four consecutive bf16-shaped tiles in one 16-byte piece.
//   block-scaled fp4:  the same tiles, and beside them a plane of scale bytes, 64 per tile in tile
//                      order: byte (16 rows x 4) [r][h] is the scale of row 16rb + r, columns
//                      128t + 32h .. + 31 (127 = 2^0 where the matrix has no such columns).
// Rows >= N and columns >= K are zero.  KT counts tiles of the matrix's own width.
struct PackedMat {
  void* data = nullptr;
  void* scales = nullptr;  // block-scaled formats only
  size_t scale_bytes = 0;
  int N = 0, K = 0;    // logical
  int NRB = 0, KT = 0; // row blocks, k tiles
  size_t bytes = 0;
};

// Weight format of a model as the kernels see it: the activation side of PI_DTYPE_FP8_E4M3 is
// that of a bf16 model; only the matrices differ.
constexpr int kWeightF32 = PI_DTYPE_F32, kWeightBF16 = PI_DTYPE_BF16, kWeightFP8 = PI_DTYPE_FP8_E4M3,
              kWeightFP4 = PI_DTYPE_FP4_E2M1, kWeightFP4B = PI_DTYPE_FP4_E2M1_B32;
__host__ __device__ constexpr bool weight_is_fp4(int wd) { return wd == kWeightFP4 || wd == kWeightFP4B; }
__host__ __device__ constexpr int weight_tile_cols(int wd) { return weight_is_fp4(wd) ? 128 : wd == kWeightFP8 ? 64 : 32; }
__host__ __device__ constexpr int weight_tile_bytes(int wd) { return wd == kWeightF32 ? 2048 : 1024; }

struct LayerWeights {
  PackedMat qkv, o, gateup, down;
  float* attn_gain = nullptr;
  float* ffn_gain = nullptr;
};

constexpr int kStageThreads = 512;  // 8 waves per workgroup, one workgroup per compute unit

// Device-visible state of the run in flight on a model.
struct RunState {
  int32_t reserved0;
  int32_t status;       // PI_OK / PI_CANCELLED (every run of the micro-batch) / PI_E_SLOT_LIVE
  int32_t layers_done;  // first layer not evaluated
  int32_t reserved1;
};

// Grid barrier state.  Every workgroup owns one arrival word and publishes the (ever growing)
// number of the barrier it has reached in the upper 16 bits (compared modulo 2^16); a barrier is
// passed when every word has reached it, so there is no shared counter to contend on and nothing
// to reset between launches.  The lower 16 bits of workgroup 0's word are the tokens whose runs
// have been cancelled so far.
constexpr int kMaxGrid = 1024;
struct StageSync {
  unsigned flags[kMaxGrid];
  unsigned reserved;
  unsigned abort;     // sticky: a barrier wait ran into its time limit
  unsigned exited;
  unsigned pad;
};

struct MatDev {
  const char* w;
  const char* s;  // scale plane of a block-scaled matrix, else null
  int N, K, NRB, KT;
};

struct LayerDev {
  MatDev qkv, o, gateup, down;
  const float* attn_gain;
  const float* ffn_gain;
};

enum Epilogue { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

// Kernel argument of the stage kernel.  All pointers are device pointers.
struct StageArgs {
  // model
  const LayerDev* layers;
  MatDev lm_head;
  const float* final_gain;
  const void* embed;
  const float2* rope;  // [max_pos][hd/2] (cos, sin)
  int max_pos;
  int dtype, d, n_q_heads, n_kv_heads, head_dim, ffn, vocab, n_layers;
  float eps;
  float wscale;  // 8-bit weights: the model's power-of-two scale (1 otherwise)
  // run
  int n;
  const int32_t* tokens;
  const int32_t* positions;
  const int32_t* slots;
  const uint64_t* mask;
  int prefix_len, window_base;
  int layer_begin, layer_end;
  const float* hidden_in;
  float* hidden_out;
  float* logits_out;
  const int32_t* cancel_flags;       // [n_groups] device-visible words, or null
  int32_t* run_status;
  // kv cache: K and V each [L][Hkv][cells][hd]
  char* kbase;
  char* vbase;
  size_t kv_layer_bytes;
  int n_cells, kv_dtype;
  const int32_t* kv_len;
  // scratch
  // x, q: fp32 [n][.]; o (attention output), a (SwiGLU output) and xs (the residual stream times the
  // next projection's RMSNorm gain): in the staged form the projection phases copy into LDS
  float *x, *q, *o, *a, *ssq;
  char* xs;
  float* part;   // three regions of [NRB][S_k][256] partial tiles that cross slices; all-ones while empty
  size_t part_half_floats;  // floats per region
  float* attn_o;   // [Hkv][units][R][hd]
  float* attn_ml;  // [Hkv][units][R][2]
  unsigned* attn_flags;  // [Hkv][attn_flag_stride]: barrier number at which a unit last published
  unsigned* attn_ticket; // one word: the tickets by which workgroups draw attention units, from 0 in every launch
  unsigned* kv_ready;    // [2 * n_kv_rows / 16]: per 16-row block of K, then of V: the tag of the QKV phase that last wrote the run's cells
  int attn_flag_stride;
  RunState* rs;
  StageSync* sync;
  // work split
  int sk[5];  // column slices per projection phase: QKV, O, gate/up, down, LM head
  // per projection phase (same order): tiles per wave that may be asked for ahead of the phase, into
  // LDS, and the byte offset at which the eight waves' regions (pf_cap KiB each) begin -- behind what
  // that phase, and any phase that may still run in the workgroup when they are asked for, keeps there
  // (eight bits per phase, phase 0 lowest; the offsets in KiB: read with a shift, where an array
  // indexed by the phase would be a load from the argument block at every use)
  unsigned long long pf_cap8, pf_base8;
  int attn_chunk, attn_units_per_head;
  unsigned long long timeout_ticks;  // 100 MHz ticks a barrier wait may last
  int slow_poll;                     // a barrier's looks at the arrival words are spaced ~0.7 us apart (else back to back)
  unsigned epoch_base;               // barriers used by earlier launches on this model
  unsigned long long* trace;  // optional: 100 MHz timestamps, one per barrier passed by workgroup 0
  int trace_cap;
  unsigned long long* wgtrace;  // optional debug: [grid][5 phases][8] timestamps of workgroup events in one layer
  int wgtrace_layer;
  // optional debug: a workgroup in the middle of the grid raises the first run's cancel word itself when
  // it enters phase `raise_key` (layer * 8 + phase kind) and stamps the clock into trace[trace_cap - 1]
  int raise_key;
  // rarely read (workgroup 0, at layer boundaries), so kept behind everything the phases use
  int32_t* group_status;             // [n_groups][2] {status, layers_done} per run, or null
  int n_groups;                      // runs sharing the micro-batch
  uint32_t group_mask[PI_MAX_GROUPS];  // bit i: token i belongs to the run
};

// What other translation units may know of a pi_kv (the handle itself is private to the ABI file).
struct KvView {
  void *k, *v;
  int dtype, n_layers, n_kv_heads, n_cells, head_dim;
  int32_t* len_dev;  // canonical length, on the device
};
KvView kv_view(pi_kv* kv);
struct ModelView {
  int n_layers, vocab, max_pos;
};
ModelView model_view(const pi_model* m);

// ---- launch wrappers (each defined next to its kernels) ---------------------------------
hipError_t launch_repack(const void* src, int src_dtype, int rows, int cols, PackedMat dst,
                         int dst_dtype, int row_mul, int row_add, hipStream_t s);
hipError_t launch_convert(const void* src, int src_dtype, void* dst, int dst_dtype, size_t count,
                          hipStream_t s);
size_t attn_lds_bytes(int head_dim, int dtype, int max_unit_cells);
size_t stage_proj_lds_bytes(int n, int nt, int r_max);  // nt in 32-column tiles
int stage_ring_size(int wdtype, int min_nt);
hipError_t stage_configure(int wdtype, int ring, size_t max_lds, int* max_blocks_per_cu);
hipError_t launch_stage(const StageArgs& a, int wdtype, int ring, int grid, size_t lds, hipStream_t s);
hipError_t stream_probe(size_t bytes, int reps, double* gbps);
hipError_t launch_verify(const int32_t* draft, const int32_t* parent, int n, const float* logits,
                         int vocab, int root_expected, const int32_t* prev_result, int prev_n,
                         const int32_t* run_status, int32_t* accepted, int32_t* result,
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
// Two floats -> two bf16, rounded to nearest even, in one word (the first in the low half): a vector
// conversion, which the compiler turns into the chip's packed conversion instruction -- one
// instruction where the integer arithmetic above takes ten.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){a, b}, bf16x2));
}
__device__ __forceinline__ float bf16_low_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_high_f32(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

}  // namespace pi
