// The stage kernel: one persistent launch evaluates a whole slice of decoder layers.
//
// One workgroup of 8 waves per compute unit stays resident for the whole stage and walks the
// phases of every layer (QKV projection, attention, output projection, gate/up, down).  Two
// grid-wide barriers per layer remain (after the output projection and at the layer boundary);
// the other three phase changes wait for the data itself: the buffers a phase reads start out
// holding an all-ones "empty" word and the reader re-reads, a bounded number of times, until
// none is left.  Each wave owns a fixed, contiguous range of weight tiles in every phase and
// keeps a ring of up to 8 outstanding 128-bit non-temporal loads per lane, which it starts
// while the phase's activations are still on their way into LDS.
//
// Early Inference Cancellation: at every layer-boundary barrier the first wave of workgroup 0
// probes the device-visible cancel flag of each run that is still alive (one lane per run) and
// publishes the set of dead tokens in the barrier word itself, so every workgroup takes the
// same decision and a cancelled run stops within one layer.
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
// the same wait as an instruction the compiler's own counter tracking takes into account
// (vmcnt = 0; the export and LDS/scalar counters are left alone)
__device__ __forceinline__ void wave_settle() { __builtin_amdgcn_s_waitcnt(0x0F70); }
__device__ __forceinline__ void wg_mark(const StageArgs& A, int l, int ev) {
  // l: layer * 8 + phase kind; one row of 8 stamps per workgroup and phase of the traced layer
  if (A.wgtrace && (l >> 3) == A.wgtrace_layer && (l & 7) < 5 && threadIdx.x == 0)
    A.wgtrace[(blockIdx.x * 5 + (l & 7)) * 8 + ev] = wall_clock64();
}

// Bounded waits read the clock only once a wait has lasted a while: a clock read is a scalar
// memory round trip, which the fast path of every barrier and reduction would otherwise pay.
struct Deadline {
  unsigned long long t0 = 0;
};
__device__ __forceinline__ bool deadline_passed(Deadline& d, unsigned spin, unsigned long long limit) {
  if ((spin & 255u) != 255u) return false;
  const unsigned long long now = wall_clock64();
  if (d.t0 == 0) {
    d.t0 = now;
    return false;
  }
  return now - d.t0 > limit;
}

// ---- grid barrier ---------------------------------------------------------------------------
// Every workgroup calls it the same number of times.  Returns false when the grid must stop
// (a wait ran into its time limit somewhere): callers then leave the kernel at once.
// probe_layer >= 0: layer boundary; the last arriver records progress and probes the cancel flag.
struct BarrierCtx {
  unsigned epoch;  // absolute number of the last barrier passed
  int* sh;         // 2 ints of LDS: {ok, tokens whose runs are cancelled}
  // first wave of workgroup 0 only: the cancelled tokens and runs so far (kept in registers: a
  // load here would delay workgroup 0's arrival, and with it the whole grid, at every barrier)
  unsigned dead, dead_groups;
};

// Every workgroup calls it the same number of times.  Returns false when the grid must stop (a
// wait ran into its time limit): callers then leave the kernel at once.  layers_done >= 0 marks
// a layer boundary: workgroup 0 records progress and, when `probe` is set, reads the cancel word
// of every run of the micro-batch that is still alive, BEFORE it arrives; the lower half of its
// arrival word carries the set of tokens whose runs are cancelled (the barrier number sits in
// the upper half), so every workgroup learns it from the poll that ends its wait -- a layer
// boundary costs no round trip more than any other barrier.  (A workgroup that is late to look
// may find workgroup 0's word of the NEXT barrier there; the set only changes at boundaries and
// boundaries are never adjacent, so it reads the same set.)  sh[1] is that set.
// `arrived` runs in every wave once the workgroup's arrival is on its way (what a wave may usefully ask
// memory for while it waits must not delay the arrival).
template <typename Arrived>
__device__ __forceinline__ bool grid_barrier(const StageArgs& A, BarrierCtx& bc, int layers_done, bool probe, int mark,
                                             Arrived&& arrived) {
  __syncthreads();  // every wave of this workgroup has drained its stores
  if (A.wgtrace && mark >= 0 && (mark >> 3) == A.wgtrace_layer && (mark & 7) < 5 && threadIdx.x == 0)
    A.wgtrace[(blockIdx.x * 5 + (mark & 7)) * 8 + 4] = wall_clock64();
  bc.epoch += 1;
  StageSync* sy = A.sync;
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    const unsigned want = bc.epoch << 16;
    unsigned word = want;
    if (blockIdx.x == 0) {
      unsigned dead = bc.dead;
      if (layers_done >= 0) {
        const unsigned all = A.n >= 32 ? 0xffffffffu : (1u << A.n) - 1u;
        unsigned groups = bc.dead_groups;
        // lane g looks after run g: all cancel words are read with one load instruction
        const bool mine = lane < A.n_groups && !((groups >> lane) & 1u);
        if (mine && A.group_status)
          __hip_atomic_store(A.group_status + 2 * lane + 1, layers_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bool hit = false;
        if (dead != all && probe && A.cancel_flags && mine)
          hit = __hip_atomic_load(A.cancel_flags + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != 0;
        if (hit && A.group_status)
          __hip_atomic_store(A.group_status + 2 * lane, PI_CANCELLED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long hits = __builtin_amdgcn_ballot_w64(hit);
        if (hits) {
          groups |= (unsigned)hits;
          for (int g = 0; g < A.n_groups; ++g)
            if ((hits >> g) & 1ull) dead |= A.group_mask[g];
          bc.dead = dead;
          bc.dead_groups = groups;
          if (lane == 0 && dead == all)
            __hip_atomic_store(&A.rs->status, PI_CANCELLED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (lane == 0) __hip_atomic_store(&A.rs->layers_done, layers_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        wave_drain();
      }
      word |= dead & 0xffffu;
    }
    if (lane == 0) __hip_atomic_store(&sy->flags[blockIdx.x], word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    arrived();
    const __amdgpu_buffer_rsrc_t fr = rsrc_of(sy->flags);
    const int G = gridDim.x;
    Deadline dl;
    int ok = 1;
    unsigned first = want;  // workgroup 0's word, in lane 0
    for (unsigned spin = 0;; ++spin) {
      bool all = true;
      for (int base = 0; base < G; base += 256) {
        const int idx = base + lane * 4;
        u32x4 f = {want, want, want, want};
        if (idx < G) f = __builtin_amdgcn_raw_buffer_load_b128(fr, idx * 4, 0, kAgent);
        if (base == 0) first = f[0];
#pragma unroll
        for (int q = 0; q < 4; ++q) all = all && (idx + q >= G || (short)((f[q] - want) >> 16) >= 0);
      }
      if (__builtin_amdgcn_ballot_w64(!all) == 0) break;
      if (A.slow_poll)
        __builtin_amdgcn_s_sleep(24);
      else
        __builtin_amdgcn_s_sleep(1);
      if (deadline_passed(dl, spin, A.timeout_ticks)) {
        ok = 0;
        break;
      }
    }
    const int dead = ok ? (int)(__builtin_amdgcn_readfirstlane(first) & 0xffffu) : 0;
    if (lane == 0) {
      if (!ok) __hip_atomic_store(&sy->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (A.trace && blockIdx.x == 0 && (int)(bc.epoch - A.epoch_base) <= A.trace_cap)
        A.trace[bc.epoch - A.epoch_base - 1] = wall_clock64();
      bc.sh[0] = ok;
      bc.sh[1] = dead;
    }
  } else {
    arrived();
  }
  __syncthreads();
  return __builtin_amdgcn_readfirstlane(bc.sh[0]) != 0;
}
__device__ __forceinline__ bool grid_barrier(const StageArgs& A, BarrierCtx& bc, int layers_done, bool probe, int mark = -1) {
  return grid_barrier(A, bc, layers_done, probe, mark, [] {});
}

// ---- per-wave weight stream -----------------------------------------------------------------
// In a projection with S_k column slices, workgroup wg serves slice wg % S_k together with the
// other gridDim/S_k workgroups of its group.  The group's workgroups own whole row blocks (an
// even split of the matrix's row blocks); the workgroup's tiles of the slice, ordered
// row-block-major, are cut into equal contiguous ranges, one per wave: flat index f -> row block
// rb0 + f / nt, k tile t0 + f % nt.  A row block is therefore reduced inside one workgroup,
// through LDS; only the S_k slices of a row block meet through memory.
struct WaveStream {
  const char* w;   // the whole matrix, read through a raw buffer of `bytes` bytes
  uint32_t bytes;
  const char* ws;  // block-scaled weights: the plane of scale bytes (64 per tile, in tile order), else null
  uint32_t sbytes;
  int KT, nt, t0, NRB;
  int rb0, R;         // this workgroup's row blocks [rb0, rb0 + R)
  int f0, f1, share;  // this wave's flat range of the workgroup's R * nt tiles; tiles per wave
  int slice, wave;
  // loader cursor: flat index, tile within the slice's part of the row block, byte offset of the tile
  int lf, lt;
  uint32_t loff;
  int pf;  // leading tiles of the range that were asked for ahead of the phase and wait in LDS
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
// The per-layer table does not change while a kernel runs and the layer index is the same in every
// lane: read through the constant address space it comes by scalar loads, straight into scalar
// registers and through the scalar cache, instead of a vector load whose ~1 us the wave would sit
// out at the top of every phase.
typedef const __attribute__((address_space(4))) LayerDev* LayerTab;
__device__ __forceinline__ MatDev tab_mat(const __attribute__((address_space(4))) MatDev& m) {
  MatDev r;
  r.w = m.w;
  r.s = m.s;
  r.N = m.N;
  r.K = m.K;
  r.NRB = m.NRB;
  r.KT = m.KT;
  return r;
}
__device__ __forceinline__ LayerDev tab_layer(LayerTab t, int l) {
  LayerDev r;
  r.qkv = tab_mat(t[l].qkv);
  r.o = tab_mat(t[l].o);
  r.gateup = tab_mat(t[l].gateup);
  r.down = tab_mat(t[l].down);
  r.attn_gain = t[l].attn_gain;
  r.ffn_gain = t[l].ffn_gain;
  return r;
}
template <int DT>
__device__ __forceinline__ MatDev table_mat(const StageArgs& A, int l, int which) {  // which: 0 QKV, 1 O
  return tab_mat(which == 0 ? ((LayerTab)A.layers)[l].qkv : ((LayerTab)A.layers)[l].o);
}
template <int DT>
__device__ __forceinline__ LayerDev table_layer(const StageArgs& A, int l) {
  return tab_layer((LayerTab)A.layers, l);
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}

// The stream state is carried across phases and around the phase loop, where the compiler has to
// assume it differs between lanes; it does not, and the streaming loop needs it in scalar
// registers (a raw buffer load with per-lane descriptor or offset operands is wrapped in a loop
// over the distinct values).
__device__ __forceinline__ void stream_make_uniform(WaveStream& S) {
  S.w = uni_ptr(S.w);
  S.bytes = (uint32_t)uni((int)S.bytes);
  S.ws = uni_ptr(S.ws);
  S.sbytes = (uint32_t)uni((int)S.sbytes);
  S.KT = uni(S.KT); S.nt = uni(S.nt); S.t0 = uni(S.t0); S.NRB = uni(S.NRB);
  S.f0 = uni(S.f0); S.f1 = uni(S.f1); S.share = uni(S.share);
  S.slice = uni(S.slice); S.wave = uni(S.wave); S.rb0 = uni(S.rb0); S.R = uni(S.R);
  S.lf = uni(S.lf); S.lt = uni(S.lt); S.loff = (uint32_t)uni((int)S.loff);
  S.pf = uni(S.pf);
}

template <int DT>
__device__ __forceinline__ void stream_init(WaveStream& S, const MatDev& M, int S_k, int wave) {
  const int wg = blockIdx.x, G = gridDim.x;
  constexpr int kTileBytes = weight_tile_bytes(DT);
  S.w = M.w;
  S.bytes = (uint32_t)M.NRB * (uint32_t)M.KT * kTileBytes;
  S.ws = M.s;
  S.sbytes = (uint32_t)M.NRB * (uint32_t)M.KT * 64u;
  S.KT = M.KT;
  S.NRB = M.NRB;
  S.nt = uni(M.KT / S_k);
  S.slice = uni(wg % S_k);
  S.t0 = S.slice * S.nt;
  S.wave = wave;
  const int Gs = uni(G / S_k), gwg = uni(wg / S_k);
  S.rb0 = uni((int)((long)gwg * M.NRB / Gs));
  S.R = uni((int)((long)(gwg + 1) * M.NRB / Gs)) - S.rb0;
  const int total = S.R * S.nt;
  S.share = max(1, uni((total + kWaves - 1) / kWaves));
  S.f0 = min(total, wave * S.share);
  S.f1 = min(total, S.f0 + S.share);
  S.lf = S.f0;
  const int q = uni(S.f0 / S.nt);
  S.lt = S.f0 - q * S.nt;
  S.loff = (uint32_t)((S.rb0 + q) * S.KT + S.t0 + S.lt) * (uint32_t)kTileBytes;
  S.pf = 0;
  stream_make_uniform(S);
}

// Tiles asked for ahead of the phase.  A wave that has finished a phase has nothing to do until the
// slowest workgroup has finished it too, and its ring lives in registers that the wait needs; but
// the first tiles of its next range can travel meanwhile straight into LDS (no register is their
// destination), `cap` of them at most and only tiles of the range's first row block, leaving that
// row block at least one tile for the ring (so the streaming loop ends the row block as always).
// The wave's own later loads (the barrier's poll, the staged activations) return behind these, in
// order, so whatever it reads from its LDS region after those has landed.
__device__ __forceinline__ int park_cap(const StageArgs& A, int pidx) { return (int)((A.pf_cap8 >> (8 * pidx)) & 0xffu); }
__device__ __forceinline__ char* park_region(const StageArgs& A, char* lds, int pidx, int wave) {
  return lds + ((int)((A.pf_base8 >> (8 * pidx)) & 0xffu) + wave * park_cap(A, pidx)) * 1024;
}
template <int DT>
__device__ __forceinline__ void stream_park(WaveStream& S, char* region, int cap, int lane) {
  if constexpr (weight_tile_bytes(DT) == 1024 && DT != kWeightFP4B) {
    const int seg = min(S.nt - S.lt, S.f1 - S.f0) - 1;
    const int P = uni(max(0, min(cap, seg)) & ~1);
    const char* src = S.w + S.loff + lane * 16;
    for (int i = 0; i < P; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + i * 1024),
                                       (__attribute__((address_space(3))) void*)(region + i * 1024), 16, 0, 2);
    S.pf = P;
    S.lf += P;
    S.lt += P;
    S.loff += (uint32_t)(P * 1024);
  }
}

// The ring of outstanding weight tiles: UR tiles, each 1 KiB (bf16: one 16-byte load per lane)
// or 2 KiB (fp32: two loads per lane).  Slot indices are compile-time, so it lives in registers.
template <int DT, int UR>
struct Ring {
  static constexpr int U = UR;
  static constexpr int kTileBytes = weight_tile_bytes(DT);
  static constexpr int kRegs = DT == kWeightF32 ? 2 * UR : UR;
  u32x4 r[kRegs];
  uint32_t s[DT == kWeightFP4B ? UR : 1];  // block-scaled weights: the lane's row's four scale bytes of the tile
};

// What one pass over the ring does, worked out in scalar registers before the pass, so that every
// per-slot decision inside it is a comparison of a scalar with the (compile-time) slot number and
// no cursor is written between slots: the instruction count per tile is what bounds the stream.
struct PassPlan {
  int nc;              // the consumer takes slots 0 .. nc-1
  int ec;              // slot ec-1 holds the last tile of the consumer's current row block
  int cbaseA, cbaseB;  // slot J's operands start (J < ec ? cbaseA : cbaseB) + J * stride bytes into x
  int stride;          // bytes of operand slots per tile: 64 n
  int zoff;            // byte offset of the all-zero operand slots behind x
  int nl;              // the loader refills slots 0 .. nl-1
  int el;              // slot el-1 gets the last tile of the loader's current row block
  uint32_t lbaseA, lbaseB;  // slot J loads the tile at (J < el ? lbaseA : lbaseB) + J * tile bytes
};

// Issue the load of the wave's next tile into slot J.  The load itself is unconditional: past
// the end of the range it has out-of-range offsets (the hardware's range check answers with
// zeros without going to memory) and the consumer never looks at the slot, so the loads of a
// pass are never inside a branch (a branch around a load makes the compiler wait for it at the
// join) and stay in flight.
template <int DT, int UR, int J>
__device__ __forceinline__ void ring_issue(Ring<DT, UR>& R, const WaveStream& S, const PassPlan& P, int lane16) {
  constexpr int TB = Ring<DT, UR>::kTileBytes;
  const int mask = J < P.nl ? -1 : 0;
  const int soff = (int)((J < P.el ? P.lbaseA : P.lbaseB) + (uint32_t)(J * TB)) & mask;
  const int voff = (lane16 & mask) | (0x7ffffff0 & ~mask);
  const __amdgpu_buffer_rsrc_t rsrc = make_rsrc(S.w, S.bytes);
  if constexpr (DT == kWeightFP4B) {
    // the tile, then the dword of its scale plane that belongs to this lane's row (tile offset / 16 + 4 row)
    R.r[J] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, soff, 2);
    const int svoff = (((lane16 >> 4) & 15) * 4 & mask) | (0x7ffffff0 & ~mask);
    R.s[J] = __builtin_amdgcn_raw_buffer_load_b32(make_rsrc(S.ws, S.sbytes), svoff, (int)((uint32_t)soff >> 4), 2);
  } else if constexpr (DT != kWeightF32) {
    R.r[J] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, soff, 2);
  } else {
    R.r[2 * J] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, soff, 2);
    R.r[2 * J + 1] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, soff + (1024 & mask), 2);
  }
  // Ring loads must be issued in slot order: the counter wait before slot J is consumed is "all but
  // the newest U - 1", and the instruction scheduler is otherwise free to reorder independent loads
  // (the oldest slot then looks newest and the compiler waits for the whole ring).
  asm volatile("" ::: "memory");
}

template <int DT, int UR, int J, int JEND>
__device__ __forceinline__ void issue_slots(Ring<DT, UR>& R, const WaveStream& S, const PassPlan& P, int lane16) {
  if constexpr (J < JEND) {
    ring_issue<DT, UR, J>(R, S, P, lane16);
    issue_slots<DT, UR, J + 1, JEND>(R, S, P, lane16);
  }
}

// The loader's part of a pass plan and of the cursor update after the pass (the host guarantees
// nt >= UR: at most one row block ends in a pass).
template <int UR>
__device__ __forceinline__ void plan_loads(PassPlan& P, const WaveStream& S, int tile_bytes) {
  P.nl = max(0, min(UR, S.f1 - S.lf));
  P.el = S.nt - S.lt;
  P.lbaseA = S.loff;
  P.lbaseB = S.loff + (uint32_t)(S.KT - S.nt) * (uint32_t)tile_bytes;
}
__device__ __forceinline__ void advance_loads(WaveStream& S, const PassPlan& P, int tile_bytes) {
  S.lf += P.nl;
  if (P.nl > 0 && P.el <= P.nl) {
    S.lt = P.nl - P.el;
    S.loff = P.lbaseB + (uint32_t)(P.nl * tile_bytes);
  } else {
    S.lt += P.nl;
    S.loff += (uint32_t)(P.nl * tile_bytes);
  }
}

// Fill the (empty) ring with the first tiles of the wave's range.  `really` false: the same
// instructions with out-of-range offsets (answered with zeros, no traffic), for a caller that must
// not put its loads behind a branch but may not want them yet.
template <int DT, int UR>
__device__ __forceinline__ void ring_prefetch(Ring<DT, UR>& R, WaveStream& S, int lane, bool really = true) {
  constexpr int TB = Ring<DT, UR>::kTileBytes;
  PassPlan P;
  plan_loads<UR>(P, S, TB);
  if (!really) P.nl = 0;
  issue_slots<DT, UR, 0, UR>(R, S, P, lane * 16);
  advance_loads(S, P, TB);
}

constexpr uint32_t kEmptyWord = 0xFFFFFFFFu;  // all-ones: "nothing here yet" in buffers that workgroups poll

// ---- activations between phases: the staged form ------------------------------------------------
// What a projection phase multiplies its weights with is the same for every workgroup -- n rows of K
// activations, times the RMSNorm gain where the phase has one -- and every workgroup needs all of it
// (or its column slice) in LDS, as the matrix instruction's second operand: split into a bf16 high
// and low part for a bf16 model.  So the PRODUCER of the activations (the residual, SwiGLU and
// attention epilogues, the stage input) writes them to memory in exactly that form, once, and a
// consumer copies its slice into LDS with loads that write LDS directly: no registers, no
// arithmetic, everything in flight at once.
//   Piece (c8, i) = columns 8 c8 .. 8 c8 + 7 of token i is 16-byte slot c8 * n + i of two arrays, the
//   second (K / 8) * n slots behind the first.  bf16 model: array 0 holds the pieces' eight high
//   parts, array 1 the eight low parts (value - high part, rounded to bf16).  fp32 model: array 0
//   holds the first four values of the piece, array 1 the last four.
// A phase's slice of k tiles [t0, t0 + nt) is the contiguous slot range [4 t0 n, 4 (t0 + nt) n) of
// both arrays; columns past K do not exist in memory (the consumer's descriptor ends with the
// arrays, and loads beyond it write zeros).
__device__ __forceinline__ uint32_t staged_array_bytes(int K, int n) { return (uint32_t)(K >> 3) * (uint32_t)n * 16u; }
// Store columns c0 .. c0 + 3 (c0 a multiple of 4) of token i.
template <int DT>
__device__ __forceinline__ void store_staged4(char* base, int K, int n, int i, int c0, f32x4 v) {
  const __amdgpu_buffer_rsrc_t r = rsrc_of(base);
  const int slot16 = ((c0 >> 3) * n + i) * 16, half = (c0 >> 2) & 1;
  const int arr = (int)staged_array_bytes(K, n);
  if constexpr (DT != kWeightF32) {
    const uint32_t h0 = pack_bf16(v[0], v[1]), h1 = pack_bf16(v[2], v[3]);
    const uint32_t l0 = pack_bf16(v[0] - bf16_low_f32(h0), v[1] - bf16_high_f32(h0));
    const uint32_t l1 = pack_bf16(v[2] - bf16_low_f32(h1), v[3] - bf16_high_f32(h1));
    st_ag2(r, slot16 + half * 8, __uint_as_float(h0), __uint_as_float(h1));
    st_ag2(r, arr + slot16 + half * 8, __uint_as_float(l0), __uint_as_float(l1));
  } else {
    st_ag4(r, half * arr + slot16, v);
  }
}
// Store columns c0, c0 + 1 (c0 even) of token i.
template <int DT>
__device__ __forceinline__ void store_staged2(char* base, int K, int n, int i, int c0, float v0, float v1) {
  const __amdgpu_buffer_rsrc_t r = rsrc_of(base);
  const int slot16 = ((c0 >> 3) * n + i) * 16;
  const int arr = (int)staged_array_bytes(K, n);
  if constexpr (DT != kWeightF32) {
    const uint32_t h = pack_bf16(v0, v1);
    const uint32_t l = pack_bf16(v0 - bf16_low_f32(h), v1 - bf16_high_f32(h));
    const int off = slot16 + ((c0 >> 1) & 3) * 4;
    __builtin_amdgcn_raw_buffer_store_b32(h, r, off, 0, kAgent);
    __builtin_amdgcn_raw_buffer_store_b32(l, r, arr + off, 0, kAgent);
  } else {
    st_ag2(r, ((c0 >> 2) & 1) * arr + slot16 + (c0 & 2) * 4, v0, v1);
  }
}

// vmcnt(N) as the wait instruction that the compiler's own counter tracking takes into account
template <int N>
__device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

// ---- activation staging (once per phase and workgroup) ---------------------------------------
// LDS slot (tt, g, i) holds the piece of token i that starts at column 32(t0+tt) + 8g, array 0 in
// the first half of the operand area and array 1 lo_off = (nt + 1) * 4 * n slots behind it.  The
// slots of one more tile (tt = nt) are all zero in both halves: the streaming loop multiplies by
// them where a slot of its ring holds nothing.
// The copy: the slice is cut into pieces of 1 KiB (one load instruction of a wave), wave w takes
// pieces w, w + 8, ... of both arrays.  `mid` (the caller's weight requests: kMidLoads load
// instructions, always) goes out behind them, so the activations, being older, are waited for
// alone.
// Also computes 1/sqrt(mean x^2 + eps) per token (scaled phases) from the per-16-column partial
// sums of squares, summed in a fixed order.  `post` runs before the closing workgroup barrier.
// poll_limit > 0: the activations may still be on their way (no grid barrier separates this phase
// from their producer): a slot with an all-ones word is "empty"; a wave whose pieces hold one asks
// for those pieces again, at most poll_limit times.  Their producer overwrites every slot, and a
// later phase puts the pattern back once every workgroup has staged them.
template <int kMidLoads, typename Mid, typename Post>
__device__ __forceinline__ void stage_x(const char* xs, int K, int n, int t0, int nt, char* lds, const float* ssq,
                                        int n_blocks, float eps, float* red, float* rscale, Mid&& mid, Post&& post,
                                        unsigned poll_limit, bool* timed_out, int wave, int lane) {
  const int lo_off = (nt + 1) * 4 * n;
  for (int z = nt * 4 * n + threadIdx.x; z < lo_off; z += kThreads) {
    ((uint4*)lds)[z] = make_uint4(0u, 0u, 0u, 0u);
    ((uint4*)lds)[lo_off + z] = make_uint4(0u, 0u, 0u, 0u);
  }
  // Partial sums of squares, [block of 16 columns][16 tokens]: a lane reads four tokens of a block
  // with one 128-bit load (lane t: tokens 4 (t & 3) .., blocks t >> 2, + 128, + 256, ...: two loads per
  // lane at d_model 4096), all in flight at once.  Unscaled phases and blocks past the last get
  // out-of-range offsets, which the hardware answers with zeros without going to memory.
  constexpr int kSsqLoads = 4;  // up to 4 * 128 = 512 blocks of 16 columns (d_model <= 8192) at once
  f32x4 part[kSsqLoads];
  {
    const __amdgpu_buffer_rsrc_t sr = make_rsrc(ssq ? ssq : (const float*)xs, ssq ? (uint32_t)n_blocks * 64u : 0u);
    const int voff = (int)threadIdx.x * 16;  // block (tid >> 2), tokens 4 (tid & 3) ..
#pragma unroll
    for (int q = 0; q < kSsqLoads; ++q) part[q] = ld_ag4(sr, voff + q * (kThreads * 16));
  }
  const uint32_t arr = staged_array_bytes(K, n);
  const __amdgpu_buffer_rsrc_t r0 = make_rsrc(xs, arr), r1 = make_rsrc(xs + arr, arr);
  const int bytes = nt * 4 * n * 16, src0 = t0 * 4 * n * 16;  // the slice, in each array
  const int pieces = (bytes + 1023) >> 10;
  typedef __attribute__((address_space(3))) void* lds_ptr;
  const auto pull = [&](int c) {  // piece c of both arrays (lanes past the slice's end stay out)
    const int off = c * 1024 + lane * 16;
    if (off < bytes) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r0, (lds_ptr)(lds + c * 1024), 16, off, src0, 0, kAgent);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r1, (lds_ptr)(lds + lo_off * 16 + c * 1024), 16, off, src0, 0, kAgent);
    }
  };
  for (int c = wave; c < pieces; c += kWaves) pull(c);
  mid();
  wait_vm<kMidLoads>();  // this wave's pieces are in LDS
  if (poll_limit) {
    for (unsigned spin = 0;; ++spin) {
      bool again = false;
      for (int c = wave; c < pieces; c += kWaves) {
        const int off = c * 1024 + lane * 16;
        bool missing = false;
        if (off < bytes) {
          const u32x4 a = *(const u32x4*)(lds + off), b = *(const u32x4*)(lds + lo_off * 16 + off);
          missing = a[0] == kEmptyWord || a[1] == kEmptyWord || a[2] == kEmptyWord || a[3] == kEmptyWord ||
                    b[0] == kEmptyWord || b[1] == kEmptyWord || b[2] == kEmptyWord || b[3] == kEmptyWord;
        }
        if (__builtin_amdgcn_ballot_w64(missing) != 0) {
          pull(c);
          again = true;
        }
      }
      if (!again) break;
      if (spin >= poll_limit) {
        *timed_out = true;
        break;
      }
      wave_settle();  // the re-reads are younger than the weight loads: leave nothing of them pending
    }
  }
  if (ssq) {
    f32x4 ssum = (part[0] + part[1]) + (part[2] + part[3]);
    for (int b = (int)(threadIdx.x >> 2) + kSsqLoads * (kThreads / 4); b < n_blocks; b += kThreads / 4)  // d_model > 8192
      ssum += ld_ag4(make_rsrc(ssq, (uint32_t)n_blocks * 64u), (b * 16 + (int)(threadIdx.x & 3) * 4) * 4);
    // lanes with the same tokens (equal lane & 3) first, by shuffles in a fixed order, then the eight
    // waves through LDS: a chain of dependent LDS reads would cost most of a microsecond here
#pragma unroll
    for (int sh = 4; sh < 64; sh *= 2) {
#pragma unroll
      for (int j = 0; j < 4; ++j) ssum[j] += __shfl_xor(ssum[j], sh);
    }
    if (lane < 4) *(f32x4*)(red + wave * 16 + lane * 4) = ssum;
    __syncthreads();
    if (threadIdx.x < 16) {
      float t = 0.0f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) t += red[w * 16 + threadIdx.x];
      rscale[threadIdx.x] = 1.0f / sqrtf(t / (float)K + eps);
    }
  }
  post();
  __syncthreads();
}

// Sum of four squares as one explicit chain of fused multiply-adds: the residual stream's sums of
// squares are produced at two places (stage input, residual epilogue) and must not depend on
// which multiply-adds the compiler would choose to fuse at each.
__device__ __forceinline__ float sum_sq4(float a, float b, float c, float d) {
  return __builtin_fmaf(d, d, __builtin_fmaf(c, c, __builtin_fmaf(b, b, a * a)));
}

// ---- epilogues --------------------------------------------------------------------------------
struct EpiCtx {
  int epi;  // Epilogue kind
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
  unsigned dead_tokens;  // QKV: tokens of cancelled runs
  unsigned* kv_ready;    // QKV: per 16-row block of K and V, raised to kv_tag once the block's cells are in memory
  unsigned kv_tag;
  const float2* rope;
  const f32x4* resid;  // RESID: LDS copy of the residual rows of the workgroup's row blocks, [row block][lane]
  int rb0;             // first row block of the workgroup
  // RESID: the new residual rows are also written in the staged form the next projection reads, times
  // that projection's RMSNorm gain (null: nobody reads them in that form)
  char* staged_out;
  const float* gain_next;  // [N]
  const f32x4* gres;       // LDS copy of the gains of the workgroup's rows, [row block][lane] (null: read in place)
};

__device__ __forceinline__ void store_kv4(char* cache, int kv_dtype, size_t elem_idx, const float* v) {
  const __amdgpu_buffer_rsrc_t r = rsrc_of(cache);
  if (kv_dtype == PI_DTYPE_BF16) {
    u32x2 p = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
    __builtin_amdgcn_raw_buffer_store_b64(p, r, (int)(elem_idx * 2), 0, kAgent);
  } else {
    st_ag4(r, (int)(elem_idx * 4), f32x4{v[0], v[1], v[2], v[3]});
  }
}

// The accumulator tile of a wave: lane l holds rows 16rb + 4(l>>4) + 0..3 for token l & 15.
template <int DT>
__device__ __forceinline__ void epilogue(const EpiCtx& e, int rb, f32x4 acc, int lane, const float* rscale) {
  const int EPI = e.epi;
  const int i = lane & 15, g = lane >> 4;
  const int row = rb * kRowBlock + g * 4;
  const bool live = i < e.n;
  if (EPI == EPI_QKV) {
    const int hd = e.head_dim;
    if (live) {
      const float r = rscale[i];
      float v[4] = {acc[0] * r, acc[1] * r, acc[2] * r, acc[3] * r};
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
        if (!((e.dead_tokens >> i) & 1u)) store_kv4(is_k ? e.kcache : e.vcache, e.kv_dtype, idx, v);  // a cancelled run writes no more K/V
      }
    }
    // Attention is not behind a grid barrier: it reads the queries until none is "empty", and the
    // window's cells once the words of their 16-row blocks say this phase has written them.  A row
    // block is all Q, all K or all V, so the whole wave takes this branch together.
    const int kv0 = rb * kRowBlock - e.n_q_rows;
    if (kv0 >= 0 && kv0 < 2 * e.n_kv_rows) {
      wave_drain();  // the block's cells are in memory
      if (lane == 0) __hip_atomic_store(e.kv_ready + kv0 / kRowBlock, e.kv_tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  } else if (EPI == EPI_RESID) {
    float s = 0.0f;
    if (live && row < e.N) {
      const __amdgpu_buffer_rsrc_t xr = rsrc_of(e.out);
      const int off = (i * e.N + row) * 4;
      // the residual rows were copied to LDS when the phase began (unless the workgroup owns too
      // many row blocks): a load issued here would queue behind the weight requests in flight
      const f32x4 x = (e.resid ? e.resid[(rb - e.rb0) * 64 + lane] : ld_ag4(xr, off)) + acc;
      st_ag4(xr, off, x);
      s = sum_sq4(x[0], x[1], x[2], x[3]);
      if (e.staged_out) {
        const f32x4 gn = e.gres ? e.gres[(rb - e.rb0) * 64 + lane] : *(const f32x4*)(e.gain_next + row);
        store_staged4<DT>(e.staged_out, e.N, e.n, i, row, x * gn);
      }
    }
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 32);
    if (g == 0) st_ag(e.ssq_out + rb * 16 + i, live ? s : 0.0f);
  } else if (EPI == EPI_SWIGLU) {
    if (!live || row >= e.N) return;
    const float r = rscale[i];
    const float g0 = acc[0] * r, u0 = acc[1] * r, g1 = acc[2] * r, u1 = acc[3] * r;
    // (in the staged form: the down projection is its only reader)
    store_staged2<DT>((char*)e.out, e.N / 2, e.n, i, row / 2, g0 / (1.0f + expf(-g0)) * u0, g1 / (1.0f + expf(-g1)) * u1);
  } else {  // EPI_LOGITS: read by later kernels only
    if (!live || row >= e.N) return;
    const float r = rscale[i];
    *(float4*)(e.out + (size_t)i * e.N + row) = make_float4(acc[0] * r, acc[1] * r, acc[2] * r, acc[3] * r);
  }
}

// One wave has finished its part of row block rb.  Inside the workgroup: a wave contributes to a
// row block it does not start only at the beginning of its own range, so each wave parks at most
// one partial tile per phase (LDS slot = wave) and raises its flag to the phase's tag; the wave
// that holds the row block's first tile reaches the row block last in its own range, waits
// (bounded) for those flags and adds the tiles in wave order.  Across slices (S_k > 1): slices
// other than 0 store their sums to memory (a tile is "empty" while it holds the all-ones
// pattern, which no sum can produce); slice 0 polls them (bounded), adds them in slice order,
// marks them empty again for the next use and runs the epilogue.
constexpr unsigned kPollLimit = 1u << 20;  // re-reads of activations on their way (each a memory round trip): seconds
constexpr int kMaxResidBlocks = 8;  // residual rows of at most this many row blocks per workgroup are kept in LDS

struct FlushCtx {
  f32x4* part;  // LDS [waves - 1][64]
  int* pflag;   // LDS [waves]: tag of the phase in which the wave last parked a tile
  unsigned tag;
  int trace_key;
  float* xpart;     // this phase's half of the cross-slice tiles in memory
  // buffers this phase puts the "empty" pattern back into (the first rearm_n floats, every workgroup
  // a share), before its stores are drained; null: none
  float* rearm[2];
  int rearm_n[2];
};

// Returns whether global memory was touched (false: the tile was parked in LDS and that is all).
template <int DT>
__device__ __forceinline__ bool flush_rowblock(const StageArgs& A, const WaveStream& S, int S_k, int rb,
                                               f32x4 acc, int lane, const EpiCtx& e, const float* rscale,
                                               const FlushCtx& F) {
  const int r = rb - S.rb0;
  const int first = uni((r * S.nt) / S.share);
  const int last = uni(((r + 1) * S.nt - 1) / S.share);
  if (last > first) {
    if (S.wave != first) {
      F.part[(S.wave - 1) * 64 + lane] = acc;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      if (lane == 0) __hip_atomic_store(F.pflag + S.wave, (int)F.tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      return false;
    }
    Deadline dl;
    for (unsigned spin = 0;; ++spin) {
      int missing = 0;
      for (int w = first + 1; w <= last; ++w)
        missing |= __hip_atomic_load(F.pflag + w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != (int)F.tag;
      if (!uni(missing)) break;
      __builtin_amdgcn_s_sleep(1);
      if (deadline_passed(dl, spin, A.timeout_ticks)) {
        if (lane == 0) __hip_atomic_store(&A.sync->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    for (int w = first + 1; w <= last; ++w) acc += F.part[(w - 1) * 64 + lane];
  }
  if (S_k > 1) {
    const bool live = (lane & 15) < e.n;
    const __amdgpu_buffer_rsrc_t pr = rsrc_of(F.xpart);
    if (S.slice != 0) {
      if (live) st_ag4(pr, ((rb * S_k + S.slice) * 64 + lane) * 16, acc);
      return true;
    }
    const u32x4 empty = {kEmptyWord, kEmptyWord, kEmptyWord, kEmptyWord};
    Deadline dl;
    for (int base = 1; base < S_k; base += 8) {  // slice 0 is this workgroup
      u32x4 t[8];
      int off[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) off[q] = ((rb * S_k + min(base + q, S_k - 1)) * 64 + lane) * 16;
      for (unsigned spin = 0;; ++spin) {
        bool ready = true;
#pragma unroll
        for (int q = 0; q < 8; ++q) t[q] = __builtin_amdgcn_raw_buffer_load_b128(pr, off[q], 0, kAgent);
#pragma unroll
        for (int q = 0; q < 8; ++q) ready = ready && (t[q][0] != kEmptyWord || t[q][1] != kEmptyWord);
        if (__builtin_amdgcn_ballot_w64(live && !ready) == 0) break;
        __builtin_amdgcn_s_sleep(1);
        if (deadline_passed(dl, spin, A.timeout_ticks)) {
          if (lane == 0) __hip_atomic_store(&A.sync->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        if (base + q < S_k && live) {
          acc += __builtin_bit_cast(f32x4, t[q]);
          __builtin_amdgcn_raw_buffer_store_b128(empty, pr, off[q], 0, kAgent);
        }
      }
    }
  }
  epilogue<DT>(e, rb, acc, lane, rscale);
  return true;
}

// ---- the MFMA inner step ----------------------------------------------------------------------
struct ConsumeState {
  int f, rb, t;  // flat cursor, absolute row block, tile within the slice's part of it
  // Two accumulators, one per operand half (bf16: hi and lo parts of the activations; fp32: first
  // and last four columns of the tile): two independent chains of matrix instructions instead of
  // one in which every instruction waits for the one before.  Their sum is the row block's tile.
  f32x4 acc0, acc1;
  int pending;   // a row block ended in the last pass: its tile is pacc, its number prb
  int prb;
  f32x4 pacc;
};

// Per-lane constants of a pass.
struct PassLane {
  int lane16;      // byte offset of the lane's 16 bytes in a weight tile
  const char* b0;  // the lane's operand halves of tile 0
  const char* b1;
  float wscale;    // 8-bit weights: the power-of-two scale the conversion applies
};

// One weight tile times its operand slots, added to the two accumulators.  `w` is the lane's 16 bytes of
// the tile (fp32: `w` and `w2`, its two halves), `sc4` the lane's row's four scale bytes (block-scaled
// weights), x0 / x1 the operand halves of the tile's 32-column parts.
template <int DT>
__device__ __forceinline__ void tile_mfma(ConsumeState& C, u32x4 w, u32x4 w2, uint32_t sc4, const u32x4* x0,
                                          const u32x4* x1, float wscale) {
  if constexpr (DT == kWeightBF16) {
    const bf16x8 av = __builtin_bit_cast(bf16x8, w);
    C.acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, x0[0]), C.acc0, 0, 0, 0);
    C.acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, x1[0]), C.acc1, 0, 0, 0);
  } else if constexpr (DT == kWeightFP8) {
    // sixteen bytes -> two bf16 operands; the conversion is exact (three mantissa bits) and
    // applies the model's power-of-two scale on the way
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      u32x4 o;
      o[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[2 * h], wscale, false));
      o[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[2 * h], wscale, true));
      o[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[2 * h + 1], wscale, false));
      o[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[2 * h + 1], wscale, true));
      const bf16x8 av = __builtin_bit_cast(bf16x8, o);
      C.acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, x0[h]), C.acc0, 0, 0, 0);
      C.acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, x1[h]), C.acc1, 0, 0, 0);
    }
  } else if constexpr (weight_is_fp4(DT)) {
    // sixteen bytes -> four bf16 operands (one per 32 columns), one byte = two weights; with
    // block scales each of the four has the scale of its own 32 columns of the lane's row,
    // 2^(byte - 127), which is the float whose exponent field is that byte
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      float sc = wscale;
      if constexpr (DT == kWeightFP4B) sc = __uint_as_float(((sc4 >> (8 * h)) & 0xffu) << 23);
      u32x4 o;
      o[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[h], sc, 0));
      o[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[h], sc, 1));
      o[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[h], sc, 2));
      o[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[h], sc, 3));
      const bf16x8 av = __builtin_bit_cast(bf16x8, o);
      C.acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, x0[h]), C.acc0, 0, 0, 0);
      C.acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, x1[h]), C.acc1, 0, 0, 0);
    }
  } else {
    const f32x4 w0 = __builtin_bit_cast(f32x4, w), w1 = __builtin_bit_cast(f32x4, w2);
    const f32x4 a0 = __builtin_bit_cast(f32x4, x0[0]), a1 = __builtin_bit_cast(f32x4, x1[0]);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      C.acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(w0[q], a0[q], C.acc0, 0, 0, 0);
      C.acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(w1[q], a1[q], C.acc1, 0, 0, 0);
    }
  }
}

// A group of slots is consumed in a straight line behind one wave-uniform branch.  All operand
// reads of the group are issued first and the matrix instructions follow, so the LDS latency is
// paid once per group rather than twice per tile; a slot past the consumer's end multiplies by
// the all-zero operand slots.
template <int DT, int UR, int J0, int J1>
__device__ __forceinline__ void consume_group(const Ring<DT, UR>& R, ConsumeState& C, const PassPlan& P,
                                              const PassLane& PLn) {
  constexpr int NG = J1 - J0;
  constexpr int NX = weight_tile_cols(DT) / 32;  // 32-column operand slots per weight tile
  u32x4 x0[NG][NX], x1[NG][NX];
#pragma unroll
  for (int j = 0; j < NG; ++j) {
    const int J = J0 + j;
    const int off = J < P.nc ? (J < P.ec ? P.cbaseA : P.cbaseB) + J * P.stride : P.zoff;
    x0[j][0] = *(const u32x4*)(PLn.b0 + off);
    x1[j][0] = *(const u32x4*)(PLn.b1 + off);
#pragma unroll
    for (int h = 1; h < NX; ++h) {  // the tile's further parts: the next operand slots (the zero slot has no neighbours)
      const int offh = J < P.nc ? off + h * (P.stride / NX) : P.zoff;
      x0[j][h] = *(const u32x4*)(PLn.b0 + offh);
      x1[j][h] = *(const u32x4*)(PLn.b1 + offh);
    }
  }
#pragma unroll
  for (int j = 0; j < NG; ++j) {
    const int J = J0 + j;
    if constexpr (DT == kWeightF32) tile_mfma<DT>(C, R.r[2 * J], R.r[2 * J + 1], 0u, x0[j], x1[j], PLn.wscale);
    else tile_mfma<DT>(C, R.r[J], R.r[J], R.s[DT == kWeightFP4B ? J : 0], x0[j], x1[j], PLn.wscale);
    if (__builtin_expect(J == P.ec - 1 && J < P.nc, 0)) {  // the row block's last tile: set its sum aside
      C.pacc = C.acc0 + C.acc1;
      C.acc0 = f32x4{0.f, 0.f, 0.f, 0.f};
      C.acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
}

// The tiles that were asked for ahead of the phase: four at a time (an even count: the last group may
// hold two) from the wave's LDS region, all of the consumer's current row block, which does not end
// among them.
template <int DT>
__device__ __forceinline__ void consume_parked(ConsumeState& C, const PassLane& PLn, const char* region, int count,
                                               int stride) {
  constexpr int NX = weight_tile_cols(DT) / 32;
  int i = 0;
  for (; i + 4 <= count; i += 4) {
    u32x4 w[4], x0[4][NX], x1[4][NX];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      w[j] = *(const u32x4*)(region + (i + j) * 1024 + PLn.lane16);
      const int off = (C.t + i + j) * stride;
#pragma unroll
      for (int h = 0; h < NX; ++h) {
        x0[j][h] = *(const u32x4*)(PLn.b0 + off + h * (stride / NX));
        x1[j][h] = *(const u32x4*)(PLn.b1 + off + h * (stride / NX));
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) tile_mfma<DT>(C, w[j], w[j], 0u, x0[j], x1[j], PLn.wscale);
  }
  if (i < count) {
    u32x4 w[2], x0[2][NX], x1[2][NX];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      w[j] = *(const u32x4*)(region + (i + j) * 1024 + PLn.lane16);
      const int off = (C.t + i + j) * stride;
#pragma unroll
      for (int h = 0; h < NX; ++h) {
        x0[j][h] = *(const u32x4*)(PLn.b0 + off + h * (stride / NX));
        x1[j][h] = *(const u32x4*)(PLn.b1 + off + h * (stride / NX));
      }
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) tile_mfma<DT>(C, w[j], w[j], 0u, x0[j], x1[j], PLn.wscale);
  }
  C.f += count;
  C.t += count;
}

// One pass over the ring, in groups of kGroup slots: the group's tiles are consumed (skipped as a
// whole when the consumer has nothing for the group), then the group's slots are refilled,
// outside any branch.
template <int DT>
constexpr int group_size() { return DT == kWeightBF16 ? 4 : 2; }  // (a 4-bit tile has four operand slots: sixteen live operand registers per slot)
template <int DT, int UR, int J0>
__device__ __forceinline__ void ring_pass(Ring<DT, UR>& R, const WaveStream& S, ConsumeState& C, const PassPlan& P,
                                          const PassLane& PLn) {
  if constexpr (J0 < UR) {
    constexpr int J1 = J0 + group_size<DT>() < UR ? J0 + group_size<DT>() : UR;
    if (J0 < P.nc) consume_group<DT, UR, J0, J1>(R, C, P, PLn);
    issue_slots<DT, UR, J0, J1>(R, S, P, PLn.lane16);
    ring_pass<DT, UR, J1>(R, S, C, P, PLn);
  }
}

// Stream this wave's range of the phase; the ring already holds its first tiles.
template <int DT, int UR>
__device__ __forceinline__ void consume_phase(const StageArgs& A, Ring<DT, UR>& R, WaveStream& S, int S_k,
                                              const char* lds, int n, int lane, const EpiCtx& e,
                                              const float* rscale, const FlushCtx& F, const MatDev next, bool has_next,
                                              int next_sk, int wave, int pidx, bool park_now) {
  constexpr int TB = Ring<DT, UR>::kTileBytes;
  ConsumeState C;
  C.f = S.f0;
  const int q0 = uni(S.f0 / S.nt);
  C.rb = S.rb0 + q0;
  C.t = S.f0 - q0 * S.nt;
  C.acc0 = C.acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
  C.pending = 0;
  C.prb = 0;
  C.pacc = C.acc0;
  PassLane PLn;
  PLn.lane16 = lane * 16;
  PLn.b0 = lds + ((lane >> 4) * n + min(lane & 15, n - 1)) * 16;
  constexpr int KX = weight_tile_cols(DT) / 32;  // 32-column operand slots per weight tile
  PLn.b1 = PLn.b0 + (KX * S.nt + 1) * 64 * n;
  PLn.wscale = A.wscale;
  if (S.pf > 0) {
    consume_parked<DT>(C, PLn, park_region(A, const_cast<char*>(lds), pidx, wave), S.pf, KX * 64 * n);
    C.f = uni(C.f);
    C.t = uni(C.t);
  }

  // The compiler treats the vector memory counter as unordered while loads AND stores are pending
  // and then waits for everything before it touches a ring slot -- in every pass of the loop, once
  // that state has reached the loop header.  So stores are waited for, in a form the compiler sees,
  // before the loop and after every flush; between flushes the passes wait for exactly one slot.
  while (C.f < S.f1) {
    PassPlan P;
    P.stride = KX * 64 * n;
    P.zoff = S.nt * P.stride;
    P.nc = min(UR, S.f1 - C.f);
    P.ec = S.nt - C.t;
    P.cbaseA = C.t * P.stride;
    P.cbaseB = -P.ec * P.stride;
    plan_loads<UR>(P, S, TB);
    ring_pass<DT, UR, 0>(R, S, C, P, PLn);
    advance_loads(S, P, TB);
    C.f += P.nc;
    if (P.ec <= P.nc) {  // a row block ended in this pass
      // (a tile parked in LDS leaves no store behind: the ring stays in flight across it)
      if (flush_rowblock<DT>(A, S, S_k, C.rb, C.pacc, lane, e, rscale, F)) wave_settle();
      C.rb += 1;
      C.t = P.nc - P.ec;
    } else {
      C.t += P.nc;
    }
    C.f = uni(C.f);
    C.t = uni(C.t);
    C.rb = uni(C.rb);
  }
  if (C.t > 0) (void)flush_rowblock<DT>(A, S, S_k, C.rb, C.acc0 + C.acc1, lane, e, rscale, F);  // range ends inside a row block
#pragma unroll  // (a loop over the two entries would index them at run time and put the context into scratch memory)
  for (int b = 0; b < 2; ++b) {
    if (!F.rearm[b]) continue;
    const int pieces = F.rearm_n[b] / 4, per = (pieces + (int)gridDim.x - 1) / (int)gridDim.x;
    const __amdgpu_buffer_rsrc_t rr = rsrc_of(F.rearm[b]);
    const u32x4 empty = {kEmptyWord, kEmptyWord, kEmptyWord, kEmptyWord};
    for (int j = (int)threadIdx.x; j < per; j += kThreads) {
      const int piece = (int)blockIdx.x * per + j;
      if (piece < pieces) __builtin_amdgcn_raw_buffer_store_b128(empty, rr, piece * 16, 0, kAgent);
    }
  }
  // The wave's place in the next phase is worked out (integer divisions) while its stores are on their
  // way.  (The next matrix by value: through a pointer it would sit in scratch memory, one round trip
  // away.)
  if (has_next) stream_init<DT>(S, next, next_sk, wave);
  wave_drain();  // this wave's stores are complete (the wait also covers loads, so it comes first)
  // (park_now is set behind gate/up only: the down projection follows; elsewhere the next phase's first
  // tiles are asked for behind the arrival at the grid barrier)
  if (has_next && park_now) stream_park<DT>(S, park_region(A, const_cast<char*>(lds), 3, wave), park_cap(A, 3), lane);
}

// ---- attention phase ----------------------------------------------------------------------------
// Work unit = (kv head, range of prefix cells); the last unit of a head also takes the run's
// window cells.  The unit's K rows and V columns are staged in LDS once (one round trip), then
//   S = K Q^T      MFMA, K rows as A operand straight from LDS, Q split into bf16 hi + lo
//   P = exp(S - rowmax), row sums          (whole unit at once: no running rescale)
//   O = P V        MFMA, V stored transposed in LDS so cells are the contraction index
// for all G*n query rows of the kv head, 32 rows at a time.  Each unit parks (max, sum, O); the
// last unit of a head to arrive merges them in unit order.
constexpr int kRG = 32;  // query rows per pass

struct AttnLds {
  int cp;       // cells of the unit padded to a multiple of 32
  int kstride;  // bytes per K / Q row
  int vstride;  // bytes per V^T / P row
  int k_off[2], v_off[2], q_off[2], p_off[2], max_off, sum_off, flag_off;
  int total;
};

__host__ __device__ inline AttnLds attn_lds_layout(int hd, int cp, int n_split) {
  AttnLds L;
  L.cp = cp;
  L.kstride = hd * 2 + 16;
  L.vstride = cp * 2 + 16;
  int off = 0;
  for (int s = 0; s < 2; ++s) {
    L.k_off[s] = off;
    if (s < n_split) off += cp * L.kstride;
  }
  for (int s = 0; s < 2; ++s) {
    L.v_off[s] = off;
    if (s < n_split) off += hd * L.vstride;
  }
  for (int s = 0; s < 2; ++s) {
    L.q_off[s] = off;
    off += kRG * L.kstride;
  }
  for (int s = 0; s < 2; ++s) {
    L.p_off[s] = off;
    off += kRG * L.vstride;
  }
  L.max_off = off;
  off += kWaves * kRG * 4;
  L.sum_off = off;
  off += kWaves * kRG * 4;
  L.flag_off = off;
  off += 16;
  L.total = off;
  return L;
}


template <int HD, int DT>
__device__ void attn_unit(const StageArgs& A, const char* kl, const char* vl, int h, int u, char* lds, unsigned tag) {
  constexpr int NS = DT != kWeightF32 ? 1 : 2;  // bf16 terms per cache value
  constexpr int ES = DT != kWeightF32 ? 2 : 4;
  constexpr int KSTEPS = HD / 32;
  constexpr int DTILES = HD / 16;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, l16 = lane & 15;
  const int G = A.n_q_heads / A.n_kv_heads;
  const int R = G * A.n;
  const int upH = A.attn_units_per_head;
  const bool has_window = u == upH - 1;
  const int p_begin = min(A.prefix_len, u * A.attn_chunk);
  const int p_end = min(A.prefix_len, p_begin + A.attn_chunk);
  const int npc = p_end - p_begin;
  uint64_t any = 0;
  for (int i = 0; i < A.n; ++i) any |= A.mask[i];
  const int wcells = has_window ? min(64 - (int)__builtin_clzll(any | 1ull), A.n_cells - A.window_base) : 0;
  const int cells = npc + wcells;
  const int CP = (cells + 31) & ~31;
  const AttnLds L = attn_lds_layout(HD, CP, NS);
  const float scale = 1.0f / sqrtf((float)HD);
  const size_t head_elems = (size_t)h * A.n_cells * HD;

  __syncthreads();  // LDS of the previous unit / phase is free
  // No grid barrier separates this phase from the QKV projection.  The unit that takes the window
  // waits (bounded) until the words of its head's K and V row blocks carry this layer's tag: the
  // run's cells are then in memory.  (Prefix cells are older than the launch.)
  if (has_window) {
    const int blocks = HD / 16, kv_blocks = A.n_kv_heads * blocks;
    for (unsigned spin = 0;; ++spin) {
      bool missing = false;
      if (tid < 2 * blocks) {
        const int w = (tid < blocks ? 0 : kv_blocks) + h * blocks + (tid % blocks);
        const unsigned f = __hip_atomic_load(A.kv_ready + w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        missing = (int)(f - tag) < 0;
      }
      if (!__syncthreads_or(missing)) break;
      if (spin >= kPollLimit) {
        if (tid == 0) __hip_atomic_store(&A.sync->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
  }
  // ---- stage K rows and V columns (as bf16 terms) ----
  {
    const __amdgpu_buffer_rsrc_t kr = rsrc_of(kl), vr = rsrc_of(vl);
    const int items = CP * (HD / 8);
    constexpr int KB = 4;  // items per thread whose loads are in flight together
    for (int it0 = 0; it0 < items; it0 += kThreads * KB) {
      u32x4 kraw[KB][NS], vraw[KB][NS];
      int lc[KB], d8[KB];
      bool live[KB];
#pragma unroll
      for (int q = 0; q < KB; ++q) {
        const int it = it0 + q * kThreads + tid;
        lc[q] = it / (HD / 8);
        d8[q] = (it % (HD / 8)) * 8;
        live[q] = it < items && lc[q] < cells;
        // Branch-free so that all loads of the batch are in flight together (a branch around a
        // load makes the compiler wait for it at the join); a dead item re-reads the head's first
        // bytes.  Every cell is read once per layer, and the window cells were written by other
        // workgroups in this launch, so all loads bypass the per-XCD L2.
        const bool win = lc[q] >= npc;
        const int cell = !live[q] ? 0 : (win ? A.window_base + (lc[q] - npc) : p_begin + lc[q]);
        const int off = (int)((head_elems + (size_t)cell * HD + (live[q] ? d8[q] : 0)) * ES);
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          kraw[q][s] = __builtin_amdgcn_raw_buffer_load_b128(kr, off + 16 * s, 0, kAgent);
          vraw[q][s] = __builtin_amdgcn_raw_buffer_load_b128(vr, off + 16 * s, 0, kAgent);
        }
      }
#pragma unroll
      for (int q = 0; q < KB; ++q) {
        const int it = it0 + q * kThreads + tid;
        if (it >= items) continue;
        uint32_t kw[2][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}}, vw[2][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
        if (live[q]) {
          if (NS == 1) {
#pragma unroll
            for (int j = 0; j < 4; ++j) { kw[0][j] = kraw[q][0][j]; vw[0][j] = vraw[q][0][j]; }
          } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const float k0 = __uint_as_float(kraw[q][j >> 1][(2 * j) & 3]), k1 = __uint_as_float(kraw[q][j >> 1][(2 * j + 1) & 3]);
              const float v0 = __uint_as_float(vraw[q][j >> 1][(2 * j) & 3]), v1 = __uint_as_float(vraw[q][j >> 1][(2 * j + 1) & 3]);
              kw[0][j] = pack_bf16(k0, k1);
              vw[0][j] = pack_bf16(v0, v1);
              kw[1][j] = pack_bf16(k0 - bf16_low_f32(kw[0][j]), k1 - bf16_high_f32(kw[0][j]));
              vw[1][j] = pack_bf16(v0 - bf16_low_f32(vw[0][j]), v1 - bf16_high_f32(vw[0][j]));
            }
          }
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          *(uint4*)(lds + L.k_off[s] + lc[q] * L.kstride + d8[q] * 2) = make_uint4(kw[s][0], kw[s][1], kw[s][2], kw[s][3]);
          uint16_t* vt = (uint16_t*)(lds + L.v_off[s]);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            vt[(d8[q] + 2 * j) * (L.vstride / 2) + lc[q]] = (uint16_t)vw[s][j];
            vt[(d8[q] + 2 * j + 1) * (L.vstride / 2) + lc[q]] = (uint16_t)(vw[s][j] >> 16);
          }
        }
      }
    }
  }
  const int n_ct = CP / 16;  // cell tiles
  float* rowmax = (float*)(lds + L.max_off);
  float* rowsum = (float*)(lds + L.sum_off);
  const size_t ubase = ((size_t)h * upH + u) * R;
  const __amdgpu_buffer_rsrc_t qr = rsrc_of(A.q), por = rsrc_of(A.attn_o);

  for (int r0 = 0; r0 < R; r0 += kRG) {
    const int rows = min(kRG, R - r0);
    __syncthreads();
    // ---- stage the query rows as bf16 hi + lo ----
    // The queries may still be on their way: a piece that reads "empty" is read again (bounded).
    constexpr int QI = (kRG * (HD / 4) + kThreads - 1) / kThreads;  // items per thread
    f32x4 qv[QI];
    int qoff[QI];
#pragma unroll
    for (int k = 0; k < QI; ++k) {
      const int it = tid + k * kThreads;
      const int rr = it / (HD / 4), d4 = (it % (HD / 4)) * 4;
      const int r = r0 + rr, gq = r / A.n, i = r % A.n;
      qoff[k] = it < kRG * (HD / 4) && rr < rows ? ((i * A.n_q_heads + h * G + gq) * HD + d4) * 4 : -1;
      qv[k] = ld_ag4(qr, qoff[k] < 0 ? 0 : qoff[k]);
    }
    for (unsigned spin = 0;; ++spin) {
      bool missing = false;
#pragma unroll
      for (int k = 0; k < QI; ++k)
        missing = missing || (qoff[k] >= 0 && __float_as_uint(qv[k][0]) == kEmptyWord && __float_as_uint(qv[k][1]) == kEmptyWord);
      if (!__syncthreads_or(missing)) break;
      if (spin >= kPollLimit) {
        if (tid == 0) __hip_atomic_store(&A.sync->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      __builtin_amdgcn_s_sleep(1);
#pragma unroll
      for (int k = 0; k < QI; ++k) qv[k] = ld_ag4(qr, qoff[k] < 0 ? 0 : qoff[k]);
    }
#pragma unroll
    for (int k = 0; k < QI; ++k) {
      const int it = tid + k * kThreads;
      if (it >= kRG * (HD / 4)) continue;
      const int rr = it / (HD / 4), d4 = (it % (HD / 4)) * 4;
      const f32x4 v = qoff[k] >= 0 ? qv[k] : f32x4{0.f, 0.f, 0.f, 0.f};
      const uint32_t h0 = pack_bf16(v[0], v[1]), h1 = pack_bf16(v[2], v[3]);
      const uint32_t l0 = pack_bf16(v[0] - bf16_low_f32(h0), v[1] - bf16_high_f32(h0));
      const uint32_t l1 = pack_bf16(v[2] - bf16_low_f32(h1), v[3] - bf16_high_f32(h1));
      *(uint2*)(lds + L.q_off[0] + rr * L.kstride + d4 * 2) = make_uint2(h0, h1);
      *(uint2*)(lds + L.q_off[1] + rr * L.kstride + d4 * 2) = make_uint2(l0, l1);
    }
    __syncthreads();
    // ---- scores: this wave's cell tiles x both row tiles ----
    f32x4 sacc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) sacc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      const int ct = wave + a * kWaves;
      if (ct < n_ct) {
#pragma unroll
        for (int j = 0; j < KSTEPS; ++j) {
          bf16x8 kop[NS];
#pragma unroll
          for (int s = 0; s < NS; ++s)
            kop[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(lds + L.k_off[s] + (ct * 16 + l16) * L.kstride + j * 64 + g * 16));
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            const bf16x8 qh = __builtin_bit_cast(bf16x8, *(const u32x4*)(lds + L.q_off[0] + (b * 16 + l16) * L.kstride + j * 64 + g * 16));
            const bf16x8 ql = __builtin_bit_cast(bf16x8, *(const u32x4*)(lds + L.q_off[1] + (b * 16 + l16) * L.kstride + j * 64 + g * 16));
            sacc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[0], qh, sacc[a][b], 0, 0, 0);
            sacc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[0], ql, sacc[a][b], 0, 0, 0);
            if (NS == 2) sacc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[NS - 1], qh, sacc[a][b], 0, 0, 0);
          }
        }
      }
    }
    // scale, mask, per-wave row maxima.  Lane (l16, g) holds cells ct*16 + 4g + 0..3 of row b*16 + l16.
    float wmax[2] = {-INFINITY, -INFINITY};
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int rr = b * 16 + l16;
      const bool row_live = rr < rows;
      const uint64_t mword = row_live ? A.mask[(r0 + rr) % A.n] : 0ull;
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const int ct = wave + a * kWaves;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int lc = ct * 16 + 4 * g + q;
          bool vis = row_live && ct < n_ct && lc < cells;
          if (vis && lc >= npc) vis = (mword >> (lc - npc)) & 1ull;
          const float sv = vis ? sacc[a][b][q] * scale : -INFINITY;
          sacc[a][b][q] = sv;
          wmax[b] = fmaxf(wmax[b], sv);
        }
      }
      wmax[b] = fmaxf(wmax[b], __shfl_xor(wmax[b], 16));
      wmax[b] = fmaxf(wmax[b], __shfl_xor(wmax[b], 32));
      if (g == 0) rowmax[wave * kRG + rr] = wmax[b];
    }
    __syncthreads();
    float M[2], wsum[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int rr = b * 16 + l16;
      float m = -INFINITY;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) m = fmaxf(m, rowmax[w * kRG + rr]);
      M[b] = m;
      wsum[b] = 0.0f;
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const int ct = wave + a * kWaves;
        if (ct < n_ct) {
          float p[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            p[q] = sacc[a][b][q] == -INFINITY ? 0.0f : expf(sacc[a][b][q] - m);
            wsum[b] += p[q];
          }
          const uint32_t h0 = pack_bf16(p[0], p[1]), h1 = pack_bf16(p[2], p[3]);
          const uint32_t l0 = pack_bf16(p[0] - bf16_low_f32(h0), p[1] - bf16_high_f32(h0));
          const uint32_t l1 = pack_bf16(p[2] - bf16_low_f32(h1), p[3] - bf16_high_f32(h1));
          *(uint2*)(lds + L.p_off[0] + rr * L.vstride + (ct * 16 + 4 * g) * 2) = make_uint2(h0, h1);
          *(uint2*)(lds + L.p_off[1] + rr * L.vstride + (ct * 16 + 4 * g) * 2) = make_uint2(l0, l1);
        }
      }
      wsum[b] += __shfl_xor(wsum[b], 16);
      wsum[b] += __shfl_xor(wsum[b], 32);
      if (g == 0) rowsum[wave * kRG + rr] = wsum[b];
    }
    __syncthreads();
    // ---- O = P V : wave w owns head-dim tile w ----
    if (wave < DTILES) {
      f32x4 oacc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
      for (int cpair = 0; cpair < CP / 32; ++cpair) {
        bf16x8 vop[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s)
          vop[s] = __builtin_bit_cast(bf16x8, *(const u32x4*)(lds + L.v_off[s] + (wave * 16 + l16) * L.vstride + (cpair * 32 + 8 * g) * 2));
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const bf16x8 ph = __builtin_bit_cast(bf16x8, *(const u32x4*)(lds + L.p_off[0] + (b * 16 + l16) * L.vstride + (cpair * 32 + 8 * g) * 2));
          const bf16x8 pl = __builtin_bit_cast(bf16x8, *(const u32x4*)(lds + L.p_off[1] + (b * 16 + l16) * L.vstride + (cpair * 32 + 8 * g) * 2));
          oacc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[0], ph, oacc[b], 0, 0, 0);
          oacc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[0], pl, oacc[b], 0, 0, 0);
          if (NS == 2) oacc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[NS - 1], ph, oacc[b], 0, 0, 0);
        }
      }
      // lane (l16, g) holds O[row b*16 + l16][d = wave*16 + 4g + 0..3]
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int rr = b * 16 + l16;
        if (rr < rows) st_ag4(por, (int)(((ubase + r0 + rr) * HD + wave * 16 + 4 * g) * 4), oacc[b]);
      }
    }
    if (tid < rows) {
      float m = -INFINITY, sum = 0.0f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) m = fmaxf(m, rowmax[w * kRG + tid]);
#pragma unroll
      for (int w = 0; w < kWaves; ++w) sum += rowsum[w * kRG + tid];
      st_ag(A.attn_ml + (ubase + r0 + tid) * 2, m);
      st_ag(A.attn_ml + (ubase + r0 + tid) * 2 + 1, sum);
    }
  }
  // publish: this unit's partial results are in memory
  wave_drain();
  __syncthreads();
  if (tid == 0) __hip_atomic_store(A.attn_flags + h * A.attn_flag_stride + u, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Merge step of unit (h, u): wait (bounded) until every unit of kv head h has published, then
// combine the units, in unit order, for this unit's share of the head's query rows.
template <int HD, int DT>
__device__ bool attn_merge(const StageArgs& A, int h, int u, unsigned tag, int* sh) {
  const int tid = threadIdx.x;
  const int G = A.n_q_heads / A.n_kv_heads;
  const int R = G * A.n;
  const int upH = A.attn_units_per_head;
  if (u >= R) return true;  // no row for this unit
  if (tid < 64) {
    Deadline dl;
    int ok = 1;
    for (unsigned spin = 0;; ++spin) {
      bool all = true;
      for (int b = tid; b < upH; b += 64) {
        const unsigned f = __hip_atomic_load(A.attn_flags + h * A.attn_flag_stride + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        all = all && (int)(f - tag) >= 0;
      }
      if (__builtin_amdgcn_ballot_w64(!all) == 0) break;
      __builtin_amdgcn_s_sleep(1);
      if (deadline_passed(dl, spin, A.timeout_ticks)) {
        ok = 0;
        break;
      }
    }
    if (tid == 0) {
      if (!ok) __hip_atomic_store(&A.sync->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      sh[0] = ok;
    }
  }
  __syncthreads();
  if (!__builtin_amdgcn_readfirstlane(sh[0])) return false;
  const __amdgpu_buffer_rsrc_t por = rsrc_of(A.attn_o), mlr = rsrc_of(A.attn_ml);
  const int my_rows = (R - u + upH - 1) / upH;
  for (int e = tid; e < my_rows * (HD / 4); e += kThreads) {
    const int r = u + (e / (HD / 4)) * upH, d4 = (e % (HD / 4)) * 4;
    const int hb = h * upH;
    // running merge in unit order, eight units' loads in flight at a time
    float Mx = -INFINITY, Ls = 0.0f;
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    for (int u0 = 0; u0 < upH; u0 += 8) {
      u32x2 ml[8];
      f32x4 po[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int uu = min(u0 + q, upH - 1);
        ml[q] = __builtin_amdgcn_raw_buffer_load_b64(mlr, (int)(((hb + uu) * R + r) * 8), 0, kAgent);
        po[q] = ld_ag4(por, (int)((((hb + uu) * R + r) * HD + d4) * 4));
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        if (u0 + q >= upH) continue;
        const float m = __uint_as_float(ml[q][0]), l = __uint_as_float(ml[q][1]);
        if (m == -INFINITY) continue;
        const float mn = fmaxf(Mx, m);
        const float a = Mx == -INFINITY ? 0.0f : expf(Mx - mn), b = expf(m - mn);
        Ls = Ls * a + l * b;
        o = o * a + po[q] * b;
        Mx = mn;
      }
    }
    const int gq = r / A.n, i = r % A.n;
    const float inv = 1.0f / Ls;
    // (in the staged form: the output projection is its only reader)
    store_staged4<DT>((char*)A.o, A.n_q_heads * HD, A.n, i, (h * G + gq) * HD + d4, o * inv);
  }
  return true;
}

// Which workgroup takes which unit is decided when the workgroups get here: each draws tickets from a
// counter (the same number of draws for everyone, so a layer's tickets start at a known value), and a
// ticket below the number of units is that unit.  The workgroups that finish the QKV projection first
// draw the units, and when there are fewer units than workgroups the slowest -- whose queries
// everyone waits for anyway -- draw none: the phase then ends one unit's work after the last query
// is in memory, not after the slowest workgroup has also staged and worked a unit of its own.
// Results do not depend on who computes what (units are merged in unit order).
// All units first, then all merges: a workgroup never waits while it still owes a unit, so the
// waits in the merge step cannot deadlock even when a workgroup serves several units.
constexpr int kMaxAttnRounds = 64;
// `between` runs in every wave when the workgroup's units are done (LDS is free from then on) and before
// its merge steps wait for the other units.
template <int DT, typename Between>
__device__ __forceinline__ bool attention_phase(const StageArgs& A, const char* kl, const char* vl, char* lds, unsigned tag,
                                                int* sh, int* tickets, int layer_rel, Between&& between) {
  const int units = A.n_kv_heads * A.attn_units_per_head;
  const int rounds = (units + (int)gridDim.x - 1) / (int)gridDim.x;  // <= kMaxAttnRounds (host)
  const unsigned base = (unsigned)layer_rel * (unsigned)rounds * gridDim.x;
  for (int r = 0; r < rounds; ++r) {
    if (threadIdx.x == 0)
      tickets[r] = (int)(__hip_atomic_fetch_add(A.attn_ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - base);
    __syncthreads();
    const int w = __builtin_amdgcn_readfirstlane(tickets[r]);
    if (w >= units) continue;
    const int h = w / A.attn_units_per_head, u = w % A.attn_units_per_head;
    switch (A.head_dim) {
      case 32: attn_unit<32, DT>(A, kl, vl, h, u, lds, tag); break;
      case 64: attn_unit<64, DT>(A, kl, vl, h, u, lds, tag); break;
      default: attn_unit<128, DT>(A, kl, vl, h, u, lds, tag); break;
    }
  }
  between();
  bool ok = true;
  for (int r = 0; ok && r < rounds; ++r) {
    const int w = __builtin_amdgcn_readfirstlane(tickets[r]);
    if (w >= units) continue;
    const int h = w / A.attn_units_per_head, u = w % A.attn_units_per_head;
    switch (A.head_dim) {
      case 32: ok = attn_merge<32, DT>(A, h, u, tag, sh); break;
      case 64: ok = attn_merge<64, DT>(A, h, u, tag, sh); break;
      default: ok = attn_merge<128, DT>(A, h, u, tag, sh); break;
    }
  }
  wave_drain();
  return ok;
}

// ---- stage input / output ---------------------------------------------------------------------
// (also writes the staged form of the residual stream, times the first layer's attention gain)
template <int DT>
__device__ void embed_phase(const StageArgs& A, const float* gain) {
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
      const f32x4 gn = *(const f32x4*)(gain + c);
      store_staged4<DT>(A.xs, A.d, A.n, i, c, f32x4{v[0], v[1], v[2], v[3]} * gn);
    }
    float s = sum_sq4(v[0], v[1], v[2], v[3]);
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
template <int DT, int UR>
__device__ __forceinline__ void proj_phase(const StageArgs& A, Ring<DT, UR>& R, WaveStream& S, int S_k,
                                           const char* xin, bool scaled, int K,
                                           const EpiCtx& e, char* lds, int* pflag, unsigned tag, int lane,
                                           const MatDev next, bool has_next, int next_sk, int wave, int trace_layer,
                                           bool poll_x, int kind) {
  const int pidx = kind == 0 ? 0 : kind - 1;  // index of the phase's plan: QKV, O, gate/up, down, LM head
  if (poll_x) __syncthreads();  // no grid barrier came before: the workgroup's slower waves are done with LDS
  stream_make_uniform(S);
  constexpr int KX = weight_tile_cols(DT) / 32;  // activations are staged in 32-column slots whatever the weight tile
  const size_t xbytes = (size_t)(KX * S.nt + 1) * 128 * A.n;
  float* red = (float*)(lds + xbytes);
  float* rscale = red + kThreads;
  FlushCtx F;
  F.part = (f32x4*)(rscale + 16);
  F.pflag = pflag;
  F.tag = tag;
  F.trace_key = trace_layer;
  // What the barrier-free phase changes wait on is put back to "empty" where every reader is known
  // to be done and a grid barrier still comes before the next writer: the attention output and
  // the queries at the end of gate/up (behind the barrier that follows O), the SwiGLU output at
  // the end of QKV (behind the layer boundary).
  F.rearm[0] = kind == 3 ? A.o : kind == 0 ? A.a : nullptr;
  F.rearm_n[0] = kind == 3 ? A.n * A.n_q_heads * A.head_dim : A.n * A.ffn;
  F.rearm[1] = kind == 3 ? A.q : nullptr;
  F.rearm_n[1] = A.n * A.n_q_heads * A.head_dim;
  // Phases in a row without a grid barrier between them (QKV, O; gate/up, down) use different
  // regions of the cross-slice tiles: a workgroup ahead in a later phase must not store into a
  // tile an earlier phase is still collecting.  Kinds 0, 2, 3, 4 -> regions 0, 2, 0, 1.
  F.xpart = A.part + (size_t)(kind % 3) * A.part_half_floats;
  f32x4* resid = F.part + (kWaves - 1) * 64;
  const int Gs = uni((int)gridDim.x / S_k);
  const int r_max = uni((S.NRB + Gs - 1) / Gs);
  f32x4* gres = resid + r_max * 64;  // behind the residual rows: the next projection's gains for the same rows
  const bool stage_resid = e.epi == EPI_RESID && r_max <= kMaxResidBlocks;  // as sized by the host
  // Nothing of the previous phase is pending any more (every wave drained before the barrier);
  // said in a form the compiler's counter tracking sees, so that the waits below are counted.
  wave_settle();
  // The residual rows of the workgroup's row blocks (at most one row block per wave): the load
  // goes out first and is parked in LDS behind the activations.
  const bool has_r = stage_resid && wave < S.R;
  f32x4 rv, gv;
  bool rv_live;
  {
    const int i = lane & 15, row = (S.rb0 + wave) * kRowBlock + (lane >> 4) * 4;
    rv_live = has_r && i < e.n && row < e.N;
    rv = ld_ag4(rsrc_of(e.out), rv_live ? (i * e.N + row) * 4 : 0);
    const bool gv_live = rv_live && e.gain_next;
    gv = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
        make_rsrc(e.gain_next ? e.gain_next : (const float*)xin, gv_live ? (uint32_t)e.N * 4u : 0u), gv_live ? row * 4 : 0, 0, 0));
  }
  bool timed_out = false;
  EpiCtx e2 = e;
  e2.resid = stage_resid ? resid : nullptr;
  e2.gres = stage_resid ? gres : nullptr;
  e2.rb0 = S.rb0;
  const auto park_resid = [&] {
    if (has_r) {
      resid[wave * 64 + lane] = rv_live ? rv : f32x4{0.f, 0.f, 0.f, 0.f};
      gres[wave * 64 + lane] = gv;
    }
  };
  // Where the phase's first tiles wait in LDS, the ring is asked for once the activations are
  // staged and fills while those tiles are consumed: nothing then travels ahead of the activations
  // (or of the re-reads of a phase that waits for them), which arrive 1.5-4 us earlier for it.
  // Elsewhere the ring goes out right behind the activation loads.
  const bool ring_late = park_cap(A, pidx) > 8;  // (fewer tiles are consumed before the ring's first tiles arrive)
  constexpr int kRingLoads = Ring<DT, UR>::kRegs + (DT == kWeightFP4B ? UR : 0);  // load instructions of one ring_prefetch
  stage_x<kRingLoads>(xin, K, A.n, KX * S.t0, KX * S.nt, lds, scaled ? A.ssq : nullptr, A.d / 16, A.eps, red, rscale,
                      [&] { ring_prefetch<DT, UR>(R, S, lane, !ring_late); }, park_resid, poll_x ? kPollLimit : 0u,
                      &timed_out, wave, lane);
  if (ring_late) ring_prefetch<DT, UR>(R, S, lane);
  if (timed_out && lane == 0) __hip_atomic_store(&A.sync->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  // (no global store may sit between the weight loads above and the streaming loop: with loads and
  // stores both pending the compiler stops counting and waits for everything at every ring slot)
  consume_phase<DT, UR>(A, R, S, S_k, lds, A.n, lane, e2, rscale, F, next, has_next, next_sk, wave, pidx,
                        /*park_now=*/kind == 3);  // drains its stores
  wg_mark(A, trace_layer, 2);
}

template <int DT, int UR>
__global__ void __launch_bounds__(kThreads, 1) stage_kernel(const StageArgs A) {
  extern __shared__ __align__(16) char lds[];
  __shared__ int bar_sh[2];
  __shared__ int attn_tickets[kMaxAttnRounds];
  __shared__ int pflag[kWaves];
  if (threadIdx.x < kWaves) pflag[threadIdx.x] = 0;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform: keep it scalar
  BarrierCtx bc;
  bc.epoch = A.epoch_base;
  bc.sh = bar_sh;
  bc.dead = 0;
  bc.dead_groups = 0;
  const int L = A.n_layers;

  // run latch (first wave of workgroup 0): validate the slots and positions (lane i: token i), probe
  // every run's cancel word once (lane g: run g)
  const unsigned all_tokens = (1u << A.n) - 1u;
  if (blockIdx.x == 0 && threadIdx.x < 64) {
    int status = PI_OK;
    unsigned dead = 0;
    const int len = *A.kv_len;
    bool bad = false, bad_pos = false;
    if (lane < A.n) {
      const int s = A.slots[lane];
      bad = s < len || s < A.window_base || s >= A.window_base + PI_WINDOW || s >= A.n_cells;
      // the rotary table has max_pos rows: a position outside it would be read out of bounds
      const int p = A.positions[lane];
      bad_pos = p < 0 || p >= A.max_pos;
    }
    const bool refused_slot = __builtin_amdgcn_ballot_w64(bad) != 0;
    const bool refused = refused_slot || __builtin_amdgcn_ballot_w64(bad_pos) != 0;
    const int refusal = refused_slot ? PI_E_SLOT_LIVE : PI_E_ARG;
    if (refused) {
      status = refusal;
      dead = all_tokens;
    }
    // a run that an earlier stage of the same pass reported cancelled stays cancelled, and its
    // entry (which says where it stopped) is left alone
    bool hit = false, before = false;
    if (!refused && A.group_status && lane < A.n_groups)
      before = __hip_atomic_load(A.group_status + 2 * lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == PI_CANCELLED;
    if (!refused && !before && A.cancel_flags && lane < A.n_groups)
      hit = __hip_atomic_load(A.cancel_flags + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != 0;
    hit = hit || before;
    const unsigned long long hits = __builtin_amdgcn_ballot_w64(hit);
    for (int g = 0; g < A.n_groups; ++g)
      if ((hits >> g) & 1ull) dead |= A.group_mask[g];
    if (!refused && dead == all_tokens) status = PI_CANCELLED;
    if (A.group_status && lane < A.n_groups && !before) {
      __hip_atomic_store(A.group_status + 2 * lane, refused ? refusal : (hit ? PI_CANCELLED : PI_OK), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(A.group_status + 2 * lane + 1, A.layer_begin, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    bc.dead = dead;
    bc.dead_groups = refused ? 0xffffffffu : (unsigned)hits;
    if (lane == 0) {
      __hip_atomic_store(&A.rs->status, status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&A.rs->layers_done, A.layer_begin, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(A.attn_ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // (two grid barriers before its first use)
    }
    wave_drain();
  }
  // the attention output, the SwiGLU output and the queries start "empty" whatever an earlier launch left behind
  for (int which = 0; which < 3; ++which) {
    const int pieces = A.n * (which == 1 ? A.ffn : A.n_q_heads * A.head_dim) / 4;
    const int per = (pieces + (int)gridDim.x - 1) / (int)gridDim.x;
    const __amdgpu_buffer_rsrc_t rr = rsrc_of(which == 0 ? A.o : which == 1 ? A.a : A.q);
    const u32x4 empty = {kEmptyWord, kEmptyWord, kEmptyWord, kEmptyWord};
    for (int j = (int)threadIdx.x; j < per; j += kThreads) {
      const int piece = (int)blockIdx.x * per + j;
      if (piece < pieces) __builtin_amdgcn_raw_buffer_store_b128(empty, rr, piece * 16, 0, kAgent);
    }
  }
  wave_drain();
  Ring<DT, UR> R;
  WaveStream S;
  bool ok = grid_barrier(A, bc, A.layer_begin, false);
  unsigned dead_tokens = (unsigned)__builtin_amdgcn_readfirstlane(bar_sh[1]);  // tokens of cancelled runs
  bool dead = dead_tokens == all_tokens;  // nothing left to do
  if (ok && !dead) {
    embed_phase<DT>(A, table_layer<DT>(A, A.layer_begin).attn_gain);
    stream_init<DT>(S, table_mat<DT>(A, A.layer_begin, 0), A.sk[0], wave);
    ok = grid_barrier(A, bc, -1, false, -1, [&] { stream_park<DT>(S, park_region(A, lds, 0, wave), park_cap(A, 0), lane); });
  }
  // One pass of this loop is one phase; phases 0, 2, 3, 4 of a layer are the projections (QKV,
  // O, gate/up, down), phase 1 is attention, and a final pass after the last layer is the LM
  // head.  A single copy of the projection code serves all of them.
  const int n_ph = (A.layer_end - A.layer_begin) * 5 + (A.layer_end == L ? 1 : 0);
  for (int ph = 0; ok && !dead && ph < n_ph; ++ph) {
    const int l = A.layer_begin + ph / 5;
    const int k = l < A.layer_end ? ph % 5 : 5;  // 5: LM head
    if (k == 1) {
      wg_mark(A, l * 8 + 1, 0);
      // The output projection's first tiles are asked for once the workgroup's units are done, ahead of its
      // merge steps: those wait for the other units anyway, and the workgroup that merges last is the one
      // the output projection waits for.  (Not where the projection is unsliced and twice as many tiles
      // are asked for: the merge steps' own loads return behind them, which costs what the order gains.)
      const bool ask_early = A.sk[1] > 1;
      const auto ask_o = [&] {
        stream_init<DT>(S, table_mat<DT>(A, l, 1), A.sk[1], wave);
        if (park_cap(A, 1) > 0) {
          // the tiles' region may overlap what slower waves of a workgroup without attention work still
          // read for the QKV projection
          __syncthreads();
          stream_park<DT>(S, park_region(A, lds, 1, wave), park_cap(A, 1), lane);
        }
      };
      if (!(ok = attention_phase<DT>(A, A.kbase + (size_t)l * A.kv_layer_bytes, A.vbase + (size_t)l * A.kv_layer_bytes, lds,
                                     bc.epoch + 1, bar_sh, attn_tickets, l - A.layer_begin, [&] { if (ask_early) ask_o(); })))
        break;
      wg_mark(A, l * 8 + 1, 2);
      if (!ask_early) ask_o();
      // No grid barrier here: the output projection asks for its weights at once and reads the
      // attention output until no piece of it is "empty" any more (the merging workgroups are
      // the last to finish this phase; everyone else's weight requests travel meanwhile).
      wg_mark(A, l * 8 + 1, 5);
      continue;
    }
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
    e.dead_tokens = dead_tokens;
    e.kv_ready = A.kv_ready;
    e.kv_tag = bc.epoch + 1;  // attention of this layer starts without a barrier in between and looks for the same number
    e.rope = A.rope;
    e.resid = nullptr;
    e.gres = nullptr;
    e.rb0 = 0;
    e.ssq_out = A.ssq;
    e.staged_out = nullptr;
    e.gain_next = nullptr;
    MatDev M, nxt;
    const char* xin;
    bool scaled = false, has_next = true;
    int sk, nsk = 1;
    if (k == 5) {  // final RMSNorm + LM head
      M = A.lm_head; sk = A.sk[4]; xin = A.xs; scaled = true;
      e.epi = EPI_LOGITS; e.out = A.logits_out; has_next = false; nxt = M;
    } else {
      const LayerDev W = table_layer<DT>(A, l);
      if (k == 0) {  // RMSNorm + QKV projection + RoPE + KV write
        M = W.qkv; sk = A.sk[0]; xin = A.xs; scaled = true;
        e.epi = EPI_QKV; e.out = A.q; has_next = false; nxt = M;
      } else if (k == 2) {  // output projection + residual
        M = W.o; sk = A.sk[1]; xin = (const char*)A.o; e.epi = EPI_RESID; e.out = A.x; nxt = W.gateup; nsk = A.sk[2];
        e.staged_out = A.xs; e.gain_next = W.ffn_gain;
      } else if (k == 3) {  // RMSNorm + gate/up + SwiGLU
        M = W.gateup; sk = A.sk[2]; xin = A.xs; scaled = true;
        e.epi = EPI_SWIGLU; e.out = A.a; nxt = W.down; nsk = A.sk[3];
      } else {  // down projection + residual; then the next layer's QKV or the LM head
        M = W.down; sk = A.sk[3]; xin = (const char*)A.a; e.epi = EPI_RESID; e.out = A.x;
        if (l + 1 < A.layer_end) {
          nxt = table_mat<DT>(A, l + 1, 0); nsk = A.sk[0];
          e.staged_out = A.xs; e.gain_next = table_layer<DT>(A, l + 1).attn_gain;
        } else if (A.layer_end == L) {
          nxt = A.lm_head; nsk = A.sk[4];
          e.staged_out = A.xs; e.gain_next = A.final_gain;
        } else {
          has_next = false; nxt = M;
        }
      }
    }
    e.N = M.N;
    wg_mark(A, l * 8 + k, 0);
    if (__builtin_expect(A.raise_key == l * 8 + k, 0) && A.cancel_flags && A.trace && blockIdx.x == gridDim.x / 2 &&
        threadIdx.x == 0) {
      // measurement aid: the cancellation signal raised from another compute unit, on the device clock
      __hip_atomic_store((int32_t*)A.cancel_flags, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      wave_drain();
      A.trace[A.trace_cap - 1] = wall_clock64();
    }
    proj_phase<DT, UR>(A, R, S, sk, xin, scaled, M.K, e, lds, pflag, (unsigned)ph + 1u, lane,
                       nxt, has_next, nsk, wave, l * 8 + k,
                       /*poll_x=*/k == 2 || k == 4, /*kind=*/k);
    wg_mark(A, l * 8 + k, 3);
    if (k == 5) break;
    // no grid barrier behind QKV and gate/up: attention waits for the queries and the run's cells,
    // the down projection for the SwiGLU output
    if (k == 0 || k == 3) continue;
    const bool boundary = k == 4;
    const int npidx = k == 2 ? 2 : (l + 1 < A.layer_end ? 0 : 4);  // what follows the barrier: gate/up; the next QKV or the LM head
    if (!(ok = grid_barrier(A, bc, boundary ? l + 1 : -1, boundary && l + 1 < A.layer_end, l * 8 + k,
                            [&] { if (has_next) stream_park<DT>(S, park_region(A, lds, npidx, wave), park_cap(A, npidx), lane); })))
      break;
    wg_mark(A, l * 8 + k, 5);
    if (boundary) {
      dead_tokens = (unsigned)__builtin_amdgcn_readfirstlane(bar_sh[1]);
      dead = dead_tokens == all_tokens;
    }
  }
  if (ok && !dead && A.layer_end < L) hidden_out_phase(A);
  // Exit: the last workgroup to leave re-arms the barrier for the next launch and reports.
  wave_drain();  // (a run that ends early may leave tiles on their way into LDS)
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

size_t attn_lds_bytes(int head_dim, int dtype, int max_unit_cells) {
  const int cp = (max_unit_cells + 31) & ~31;
  return (size_t)attn_lds_layout(head_dim, cp, dtype == PI_DTYPE_BF16 ? 1 : 2).total;
}

size_t stage_proj_lds_bytes(int n, int nt, int r_max) {
  if (r_max > kMaxResidBlocks) r_max = 0;  // too many row blocks per workgroup: residual rows are read in place
  // operand slots (+ the zero tile), the reduction scratch, seven parked partial tiles, and per row
  // block of the workgroup its residual rows and the next projection's gains for them
  return (size_t)(nt + 1) * 128 * n + (kStageThreads + 16) * sizeof(float) + (kStageThreads / 64 - 1 + 2 * r_max) * 1024;
}

namespace {
const void* stage_fn(int dtype, int ring) {
  if (dtype == kWeightFP4B) return ring == 8 ? (const void*)stage_kernel<kWeightFP4B, 8> : (const void*)stage_kernel<kWeightFP4B, 4>;
  if (dtype == kWeightFP4) return ring == 8 ? (const void*)stage_kernel<kWeightFP4, 8> : (const void*)stage_kernel<kWeightFP4, 4>;
  if (dtype == kWeightFP8) return ring == 8 ? (const void*)stage_kernel<kWeightFP8, 8> : (const void*)stage_kernel<kWeightFP8, 4>;
  if (dtype == PI_DTYPE_BF16) return ring == 8 ? (const void*)stage_kernel<PI_DTYPE_BF16, 8> : (const void*)stage_kernel<PI_DTYPE_BF16, 4>;
  return ring == 8 ? (const void*)stage_kernel<PI_DTYPE_F32, 8> : (const void*)stage_kernel<PI_DTYPE_F32, 4>;
}
}  // namespace

// Tiles a wave keeps in flight.  Eight 1 KiB tiles per wave (64 KiB per compute unit) stream as
// fast as sixteen on every shape measured and leave the phase changes -- where a small model
// spends most of its time -- with less code to walk through and fewer registers to hold: the
// 7B-shaped bf16 forward is unchanged within 1 %, the 8-bit and 4-bit ones and the TinyLlama
// shape gain 6-9 %.  Four remain for contractions shorter than eight tiles per slice.
int stage_ring_size(int dtype, int min_nt) {
  (void)dtype;
  if (min_nt >= 8) return 8;
  return min_nt >= 4 ? 4 : 0;
}

hipError_t stage_configure(int dtype, int ring, size_t max_lds, int* max_blocks_per_cu) {
  const void* fn = stage_fn(dtype, ring);
  hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_lds);
  if (e != hipSuccess) return e;
  return hipOccupancyMaxActiveBlocksPerMultiprocessor(max_blocks_per_cu, fn, kStageThreads, max_lds);
}

// ---- read-bandwidth probe --------------------------------------------------------------------
// What this chip delivers to a launch of the stage kernel's shape that does nothing but stream: one
// workgroup of 8 waves per compute unit, each wave reading its own contiguous range of 1 KiB tiles
// with a ring of eight 128-bit non-temporal loads per lane and folding them into a checksum.
namespace {
__global__ void __launch_bounds__(kStageThreads, 1) stream_probe_kernel(const u32x4* __restrict__ w, long tiles_per_wave,
                                                                      unsigned* sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const u32x4* p = w + ((size_t)(blockIdx.x * kWaves + wave) * tiles_per_wave) * 64 + lane;
  u32x4 acc = {0, 0, 0, 0};
  for (long i = 0; i < tiles_per_wave; i += 8) {
    u32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(p + (size_t)(i + j) * 64);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= v[j];
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[0] = 1;  // keeps the loads alive
}
}  // namespace

hipError_t stream_probe(size_t bytes, int reps, double* gbps) {
  int dev = 0;
  hipDeviceProp_t prop;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) return e;
  const int grid = prop.multiProcessorCount;
  const size_t per_wave = bytes / ((size_t)grid * kWaves) / 8192 * 8;  // tiles per wave, a multiple of the ring
  if (per_wave == 0) return hipErrorInvalidValue;
  const size_t used = per_wave * 1024 * grid * kWaves;
  void* buf = nullptr;
  unsigned* sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  e = hipMalloc(&buf, used);
  if (e == hipSuccess) e = hipMalloc((void**)&sink, 64);
  if (e == hipSuccess) e = hipMemset(buf, 1, used);
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  float best_ms = 0.0f;
  for (int r = 0; e == hipSuccess && r < reps + 1; ++r) {  // the first launch warms up
    e = hipEventRecord(e0, nullptr);
    if (e == hipSuccess) {
      stream_probe_kernel<<<dim3((unsigned)grid), dim3(kStageThreads), 0, nullptr>>>((const u32x4*)buf, (long)per_wave, sink);
      e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(e1, nullptr);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (r > 0 && (best_ms == 0.0f || ms < best_ms)) best_ms = ms;
  }
  if (e == hipSuccess && gbps) *gbps = (double)used / 1e9 / ((double)best_ms * 1e-3);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (sink) (void)hipFree(sink);
  if (buf) (void)hipFree(buf);
  return e;
}

hipError_t launch_stage(const StageArgs& a, int dtype, int ring, int grid, size_t lds, hipStream_t s) {
  StageArgs args = a;
  void* params[] = {(void*)&args};
  return hipLaunchKernel(stage_fn(dtype, ring), dim3((unsigned)grid), dim3(kStageThreads), params, lds, s);
}

}  // namespace pi
