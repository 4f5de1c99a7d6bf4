// The C ABI (include/pipeinfer.h): handles, host-side validation, the per-layer launch sequence.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "pi_internal.h"

using namespace pi;

namespace {

constexpr size_t kProjLdsBudget = 96 * 1024;  // bytes of LDS the QKV phase should take (there a second slice beats a fuller LDS)
constexpr size_t kLdsLimit = 159 * 1024;      // dynamic LDS of a workgroup (160 KiB per compute unit; a little is static)
constexpr int kParkMax = 16;                  // tiles a wave may ask for ahead of a phase (1 KiB of LDS each)
constexpr size_t kProjLdsLimit = 150 * 1024;  // ... and may take where no split fits the budget (160 KiB; a little is static)
constexpr size_t kSlowPollLayerBytes = 256u << 20;  // a layer's weights from which barrier waits space their looks
constexpr unsigned long long kBarrierTimeoutTicks = 200000000ull;  // 2 s of the 100 MHz clock

}  // namespace

struct pi_model {
  pi_model_config cfg;
  std::vector<LayerWeights> layers;
  PackedMat lm_head;
  void* embed = nullptr;  // [vocab][d] row-major in cfg.dtype
  float* final_gain = nullptr;
  float2* rope = nullptr;  // [max_pos][hd/2]
  LayerDev* layers_dev = nullptr;
  // activation scratch of the one run in flight
  float *x = nullptr, *q = nullptr, *o = nullptr, *a = nullptr, *ssq = nullptr, *part = nullptr;
  char* xs = nullptr;  // the residual stream in the form the projections stage (o and a are in that form too)
  int last_n = 0;      // tokens of the last forward (the staged form's layout depends on it)
  unsigned* kv_ready = nullptr;
  RunState* rs = nullptr;
  StageSync* sync = nullptr;
  unsigned long long* trace = nullptr;  // timestamps of the barriers of the last run
  int trace_cap = 0;
  bool trace_on = false;
  unsigned long long* wgtrace = nullptr;
  int wgtrace_layer = -1;
  int raise_key = -1;  // debug: phase (layer * 8 + kind) at which the kernel raises the run's cancel word itself
  int grid = 0;  // workgroups of the stage kernel = compute units
  unsigned epoch = 0;  // grid barriers reserved by earlier launches
  size_t configured_lds[17] = {0};  // per ring size: dynamic LDS the kernel was configured for
  std::vector<void*> allocs;
  std::vector<uint8_t> set_flags;  // per (kind, layer)
  int sk_override[5] = {0, 0, 0, 0, 0};
  int attn_share_override = 0;  // tuning hook: attention units per 100 workgroups aimed at (0: built-in)
  int park_override = 0;  // tuning hook: 0 = built-in rule, 1 = no tiles ahead of a phase, else the cap per wave
  size_t lds_budget = 0;  // tuning hook: what every projection phase's split aims to stay under (0: built-in per phase)
  size_t part_tiles = 0;  // capacity of each region of `part`, in 1 KiB tiles
  int wdtype = PI_DTYPE_BF16;  // format of the weight matrices (cfg.dtype, or 8-bit)
  int kt32() const { return weight_tile_cols(wdtype) / 32; }  // 32-column tiles per weight tile
  int n_q_rows() const { return cfg.n_q_heads * cfg.head_dim; }
  int n_kv_rows() const { return cfg.n_kv_heads * cfg.head_dim; }
};

struct pi_kv {
  const pi_model* model;
  int dtype, n_cells, n_layers, n_kv_heads, head_dim;
  void *k = nullptr, *v = nullptr;
  size_t bytes_each = 0, layer_bytes = 0;
  int32_t* len_dev = nullptr;
  int* cnt = nullptr;
  float *attn_o = nullptr, *attn_ml = nullptr;
  unsigned* attn_flags = nullptr;
  int attn_flag_stride = 0;
};

namespace pi {
ModelView model_view(const pi_model* m) { return ModelView{m->cfg.n_layers, m->cfg.vocab, m->cfg.max_pos}; }
KvView kv_view(pi_kv* kv) {
  return KvView{kv->k, kv->v, kv->dtype, kv->n_layers, kv->n_kv_heads, kv->n_cells, kv->head_dim, kv->len_dev};
}
}  // namespace pi

namespace {

int32_t hip_status(hipError_t e) {
  if (e == hipSuccess) return PI_OK;
  return e == hipErrorOutOfMemory ? PI_E_OOM : PI_E_HIP;
}

PackedMat make_packed(int N, int K, int dtype) {
  PackedMat p;
  p.N = N;
  p.K = K;
  p.NRB = (N + kRowBlock - 1) / kRowBlock;
  p.KT = (K + weight_tile_cols(dtype) - 1) / weight_tile_cols(dtype);
  // 4-bit tiles are 128 columns wide: rounded up to a multiple of eight tiles (zero weights), so that the
  // tile count still splits into power-of-two column slices and a short contraction still fills a ring
  if (weight_is_fp4(dtype)) p.KT = (p.KT + 7) / 8 * 8;
  p.bytes = (size_t)p.NRB * p.KT * weight_tile_bytes(dtype);
  if (dtype == kWeightFP4B) p.scale_bytes = (size_t)p.NRB * p.KT * 64;
  return p;
}

template <typename T>
hipError_t dev_alloc(pi_model* m, T** p, size_t bytes, bool zero) {
  void* raw = nullptr;
  hipError_t e = hipMalloc(&raw, bytes ? bytes : 16);
  if (e != hipSuccess) return e;
  m->allocs.push_back(raw);
  *p = (T*)raw;
  if (zero) e = hipMemset(raw, 0, bytes ? bytes : 16);
  return e;
}

// Column slices for one projection phase (0 QKV, 1 O, 2 gate/up, 3 down, 4 LM head).  A split must
// be a power of two that divides the tile count and the grid, keep the phase's LDS needs for n
// tokens within reach and leave a slice at least 16 tiles per row block (fewer would starve the
// ring).  Among those, measured on the 7B and 70B shapes:
//  * the fewest slices whose staged activations fit the budget are best for the wide matrices
//    (QKV, gate/up, LM head), which have several row blocks per workgroup anyway;
//  * the output and down projections have about one row block per workgroup: unsliced, the
//    workgroup's eight waves share that one row block and one wave reduces and finishes it
//    alone at the very end of the phase.  Sliced so that a workgroup holds eight row blocks, every
//    wave owns one and the eight finish side by side; that is worth more than the partial tiles
//    that then cross slices through memory (3-5 us per 7B layer) -- for the down projection
//    always, for the output projection from four tokens on;
//  * a matrix with fewer row blocks than the grid has workgroups is sliced until every
//    workgroup has a row block.
// 0 = impossible.
int choose_sk(const pi_model* m, int phase, const PackedMat& w, int n, size_t budget) {
  const int ov = m->sk_override[phase];
  const auto usable = [&](int sk, size_t cap) {
    if (sk < 1 || sk > m->grid || sk > w.KT || w.KT % sk || m->grid % sk) return false;
    const int gs = m->grid / sk;
    return stage_proj_lds_bytes(n, m->kt32() * (w.KT / sk), (w.NRB + gs - 1) / gs) <= cap;
  };
  int fits = 0;
  for (int sk = 1; sk <= m->grid && sk <= w.KT; sk *= 2) {
    if (!usable(sk, budget)) continue;
    if (ov > sk) continue;  // an override asks for at least this many slices
    if (fits && w.KT / sk < 16) break;  // more slices would starve the ring
    fits = sk;
    if ((long)w.NRB * sk >= m->grid) break;
  }
  if (!fits && budget < kProjLdsLimit) return choose_sk(m, phase, w, n, kProjLdsLimit);
  if (fits && !ov && (phase == 3 || (phase == 1 && n >= 4))) {
    // one row block per wave: the largest split with at most eight row blocks per workgroup (the
    // down projection below eight tokens: four, two waves to a row block -- 1 % on the 7B shape)
    const long per_wg = phase == 3 && n < 8 ? 4 : 8;
    int star = fits;
    for (int sk = fits * 2; sk <= m->grid && (long)w.NRB * sk <= per_wg * m->grid && w.KT / sk >= 16; sk *= 2)
      if (usable(sk, budget)) star = sk;
    fits = star;
  }
  return fits;
}

struct StagePlan {
  int sk[5];
  int min_nt;
  size_t lds;
  size_t part_tiles;  // 1 KiB tiles that cross slices
  int pf_cap[5], pf_base[5];  // per phase: tiles per wave asked for ahead of it; where their LDS regions begin
};

bool make_stage_plan(const pi_model* m, int n, StagePlan* p) {
  const PackedMat* mats[5] = {&m->layers[0].qkv, &m->layers[0].o, &m->layers[0].gateup, &m->layers[0].down,
                              &m->lm_head};
  p->min_nt = 1 << 30;
  p->lds = 0;
  p->part_tiles = 1;
  for (int ph = 0; ph < 5; ++ph) {
    // the QKV projection does better with a second slice than with more than 96 KiB of staged
    // activations; the others take what LDS there is
    const size_t budget = m->lds_budget ? m->lds_budget : (ph == 0 ? kProjLdsBudget : kProjLdsLimit);
    const int sk = choose_sk(m, ph, *mats[ph], n, budget);
    if (sk == 0) return false;
    p->sk[ph] = sk;
    const int nt = mats[ph]->KT / sk;
    if (nt < p->min_nt) p->min_nt = nt;
    const int gs = m->grid / sk;
    const size_t lds = stage_proj_lds_bytes(n, m->kt32() * nt, (mats[ph]->NRB + gs - 1) / gs);
    if (lds > p->lds) p->lds = lds;
    if (sk > 1 && (size_t)sk * mats[ph]->NRB > p->part_tiles) p->part_tiles = (size_t)sk * mats[ph]->NRB;
  }
  // What LDS a projection phase leaves free holds tiles asked for ahead of it (an equal region per
  // wave).  They are asked for while the workgroup waits at the grid barrier before the phase, or
  // after attention -- nothing else of the workgroup is in LDS then -- except those of the down
  // projection, which a wave asks for while other waves still stream gate/up.  (The attention phase
  // may use the same bytes: no tiles wait while it runs.)
  size_t need[5];
  for (int ph = 0; ph < 5; ++ph) {
    const int gs = m->grid / p->sk[ph];
    need[ph] = stage_proj_lds_bytes(n, m->kt32() * (mats[ph]->KT / p->sk[ph]), (mats[ph]->NRB + gs - 1) / gs);
  }
  // (one geometry for both, so that a wave's region for the down projection is its own region of
  // gate/up, which only it has touched)
  need[2] = need[3] = std::max(need[2], need[3]);
  const bool parks = weight_tile_bytes(m->wdtype) == 1024 && m->wdtype != kWeightFP4B && m->park_override != 1;
  for (int ph = 0; ph < 5; ++ph) {
    p->pf_base[ph] = (int)((need[ph] + 1023) / 1024 * 1024);
    const int room = (int)(((long)kLdsLimit - p->pf_base[ph]) / (1024 * (kStageThreads / 64)));
    // (a sliced output projection has sixteen tiles per wave and no time to spare before it: asking for
    // more than half of them ahead measures slower)
    const int want = m->park_override > 1 ? m->park_override : (ph == 1 && p->sk[1] > 1 ? kParkMax / 2 : kParkMax);
    p->pf_cap[ph] = parks ? std::max(0, std::min(room, want)) & ~1 : 0;
    const size_t with_parked = (size_t)p->pf_base[ph] + (size_t)p->pf_cap[ph] * 1024 * (kStageThreads / 64);
    if (p->pf_cap[ph] > 0 && with_parked > p->lds) p->lds = with_parked;
  }
  return true;
}

int32_t stage_forward_groups(pi_model* m, pi_kv* kv, const pi_run_desc* run, int n_groups, const uint32_t* group_mask,
                             const int32_t* cancel_flags, int32_t* group_status, int32_t layer_begin,
                             int32_t layer_end, const float* hidden_in, float* hidden_out, float* logits_out,
                             int32_t* run_status, void* stream);

bool is_layer_kind(int kind) { return kind >= PI_T_ATTN_NORM && kind <= PI_T_WD; }

size_t flag_index(const pi_model* m, int kind, int layer) {
  return (size_t)kind * m->cfg.n_layers + (is_layer_kind(kind) ? layer : 0);
}

// Per-device process-wide state (kMaxDevices devices at most; a device beyond that is refused).
constexpr int kMaxDevices = 16;
struct VerifyScratch {
  float* best_val = nullptr;
  int32_t* best_idx = nullptr;
  int* cnt = nullptr;
  hipError_t err = hipSuccess;
  bool ready = false;
};
VerifyScratch g_verify[kMaxDevices];
std::mutex g_verify_mutex;

// The stage kernel's workgroups wait for each other, so two stage kernels must never share the
// device: each launch waits (on its own stream) for the event recorded behind the previous one.
struct LaunchOrder {
  hipEvent_t ev = nullptr;
  hipStream_t last_stream = nullptr;
  bool any = false;
};
LaunchOrder g_order[kMaxDevices];
std::mutex g_order_mutex;

hipError_t launch_stage_in_order(const StageArgs& a, int wdtype, int ring, int grid, size_t lds, hipStream_t s) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_order_mutex);
  LaunchOrder& o = g_order[dev];
  if (!o.ev) {
    e = hipEventCreateWithFlags(&o.ev, hipEventDisableTiming);
    if (e != hipSuccess) return e;
  }
  if (o.any && o.last_stream != s) {
    e = hipStreamWaitEvent(s, o.ev, 0);
    if (e != hipSuccess) return e;
  }
  e = launch_stage(a, wdtype, ring, grid, lds, s);
  if (e != hipSuccess) return e;
  e = hipEventRecord(o.ev, s);
  o.last_stream = s;
  o.any = true;
  return e;
}

}  // namespace

extern "C" {

const char* pi_strerror(int32_t s) {
  switch (s) {
    case PI_OK: return "ok";
    case PI_CANCELLED: return "run cancelled";
    case PI_E_ARG: return "invalid argument";
    case PI_E_SHAPE: return "unsupported shape or size";
    case PI_E_OOM: return "out of device memory";
    case PI_E_SLOT_LIVE: return "speculative write targets a live canonical cell or leaves the window";
    case PI_E_HIP: return "HIP runtime error";
    case PI_E_STATE: return "model not fully loaded or handle misused";
    case PI_E_FULL: return "no free cell in the window or no free sequence identifier";
    case PI_E_BUSY: return "a partition still holds a cell of the window";
    default: return "unknown status";
  }
}

int32_t pi_model_load(const pi_model_config* cfg, pi_model** out) {
  if (!cfg || !out) return PI_E_ARG;
  *out = nullptr;
  const pi_model_config& c = *cfg;
  if (c.n_layers < 1 || c.d_model < 32 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.ffn < 16 ||
      c.vocab < 16 || c.max_pos < 1)
    return PI_E_SHAPE;
  if (c.head_dim != 32 && c.head_dim != 64 && c.head_dim != 128) return PI_E_SHAPE;
  if (c.d_model % 32 || (c.n_q_heads * c.head_dim) % 32 || c.ffn % 16 || c.vocab % 16) return PI_E_SHAPE;
  if (c.n_q_heads % c.n_kv_heads || c.n_q_heads / c.n_kv_heads > 8) return PI_E_SHAPE;
  if (c.dtype != PI_DTYPE_F32 && c.dtype != PI_DTYPE_BF16) return PI_E_SHAPE;
  const bool w8 = c.weight_dtype == PI_DTYPE_FP8_E4M3 || c.weight_dtype == PI_DTYPE_FP4_E2M1 ||
                  c.weight_dtype == PI_DTYPE_FP4_E2M1_B32;
  if (c.weight_dtype == PI_DTYPE_FP4_E2M1_B32 && c.weight_scale_exp2 != 0) return PI_E_SHAPE;  // the blocks carry the scales
  if (w8 ? (c.dtype != PI_DTYPE_BF16 || c.weight_scale_exp2 < -32 || c.weight_scale_exp2 > 32)
         : (c.weight_dtype != c.dtype && !(c.weight_dtype == 0 && c.dtype == PI_DTYPE_BF16)))
    return PI_E_SHAPE;
  if (c.vocab > (1 << 24) || !(c.rms_eps >= 0.0f) || !(c.rope_base > 1.0f)) return PI_E_SHAPE;

  pi_model* m = new (std::nothrow) pi_model();
  if (!m) return PI_E_OOM;
  m->cfg = c;
  m->wdtype = w8 ? c.weight_dtype : c.dtype;
  const int wd = m->wdtype;
  const int d = c.d_model, nq = c.n_q_heads * c.head_dim, nkv = c.n_kv_heads * c.head_dim;
  const int es = c.dtype == PI_DTYPE_BF16 ? 2 : 4;
  hipError_t e = hipSuccess;
  auto fail = [&](int32_t st) {
    pi_model_free(m);
    return st;
  };
  m->layers.resize(c.n_layers);
  for (int l = 0; l < c.n_layers && e == hipSuccess; ++l) {
    LayerWeights& L = m->layers[l];
    L.qkv = make_packed(nq + 2 * nkv, d, wd);
    L.o = make_packed(d, nq, wd);
    L.gateup = make_packed(2 * c.ffn, d, wd);
    L.down = make_packed(d, c.ffn, wd);
    for (PackedMat* p : {&L.qkv, &L.o, &L.gateup, &L.down}) {
      if (e == hipSuccess) e = dev_alloc(m, (char**)&p->data, p->bytes, true);
      if (e == hipSuccess && p->scale_bytes) e = dev_alloc(m, (char**)&p->scales, p->scale_bytes, true);
    }
    if (e == hipSuccess) e = dev_alloc(m, &L.attn_gain, d * sizeof(float), true);
    if (e == hipSuccess) e = dev_alloc(m, &L.ffn_gain, d * sizeof(float), true);
  }
  m->lm_head = make_packed(c.vocab, d, wd);
  if (e == hipSuccess) e = dev_alloc(m, (char**)&m->lm_head.data, m->lm_head.bytes, true);
  if (e == hipSuccess && m->lm_head.scale_bytes) e = dev_alloc(m, (char**)&m->lm_head.scales, m->lm_head.scale_bytes, true);
  if (e == hipSuccess) e = dev_alloc(m, (char**)&m->embed, (size_t)c.vocab * d * es, true);
  if (e == hipSuccess) e = dev_alloc(m, &m->final_gain, d * sizeof(float), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->rope, (size_t)c.max_pos * (c.head_dim / 2) * sizeof(float2), false);
  if (e == hipSuccess) e = dev_alloc(m, &m->x, (size_t)PI_MAX_BATCH * d * sizeof(float), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->q, (size_t)PI_MAX_BATCH * nq * sizeof(float), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->xs, (size_t)PI_MAX_BATCH * d * sizeof(float), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->o, (size_t)PI_MAX_BATCH * nq * sizeof(float), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->a, (size_t)PI_MAX_BATCH * c.ffn * sizeof(float), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->ssq, (size_t)(d / 16) * 16 * sizeof(float), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->kv_ready, (size_t)(2 * c.n_kv_heads * c.head_dim / 16) * sizeof(unsigned), true);
  if (e == hipSuccess) {
    int dev = 0;
    hipDeviceProp_t prop;
    e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e == hipSuccess) m->grid = prop.multiProcessorCount < kMaxGrid ? prop.multiProcessorCount : kMaxGrid;
  }
  if (e == hipSuccess) {
    // tiles that cross slices, for the largest plan over all token counts; every tile starts "empty"
    size_t tiles = 1;
    for (int n = 1; n <= PI_MAX_BATCH; ++n) {
      StagePlan sp;
      if (make_stage_plan(m, n, &sp) && sp.part_tiles > tiles) tiles = sp.part_tiles;
    }
    e = dev_alloc(m, &m->part, 3 * tiles * 1024, false);  // three regions, one per kind of phase in a barrier-free chain
    if (e == hipSuccess) e = hipMemset(m->part, 0xFF, 3 * tiles * 1024);
    if (e == hipSuccess) m->part_tiles = tiles;
  }
  if (e == hipSuccess) e = dev_alloc(m, &m->rs, sizeof(RunState), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->sync, sizeof(StageSync), true);
  m->trace_cap = 5 * c.n_layers + 8;
  if (e == hipSuccess) e = dev_alloc(m, &m->trace, (size_t)m->trace_cap * sizeof(unsigned long long), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->wgtrace, (size_t)kMaxGrid * 40 * sizeof(unsigned long long), true);
  if (e == hipSuccess) {
    std::vector<LayerDev> ld(c.n_layers);
    auto md = [](const PackedMat& p) {
      MatDev r;
      r.w = (const char*)p.data;
      r.s = (const char*)p.scales;
      r.N = p.N;
      r.K = p.K;
      r.NRB = p.NRB;
      r.KT = p.KT;
      return r;
    };
    for (int l = 0; l < c.n_layers; ++l) {
      const LayerWeights& L = m->layers[l];
      ld[l].qkv = md(L.qkv);
      ld[l].o = md(L.o);
      ld[l].gateup = md(L.gateup);
      ld[l].down = md(L.down);
      ld[l].attn_gain = L.attn_gain;
      ld[l].ffn_gain = L.ffn_gain;
    }
    e = dev_alloc(m, &m->layers_dev, ld.size() * sizeof(LayerDev), false);
    if (e == hipSuccess) e = hipMemcpy(m->layers_dev, ld.data(), ld.size() * sizeof(LayerDev), hipMemcpyHostToDevice);
  }
  if (e != hipSuccess) return fail(hip_status(e));
  // rotary table: angle = pos * base^(-2t/hd), evaluated in double on the host
  {
    const int half = c.head_dim / 2;
    std::vector<float2> tab((size_t)c.max_pos * half);
    for (int t = 0; t < half; ++t) {
      const double theta = std::pow((double)c.rope_base, -2.0 * t / c.head_dim);
      for (int p = 0; p < c.max_pos; ++p) {
        const double ang = (double)p * theta;
        tab[(size_t)p * half + t] = make_float2((float)std::cos(ang), (float)std::sin(ang));
      }
    }
    e = hipMemcpy(m->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail(hip_status(e));
  }
  m->set_flags.assign((size_t)12 * c.n_layers, 0);
  *out = m;
  return PI_OK;
}

int32_t pi_model_free(pi_model* m) {
  if (!m) return PI_E_ARG;
  (void)hipDeviceSynchronize();
  for (void* p : m->allocs) (void)hipFree(p);
  delete m;
  return PI_OK;
}

int32_t pi_model_weight_bytes(const pi_model* m, int64_t* layer_bytes, int64_t* lm_head_bytes) {
  if (!m) return PI_E_ARG;
  const LayerWeights& L = m->layers[0];
  if (layer_bytes)
    *layer_bytes = (int64_t)(L.qkv.bytes + L.o.bytes + L.gateup.bytes + L.down.bytes + L.qkv.scale_bytes + L.o.scale_bytes +
                             L.gateup.scale_bytes + L.down.scale_bytes);
  if (lm_head_bytes) *lm_head_bytes = (int64_t)(m->lm_head.bytes + m->lm_head.scale_bytes);
  return PI_OK;
}

int32_t pi_model_set_tensor(pi_model* m, int32_t kind, int32_t layer, const void* src, int32_t src_dtype,
                            int32_t src_loc) {
  if (!m || !src) return PI_E_ARG;
  if (kind < PI_T_EMBED || kind > PI_T_LM_HEAD) return PI_E_ARG;
  if (src_dtype < PI_DTYPE_F32 || src_dtype > PI_DTYPE_FP4_E2M1_B32) return PI_E_ARG;
  if (src_loc != PI_LOC_HOST && src_loc != PI_LOC_DEVICE) return PI_E_ARG;
  if (is_layer_kind(kind) && (layer < 0 || layer >= m->cfg.n_layers)) return PI_E_ARG;
  const pi_model_config& c = m->cfg;
  const int d = c.d_model, nq = m->n_q_rows(), nkv = m->n_kv_rows();
  const bool is_gain = kind == PI_T_ATTN_NORM || kind == PI_T_FFN_NORM || kind == PI_T_FINAL_NORM;
  if (is_gain && src_dtype != PI_DTYPE_F32) return PI_E_ARG;
  if (!is_gain && src_dtype == PI_DTYPE_BF16 && c.dtype == PI_DTYPE_F32) return PI_E_ARG;
  // quantised weights: the streamed matrices come in the model's weight format and nothing else does
  const bool is_matrix = !is_gain && kind != PI_T_EMBED;
  const bool quantised_src = src_dtype == PI_DTYPE_FP8_E4M3 || src_dtype == PI_DTYPE_FP4_E2M1 ||
                             src_dtype == PI_DTYPE_FP4_E2M1_B32;
  const bool quantised_dst = is_matrix && (m->wdtype == kWeightFP8 || weight_is_fp4(m->wdtype));
  if (quantised_src != quantised_dst || (quantised_src && src_dtype != m->wdtype)) return PI_E_ARG;
  const int wd = m->wdtype;
  int rows = 1, cols = d;
  switch (kind) {
    case PI_T_EMBED: case PI_T_LM_HEAD: rows = c.vocab; break;
    case PI_T_WQ: rows = nq; break;
    case PI_T_WK: case PI_T_WV: rows = nkv; break;
    case PI_T_WO: rows = d; cols = nq; break;
    case PI_T_WG: case PI_T_WU: rows = c.ffn; break;
    case PI_T_WD: rows = d; cols = c.ffn; break;
    default: break;
  }
  if (weight_is_fp4(src_dtype) && cols % 2) return PI_E_SHAPE;
  const size_t src_bytes = src_dtype == PI_DTYPE_FP4_E2M1_B32 ? (size_t)rows * cols / 2 + (size_t)rows * ((cols + 31) / 32)
                           : src_dtype == PI_DTYPE_FP4_E2M1 ? (size_t)rows * cols / 2
                           : (size_t)rows * cols * (src_dtype == PI_DTYPE_FP8_E4M3 ? 1 : src_dtype == PI_DTYPE_BF16 ? 2 : 4);
  const void* dsrc = src;
  void* staging = nullptr;
  hipError_t e = hipSuccess;
  if (src_loc == PI_LOC_HOST) {
    e = hipMalloc(&staging, src_bytes);
    if (e != hipSuccess) return hip_status(e);
    e = hipMemcpy(staging, src, src_bytes, hipMemcpyHostToDevice);
    dsrc = staging;
  }
  if (e == hipSuccess) {
    LayerWeights* L = is_layer_kind(kind) ? &m->layers[layer] : nullptr;
    switch (kind) {
      case PI_T_ATTN_NORM: e = hipMemcpy(L->attn_gain, dsrc, src_bytes, hipMemcpyDeviceToDevice); break;
      case PI_T_FFN_NORM: e = hipMemcpy(L->ffn_gain, dsrc, src_bytes, hipMemcpyDeviceToDevice); break;
      case PI_T_FINAL_NORM: e = hipMemcpy(m->final_gain, dsrc, src_bytes, hipMemcpyDeviceToDevice); break;
      case PI_T_EMBED: {
        e = launch_convert(dsrc, src_dtype, m->embed, c.dtype, (size_t)rows * cols, nullptr);
        break;
      }
      case PI_T_WQ: e = launch_repack(dsrc, src_dtype, rows, cols, L->qkv, wd, 1, 0, nullptr); break;
      case PI_T_WK: e = launch_repack(dsrc, src_dtype, rows, cols, L->qkv, wd, 1, nq, nullptr); break;
      case PI_T_WV: e = launch_repack(dsrc, src_dtype, rows, cols, L->qkv, wd, 1, nq + nkv, nullptr); break;
      case PI_T_WO: e = launch_repack(dsrc, src_dtype, rows, cols, L->o, wd, 1, 0, nullptr); break;
      case PI_T_WG: e = launch_repack(dsrc, src_dtype, rows, cols, L->gateup, wd, 2, 0, nullptr); break;
      case PI_T_WU: e = launch_repack(dsrc, src_dtype, rows, cols, L->gateup, wd, 2, 1, nullptr); break;
      case PI_T_WD: e = launch_repack(dsrc, src_dtype, rows, cols, L->down, wd, 1, 0, nullptr); break;
      case PI_T_LM_HEAD: e = launch_repack(dsrc, src_dtype, rows, cols, m->lm_head, wd, 1, 0, nullptr); break;
      default: break;
    }
  }
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (staging) (void)hipFree(staging);
  if (e != hipSuccess) return hip_status(e);
  m->set_flags[flag_index(m, kind, layer)] = 1;
  return PI_OK;
}

int32_t pi_debug_read_scratch(pi_model* m, int32_t which, float* dst_host, int64_t count) {
  if (!m || !dst_host || count < 0) return PI_E_ARG;
  const float* src = which == 0 ? m->x : which == 1 ? m->q : which == 2 ? m->o : which == 3 ? m->a : nullptr;
  if (!src) return PI_E_ARG;
  hipError_t e = hipDeviceSynchronize();
  if (which < 2) {
    if (e == hipSuccess) e = hipMemcpy(dst_host, src, (size_t)count * sizeof(float), hipMemcpyDeviceToHost);
    return hip_status(e);
  }
  // The attention and SwiGLU outputs live in the form the next projection stages: per piece of eight
  // columns and token a 16-byte slot in each of two arrays (bf16 model: eight high parts / eight low
  // parts; fp32 model: the first / the last four values).  Put back as [n][K] floats.
  const int n = m->last_n;
  const int K = which == 2 ? m->n_q_rows() : m->cfg.ffn;
  if (n < 1 || count != (int64_t)n * K) return PI_E_ARG;
  std::vector<uint32_t> raw((size_t)count);
  if (e == hipSuccess) e = hipMemcpy(raw.data(), src, (size_t)count * sizeof(float), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_status(e);
  const size_t arr_words = (size_t)(K / 8) * n * 4;
  const auto word = [&](int array, int c8, int i, int w) { return raw[array * arr_words + ((size_t)c8 * n + i) * 4 + w]; };
  const auto as_float = [](uint32_t u) { float f; memcpy(&f, &u, 4); return f; };
  for (int i = 0; i < n; ++i)
    for (int c = 0; c < K; ++c) {
      const int c8 = c / 8, p = c % 8;
      float v;
      if (m->cfg.dtype == PI_DTYPE_BF16) {
        const uint32_t h = word(0, c8, i, p / 2), l = word(1, c8, i, p / 2);
        v = as_float(p % 2 ? h & 0xffff0000u : h << 16) + as_float(p % 2 ? l & 0xffff0000u : l << 16);
      } else {
        v = as_float(word(p / 4, c8, i, p % 4));
      }
      dst_host[(size_t)i * K + c] = v;
    }
  return PI_OK;
}

int32_t pi_debug_wgtrace(pi_model* m, int32_t layer, uint64_t* dst_host) {
  if (!m) return PI_E_ARG;
  m->wgtrace_layer = layer;
  if (!dst_host) return PI_OK;
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess) e = hipMemcpy(dst_host, m->wgtrace, (size_t)m->grid * 40 * sizeof(uint64_t), hipMemcpyDeviceToHost);
  return hip_status(e);
}

int32_t pi_debug_raise_cancel(pi_model* m, int32_t layer, int32_t phase) {
  if (!m || phase < 0 || phase > 4 || phase == 1) return PI_E_ARG;
  if (layer >= m->cfg.n_layers) return PI_E_ARG;
  m->raise_key = layer < 0 ? -1 : layer * 8 + phase;
  return PI_OK;
}

int32_t pi_debug_stream_probe(int64_t bytes, int32_t reps, double* gbps) {
  if (bytes < (1 << 26) || reps < 1 || reps > 1000 || !gbps) return PI_E_ARG;
  return hip_status(stream_probe((size_t)bytes, reps, gbps));
}

int32_t pi_debug_read_trace(pi_model* m, uint64_t* dst_host, int32_t count) {
  if (!m || !dst_host || count < 0 || count > m->trace_cap) return PI_E_ARG;
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess) e = hipMemcpy(dst_host, m->trace, (size_t)count * sizeof(uint64_t), hipMemcpyDeviceToHost);
  return hip_status(e);
}

int32_t pi_debug_set_plan(pi_model* m, int32_t phase, int32_t s_k) {
  if (!m || phase < 0 || phase > 8 || s_k < 0) return PI_E_ARG;
  if (phase == 8) {
    if (s_k > 400) return PI_E_ARG;
    m->attn_share_override = s_k;
    return PI_OK;
  }
  if (phase == 5) {
    m->trace_on = s_k != 0;
    return PI_OK;
  }
  if (phase == 7) {
    if (s_k > 64) return PI_E_ARG;
    m->park_override = s_k;
    return PI_OK;
  }
  if (phase == 6) {
    if (s_k != 0 && (s_k < 16 || (size_t)s_k * 1024 > kProjLdsLimit)) return PI_E_ARG;
    m->lds_budget = (size_t)s_k * 1024;
  } else {
    m->sk_override[phase] = s_k;
  }
  // The buffer of cross-slice tiles was sized for the plans in force so far; grow it for this one.
  size_t tiles = 1;
  for (int n = 1; n <= PI_MAX_BATCH; ++n) {
    StagePlan sp;
    if (make_stage_plan(m, n, &sp) && sp.part_tiles > tiles) tiles = sp.part_tiles;
  }
  if (tiles > m->part_tiles) {
    hipError_t e = hipDeviceSynchronize();
    float* grown = nullptr;
    if (e == hipSuccess) e = dev_alloc(m, &grown, 3 * tiles * 1024, false);
    if (e == hipSuccess) e = hipMemset(grown, 0xFF, 3 * tiles * 1024);
    if (e != hipSuccess) {
      if (phase == 6) m->lds_budget = 0;
      else m->sk_override[phase] = 0;
      return hip_status(e);
    }
    m->part = grown;  // the old buffer stays with the model until it is freed
    m->part_tiles = tiles;
  }
  return PI_OK;
}

// ---------------------------------------------------------------------------------- KV cache

int32_t pi_kv_alloc(const pi_model* m, int32_t n_cells, int32_t kv_dtype, pi_kv** out) {
  if (!m || !out) return PI_E_ARG;
  *out = nullptr;
  if (n_cells < 16 || n_cells % 16 || n_cells > (1 << 20)) return PI_E_SHAPE;
  if (kv_dtype != PI_DTYPE_F32 && kv_dtype != PI_DTYPE_BF16) return PI_E_SHAPE;
  pi_kv* kv = new (std::nothrow) pi_kv();
  if (!kv) return PI_E_OOM;
  kv->model = m;
  kv->dtype = kv_dtype;
  kv->n_cells = n_cells;
  kv->n_layers = m->cfg.n_layers;
  kv->n_kv_heads = m->cfg.n_kv_heads;
  kv->head_dim = m->cfg.head_dim;
  const size_t es = kv_dtype == PI_DTYPE_BF16 ? 2 : 4;
  kv->layer_bytes = (size_t)kv->n_kv_heads * n_cells * kv->head_dim * es;
  kv->bytes_each = kv->layer_bytes * kv->n_layers;
  const int G = m->cfg.n_q_heads / m->cfg.n_kv_heads;
  const size_t max_units = (size_t)n_cells / 32 + 2;
  const size_t rows = (size_t)kv->n_kv_heads * max_units * G * PI_MAX_BATCH;
  hipError_t e = hipMalloc(&kv->k, kv->bytes_each);
  if (e == hipSuccess) e = hipMalloc(&kv->v, kv->bytes_each);
  if (e == hipSuccess) e = hipMalloc((void**)&kv->len_dev, sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc((void**)&kv->cnt, sizeof(int));
  if (e == hipSuccess) e = hipMalloc((void**)&kv->attn_o, rows * kv->head_dim * sizeof(float));
  if (e == hipSuccess) e = hipMalloc((void**)&kv->attn_ml, rows * 2 * sizeof(float));
  kv->attn_flag_stride = (int)max_units;
  // (one word more: the counter from which workgroups draw their attention units)
  if (e == hipSuccess) e = hipMalloc((void**)&kv->attn_flags, (kv->n_kv_heads * max_units + 1) * sizeof(unsigned));
  if (e == hipSuccess) e = hipMemset(kv->attn_flags, 0, (kv->n_kv_heads * max_units + 1) * sizeof(unsigned));
  if (e == hipSuccess) e = hipMemset(kv->k, 0, kv->bytes_each);
  if (e == hipSuccess) e = hipMemset(kv->v, 0, kv->bytes_each);
  if (e == hipSuccess) e = hipMemset(kv->len_dev, 0, sizeof(int32_t));
  if (e == hipSuccess) e = hipMemset(kv->cnt, 0, sizeof(int));
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    pi_kv_free(kv);
    return hip_status(e);
  }
  *out = kv;
  return PI_OK;
}

int32_t pi_kv_free(pi_kv* kv) {
  if (!kv) return PI_E_ARG;
  (void)hipDeviceSynchronize();
  for (void* p : {kv->k, kv->v, (void*)kv->len_dev, (void*)kv->cnt, (void*)kv->attn_o, (void*)kv->attn_ml, (void*)kv->attn_flags})
    if (p) (void)hipFree(p);
  delete kv;
  return PI_OK;
}

int32_t pi_kv_set_cells(pi_kv* kv, int32_t layer, int32_t cell_begin, int32_t n, const void* k_src,
                        const void* v_src, int32_t src_dtype, int32_t src_loc) {
  if (!kv || !k_src || !v_src) return PI_E_ARG;
  if (layer < 0 || layer >= kv->n_layers || cell_begin < 0 || n < 0 || cell_begin + n > kv->n_cells) return PI_E_ARG;
  if (src_dtype != PI_DTYPE_F32 && src_dtype != PI_DTYPE_BF16) return PI_E_ARG;
  if (n == 0) return PI_OK;
  const size_t bytes = (size_t)n * kv->n_kv_heads * kv->head_dim * (src_dtype == PI_DTYPE_BF16 ? 2 : 4);
  void *ks = nullptr, *vs = nullptr;
  const void *kd = k_src, *vd = v_src;
  hipError_t e = hipSuccess;
  if (src_loc == PI_LOC_HOST) {
    e = hipMalloc(&ks, bytes);
    if (e == hipSuccess) e = hipMalloc(&vs, bytes);
    if (e == hipSuccess) e = hipMemcpy(ks, k_src, bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(vs, v_src, bytes, hipMemcpyHostToDevice);
    kd = ks;
    vd = vs;
  } else if (src_loc != PI_LOC_DEVICE) {
    return PI_E_ARG;
  }
  if (e == hipSuccess)
    e = launch_kv_set(kv->k, kv->v, kv->dtype, kv->n_kv_heads, kv->n_cells, kv->head_dim, layer, cell_begin, n,
                      kd, vd, src_dtype, nullptr);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (ks) (void)hipFree(ks);
  if (vs) (void)hipFree(vs);
  return hip_status(e);
}

int32_t pi_kv_get_cells(const pi_kv* kv, int32_t layer, int32_t cell_begin, int32_t n, float* k_dst_host,
                        float* v_dst_host) {
  if (!kv || !k_dst_host || !v_dst_host) return PI_E_ARG;
  if (layer < 0 || layer >= kv->n_layers || cell_begin < 0 || n < 0 || cell_begin + n > kv->n_cells) return PI_E_ARG;
  if (n == 0) return PI_OK;
  const size_t bytes = (size_t)n * kv->n_kv_heads * kv->head_dim * sizeof(float);
  float *kd = nullptr, *vd = nullptr;
  hipError_t e = hipMalloc((void**)&kd, bytes);
  if (e == hipSuccess) e = hipMalloc((void**)&vd, bytes);
  if (e == hipSuccess)
    e = launch_kv_get(kv->k, kv->v, kv->dtype, kv->n_kv_heads, kv->n_cells, kv->head_dim, layer, cell_begin, n,
                      kd, vd, nullptr);
  if (e == hipSuccess) e = hipMemcpy(k_dst_host, kd, bytes, hipMemcpyDeviceToHost);
  if (e == hipSuccess) e = hipMemcpy(v_dst_host, vd, bytes, hipMemcpyDeviceToHost);
  if (kd) (void)hipFree(kd);
  if (vd) (void)hipFree(vd);
  return hip_status(e);
}

int32_t pi_kv_set_len(pi_kv* kv, int32_t kv_len) {
  if (!kv || kv_len < 0 || kv_len > kv->n_cells) return PI_E_ARG;
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess) e = hipMemcpy(kv->len_dev, &kv_len, sizeof(int32_t), hipMemcpyHostToDevice);
  return hip_status(e);
}

int32_t pi_kv_len(const pi_kv* kv, int32_t* out) {
  if (!kv || !out) return PI_E_ARG;
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess) e = hipMemcpy(out, kv->len_dev, sizeof(int32_t), hipMemcpyDeviceToHost);
  return hip_status(e);
}

int32_t pi_kv_raw(const pi_kv* kv, void* dst_host, int64_t* nbytes) {
  if (!kv || !nbytes) return PI_E_ARG;
  const int64_t need = (int64_t)(2 * kv->bytes_each);
  if (!dst_host) {
    *nbytes = need;
    return PI_OK;
  }
  if (*nbytes < need) return PI_E_ARG;
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess) e = hipMemcpy(dst_host, kv->k, kv->bytes_each, hipMemcpyDeviceToHost);
  if (e == hipSuccess) e = hipMemcpy((char*)dst_host + kv->bytes_each, kv->v, kv->bytes_each, hipMemcpyDeviceToHost);
  *nbytes = need;
  return hip_status(e);
}

// ---------------------------------------------------------------------------------- forward

int32_t pi_stage_forward(pi_model* m, pi_kv* kv, const pi_run_desc* run, int32_t layer_begin, int32_t layer_end,
                         const float* hidden_in, float* hidden_out, float* logits_out,
                         const int32_t* cancel_flag, int32_t* run_status, void* stream) {
  if (!run) return PI_E_ARG;
  const uint32_t everyone = run->n >= 1 && run->n < 32 ? (1u << run->n) - 1u : 0u;
  return stage_forward_groups(m, kv, run, 1, &everyone, cancel_flag, nullptr, layer_begin, layer_end, hidden_in,
                              hidden_out, logits_out, run_status, stream);
}

int32_t pi_stage_forward_multi(pi_model* m, pi_kv* kv, const pi_run_desc* run, const pi_group_desc* groups,
                               int32_t layer_begin, int32_t layer_end, const float* hidden_in, float* hidden_out,
                               float* logits_out, int32_t* run_status, void* stream) {
  if (!run || !groups || !groups->group_of_token) return PI_E_ARG;
  if (groups->n_groups < 1 || groups->n_groups > PI_MAX_GROUPS) return PI_E_SHAPE;
  if (run->n < 1 || run->n > PI_MAX_BATCH) return PI_E_SHAPE;
  uint32_t masks[PI_MAX_GROUPS] = {0};
  for (int i = 0; i < run->n; ++i) {
    const int g = groups->group_of_token[i];
    if (g < 0 || g >= groups->n_groups) return PI_E_ARG;
    masks[g] |= 1u << i;
  }
  for (int g = 0; g < groups->n_groups; ++g)
    if (!masks[g]) return PI_E_ARG;  // a run without tokens
  return stage_forward_groups(m, kv, run, groups->n_groups, masks, groups->cancel_flags, groups->group_status,
                              layer_begin, layer_end, hidden_in, hidden_out, logits_out, run_status, stream);
}

}  // extern "C"

namespace {

int32_t stage_forward_groups(pi_model* m, pi_kv* kv, const pi_run_desc* run, int n_groups, const uint32_t* group_mask,
                             const int32_t* cancel_flags, int32_t* group_status, int32_t layer_begin,
                             int32_t layer_end, const float* hidden_in, float* hidden_out, float* logits_out,
                             int32_t* run_status, void* stream) {
  if (!m || !kv || !run) return PI_E_ARG;
  if (kv->model != m) return PI_E_STATE;
  const pi_model_config& c = m->cfg;
  const int n = run->n, L = c.n_layers;
  if (n < 1 || n > PI_MAX_BATCH) return PI_E_SHAPE;
  if (layer_begin < 0 || layer_end > L || layer_begin >= layer_end) return PI_E_ARG;
  if (!run->positions || !run->slots || !run->mask) return PI_E_ARG;
  if (layer_begin == 0 ? !run->tokens : !hidden_in) return PI_E_ARG;
  if (layer_end == L ? !logits_out : !hidden_out) return PI_E_ARG;
  if (run->prefix_len < 0 || run->prefix_len > kv->n_cells) return PI_E_ARG;
  if (run->window_base < 0 || run->window_base >= kv->n_cells) return PI_E_ARG;
  {
    // every tensor must have been supplied
    for (int kind = PI_T_EMBED; kind <= PI_T_LM_HEAD; ++kind) {
      const int cnt = is_layer_kind(kind) ? L : 1;
      for (int l = 0; l < cnt; ++l)
        if (!m->set_flags[flag_index(m, kind, l)]) return PI_E_STATE;
    }
  }
  if (kv->dtype != c.dtype) return PI_E_SHAPE;  // the attention kernels read the cache in the model's type
  StagePlan sp;
  if (!make_stage_plan(m, n, &sp)) return PI_E_SHAPE;
  if (sp.part_tiles > m->part_tiles) return PI_E_SHAPE;  // the plan's cross-slice tiles must fit what was allocated
  const int ring = stage_ring_size(m->wdtype, sp.min_nt);
  if (ring == 0) return PI_E_SHAPE;
  // attention work units: per kv head, the prefix in chunks (multiples of 32 cells) sized so that
  // about one unit per workgroup exists and a unit's K/V (chunk + window) fits in LDS; the last
  // unit of a head also takes the window
  int attn_chunk, attn_units;
  {
    constexpr size_t kAttnLdsBudget = 140 * 1024;
    // about three units per four workgroups: the workgroups that finish the QKV projection last then
    // draw no unit (the kernel hands units out in the order of arrival)
    const int share = m->attn_share_override ? m->attn_share_override : 75;
    long per_head = (long)m->grid * share / 100 / c.n_kv_heads;
    if (per_head < 1) per_head = 1;
    int chunk = (int)((run->prefix_len + per_head - 1) / per_head);
    chunk = ((chunk + 31) / 32) * 32;
    if (chunk < 32) chunk = 32;
    while (chunk > 32 && (attn_lds_bytes(c.head_dim, c.dtype, chunk + PI_WINDOW) > kAttnLdsBudget ||
                          chunk + PI_WINDOW > 256))
      chunk -= 32;
    if (attn_lds_bytes(c.head_dim, c.dtype, chunk + PI_WINDOW) > kAttnLdsBudget) return PI_E_SHAPE;
    attn_chunk = chunk;
    attn_units = (run->prefix_len + chunk - 1) / chunk;
    if (attn_units < 1) attn_units = 1;
    if ((long)attn_units * c.n_kv_heads > 64L * m->grid) return PI_E_SHAPE;  // a workgroup draws at most 64 units per layer
    const size_t al = attn_lds_bytes(c.head_dim, c.dtype, chunk + PI_WINDOW);
    if (al > sp.lds) sp.lds = al;
  }
  if (sp.lds > m->configured_lds[ring]) {
    int blocks = 0;
    hipError_t ce = stage_configure(m->wdtype, ring, sp.lds, &blocks);
    if (ce != hipSuccess) return hip_status(ce);
    if (blocks < 1) return PI_E_SHAPE;
    m->configured_lds[ring] = sp.lds;
  }
  StageArgs a;
  memset(&a, 0, sizeof(a));
  a.layers = m->layers_dev;
  a.lm_head.w = (const char*)m->lm_head.data;
  a.lm_head.N = m->lm_head.N;
  a.lm_head.K = m->lm_head.K;
  a.lm_head.NRB = m->lm_head.NRB;
  a.lm_head.KT = m->lm_head.KT;
  a.final_gain = m->final_gain;
  a.embed = m->embed;
  a.rope = m->rope;
  a.max_pos = c.max_pos;
  a.dtype = c.dtype;
  a.d = c.d_model;
  a.n_q_heads = c.n_q_heads;
  a.n_kv_heads = c.n_kv_heads;
  a.head_dim = c.head_dim;
  a.ffn = c.ffn;
  a.vocab = c.vocab;
  a.n_layers = L;
  a.eps = c.rms_eps;
  a.wscale = m->wdtype == kWeightFP8 || m->wdtype == kWeightFP4 ? std::ldexp(1.0f, c.weight_scale_exp2) : 1.0f;
  a.lm_head.s = (const char*)m->lm_head.scales;
  a.n = n;
  a.tokens = run->tokens;
  a.positions = run->positions;
  a.slots = run->slots;
  a.mask = run->mask;
  a.prefix_len = run->prefix_len;
  a.window_base = run->window_base;
  a.layer_begin = layer_begin;
  a.layer_end = layer_end;
  a.hidden_in = hidden_in;
  a.hidden_out = hidden_out;
  a.logits_out = logits_out;
  a.cancel_flags = cancel_flags;
  a.group_status = group_status;
  a.n_groups = n_groups;
  for (int g = 0; g < n_groups; ++g) a.group_mask[g] = group_mask[g];
  a.run_status = run_status;
  a.kbase = (char*)kv->k;
  a.vbase = (char*)kv->v;
  a.kv_layer_bytes = kv->layer_bytes;
  a.n_cells = kv->n_cells;
  a.kv_dtype = kv->dtype;
  a.kv_len = kv->len_dev;
  a.x = m->x;
  a.xs = m->xs;
  m->last_n = n;
  a.q = m->q;
  a.o = m->o;
  a.a = m->a;
  a.ssq = m->ssq;
  a.kv_ready = m->kv_ready;
  a.part = m->part;
  a.part_half_floats = m->part_tiles * 256;
  a.attn_o = kv->attn_o;
  a.attn_ml = kv->attn_ml;
  a.attn_flags = kv->attn_flags;
  a.attn_flag_stride = kv->attn_flag_stride;
  a.attn_ticket = kv->attn_flags + (size_t)kv->n_kv_heads * kv->attn_flag_stride;
  a.rs = m->rs;
  a.sync = m->sync;
  for (int ph = 0; ph < 5; ++ph) a.sk[ph] = sp.sk[ph];
  for (int ph = 0; ph < 5; ++ph) {
    a.pf_cap8 |= (unsigned long long)sp.pf_cap[ph] << (8 * ph);
    a.pf_base8 |= (unsigned long long)(sp.pf_base[ph] / 1024) << (8 * ph);
  }
  a.attn_chunk = attn_chunk;
  a.attn_units_per_head = attn_units;
  a.timeout_ticks = kBarrierTimeoutTicks;
  {
    // 256 workgroups looking at the arrival words back to back slow down the workgroups still streaming;
    // where a layer streams long enough for that to show (measured: the bf16 7B shape, -0.6 % from four
    // tokens on; 8-bit and 4-bit weights, the 70B shape and small models +-0 or worse), the looks are spaced.
    const LayerWeights& L0 = m->layers[0];
    const size_t layer_bytes = L0.qkv.bytes + L0.o.bytes + L0.gateup.bytes + L0.down.bytes;
    a.slow_poll = layer_bytes >= kSlowPollLayerBytes && run->n >= 4 ? 1 : 0;
  }
  a.epoch_base = m->epoch;
  m->epoch += (unsigned)(5 * (layer_end - layer_begin) + 4);  // every barrier this launch can reach
  a.trace = m->trace_on ? m->trace : nullptr;  // a clock read per barrier is not free: only on request
  a.trace_cap = m->trace_cap;
  a.wgtrace = m->wgtrace_layer >= 0 ? m->wgtrace : nullptr;
  a.wgtrace_layer = m->wgtrace_layer;
  a.raise_key = m->trace_on ? m->raise_key : -1;
  return hip_status(launch_stage_in_order(a, m->wdtype, ring, m->grid, sp.lds, (hipStream_t)stream));
}

}  // namespace

extern "C" {

int32_t pi_verify_greedy_chained(const int32_t* draft, const int32_t* parent, int32_t n, const float* logits,
                                 int32_t vocab, int32_t root_expected, const int32_t* prev_result, int32_t prev_n,
                                 const int32_t* run_status, int32_t* accepted_nodes, int32_t* result, void* stream) {
  if (!draft || !logits || !accepted_nodes || !result) return PI_E_ARG;
  if (n < 1 || n > PI_MAX_BATCH || vocab < 1 || vocab > (1 << 24)) return PI_E_SHAPE;
  if (prev_result && (prev_n < 1 || prev_n > PI_MAX_BATCH)) return PI_E_SHAPE;
  int dev = 0;
  hipError_t de = hipGetDevice(&dev);
  if (de != hipSuccess) return hip_status(de);
  if (dev < 0 || dev >= kMaxDevices) return PI_E_SHAPE;
  VerifyScratch& vs = g_verify[dev];
  {
    std::lock_guard<std::mutex> lock(g_verify_mutex);
    if (!vs.ready) {
      hipError_t e = hipMalloc((void**)&vs.best_val, PI_MAX_BATCH * sizeof(float));
      if (e == hipSuccess) e = hipMalloc((void**)&vs.best_idx, PI_MAX_BATCH * sizeof(int32_t));
      if (e == hipSuccess) e = hipMalloc((void**)&vs.cnt, sizeof(int));
      if (e == hipSuccess) e = hipMemset(vs.cnt, 0, sizeof(int));
      if (e == hipSuccess) e = hipDeviceSynchronize();
      vs.err = e;
      vs.ready = true;
    }
  }
  if (vs.err != hipSuccess) return hip_status(vs.err);
  return hip_status(launch_verify(draft, parent, n, logits, vocab, root_expected, prev_result, prev_n, run_status,
                                  accepted_nodes, result, vs.best_val, vs.best_idx, vs.cnt, (hipStream_t)stream));
}

int32_t pi_verify_greedy(const int32_t* draft, const int32_t* parent, int32_t n, const float* logits,
                         int32_t vocab, int32_t root_expected, int32_t* accepted_nodes, int32_t* result,
                         void* stream) {
  return pi_verify_greedy_chained(draft, parent, n, logits, vocab, root_expected, nullptr, 0, nullptr, accepted_nodes,
                                  result, stream);
}

int32_t pi_mapped_device_pointer(void* host_ptr, void** device_ptr) {
  if (!host_ptr || !device_ptr) return PI_E_ARG;
  *device_ptr = nullptr;
  return hip_status(hipHostGetDevicePointer(device_ptr, host_ptr, 0));
}

int32_t pi_kv_rollback(pi_kv* kv, const int32_t* slots, int32_t n, const int32_t* accepted_nodes,
                       const int32_t* result, void* stream) {
  if (!kv || !slots) return PI_E_ARG;
  if (n < 1 || n > PI_MAX_BATCH) return PI_E_SHAPE;
  if (result && !accepted_nodes) return PI_E_ARG;
  return hip_status(launch_rollback(kv->k, kv->v, kv->dtype, kv->n_layers, kv->n_kv_heads, kv->n_cells,
                                    kv->head_dim, slots, n, accepted_nodes, result, kv->len_dev, kv->cnt,
                                    (hipStream_t)stream));
}

}  // extern "C"
