// The C ABI (include/pipeinfer.h): handles, host-side validation, the per-layer launch sequence.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "pi_internal.h"

using namespace pi;

namespace {

constexpr size_t kProjLdsBudget = 40 * 1024;

struct Plan {
  int S_k, RBU, grid;
};

}  // namespace

struct pi_model {
  pi_model_config cfg;
  std::vector<LayerWeights> layers;
  PackedMat lm_head;
  void* embed = nullptr;  // [vocab][d] row-major in cfg.dtype
  float* final_gain = nullptr;
  float2* rope = nullptr;  // [max_pos][hd/2]
  // activation scratch of the one run in flight
  float *x = nullptr, *q = nullptr, *o = nullptr, *a = nullptr, *ssq = nullptr, *part = nullptr;
  int* cnt = nullptr;       // row-block arrival counters
  int* done_cnt = nullptr;  // layer completion counter
  RunState* rs = nullptr;
  std::vector<void*> allocs;
  std::vector<uint8_t> set_flags;  // per (kind, layer)
  int plan_override[5][3] = {{0}};  // debug: per phase {S_k, RBU, grid}; 0 = heuristic
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
};

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
  p.KT = (K + kKTile - 1) / kKTile;
  p.bytes = (size_t)p.NRB * p.KT * (dtype == PI_DTYPE_BF16 ? 1024 : 2048);
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

int lds_max_tiles(int n) { return (int)((kProjLdsBudget) / (128 * (size_t)n)); }

// Smallest number of k slices whose staged activations fit in LDS, and the largest number
// the planner may choose (at least 8 tiles per slice unless LDS forces more slices).
int s_k_min(const PackedMat& w, int n) { return (w.KT + lds_max_tiles(n) - 1) / lds_max_tiles(n); }
int s_k_cap(const PackedMat& w, int n) {
  const int lo = s_k_min(w, n);
  const int hi = w.KT / 8 > 0 ? w.KT / 8 : 1;
  return lo > hi ? lo : hi;
}

// Heuristic split of one projection into (k slices) x (row chunks): enough k slices for the
// staged activations to fit in LDS and for ~1000 work units, one row block per wave per unit.
Plan make_plan(const pi_model* m, int phase, const PackedMat& w, int n) {
  Plan p;
  const int s_lds = s_k_min(w, n), s_cap = s_k_cap(w, n);
  p.RBU = kProjThreads / 64;
  const int s_par = (1024 * p.RBU + w.NRB - 1) / w.NRB;
  p.S_k = s_lds > s_par ? s_lds : s_par;
  if (p.S_k > s_cap) p.S_k = s_cap;
  if (m->plan_override[phase][0] > 0) {
    const int sk = m->plan_override[phase][0];
    if (sk >= s_lds && sk <= s_cap) p.S_k = sk;
  }
  if (m->plan_override[phase][1] > 0) p.RBU = m->plan_override[phase][1];
  const int units = p.S_k * ((w.NRB + p.RBU - 1) / p.RBU);
  p.grid = units < 2048 ? units : 2048;
  if (m->plan_override[phase][2] > 0 && m->plan_override[phase][2] < units) p.grid = m->plan_override[phase][2];
  return p;
}

int max_split_tiles(const pi_model* m) {
  // upper bound of S_k * NRB over all phases and token counts (S_k never exceeds KT/8 or the
  // LDS-driven minimum, whichever is larger)
  size_t best = 0;
  auto upd = [&](const PackedMat& w) {
    for (int n = 1; n <= PI_MAX_BATCH; ++n) {
      const size_t v = (size_t)s_k_cap(w, n) * w.NRB;
      if (v > best) best = v;
    }
  };
  upd(m->layers[0].qkv);
  upd(m->layers[0].o);
  upd(m->layers[0].gateup);
  upd(m->layers[0].down);
  upd(m->lm_head);
  return (int)best;
}

bool is_layer_kind(int kind) { return kind >= PI_T_ATTN_NORM && kind <= PI_T_WD; }

size_t flag_index(const pi_model* m, int kind, int layer) {
  return (size_t)kind * m->cfg.n_layers + (is_layer_kind(kind) ? layer : 0);
}

struct VerifyScratch {
  float* best_val = nullptr;
  int32_t* best_idx = nullptr;
  int* cnt = nullptr;
};
VerifyScratch g_verify;
std::once_flag g_verify_once;
hipError_t g_verify_err = hipSuccess;

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
  if (c.vocab > (1 << 24) || !(c.rms_eps >= 0.0f) || !(c.rope_base > 1.0f)) return PI_E_SHAPE;

  pi_model* m = new (std::nothrow) pi_model();
  if (!m) return PI_E_OOM;
  m->cfg = c;
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
    L.qkv = make_packed(nq + 2 * nkv, d, c.dtype);
    L.o = make_packed(d, nq, c.dtype);
    L.gateup = make_packed(2 * c.ffn, d, c.dtype);
    L.down = make_packed(d, c.ffn, c.dtype);
    for (PackedMat* p : {&L.qkv, &L.o, &L.gateup, &L.down}) {
      if (e == hipSuccess) e = dev_alloc(m, (char**)&p->data, p->bytes, true);
    }
    if (e == hipSuccess) e = dev_alloc(m, &L.attn_gain, d * sizeof(float), true);
    if (e == hipSuccess) e = dev_alloc(m, &L.ffn_gain, d * sizeof(float), true);
  }
  m->lm_head = make_packed(c.vocab, d, c.dtype);
  if (e == hipSuccess) e = dev_alloc(m, (char**)&m->lm_head.data, m->lm_head.bytes, true);
  if (e == hipSuccess) e = dev_alloc(m, (char**)&m->embed, (size_t)c.vocab * d * es, true);
  if (e == hipSuccess) e = dev_alloc(m, &m->final_gain, d * sizeof(float), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->rope, (size_t)c.max_pos * (c.head_dim / 2) * sizeof(float2), false);
  if (e == hipSuccess) e = dev_alloc(m, &m->x, (size_t)PI_MAX_BATCH * d * sizeof(float), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->q, (size_t)PI_MAX_BATCH * nq * sizeof(float), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->o, (size_t)PI_MAX_BATCH * nq * sizeof(float), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->a, (size_t)PI_MAX_BATCH * c.ffn * sizeof(float), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->ssq, (size_t)(d / 16) * 16 * sizeof(float), true);
  if (e == hipSuccess) {
    int max_nrb = m->lm_head.NRB;
    for (const PackedMat* p : {&m->layers[0].qkv, &m->layers[0].gateup}) max_nrb = p->NRB > max_nrb ? p->NRB : max_nrb;
    e = dev_alloc(m, &m->cnt, (size_t)max_nrb * sizeof(int), true);
  }
  if (e == hipSuccess) e = dev_alloc(m, &m->part, (size_t)max_split_tiles(m) * 1024, false);
  if (e == hipSuccess) e = dev_alloc(m, &m->done_cnt, sizeof(int), true);
  if (e == hipSuccess) e = dev_alloc(m, &m->rs, sizeof(RunState), true);
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
  if (layer_bytes) *layer_bytes = (int64_t)(L.qkv.bytes + L.o.bytes + L.gateup.bytes + L.down.bytes);
  if (lm_head_bytes) *lm_head_bytes = (int64_t)m->lm_head.bytes;
  return PI_OK;
}

int32_t pi_model_set_tensor(pi_model* m, int32_t kind, int32_t layer, const void* src, int32_t src_dtype,
                            int32_t src_loc) {
  if (!m || !src) return PI_E_ARG;
  if (kind < PI_T_EMBED || kind > PI_T_LM_HEAD) return PI_E_ARG;
  if (src_dtype != PI_DTYPE_F32 && src_dtype != PI_DTYPE_BF16) return PI_E_ARG;
  if (src_loc != PI_LOC_HOST && src_loc != PI_LOC_DEVICE) return PI_E_ARG;
  if (is_layer_kind(kind) && (layer < 0 || layer >= m->cfg.n_layers)) return PI_E_ARG;
  const pi_model_config& c = m->cfg;
  const int d = c.d_model, nq = m->n_q_rows(), nkv = m->n_kv_rows();
  const bool is_gain = kind == PI_T_ATTN_NORM || kind == PI_T_FFN_NORM || kind == PI_T_FINAL_NORM;
  if (is_gain && src_dtype != PI_DTYPE_F32) return PI_E_ARG;
  if (!is_gain && src_dtype == PI_DTYPE_BF16 && c.dtype == PI_DTYPE_F32) return PI_E_ARG;
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
  const size_t src_bytes = (size_t)rows * cols * (src_dtype == PI_DTYPE_BF16 ? 2 : 4);
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
      case PI_T_WQ: e = launch_repack(dsrc, src_dtype, rows, cols, L->qkv, c.dtype, 1, 0, nullptr); break;
      case PI_T_WK: e = launch_repack(dsrc, src_dtype, rows, cols, L->qkv, c.dtype, 1, nq, nullptr); break;
      case PI_T_WV: e = launch_repack(dsrc, src_dtype, rows, cols, L->qkv, c.dtype, 1, nq + nkv, nullptr); break;
      case PI_T_WO: e = launch_repack(dsrc, src_dtype, rows, cols, L->o, c.dtype, 1, 0, nullptr); break;
      case PI_T_WG: e = launch_repack(dsrc, src_dtype, rows, cols, L->gateup, c.dtype, 2, 0, nullptr); break;
      case PI_T_WU: e = launch_repack(dsrc, src_dtype, rows, cols, L->gateup, c.dtype, 2, 1, nullptr); break;
      case PI_T_WD: e = launch_repack(dsrc, src_dtype, rows, cols, L->down, c.dtype, 1, 0, nullptr); break;
      case PI_T_LM_HEAD: e = launch_repack(dsrc, src_dtype, rows, cols, m->lm_head, c.dtype, 1, 0, nullptr); break;
      default: break;
    }
  }
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (staging) (void)hipFree(staging);
  if (e != hipSuccess) return hip_status(e);
  m->set_flags[flag_index(m, kind, layer)] = 1;
  return PI_OK;
}

int32_t pi_debug_set_plan(pi_model* m, int32_t phase, int32_t s_k, int32_t rbu, int32_t grid) {
  if (!m || phase < 0 || phase > 4) return PI_E_ARG;
  m->plan_override[phase][0] = s_k;
  m->plan_override[phase][1] = rbu;
  m->plan_override[phase][2] = grid;
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
  const size_t max_units = (size_t)n_cells / attn_sub_chunk(kv_dtype) + 2;
  const size_t rows = (size_t)kv->n_kv_heads * max_units * G * PI_MAX_BATCH;
  hipError_t e = hipMalloc(&kv->k, kv->bytes_each);
  if (e == hipSuccess) e = hipMalloc(&kv->v, kv->bytes_each);
  if (e == hipSuccess) e = hipMalloc((void**)&kv->len_dev, sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc((void**)&kv->cnt, sizeof(int));
  if (e == hipSuccess) e = hipMalloc((void**)&kv->attn_o, rows * kv->head_dim * sizeof(float));
  if (e == hipSuccess) e = hipMalloc((void**)&kv->attn_ml, rows * 2 * sizeof(float));
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
  for (void* p : {kv->k, kv->v, (void*)kv->len_dev, (void*)kv->cnt, (void*)kv->attn_o, (void*)kv->attn_ml})
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
  hipStream_t s = (hipStream_t)stream;
  const int d = c.d_model, nq = m->n_q_rows(), nkv = m->n_kv_rows();
  hipError_t e = launch_latch(m->rs, cancel_flag, run->slots, n, kv->len_dev, run->window_base, kv->n_cells,
                              layer_begin, s);
  if (e != hipSuccess) return hip_status(e);
  e = launch_embed(m->embed, c.dtype, run->tokens, layer_begin == 0 ? nullptr : hidden_in, n, d, c.vocab, m->x,
                   m->ssq, m->rs, s);
  if (e != hipSuccess) return hip_status(e);

  ProjArgs base;
  memset(&base, 0, sizeof(base));
  base.n = n;
  base.NP = n;
  base.eps = c.rms_eps;
  base.part = m->part;
  base.cnt = m->cnt;
  base.rs = m->rs;
  base.n_ssq_blocks = d / 16;
  auto fill = [&](ProjArgs& a, const PackedMat& w, int phase, int* grid) {
    a.W = w.data;
    a.N = w.N;
    a.K = w.K;
    a.NRB = w.NRB;
    a.KT = w.KT;
    const Plan p = make_plan(m, phase, w, n);
    a.S_k = p.S_k;
    a.RBU = p.RBU;
    *grid = p.grid;
  };
  const size_t kv_layer_elems = (size_t)kv->n_kv_heads * kv->n_cells * kv->head_dim;
  const size_t kv_es = kv->dtype == PI_DTYPE_BF16 ? 2 : 4;

  for (int l = layer_begin; l < layer_end; ++l) {
    const LayerWeights& W = m->layers[l];
    int grid = 0;
    char* kl = (char*)kv->k + (size_t)l * kv_layer_elems * kv_es;
    char* vl = (char*)kv->v + (size_t)l * kv_layer_elems * kv_es;
    {  // RMSNorm + QKV projection + RoPE + KV write
      ProjArgs a = base;
      fill(a, W.qkv, 0, &grid);
      a.xin = m->x;
      a.gain = W.attn_gain;
      a.ssq_in = m->ssq;
      a.out = m->q;
      a.n_q_rows = nq;
      a.n_kv_rows = nkv;
      a.head_dim = c.head_dim;
      a.kcache = kl;
      a.vcache = vl;
      a.n_cells = kv->n_cells;
      a.kv_dtype = kv->dtype;
      a.positions = run->positions;
      a.slots = run->slots;
      a.rope = m->rope;
      e = launch_proj(a, EPI_QKV, c.dtype, grid, s);
      if (e != hipSuccess) return hip_status(e);
    }
    {  // attention
      AttnArgs t;
      memset(&t, 0, sizeof(t));
      t.q = m->q;
      t.kcache = kl;
      t.vcache = vl;
      t.kv_dtype = kv->dtype;
      t.n_cells = kv->n_cells;
      t.n = n;
      t.n_q_heads = c.n_q_heads;
      t.n_kv_heads = c.n_kv_heads;
      t.head_dim = c.head_dim;
      t.prefix_len = run->prefix_len;
      t.window_base = run->window_base;
      t.mask = run->mask;
      const int sc = attn_sub_chunk(kv->dtype);
      int chunk = (int)(((int64_t)run->prefix_len * c.n_kv_heads + 383) / 384);
      chunk = ((chunk + sc - 1) / sc) * sc;
      if (chunk < sc) chunk = sc;
      t.chunk_cells = chunk;
      t.n_prefix_units = (run->prefix_len + chunk - 1) / chunk;
      t.part_o = kv->attn_o;
      t.part_ml = kv->attn_ml;
      t.out = m->o;
      t.rs = m->rs;
      e = launch_attention(t, s);
      if (e != hipSuccess) return hip_status(e);
    }
    {  // output projection + residual
      ProjArgs a = base;
      fill(a, W.o, 1, &grid);
      a.xin = m->o;
      a.out = m->x;
      a.ssq_out = m->ssq;
      e = launch_proj(a, EPI_RESID, c.dtype, grid, s);
      if (e != hipSuccess) return hip_status(e);
    }
    {  // RMSNorm + gate/up projection + SwiGLU
      ProjArgs a = base;
      fill(a, W.gateup, 2, &grid);
      a.xin = m->x;
      a.gain = W.ffn_gain;
      a.ssq_in = m->ssq;
      a.out = m->a;
      e = launch_proj(a, EPI_SWIGLU, c.dtype, grid, s);
      if (e != hipSuccess) return hip_status(e);
    }
    {  // down projection + residual; layer boundary: record progress, probe the cancel flag
      ProjArgs a = base;
      fill(a, W.down, 3, &grid);
      a.xin = m->a;
      a.out = m->x;
      a.ssq_out = m->ssq;
      a.rs_mut = m->rs;
      a.done_cnt = m->done_cnt;
      a.cancel_flag = cancel_flag;
      a.next_layer = l + 1;
      a.probe = (l + 1 < layer_end) ? 1 : 0;
      e = launch_proj(a, EPI_RESID, c.dtype, grid, s);
      if (e != hipSuccess) return hip_status(e);
    }
  }
  if (layer_end == L) {  // final RMSNorm + LM head
    int grid = 0;
    ProjArgs a = base;
    fill(a, m->lm_head, 4, &grid);
    a.xin = m->x;
    a.gain = m->final_gain;
    a.ssq_in = m->ssq;
    a.out = logits_out;
    e = launch_proj(a, EPI_LOGITS, c.dtype, grid, s);
    if (e != hipSuccess) return hip_status(e);
  }
  e = launch_finish(m->rs, run_status, m->x, layer_end == L ? nullptr : hidden_out, n, d, s);
  return hip_status(e);
}

int32_t pi_verify_greedy(const int32_t* draft, const int32_t* parent, int32_t n, const float* logits,
                         int32_t vocab, int32_t root_expected, int32_t* accepted_nodes, int32_t* result,
                         void* stream) {
  if (!draft || !logits || !accepted_nodes || !result) return PI_E_ARG;
  if (n < 1 || n > PI_MAX_BATCH || vocab < 1 || vocab > (1 << 24)) return PI_E_SHAPE;
  std::call_once(g_verify_once, [] {
    hipError_t e = hipMalloc((void**)&g_verify.best_val, PI_MAX_BATCH * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&g_verify.best_idx, PI_MAX_BATCH * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void**)&g_verify.cnt, sizeof(int));
    if (e == hipSuccess) e = hipMemset(g_verify.cnt, 0, sizeof(int));
    if (e == hipSuccess) e = hipDeviceSynchronize();
    g_verify_err = e;
  });
  if (g_verify_err != hipSuccess) return hip_status(g_verify_err);
  return hip_status(launch_verify(draft, parent, n, logits, vocab, root_expected, accepted_nodes, result,
                                  g_verify.best_val, g_verify.best_idx, g_verify.cnt, (hipStream_t)stream));
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
