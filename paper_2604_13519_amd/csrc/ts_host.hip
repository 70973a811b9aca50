// Host side of libtoolspec_hip.so: the C ABI of include/toolspec.h, model / cache
// ownership, argument validation, and the launch sequence of one verify pass.
// All arithmetic of the pass runs in the kernels; the host only validates the tree,
// derives per-row bookkeeping (depth, position, ancestor bit set) and orders launches.
#include <stdarg.h>
#include <stdlib.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <new>

#include "ts_internal.h"
#include "ts_device_utils.h"

// ---------------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------------
static thread_local std::string g_last_error;

ts_status ts_fail(ts_status code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return code;
}

extern "C" const char* ts_last_error(void) { return g_last_error.c_str(); }

// ---------------------------------------------------------------------------------
// profiling brackets
// ---------------------------------------------------------------------------------
void prof_begin(ts_model* m, const char* name) {
  while (m->ev_pool.size() < m->ev_used + 2) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return;
    m->ev_pool.push_back(e);
  }
  ProfRec r;
  r.name = name;
  r.a = m->ev_pool[m->ev_used++];
  r.b = m->ev_pool[m->ev_used++];
  hipEventRecord(r.a, m->stream);
  m->prof.push_back(r);
}
void prof_end(ts_model* m) {
  if (!m->prof.empty()) hipEventRecord(m->prof.back().b, m->stream);
}

// ---------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------
static inline float bf16_bits_to_float(uint16_t u) {
  uint32_t b = (uint32_t)u << 16;
  float f;
  memcpy(&f, &b, 4);
  return f;
}
static inline float half_bits_to_float(uint16_t h) {
  const uint32_t sign = (uint32_t)(h & 0x8000u) << 16, e = (h >> 10) & 0x1fu, f = h & 0x3ffu;
  uint32_t bits;
  if (e == 0x1fu) bits = sign | 0x7f800000u | (f << 13);                      // inf / NaN
  else if (e != 0) bits = sign | ((e + 112u) << 23) | (f << 13);              // normal
  else if (f == 0) bits = sign;                                               // zero
  else {                                                                      // subnormal: f * 2^-24
    float v = (float)f * 5.9604644775390625e-08f;
    memcpy(&bits, &v, 4);
    bits |= sign;
  }
  float out;
  memcpy(&out, &bits, 4);
  return out;
}

template <typename T>
static ts_status dev_alloc(T** p, size_t count) {
  void* q = nullptr;
  hipError_t e = hipMalloc(&q, std::max<size_t>(count * sizeof(T), 256));
  if (e != hipSuccess) return ts_fail(TS_ERR_OOM, "hipMalloc of %zu bytes failed: %s", count * sizeof(T), hipGetErrorString(e));
  *p = (T*)q;
  return TS_OK;
}
static ts_status dev_alloc_bytes(void** p, size_t bytes, bool zero) {
  hipError_t e = hipMalloc(p, std::max<size_t>(bytes, 256));
  if (e != hipSuccess) return ts_fail(TS_ERR_OOM, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
  if (zero) {
    e = hipMemset(*p, 0, std::max<size_t>(bytes, 256));
    if (e == hipSuccess) e = hipDeviceSynchronize();   // allocations are rare; later work runs on a non-blocking stream
    if (e != hipSuccess) return ts_fail(TS_ERR_DEVICE, "hipMemset failed: %s", hipGetErrorString(e));
  }
  return TS_OK;
}
static void dev_free(void* p) { if (p) (void)hipFree(p); }

// Stream-ordered copy followed by a wait: the model's stream is non-blocking, so copies on
// the null stream would not be ordered against its kernels.
static hipError_t copy_sync(hipStream_t s, void* dst, const void* src, size_t bytes, hipMemcpyKind kind) {
  hipError_t e = hipMemcpyAsync(dst, src, bytes, kind, s);
  if (e != hipSuccess) return e;
  return hipStreamSynchronize(s);
}

// Static staging area of ts_kv_export_noalloc (the entry point for callers that cannot allocate).
constexpr size_t kExportScratchBytes = (size_t)2 << 20;            // K slab in the first half, V slab in the second
static __device__ __align__(256) unsigned char scratch[kExportScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];                            // device address of `scratch`, per device

// Device address of this device's copy of `scratch` (each GPU holds its own copy at its own
// address).  `device` must be the current device.  Host code never passes the array's name to a
// kernel or a copy: on the host that name is only a handle for this lookup.
static ts_status scratch_address(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return ts_fail(TS_ERR_INVALID_ARG, "device index %d outside [0,%d)", device, kMaxDevices);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return ts_fail(TS_ERR_DEVICE, "hipGetSymbolAddress(scratch) failed on device %d: %s", device, hipGetErrorString(e));
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return TS_OK;
}

static bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

// ---------------------------------------------------------------------------------
// model
// ---------------------------------------------------------------------------------
static ts_status check_config(const ts_model_config& c) {
  if (c.n_layers < 1 || c.d_model < 1 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.head_dim < 1 || c.d_ffn < 1 || c.vocab < 1)
    return ts_fail(TS_ERR_INVALID_ARG, "model config: all sizes must be positive");
  if (c.n_q_heads % c.n_kv_heads) return ts_fail(TS_ERR_INVALID_ARG, "n_q_heads must be a multiple of n_kv_heads");
  if (!(c.rms_eps > 0.f) || !(c.rope_theta > 0.f)) return ts_fail(TS_ERR_INVALID_ARG, "rms_eps and rope_theta must be positive");
  if (c.d_ffn % 16) return ts_fail(TS_ERR_INVALID_ARG, "d_ffn must be a multiple of 16");
  if (c.d_model % 4) return ts_fail(TS_ERR_INVALID_ARG, "d_model must be a multiple of 4");
  if (c.dtype == TS_DTYPE_BF16) {
    if (c.d_model % 128 || (c.n_q_heads * c.head_dim) % 128 || c.d_ffn % 128)
      return ts_fail(TS_ERR_INVALID_ARG, "bf16 path: d_model, n_q_heads*head_dim and d_ffn must be multiples of 128");
    if (c.head_dim != 64 && c.head_dim != 128) return ts_fail(TS_ERR_INVALID_ARG, "bf16 path: head_dim must be 64 or 128");
    if (!is_pow2(c.n_q_heads / c.n_kv_heads)) return ts_fail(TS_ERR_INVALID_ARG, "bf16 path: query heads per KV head must be a power of two");
  } else if (c.dtype == TS_DTYPE_F32) {
    if (!is_pow2(c.head_dim) || c.head_dim < 8 || c.head_dim > 128)
      return ts_fail(TS_ERR_INVALID_ARG, "fp32 path: head_dim must be a power of two in [8,128]");
  } else {
    return ts_fail(TS_ERR_INVALID_ARG, "dtype must be TS_DTYPE_F32 or TS_DTYPE_BF16");
  }
  return TS_OK;
}

static void free_workspace(ts_model* m) {
  dev_free(m->H); dev_free(m->Xn); dev_free(m->Qb); dev_free(m->Ab); dev_free(m->Fb); dev_free(m->part);
  dev_free(m->attn_part_o); dev_free(m->attn_part_ml); dev_free(m->rope_cs); dev_free(m->row_dst); dev_free(m->amax_val);
  dev_free(m->amax_idx); dev_free(m->logits); dev_free(m->meta_dev); dev_free(m->seq_dev);
  dev_free(m->samp_lse); dev_free(m->samp_tok);
  if (m->meta_host) (void)hipHostFree(m->meta_host);
  if (m->res_host) (void)hipHostFree(m->res_host);
  m->H = nullptr; m->Xn = m->Qb = m->Ab = m->Fb = nullptr; m->part = nullptr;
  m->attn_part_o = nullptr; m->attn_part_ml = nullptr; m->rope_cs = nullptr; m->row_dst = nullptr; m->amax_val = nullptr; m->amax_idx = nullptr;
  m->logits = nullptr; m->meta_dev = nullptr; m->seq_dev = nullptr; m->meta_host = nullptr; m->res_host = nullptr;
  m->samp_lse = nullptr; m->samp_tok = nullptr;
  m->ws_rows = 0; m->ws_seqs = 0; m->logits_rows = 0; m->attn_max_splits = 0; m->part_elems = 0;
}

static size_t meta_bytes_for(int rows) { return (size_t)rows * (6 * sizeof(int32_t) + sizeof(uint64_t) + sizeof(float)); }

// Row buffers carry TS_MROWS_PER_BLOCK spare rows: tile-granular kernels read (never use)
// rows past the last real one.
static ts_status ensure_workspace(ts_model* m, int rows, int seqs, bool want_logits = false) {
  const ts_model_config& c = m->cfg;
  ts_status st;
  if (rows > m->ws_rows || seqs > m->ws_seqs) {
    TS_HIP(hipStreamSynchronize(m->stream));
    const bool keep = m->keep_logits;
    free_workspace(m);
    const int cap = ((rows + TS_MROWS_PER_BLOCK - 1) / TS_MROWS_PER_BLOCK) * TS_MROWS_PER_BLOCK;
    const int alloc_rows = cap + TS_MROWS_PER_BLOCK;
    const int scap = std::max(seqs, 1);
    const size_t esz = m->esz;
    if ((st = dev_alloc_bytes((void**)&m->H, (size_t)alloc_rows * c.d_model * 4, true))) return st;
    // projection inputs of bf16 models: a hi plane and a lo plane of IEEE halves, alloc_rows apart
    const size_t planes = c.dtype == TS_DTYPE_BF16 ? 2 : 1;
    if ((st = dev_alloc_bytes(&m->Xn, planes * alloc_rows * c.d_model * esz, true))) return st;
    if ((st = dev_alloc_bytes(&m->Qb, (size_t)alloc_rows * m->q_dim * esz, true))) return st;
    if ((st = dev_alloc_bytes(&m->Ab, planes * alloc_rows * m->q_dim * esz, true))) return st;
    if ((st = dev_alloc_bytes(&m->Fb, planes * alloc_rows * c.d_ffn * esz, true))) return st;
    size_t pe = 0;
    if (c.dtype == TS_DTYPE_BF16) {
      const int Ns[4] = {m->qkv_dim, c.d_model, 2 * c.d_ffn, c.d_model};
      const int Ks[4] = {c.d_model, m->q_dim, c.d_model, c.d_ffn};
      // the plan depends on the row count of a call; project() falls back to fewer splits if a
      // plan would not fit, so size for the planned splits at capacity and for 16 splits of one row block
      for (int i = 0; i < 4; ++i) {
        pe = std::max(pe, (size_t)gemm_bf16_plan(m, cap, Ns[i], Ks[i], 0).splits * cap * Ns[i]);
        pe = std::max(pe, (size_t)16 * std::min(cap, TS_MROWS_PER_BLOCK) * Ns[i]);
        // batches: room for up to 8 splits of the un-fused projections (the planner stays within part_elems)
        if (cap > TS_MROWS_PER_BLOCK && i != 2) pe = std::max(pe, std::min((size_t)8 * cap * Ns[i], (size_t)64 << 20));
      }
    } else {
      pe = (size_t)cap * std::max(std::max(m->qkv_dim, 2 * c.d_ffn), c.d_model);
    }
    m->part_elems = pe;
    if ((st = dev_alloc_bytes((void**)&m->part, pe * 4, true))) return st;
    if ((st = dev_alloc_bytes((void**)&m->rope_cs, (size_t)alloc_rows * (c.head_dim / 2) * sizeof(float2), true))) return st;
    if ((st = dev_alloc_bytes((void**)&m->row_dst, (size_t)alloc_rows * sizeof(RowDst), true))) return st;
    if ((st = dev_alloc_bytes((void**)&m->amax_val, (size_t)alloc_rows * m->amax_parts * 4, true))) return st;
    if ((st = dev_alloc_bytes((void**)&m->amax_idx, (size_t)alloc_rows * m->amax_parts * 4, true))) return st;
    if ((st = dev_alloc_bytes((void**)&m->samp_lse, (size_t)alloc_rows * 4, true))) return st;
    if ((st = dev_alloc_bytes((void**)&m->samp_tok, (size_t)alloc_rows * 4, true))) return st;
    m->meta_bytes = meta_bytes_for(alloc_rows);
    if ((st = dev_alloc_bytes(&m->meta_dev, m->meta_bytes, true))) return st;
    if ((st = dev_alloc_bytes((void**)&m->seq_dev, (size_t)scap * sizeof(SeqDesc), true))) return st;
    TS_HIP(hipHostMalloc(&m->meta_host, m->meta_bytes + (size_t)scap * sizeof(SeqDesc), hipHostMallocDefault));
    TS_HIP(hipHostMalloc((void**)&m->res_host, (size_t)scap * TS_RESULT_INTS * sizeof(int32_t), hipHostMallocDefault));
    m->ws_rows = cap;
    m->ws_seqs = scap;
    m->keep_logits = keep;
  }
  const bool need_logits = m->keep_logits || want_logits || c.dtype == TS_DTYPE_F32;
  if (need_logits && m->logits_rows < m->ws_rows) {
    TS_HIP(hipStreamSynchronize(m->stream));
    dev_free(m->logits);
    m->logits = nullptr;
    if ((st = dev_alloc_bytes((void**)&m->logits, (size_t)(m->ws_rows + TS_MROWS_PER_BLOCK) * c.vocab * 4, true))) return st;
    m->logits_rows = m->ws_rows;
  }
  return TS_OK;
}

static ts_status ensure_attn_partials(ts_model* m, int splits, int R) {
  if (m->cfg.dtype != TS_DTYPE_BF16) return TS_OK;
  const size_t need = (size_t)splits * R;
  if (need <= (size_t)m->attn_max_splits) return TS_OK;   // attn_max_splits counts split*row slots
  TS_HIP(hipStreamSynchronize(m->stream));
  dev_free(m->attn_part_o); dev_free(m->attn_part_ml);
  m->attn_part_o = nullptr; m->attn_part_ml = nullptr;
  m->attn_max_splits = 0;
  ts_status st;
  if ((st = dev_alloc_bytes((void**)&m->attn_part_o, need * m->q_dim * 2, true))) return st;
  if ((st = dev_alloc_bytes((void**)&m->attn_part_ml, need * m->cfg.n_q_heads * 2 * 4, true))) return st;
  m->attn_max_splits = (int)need;
  return TS_OK;
}

// Upload one host matrix [N][K] and leave it on the device in the layout its GEMM reads.
// bf16: staged row-major, then re-tiled as IEEE half into dst at tile offset n_tile0 (stride
//       n_tile_stride); m->range_flag collects weights that half cannot hold.
// f32 : copied row-major to dst + row_off rows.
static ts_status upload_matrix(ts_model* m, const void* host, int N, int K, void* dst, void* staging, int n_tile0,
                               int n_tile_stride, int f32_row_off) {
  if (!host) return ts_fail(TS_ERR_INVALID_ARG, "null weight pointer");
  if (m->cfg.dtype == TS_DTYPE_BF16) {
    TS_HIP(copy_sync(m->stream, staging, host, (size_t)N * K * 2, hipMemcpyHostToDevice));
    launch_repack_tiles(m->stream, (const bf16_t*)staging, (f16_t*)dst, N, K, n_tile0, n_tile_stride, m->range_flag);
    TS_HIP(hipGetLastError());
    TS_HIP(hipStreamSynchronize(m->stream));
  } else {
    TS_HIP(copy_sync(m->stream, (float*)dst + (size_t)f32_row_off * K, host, (size_t)N * K * 4, hipMemcpyHostToDevice));
  }
  return TS_OK;
}

static ts_status upload_gain(ts_model* m, const void* host, float** dst) {
  if (!host) return ts_fail(TS_ERR_INVALID_ARG, "null norm pointer");
  const int d = m->cfg.d_model;
  std::vector<float> tmp(d);
  if (m->cfg.dtype == TS_DTYPE_BF16)
    for (int i = 0; i < d; ++i) tmp[i] = bf16_bits_to_float(((const uint16_t*)host)[i]);
  else
    memcpy(tmp.data(), host, (size_t)d * 4);
  ts_status st = dev_alloc(dst, (size_t)d);
  if (st) return st;
  TS_HIP(copy_sync(m->stream, *dst, tmp.data(), (size_t)d * 4, hipMemcpyHostToDevice));
  return TS_OK;
}

static size_t tiled_elems(int N, int K) { return (size_t)((N + 15) / 16) * 16 * K; }

static ts_status model_load_impl(ts_model* m, const ts_weights* w) {
  const ts_model_config& c = m->cfg;
  ts_status st;
  const bool bf = c.dtype == TS_DTYPE_BF16;
  const size_t esz = m->esz;
  const int d = c.d_model, F = c.d_ffn, V = c.vocab;
  if (!w->embed || !w->lm_head || !w->norm_f || !w->wq || !w->wk || !w->wv || !w->wo || !w->wg || !w->wu || !w->wd ||
      !w->norm1 || !w->norm2)
    return ts_fail(TS_ERR_INVALID_ARG, "ts_weights has a null member");

  void* staging = nullptr;
  if (bf) {
    size_t big = std::max((size_t)V * d, (size_t)F * d);
    big = std::max(big, (size_t)m->q_dim * d);
    if ((st = dev_alloc_bytes(&staging, big * 2, false))) return st;
    if ((st = dev_alloc_bytes((void**)&m->range_flag, sizeof(int), true))) { dev_free(staging); return st; }
    if ((st = dev_alloc_bytes((void**)&m->sat_count, sizeof(unsigned long long), true))) { dev_free(staging); return st; }
  }
  auto matrix_bytes = [&](int N, int K) { return (bf ? tiled_elems(N, K) : (size_t)N * K) * esz; };

  // embedding stays row-major in the storage dtype (it is gathered, not multiplied)
  if ((st = dev_alloc_bytes(&m->embed, (size_t)V * d * esz, false))) { dev_free(staging); return st; }
  {
    hipError_t e = copy_sync(m->stream, m->embed, w->embed, (size_t)V * d * esz, hipMemcpyHostToDevice);
    if (e != hipSuccess) { dev_free(staging); return ts_fail(TS_ERR_DEVICE, "embedding upload failed: %s", hipGetErrorString(e)); }
  }
  st = dev_alloc_bytes(&m->lm_head, matrix_bytes(V, d), false);
  if (!st) st = upload_matrix(m, w->lm_head, V, d, m->lm_head, staging, 0, 1, 0);
  if (!st) st = upload_gain(m, w->norm_f, &m->norm_f);

  m->layers.assign(c.n_layers, LayerW{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr});
  std::vector<float> gu_host;
  for (int l = 0; l < c.n_layers && !st; ++l) {
    LayerW& L = m->layers[l];
    if (!w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->wg[l] || !w->wu[l] || !w->wd[l] || !w->norm1[l] || !w->norm2[l]) {
      st = ts_fail(TS_ERR_INVALID_ARG, "null weight pointer in layer %d", l);
      break;
    }
    if ((st = dev_alloc_bytes(&L.wqkv, matrix_bytes(m->qkv_dim, d), false))) break;
    if ((st = dev_alloc_bytes(&L.wo, matrix_bytes(d, m->q_dim), false))) break;
    if ((st = dev_alloc_bytes(&L.wgu, matrix_bytes(2 * F, d), false))) break;
    if ((st = dev_alloc_bytes(&L.wd, matrix_bytes(d, F), false))) break;
    // fused QKV: rows [q | k | v]
    if ((st = upload_matrix(m, w->wq[l], m->q_dim, d, L.wqkv, staging, 0, 1, 0))) break;
    if ((st = upload_matrix(m, w->wk[l], m->kv_dim, d, L.wqkv, staging, m->q_dim / 16, 1, m->q_dim))) break;
    if ((st = upload_matrix(m, w->wv[l], m->kv_dim, d, L.wqkv, staging, (m->q_dim + m->kv_dim) / 16, 1, m->q_dim + m->kv_dim))) break;
    if ((st = upload_matrix(m, w->wo[l], d, m->q_dim, L.wo, staging, 0, 1, 0))) break;
    // fused gate/up: 16-row tiles alternate gate, up, gate, up, ...
    if (bf) {
      if ((st = upload_matrix(m, w->wg[l], F, d, L.wgu, staging, 0, 2, 0))) break;
      if ((st = upload_matrix(m, w->wu[l], F, d, L.wgu, staging, 1, 2, 0))) break;
    } else {
      gu_host.resize((size_t)2 * F * d);
      const float* g = (const float*)w->wg[l];
      const float* u = (const float*)w->wu[l];
      for (int t = 0; t < F / 16; ++t) {
        memcpy(&gu_host[(size_t)(2 * t) * 16 * d], g + (size_t)t * 16 * d, (size_t)16 * d * 4);
        memcpy(&gu_host[(size_t)(2 * t + 1) * 16 * d], u + (size_t)t * 16 * d, (size_t)16 * d * 4);
      }
      if ((st = upload_matrix(m, gu_host.data(), 2 * F, d, L.wgu, staging, 0, 1, 0))) break;
    }
    if ((st = upload_matrix(m, w->wd[l], d, F, L.wd, staging, 0, 1, 0))) break;
    if ((st = upload_gain(m, w->norm1[l], &L.norm1))) break;
    if ((st = upload_gain(m, w->norm2[l], &L.norm2))) break;
  }
  dev_free(staging);
  if (!st && bf) {       // the projections multiply in IEEE half: every finite weight has to fit its range
    int flag = 0;
    TS_HIP(copy_sync(m->stream, &flag, m->range_flag, sizeof(int), hipMemcpyDeviceToHost));
    if (flag) st = ts_fail(TS_ERR_INVALID_ARG, "a projection weight exceeds the IEEE half range (|w| > 65504)");
  }
  return st;
}

extern "C" ts_status ts_model_free(ts_model* m) {
  if (!m) return TS_OK;
  (void)hipSetDevice(m->device);
  if (m->stream) (void)hipStreamSynchronize(m->stream);
  free_workspace(m);
  dev_free(m->embed); dev_free(m->lm_head); dev_free(m->norm_f); dev_free(m->range_flag); dev_free(m->sat_count);
  for (LayerW& L : m->layers) {
    dev_free(L.wqkv); dev_free(L.wo); dev_free(L.wgu); dev_free(L.wd); dev_free(L.norm1); dev_free(L.norm2);
  }
  for (hipEvent_t e : m->ev_pool) (void)hipEventDestroy(e);
  if (m->stream) (void)hipStreamDestroy(m->stream);
  delete m;
  return TS_OK;
}

extern "C" ts_status ts_model_load(const ts_model_config* cfg, const ts_weights* w, ts_model** out) {
  if (!cfg || !w || !out) return ts_fail(TS_ERR_INVALID_ARG, "ts_model_load: null argument");
  *out = nullptr;
  ts_status st = check_config(*cfg);
  if (st) return st;
  ts_model* m = new (std::nothrow) ts_model();
  if (!m) return ts_fail(TS_ERR_OOM, "host allocation failed");
  m->cfg = *cfg;
  m->esz = cfg->dtype == TS_DTYPE_BF16 ? 2 : 4;
  m->q_dim = cfg->n_q_heads * cfg->head_dim;
  m->kv_dim = cfg->n_kv_heads * cfg->head_dim;
  m->qkv_dim = m->q_dim + 2 * m->kv_dim;
  m->stream = nullptr;
  m->embed = m->lm_head = nullptr; m->norm_f = nullptr; m->range_flag = nullptr; m->sat_count = nullptr;
  m->H = nullptr; m->Xn = m->Qb = m->Ab = m->Fb = nullptr; m->part = nullptr; m->part_elems = 0;
  m->attn_part_o = nullptr; m->attn_part_ml = nullptr; m->attn_max_splits = 0;
  m->rope_cs = nullptr; m->row_dst = nullptr; m->amax_val = nullptr; m->amax_idx = nullptr; m->logits = nullptr;
  m->keep_logits = false; m->logits_rows = 0; m->meta_dev = nullptr; m->meta_host = nullptr; m->meta_bytes = 0;
  m->seq_dev = nullptr; m->res_host = nullptr; m->ws_rows = 0; m->ws_seqs = 0;
  m->samp_lse = nullptr; m->samp_tok = nullptr;
  m->prof_on = false; m->ev_used = 0; m->last_rows = 0;
  hipError_t e = hipGetDevice(&m->device);
  hipDeviceProp_t prop;
  if (e == hipSuccess) e = hipGetDeviceProperties(&prop, m->device);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&m->stream, hipStreamNonBlocking);
  if (e != hipSuccess) {
    delete m;
    return ts_fail(TS_ERR_DEVICE, "device setup failed: %s", hipGetErrorString(e));
  }
  m->n_cu = prop.multiProcessorCount;
  {   // set-up: resolve this device's copy of the static staging area once, while the device is current
    void* unused = nullptr;
    if (scratch_address(m->device, &unused) != TS_OK) {
      (void)hipStreamDestroy(m->stream);
      delete m;
      return TS_ERR_DEVICE;
    }
  }
  if (cfg->dtype == TS_DTYPE_BF16) {
    const GemmPlan p = gemm_bf16_plan(m, TS_MROWS_PER_BLOCK, cfg->vocab, cfg->d_model, 1);
    const int cols = gemm_bf16_cols_per_group(p.shape);
    m->amax_parts = (cfg->vocab + cols - 1) / cols;
  } else {
    m->amax_parts = 1;
  }
  m->amax_used = m->amax_parts;
  st = model_load_impl(m, w);
  if (!st) st = ensure_workspace(m, TS_MAX_NODES + 1, 1);
  if (st) {
    std::string keep = g_last_error;
    ts_model_free(m);
    g_last_error = keep;
    return st;
  }
  *out = m;
  return TS_OK;
}

extern "C" ts_status ts_model_keep_logits(ts_model* m, int32_t enable) {
  if (!m) return ts_fail(TS_ERR_INVALID_ARG, "null model");
  (void)hipSetDevice(m->device);
  m->keep_logits = enable != 0;
  return ensure_workspace(m, m->ws_rows, m->ws_seqs);
}

extern "C" ts_status ts_get_logits(ts_model* m, int32_t row0, int32_t n_rows, float* host) {
  if (!m || !host) return ts_fail(TS_ERR_INVALID_ARG, "null argument");
  if (!m->logits || !(m->keep_logits || m->cfg.dtype == TS_DTYPE_F32) || m->last_rows == 0)
    return ts_fail(TS_ERR_STATE, "no logits kept: call ts_model_keep_logits(m, 1) before ts_verify");
  if (row0 < 0 || n_rows < 0 || row0 + n_rows > m->last_rows)
    return ts_fail(TS_ERR_INVALID_ARG, "rows [%d,%d) outside the last pass (%d rows)", row0, row0 + n_rows, m->last_rows);
  (void)hipSetDevice(m->device);
  TS_HIP(hipStreamSynchronize(m->stream));
  TS_HIP(copy_sync(m->stream, host, m->logits + (size_t)row0 * m->cfg.vocab, (size_t)n_rows * m->cfg.vocab * 4, hipMemcpyDeviceToHost));
  return TS_OK;
}

extern "C" ts_status ts_model_saturations(ts_model* m, uint64_t* count) {
  if (!m || !count) return ts_fail(TS_ERR_INVALID_ARG, "null argument");
  *count = 0;
  if (!m->sat_count) return TS_OK;                 // fp32 models have no half-precision projection inputs
  (void)hipSetDevice(m->device);
  unsigned long long v = 0;
  TS_HIP(copy_sync(m->stream, &v, m->sat_count, sizeof(v), hipMemcpyDeviceToHost));
  *count = (uint64_t)v;
  return TS_OK;
}

extern "C" ts_status ts_get_row_tokens(ts_model* m, int32_t row0, int32_t n_rows, int32_t* host_tokens) {
  if (!m || (n_rows > 0 && !host_tokens)) return ts_fail(TS_ERR_INVALID_ARG, "null argument");
  if (m->last_rows == 0) return ts_fail(TS_ERR_STATE, "no verify pass on this model yet");
  if (row0 < 0 || n_rows < 0 || row0 + n_rows > m->last_rows)
    return ts_fail(TS_ERR_INVALID_ARG, "rows [%d,%d) outside the last pass (%d rows)", row0, row0 + n_rows, m->last_rows);
  if (n_rows == 0) return TS_OK;
  (void)hipSetDevice(m->device);
  TS_HIP(copy_sync(m->stream, host_tokens, m->samp_tok + row0, (size_t)n_rows * 4, hipMemcpyDeviceToHost));
  return TS_OK;
}

// ---------------------------------------------------------------------------------
// KV cache
// ---------------------------------------------------------------------------------
extern "C" ts_status ts_kv_free(ts_kv* kv) {
  if (!kv) return TS_OK;
  (void)hipSetDevice(kv->model->device);
  (void)hipStreamSynchronize(kv->model->stream);
  if (kv->pool) {                                   // the pages go back to the pool they came from
    ts_kv_pool* pool = kv->pool;
    for (int i = (int)kv->page_table_host.size() - 1; i >= 0; --i) pool->free_pages.push_back(kv->page_table_host[i]);
    pool->live -= 1;
  } else {
    dev_free(kv->k_pool); dev_free(kv->v_pool);
  }
  dev_free(kv->page_table); dev_free(kv->result);
  delete kv;
  return TS_OK;
}

// A cache over `pages` (physical page numbers within an allocation of pool_pages pages at k_pool / v_pool);
// pool == nullptr: the allocation is the cache's own and is freed with it.
static ts_status kv_create(ts_model* m, ts_kv_pool* pool, void* k_pool, void* v_pool, int32_t pool_pages, int32_t capacity,
                           std::vector<int32_t>&& pages, ts_kv** out) {
  ts_kv* kv = new (std::nothrow) ts_kv();
  if (!kv) {
    if (!pool) { dev_free(k_pool); dev_free(v_pool); }
    else for (int i = (int)pages.size() - 1; i >= 0; --i) pool->free_pages.push_back(pages[i]);
    return ts_fail(TS_ERR_OOM, "host allocation failed");
  }
  const ts_model_config& c = m->cfg;
  kv->model = m;
  kv->pool = pool;
  kv->capacity = capacity;
  kv->page_size = TS_PAGE_SIZE;
  kv->n_pages = (int32_t)pages.size();
  kv->pool_pages = pool_pages;
  kv->P = 0;
  kv->pending = -1;
  kv->have_result = false;
  kv->last_M = 0;
  kv->k_pool = k_pool; kv->v_pool = v_pool; kv->page_table = nullptr; kv->result = nullptr;
  kv->layer_stride_elems = (size_t)pool_pages * c.n_kv_heads * 16 * c.head_dim;
  kv->page_table_host = std::move(pages);
  // the attention kernel fetches the table four entries (one key block) at a time: pad with page 0
  ts_status st = dev_alloc_bytes((void**)&kv->page_table, (size_t)(kv->n_pages + 4) * 4, true);
  if (!st) st = dev_alloc_bytes((void**)&kv->result, TS_RESULT_INTS * 4, true);
  if (!st) {
    hipError_t e = copy_sync(m->stream, kv->page_table, kv->page_table_host.data(), (size_t)kv->n_pages * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) st = ts_fail(TS_ERR_DEVICE, "page table upload failed: %s", hipGetErrorString(e));
  }
  if (st) {
    std::string keep = g_last_error;
    if (pool) pool->live += 1;          // ts_kv_free gives the pages back and counts the cache out again
    ts_kv_free(kv);
    g_last_error = keep;
    return st;
  }
  if (pool) pool->live += 1;
  *out = kv;
  return TS_OK;
}

extern "C" ts_status ts_kv_alloc(ts_model* m, int32_t capacity, int32_t page_size, ts_kv** out) {
  if (!m || !out) return ts_fail(TS_ERR_INVALID_ARG, "ts_kv_alloc: null argument");
  *out = nullptr;
  if (page_size != TS_PAGE_SIZE) return ts_fail(TS_ERR_INVALID_ARG, "page_size must be %d", TS_PAGE_SIZE);
  if (capacity < 1) return ts_fail(TS_ERR_INVALID_ARG, "capacity_tokens must be positive");
  (void)hipSetDevice(m->device);
  const ts_model_config& c = m->cfg;
  const int32_t n_pages = (capacity + page_size - 1) / page_size;
  const size_t bytes = (size_t)n_pages * c.n_kv_heads * 16 * c.head_dim * c.n_layers * m->esz;
  void* k_pool = nullptr; void* v_pool = nullptr;
  ts_status st = dev_alloc_bytes(&k_pool, bytes, true);
  if (!st) st = dev_alloc_bytes(&v_pool, bytes, true);
  if (st) { dev_free(k_pool); dev_free(v_pool); return st; }
  std::vector<int32_t> pages(n_pages);
  for (int i = 0; i < n_pages; ++i) pages[i] = i;
  return kv_create(m, nullptr, k_pool, v_pool, n_pages, capacity, std::move(pages), out);
}

// ---------------------------------------------------------------------------------
// shared page pool
// ---------------------------------------------------------------------------------
extern "C" ts_status ts_kv_pool_create(ts_model* m, int32_t n_pages, ts_kv_pool** out) {
  if (!m || !out) return ts_fail(TS_ERR_INVALID_ARG, "ts_kv_pool_create: null argument");
  *out = nullptr;
  if (n_pages < 1) return ts_fail(TS_ERR_INVALID_ARG, "n_pages must be positive");
  (void)hipSetDevice(m->device);
  ts_kv_pool* pool = new (std::nothrow) ts_kv_pool();
  if (!pool) return ts_fail(TS_ERR_OOM, "host allocation failed");
  const ts_model_config& c = m->cfg;
  pool->model = m;
  pool->n_pages = n_pages;
  pool->k_pool = pool->v_pool = nullptr;
  pool->live = 0;
  const size_t bytes = (size_t)n_pages * c.n_kv_heads * 16 * c.head_dim * c.n_layers * m->esz;
  ts_status st = dev_alloc_bytes(&pool->k_pool, bytes, true);
  if (!st) st = dev_alloc_bytes(&pool->v_pool, bytes, true);
  if (st) { dev_free(pool->k_pool); dev_free(pool->v_pool); delete pool; return st; }
  pool->free_pages.resize(n_pages);
  for (int i = 0; i < n_pages; ++i) pool->free_pages[i] = n_pages - 1 - i;      // page 0 is handed out first
  *out = pool;
  return TS_OK;
}

extern "C" ts_status ts_kv_pool_free(ts_kv_pool* pool) {
  if (!pool) return TS_OK;
  if (pool->live != 0) return ts_fail(TS_ERR_STATE, "%d caches drawn from the pool are still alive", pool->live);
  (void)hipSetDevice(pool->model->device);
  (void)hipStreamSynchronize(pool->model->stream);
  dev_free(pool->k_pool); dev_free(pool->v_pool);
  delete pool;
  return TS_OK;
}

extern "C" ts_status ts_kv_pool_pages_free(const ts_kv_pool* pool, int32_t* n_free_pages) {
  if (!pool || !n_free_pages) return ts_fail(TS_ERR_INVALID_ARG, "null argument");
  *n_free_pages = (int32_t)pool->free_pages.size();
  return TS_OK;
}

extern "C" ts_status ts_kv_alloc_pooled(ts_kv_pool* pool, int32_t capacity, ts_kv** out) {
  if (!pool || !out) return ts_fail(TS_ERR_INVALID_ARG, "ts_kv_alloc_pooled: null argument");
  *out = nullptr;
  if (capacity < 1) return ts_fail(TS_ERR_INVALID_ARG, "capacity_tokens must be positive");
  const int32_t need = (capacity + TS_PAGE_SIZE - 1) / TS_PAGE_SIZE;
  if ((size_t)need > pool->free_pages.size())
    return ts_fail(TS_ERR_OOM, "the pool has %d free pages, capacity %d needs %d", (int)pool->free_pages.size(), capacity, need);
  (void)hipSetDevice(pool->model->device);
  std::vector<int32_t> pages(need);
  for (int i = 0; i < need; ++i) { pages[i] = pool->free_pages.back(); pool->free_pages.pop_back(); }
  return kv_create(pool->model, pool, pool->k_pool, pool->v_pool, pool->n_pages, capacity, std::move(pages), out);
}

extern "C" ts_status ts_kv_set_page_table(ts_kv* kv, const int32_t* phys, int32_t n_pages) {
  if (!kv || !phys) return ts_fail(TS_ERR_INVALID_ARG, "null argument");
  if (kv->pool) return ts_fail(TS_ERR_STATE, "the pages of a pooled cache are assigned by its pool");
  if (kv->P != 0) return ts_fail(TS_ERR_STATE, "page table can only change while the cache is empty");
  if (n_pages != kv->n_pages) return ts_fail(TS_ERR_INVALID_ARG, "n_pages must be %d", kv->n_pages);
  std::vector<char> seen(n_pages, 0);
  for (int i = 0; i < n_pages; ++i) {
    if (phys[i] < 0 || phys[i] >= n_pages || seen[phys[i]]) return ts_fail(TS_ERR_INVALID_ARG, "page table is not a permutation");
    seen[phys[i]] = 1;
  }
  (void)hipSetDevice(kv->model->device);
  TS_HIP(hipStreamSynchronize(kv->model->stream));
  kv->page_table_host.assign(phys, phys + n_pages);
  TS_HIP(copy_sync(kv->model->stream, kv->page_table, phys, (size_t)n_pages * 4, hipMemcpyHostToDevice));
  return TS_OK;
}

static ts_status kv_xfer_impl(ts_kv* kv, int pos0, int n_pos, const void* k_in, const void* v_in, void* k_out, void* v_out) {
  ts_model* m = kv->model;
  const ts_model_config& c = m->cfg;
  if (n_pos == 0) return TS_OK;
  (void)hipSetDevice(m->device);
  const size_t slab = (size_t)n_pos * c.n_kv_heads * c.head_dim * m->esz;   // one layer
  void *sk = nullptr, *sv = nullptr;
  ts_status st = dev_alloc_bytes(&sk, slab, false);
  if (!st) st = dev_alloc_bytes(&sv, slab, false);
  hipError_t e = hipSuccess;
  for (int l = 0; l < c.n_layers && !st && e == hipSuccess; ++l) {
    if (k_in) {
      e = copy_sync(m->stream, sk, (const char*)k_in + (size_t)l * slab, slab, hipMemcpyHostToDevice);
      if (e == hipSuccess) e = copy_sync(m->stream, sv, (const char*)v_in + (size_t)l * slab, slab, hipMemcpyHostToDevice);
      if (e == hipSuccess) { launch_kv_import(kv, pos0, n_pos, sk, sv, l); e = hipGetLastError(); }
      if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
    } else {
      launch_kv_export(kv, pos0, n_pos, sk, sv, l);
      e = hipGetLastError();
      if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
      if (e == hipSuccess) e = copy_sync(m->stream, (char*)k_out + (size_t)l * slab, sk, slab, hipMemcpyDeviceToHost);
      if (e == hipSuccess) e = copy_sync(m->stream, (char*)v_out + (size_t)l * slab, sv, slab, hipMemcpyDeviceToHost);
    }
  }
  dev_free(sk); dev_free(sv);
  if (st) return st;
  if (e != hipSuccess) return ts_fail(TS_ERR_DEVICE, "KV transfer failed: %s", hipGetErrorString(e));
  return TS_OK;
}

extern "C" ts_status ts_kv_import(ts_kv* kv, int32_t n_pos, const void* k_host, const void* v_host) {
  if (!kv || (n_pos > 0 && (!k_host || !v_host))) return ts_fail(TS_ERR_INVALID_ARG, "null argument");
  if (n_pos < 0 || n_pos > kv->capacity) return ts_fail(TS_ERR_KV_CAPACITY, "n_pos %d outside [0, capacity %d]", n_pos, kv->capacity);
  ts_status st = kv_xfer_impl(kv, 0, n_pos, k_host, v_host, nullptr, nullptr);
  if (st) return st;
  kv->P = n_pos;
  kv->have_result = false;
  return TS_OK;
}

extern "C" ts_status ts_kv_export(ts_kv* kv, int32_t pos0, int32_t n_pos, void* k_host, void* v_host) {
  if (!kv || (n_pos > 0 && (!k_host || !v_host))) return ts_fail(TS_ERR_INVALID_ARG, "null argument");
  if (pos0 < 0 || n_pos < 0 || pos0 + n_pos > kv->capacity)
    return ts_fail(TS_ERR_INVALID_ARG, "positions [%d,%d) outside the capacity %d", pos0, pos0 + n_pos, kv->capacity);
  return kv_xfer_impl(kv, pos0, n_pos, nullptr, nullptr, k_host, v_host);
}

// ---------------------------------------------------------------------------------
// export without allocation: the per-layer staging slabs live in a file-scope device array
// ---------------------------------------------------------------------------------
extern "C" ts_status ts_kv_export_noalloc(ts_kv* kv, int32_t pos0, int32_t n_pos, void* k_host, void* v_host) {
  if (!kv || (n_pos > 0 && (!k_host || !v_host))) return ts_fail(TS_ERR_INVALID_ARG, "null argument");
  if (pos0 < 0 || n_pos < 0 || pos0 + n_pos > kv->capacity)
    return ts_fail(TS_ERR_INVALID_ARG, "positions [%d,%d) outside the capacity %d", pos0, pos0 + n_pos, kv->capacity);
  ts_model* m = kv->model;
  const ts_model_config& c = m->cfg;
  const size_t slab = (size_t)n_pos * c.n_kv_heads * c.head_dim * m->esz;   // one layer, K or V
  if (slab > kExportScratchBytes / 2)
    return ts_fail(TS_ERR_INVALID_ARG, "ts_kv_export_noalloc: %d positions need %zu bytes per layer slab, the static staging area holds %zu (at most %zu positions of this model per call)",
                   n_pos, slab, kExportScratchBytes / 2, kExportScratchBytes / 2 / ((size_t)c.n_kv_heads * c.head_dim * m->esz));
  if (n_pos == 0) return TS_OK;
  (void)hipSetDevice(m->device);
  void* base = nullptr;
  ts_status st = scratch_address(m->device, &base);
  if (st) return st;
  void* sk = base;
  void* sv = (char*)base + kExportScratchBytes / 2;
  for (int l = 0; l < c.n_layers; ++l) {
    launch_kv_export(kv, pos0, n_pos, sk, sv, l);
    TS_HIP(hipGetLastError());
    // both copies wait for completion, so the next layer may overwrite the slabs
    TS_HIP(copy_sync(m->stream, (char*)k_host + (size_t)l * slab, sk, slab, hipMemcpyDeviceToHost));
    TS_HIP(copy_sync(m->stream, (char*)v_host + (size_t)l * slab, sv, slab, hipMemcpyDeviceToHost));
  }
  return TS_OK;
}

extern "C" ts_status ts_set_pending(ts_kv* kv, int32_t token) {
  if (!kv) return ts_fail(TS_ERR_INVALID_ARG, "null cache");
  if (token < 0 || token >= kv->model->cfg.vocab) return ts_fail(TS_ERR_TOKEN_RANGE, "token %d outside [0,%d)", token, kv->model->cfg.vocab);
  kv->pending = token;
  kv->have_result = false;
  return TS_OK;
}

extern "C" ts_status ts_kv_len(const ts_kv* kv, int32_t* len) {
  if (!kv || !len) return ts_fail(TS_ERR_INVALID_ARG, "null argument");
  *len = kv->P;
  return TS_OK;
}

extern "C" ts_status ts_kv_truncate(ts_kv* kv, int32_t new_len) {
  if (!kv) return ts_fail(TS_ERR_INVALID_ARG, "null cache");
  if (new_len < 0 || new_len > kv->P) return ts_fail(TS_ERR_INVALID_ARG, "new_len %d outside [0,%d]", new_len, kv->P);
  kv->P = new_len;
  kv->have_result = false;
  return TS_OK;
}

// ---------------------------------------------------------------------------------
// verify
// ---------------------------------------------------------------------------------
static RowMeta carve_meta(void* base, int rows) {
  RowMeta rm;
  char* p = (char*)base;
  rm.anc = (uint64_t*)p; p += (size_t)rows * sizeof(uint64_t);
  rm.tok = (int32_t*)p;  p += (size_t)rows * 4;
  rm.pos = (int32_t*)p;  p += (size_t)rows * 4;
  rm.seq = (int32_t*)p;  p += (size_t)rows * 4;
  rm.lrow = (int32_t*)p; p += (size_t)rows * 4;
  rm.par = (int32_t*)p;  p += (size_t)rows * 4;
  rm.depth = (int32_t*)p; p += (size_t)rows * 4;
  rm.u = (float*)p;
  return rm;
}

// ingest_only: run the layers (K/V of every row land in the tree slots) but not the final
// norm, lm_head, arg-max and walk, and leave no verify result behind (context ingestion).
// sample: stochastic acceptance instead of the greedy walk (one sequence; logits are materialised).
struct SampleArgs { float temperature; const float* node_uniform; uint64_t seed; };
// Context ingestion runs several consecutive row blocks of ONE cache in a pass: block b is given
// as a sequence of its own whose committed length (P) and root token are overridden - the rows of
// the blocks before it are part of its context, which is exactly the causal mask.
struct BlockOverride { const int32_t* P; const int32_t* root; };

static ts_status verify_impl(ts_model* m, ts_kv* const* kvs, int n_seqs, const int32_t* toks, const int32_t* pars,
                             const int32_t* offs, int32_t* accept_len, int32_t* acc_tokens, int32_t* acc_nodes,
                             int32_t* bonus, bool ingest_only = false, const SampleArgs* sample = nullptr,
                             const BlockOverride* blocks = nullptr) {
  const ts_model_config& c = m->cfg;
  const bool bf = c.dtype == TS_DTYPE_BF16;
  // ---- validation (nothing is modified before it passes) ---------------------------
  int R = 0, max_M = 0, max_keys = 0;
  long sum_keys = 0;
  for (int s = 0; s < n_seqs; ++s) {
    ts_kv* kv = kvs[s];
    if (!kv) return ts_fail(TS_ERR_INVALID_ARG, "null cache handle (sequence %d)", s);
    if (kv->model != m) return ts_fail(TS_ERR_INVALID_ARG, "cache %d belongs to another model", s);
    for (int t = 0; t < s && !blocks; ++t)
      if (kvs[t] == kv) return ts_fail(TS_ERR_INVALID_ARG, "cache handle used twice in one batch");
    const int P_s = blocks ? blocks->P[s] : kv->P;
    const int n = offs[s + 1] - offs[s];
    if (n < 0 || n > TS_MAX_NODES) return ts_fail(TS_ERR_INVALID_TREE, "n_nodes %d outside [0,%d] (sequence %d)", n, TS_MAX_NODES, s);
    if (n > 0 && (!toks || !pars)) return ts_fail(TS_ERR_INVALID_ARG, "null draft arrays with n_nodes > 0");
    if (!blocks && kv->pending < 0) return ts_fail(TS_ERR_STATE, "no pending token (sequence %d): call ts_set_pending or commit a verify", s);
    if (P_s + n + 1 > kv->capacity)
      return ts_fail(TS_ERR_KV_CAPACITY, "committed %d + tree rows %d exceed the capacity %d (sequence %d)", P_s, n + 1, kv->capacity, s);
    for (int i = 0; i < n; ++i) {
      const int p = pars[offs[s] + i], t = toks[offs[s] + i];
      if (p < -1 || p >= i) return ts_fail(TS_ERR_INVALID_TREE, "parent_idx[%d] = %d outside [-1,%d) (sequence %d)", i, p, i, s);
      if (t < 0 || t >= c.vocab) return ts_fail(TS_ERR_TOKEN_RANGE, "draft token %d outside [0,%d) (node %d, sequence %d)", t, c.vocab, i, s);
    }
    R += n + 1;
    max_M = std::max(max_M, n + 1);
    max_keys = std::max(max_keys, P_s + n + 1);
    sum_keys += P_s + n + 1;
  }
  if (!bf && (size_t)max_keys > attn_f32_max_keys())
    return ts_fail(TS_ERR_KV_CAPACITY, "fp32 path supports at most %zu keys per sequence", attn_f32_max_keys());

  (void)hipSetDevice(m->device);
  ts_status st = ensure_workspace(m, R, n_seqs, sample != nullptr);
  if (st) return st;
  const int splits = bf ? attn_bf16_splits(m, max_keys, n_seqs, sum_keys) : 1;
  if ((st = ensure_attn_partials(m, splits, R))) return st;

  // ---- per-row bookkeeping (Alg. 1: flattened sequence + tree mask) ------------------
  const int alloc_rows = m->ws_rows + TS_MROWS_PER_BLOCK;
  RowMeta hm = carve_meta(m->meta_host, alloc_rows);
  RowMeta dm = carve_meta(m->meta_dev, alloc_rows);
  SeqDesc* hseq = (SeqDesc*)((char*)m->meta_host + m->meta_bytes);
  int r0 = 0;
  for (int s = 0; s < n_seqs; ++s) {
    ts_kv* kv = kvs[s];
    const int n = offs[s + 1] - offs[s];
    const int P_s = blocks ? blocks->P[s] : kv->P;
    hm.tok[r0] = blocks ? blocks->root[s] : kv->pending; hm.pos[r0] = P_s; hm.seq[r0] = s; hm.lrow[r0] = 0;
    hm.par[r0] = -1; hm.depth[r0] = 0; hm.anc[r0] = 0; hm.u[r0] = 0.f;
    for (int i = 0; i < n; ++i) {
      const int r = r0 + i + 1;
      const int prow = pars[offs[s] + i] + 1;             // local parent row
      hm.tok[r] = toks[offs[s] + i];
      hm.seq[r] = s; hm.lrow[r] = i + 1; hm.par[r] = prow;
      hm.depth[r] = hm.depth[r0 + prow] + 1;
      hm.pos[r] = P_s + hm.depth[r];
      hm.anc[r] = hm.anc[r0 + prow] | (1ull << i);
      hm.u[r] = sample ? sample->node_uniform[offs[s] + i] : 0.f;
    }
    SeqDesc& sd = hseq[s];
    sd.P = P_s; sd.M = n + 1; sd.row0 = r0; sd.n_pages = kv->pool_pages;
    sd.page_table = kv->page_table; sd.k_pool = kv->k_pool; sd.v_pool = kv->v_pool; sd.result = kv->result;
    kv->have_result = false;
    r0 += n + 1;
  }
  TS_HIP(hipMemcpyAsync(m->meta_dev, m->meta_host, m->meta_bytes, hipMemcpyHostToDevice, m->stream));
  TS_HIP(hipMemcpyAsync(m->seq_dev, hseq, (size_t)n_seqs * sizeof(SeqDesc), hipMemcpyHostToDevice, m->stream));

  // ---- the pass ---------------------------------------------------------------------
  m->prof.clear();
  m->ev_used = 0;
  const int d = c.d_model, F = c.d_ffn;
  // bracket of the whole pass (first launch .. acceptance walk), only when asked for by name
  const bool time_pass = m->prof_on && m->prof_filter == "verify_pass";
  if (time_pass) prof_begin(m, "verify_pass");
  const size_t pass_rec = m->prof.size();
  launch_embed(m, dm, R);       // + rotary table and K/V destinations of the rows
  int pending_parts = 0;          // split-K partials of the previous projection still to be added to H
  size_t pending_stride = 0;
  auto project = [&](const char* name, const void* X, const void* W, int N, int K, int* n_parts, size_t* stride) {
    if (bf) {
      GemmPlan p = gemm_bf16_plan(m, R, N, K, 0);
      while (p.splits > 1 && (size_t)p.splits * R * N > m->part_elems) p.splits = K / gemm_bf16_chunk(p.shape) % (p.splits / 2) == 0 ? p.splits / 2 : 1;
      ProfScope ps(m, name);
      launch_gemm_bf16(m, (const f16_t*)X, (const f16_t*)W, m->part, R, N, K, p, 0, nullptr, nullptr);
      *n_parts = p.splits;
      *stride = (size_t)R * N;
    } else {
      launch_gemm_f32(m, (const float*)X, (const float*)W, m->part, R, N, K);
      *n_parts = 1;
      *stride = (size_t)R * N;
    }
  };
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerW& L = m->layers[l];
    int np; size_t ps;
    launch_norm(m, R, L.norm1, pending_parts, pending_stride, l == 0);
    project("gemm_qkv", m->Xn, L.wqkv, m->qkv_dim, d, &np, &ps);
    launch_rope_kv(m, dm, R, l, np, ps);
    if (bf) {
      launch_attn_bf16(m, dm, R, n_seqs, l, splits, max_M);
      launch_attn_merge(m, R, splits);
    } else {
      launch_attn_f32(m, dm, R, n_seqs, l, max_keys);
    }
    project("gemm_o", m->Ab, L.wo, d, m->q_dim, &np, &ps);
    launch_norm(m, R, L.norm2, np, ps, false);
    if (bf) {   // gate/up projection with the SwiGLU product in its epilogue
      const GemmPlan p = gemm_bf16_plan(m, R, 2 * F, d, 2);
      ProfScope psc(m, "gemm_gate_up");
      launch_gemm_bf16(m, (const f16_t*)m->Xn, (const f16_t*)L.wgu, nullptr, R, 2 * F, d, p, 2, nullptr, (f16_t*)m->Fb);
    } else {
      project("gemm_gate_up", m->Xn, L.wgu, 2 * F, d, &np, &ps);
      launch_swiglu(m, R, np, ps);
    }
    project("gemm_down", m->Fb, L.wd, d, F, &pending_parts, &pending_stride);
  }
  if (ingest_only) {
    TS_HIP(hipGetLastError());
    TS_HIP(hipStreamSynchronize(m->stream));
    m->last_rows = 0;
    return TS_OK;
  }
  launch_norm(m, R, m->norm_f, pending_parts, pending_stride, false);
  if (bf) {
    // one row block: the plan made at load (it sized the partial buffers); batches: the many-row kernel,
    // whose 512-column groups need fewer partials
    const GemmPlan p = gemm_bf16_plan(m, std::max(R, TS_MROWS_PER_BLOCK), c.vocab, d, 1);
    ProfScope ps(m, "gemm_lm_head_argmax");
    launch_gemm_bf16(m, (const f16_t*)m->Xn, (const f16_t*)m->lm_head, nullptr, R, c.vocab, d, p, 1,
                     (m->keep_logits || sample) ? m->logits : nullptr, nullptr);
  } else {
    launch_gemm_f32(m, (const float*)m->Xn, (const float*)m->lm_head, m->logits, R, c.vocab, d);
    launch_argmax_rows(m, R);
  }
  if (sample) launch_sample(m, dm, R, n_seqs, sample->temperature, sample->seed);
  else launch_walk(m, dm, R, n_seqs);
  if (time_pass && pass_rec >= 1) TS_HIP(hipEventRecord(m->prof[pass_rec - 1].b, m->stream));
  TS_HIP(hipGetLastError());
  for (int s = 0; s < n_seqs; ++s)
    TS_HIP(hipMemcpyAsync(m->res_host + (size_t)s * TS_RESULT_INTS, kvs[s]->result, TS_RESULT_INTS * 4, hipMemcpyDeviceToHost, m->stream));
  TS_HIP(hipStreamSynchronize(m->stream));
  m->last_rows = R;

  // ---- hand the result back -----------------------------------------------------------
  for (int s = 0; s < n_seqs; ++s) {
    ts_kv* kv = kvs[s];
    const int32_t* res = m->res_host + (size_t)s * TS_RESULT_INTS;
    const int len = res[0];
    const int n = offs[s + 1] - offs[s];
    if (len < 0 || len > n) return ts_fail(TS_ERR_DEVICE, "device returned accept_len %d for %d nodes", len, n);
    accept_len[s] = len;
    bonus[s] = res[1];
    for (int i = 0; i < len; ++i) {
      const int row = res[4 + i];
      acc_tokens[offs[s] + i] = res[4 + TS_MAX_NODES + i];
      if (acc_nodes) acc_nodes[offs[s] + i] = row - 1;
      kv->res_rows[i] = row;
    }
    kv->res_accept_len = len;
    kv->res_bonus = res[1];
    kv->last_M = n + 1;
    kv->have_result = true;
  }
  return TS_OK;
}

extern "C" ts_status ts_verify(ts_model* m, ts_kv* kv, const int32_t* draft_tokens, const int32_t* parent_idx,
                               int32_t n_nodes, int32_t* accept_len, int32_t* accepted_tokens, int32_t* accepted_nodes,
                               int32_t* bonus_token) {
  if (!m || !kv || !accept_len || !bonus_token || (n_nodes > 0 && !accepted_tokens))
    return ts_fail(TS_ERR_INVALID_ARG, "ts_verify: null argument");
  if (n_nodes < 0 || n_nodes > TS_MAX_NODES) return ts_fail(TS_ERR_INVALID_TREE, "n_nodes %d outside [0,%d]", n_nodes, TS_MAX_NODES);
  const int32_t offs[2] = {0, n_nodes};
  ts_kv* kvs[1] = {kv};
  return verify_impl(m, kvs, 1, draft_tokens, parent_idx, offs, accept_len, accepted_tokens, accepted_nodes, bonus_token);
}

extern "C" ts_status ts_verify_sample(ts_model* m, ts_kv* kv, const int32_t* draft_tokens, const int32_t* parent_idx,
                                      int32_t n_nodes, float temperature, const float* node_uniform, uint64_t noise_seed,
                                      int32_t* accept_len, int32_t* accepted_tokens, int32_t* accepted_nodes,
                                      int32_t* bonus_token) {
  if (!m || !kv || !accept_len || !bonus_token || (n_nodes > 0 && (!accepted_tokens || !node_uniform)))
    return ts_fail(TS_ERR_INVALID_ARG, "ts_verify_sample: null argument");
  if (n_nodes < 0 || n_nodes > TS_MAX_NODES) return ts_fail(TS_ERR_INVALID_TREE, "n_nodes %d outside [0,%d]", n_nodes, TS_MAX_NODES);
  if (!(temperature > 0.f) || !(temperature < 1e6f)) return ts_fail(TS_ERR_INVALID_ARG, "temperature %g must be positive and finite", temperature);
  for (int i = 0; i < n_nodes; ++i)
    if (!(node_uniform[i] >= 0.f && node_uniform[i] < 1.f))
      return ts_fail(TS_ERR_INVALID_ARG, "node_uniform[%d] = %g outside [0,1)", i, node_uniform[i]);
  const int32_t offs[2] = {0, n_nodes};
  ts_kv* kvs[1] = {kv};
  const SampleArgs sa{temperature, node_uniform, noise_seed};
  return verify_impl(m, kvs, 1, draft_tokens, parent_idx, offs, accept_len, accepted_tokens, accepted_nodes, bonus_token, false, &sa);
}

extern "C" ts_status ts_verify_batch(ts_model* m, ts_kv* const* kvs, int32_t n_seqs, const int32_t* draft_tokens,
                                     const int32_t* parent_idx, const int32_t* node_offsets, int32_t* accept_len,
                                     int32_t* accepted_tokens, int32_t* accepted_nodes, int32_t* bonus_token) {
  if (!m || !kvs || !node_offsets || !accept_len || !bonus_token) return ts_fail(TS_ERR_INVALID_ARG, "ts_verify_batch: null argument");
  if (n_seqs < 1 || n_seqs > 4096) return ts_fail(TS_ERR_INVALID_ARG, "n_seqs %d outside [1,4096]", n_seqs);
  if (node_offsets[0] != 0) return ts_fail(TS_ERR_INVALID_ARG, "node_offsets[0] must be 0");
  for (int s = 0; s < n_seqs; ++s)
    if (node_offsets[s + 1] < node_offsets[s]) return ts_fail(TS_ERR_INVALID_ARG, "node_offsets must be non-decreasing");
  if (node_offsets[n_seqs] > 0 && !accepted_tokens) return ts_fail(TS_ERR_INVALID_ARG, "null accepted_tokens");
  return verify_impl(m, kvs, n_seqs, draft_tokens, parent_idx, node_offsets, accept_len, accepted_tokens, accepted_nodes, bonus_token);
}

// ---------------------------------------------------------------------------------
// final hidden state of a row of the most recent verify (query representation for retrieval)
// ---------------------------------------------------------------------------------
extern "C" ts_status ts_get_hidden(ts_model* m, int32_t row, float* host_hidden) {
  if (!m || !host_hidden) return ts_fail(TS_ERR_INVALID_ARG, "ts_get_hidden: null argument");
  if (row < 0 || row >= m->last_rows) return ts_fail(TS_ERR_STATE, "row %d outside the %d rows of the last verify", row, m->last_rows);
  (void)hipSetDevice(m->device);
  const int d = m->cfg.d_model;
  if (m->cfg.dtype == TS_DTYPE_F32) {
    TS_HIP(copy_sync(m->stream, host_hidden, (const float*)m->Xn + (size_t)row * d, (size_t)d * 4, hipMemcpyDeviceToHost));
    return TS_OK;
  }
  // bf16 models keep the normalised activations as a hi and a lo IEEE half: widened and added
  std::vector<uint16_t> hx(d), lx(d);
  const size_t plane = (size_t)(m->ws_rows + TS_MROWS_PER_BLOCK) * d;
  TS_HIP(copy_sync(m->stream, hx.data(), (const f16_t*)m->Xn + (size_t)row * d, (size_t)d * 2, hipMemcpyDeviceToHost));
  TS_HIP(copy_sync(m->stream, lx.data(), (const f16_t*)m->Xn + plane + (size_t)row * d, (size_t)d * 2, hipMemcpyDeviceToHost));
  for (int i = 0; i < d; ++i) host_hidden[i] = half_bits_to_float(hx[i]) + half_bits_to_float(lx[i]);
  return TS_OK;
}

// ---------------------------------------------------------------------------------
// context ingestion through the same kernels: causal chains of up to 65 rows, every row kept
// ---------------------------------------------------------------------------------
extern "C" ts_status ts_prefill(ts_model* m, ts_kv* kv, const int32_t* tokens, int32_t n_tokens) {
  if (!m || !kv || (n_tokens > 0 && !tokens)) return ts_fail(TS_ERR_INVALID_ARG, "ts_prefill: null argument");
  if (kv->model != m) return ts_fail(TS_ERR_INVALID_ARG, "cache belongs to another model");
  if (n_tokens < 0) return ts_fail(TS_ERR_INVALID_ARG, "n_tokens %d is negative", n_tokens);
  if (n_tokens == 0) return TS_OK;
  for (int i = 0; i < n_tokens; ++i)
    if (tokens[i] < 0 || tokens[i] >= m->cfg.vocab)
      return ts_fail(TS_ERR_TOKEN_RANGE, "context token %d outside [0,%d) (index %d)", tokens[i], m->cfg.vocab, i);
  // sequence to ingest: the pending token (if any), then tokens; the last one stays pending
  std::vector<int32_t> seq;
  seq.reserve((size_t)n_tokens + 1);
  if (kv->pending >= 0) seq.push_back(kv->pending);
  seq.insert(seq.end(), tokens, tokens + n_tokens);
  const int rows_total = (int)seq.size() - 1;
  if (kv->P + rows_total + 1 > kv->capacity)
    return ts_fail(TS_ERR_KV_CAPACITY, "committed %d + context %d + 1 exceed the capacity %d", kv->P, rows_total, kv->capacity);
  // A pass ingests up to kPrefillBlocks consecutive row blocks of kPrefillRows rows.  Each block
  // is a causal chain (root + 63 nodes: a chain's ancestor set is the causal mask) whose context
  // is everything before it - the committed positions and the blocks in front of it in the same
  // pass, whose K/V the pass writes before any attention launch of the layer reads them.
  constexpr int kPrefillRows = 64, kPrefillBlocks = 32;
  std::vector<int32_t> chain_par((size_t)kPrefillBlocks * (kPrefillRows - 1));
  for (int b = 0; b < kPrefillBlocks; ++b)
    for (int i = 0; i < kPrefillRows - 1; ++i) chain_par[(size_t)b * (kPrefillRows - 1) + i] = i - 1;
  const int saved_P = kv->P, saved_pending = kv->pending;
  int done = 0;
  while (done < rows_total) {
    const int rows = std::min(rows_total - done, kPrefillRows * kPrefillBlocks);
    const int n_blocks = (rows + kPrefillRows - 1) / kPrefillRows;
    std::vector<int32_t> offs(n_blocks + 1, 0), blk_P(n_blocks), blk_root(n_blocks), nodes;
    std::vector<ts_kv*> kvs(n_blocks, kv);
    nodes.reserve(rows);
    for (int b = 0; b < n_blocks; ++b) {
      const int r0 = b * kPrefillRows, rb = std::min(rows - r0, kPrefillRows);
      blk_P[b] = kv->P + r0;
      blk_root[b] = seq[done + r0];
      // only the last block can be short, so block b's nodes start at b * (kPrefillRows - 1),
      // where chain_par restarts as well
      nodes.insert(nodes.end(), seq.begin() + done + r0 + 1, seq.begin() + done + r0 + rb);
      offs[b + 1] = offs[b] + rb - 1;
    }
    std::vector<int32_t> dummy_len(n_blocks), dummy_bonus(n_blocks);
    const BlockOverride bo{blk_P.data(), blk_root.data()};
    ts_status st = verify_impl(m, kvs.data(), n_blocks, nodes.data(), chain_par.data(), offs.data(), dummy_len.data(), nullptr,
                               nullptr, dummy_bonus.data(), true, nullptr, &bo);
    if (st) { kv->P = saved_P; kv->pending = saved_pending; kv->have_result = false; return st; }
    kv->P += rows;                                   // the rows already sit in slots P .. P+rows-1
    done += rows;
  }
  kv->pending = seq.back();
  kv->have_result = false;
  return TS_OK;
}

// ---------------------------------------------------------------------------------
// commit
// ---------------------------------------------------------------------------------
extern "C" ts_status ts_kv_commit(ts_kv* kv) {
  if (!kv) return ts_fail(TS_ERR_INVALID_ARG, "null cache");
  if (!kv->have_result) return ts_fail(TS_ERR_STATE, "no unapplied verify result on this cache");
  ts_model* m = kv->model;
  (void)hipSetDevice(m->device);
  const int len = kv->res_accept_len;
  bool moves = false;
  for (int i = 0; i < len; ++i) moves |= (kv->res_rows[i] != i + 1);
  if (moves) {
    launch_commit(kv, len);
    TS_HIP(hipGetLastError());
    TS_HIP(hipStreamSynchronize(m->stream));
  }
  kv->P += len + 1;
  kv->pending = kv->res_bonus;
  kv->have_result = false;
  return TS_OK;
}

// ---------------------------------------------------------------------------------
// profiling
// ---------------------------------------------------------------------------------
extern "C" ts_status ts_profile_enable(ts_model* m, int32_t enable) {
  if (!m) return ts_fail(TS_ERR_INVALID_ARG, "null model");
  m->prof_on = enable != 0;
  m->prof.clear();
  m->ev_used = 0;
  return TS_OK;
}

extern "C" ts_status ts_profile_filter(ts_model* m, const char* kind) {
  if (!m) return ts_fail(TS_ERR_INVALID_ARG, "null model");
  m->prof_filter = kind ? kind : "";
  return TS_OK;
}

extern "C" ts_status ts_profile_plain_read(ts_model* m, int32_t launches, uint64_t* bytes_per_launch) {
  if (!m || launches < 0) return ts_fail(TS_ERR_INVALID_ARG, "null model or negative launch count");
  if (m->layers.empty()) return ts_fail(TS_ERR_STATE, "model has no layers");
  // the kernel's never-taken store needs a valid sink word: bf16 models own one (range_flag)
  if (m->cfg.dtype != TS_DTYPE_BF16 || !m->range_flag)
    return ts_fail(TS_ERR_INVALID_ARG, "ts_profile_plain_read: bf16 models only");
  (void)hipSetDevice(m->device);
  const size_t bytes = (size_t)2 * m->cfg.d_ffn * m->cfg.d_model * 2;
  for (int i = 0; i < launches; ++i)
    launch_plain_read(m, m->layers[i % m->layers.size()].wgu, bytes, (uint32_t*)m->range_flag);
  TS_HIP(hipGetLastError());
  TS_HIP(hipStreamSynchronize(m->stream));
  if (bytes_per_launch) *bytes_per_launch = bytes;
  return TS_OK;
}

extern "C" ts_status ts_profile_read(ts_model* m, ts_profile_entry* entries, int32_t max_entries, int32_t* n_entries) {
  if (!m || !n_entries || (max_entries > 0 && !entries)) return ts_fail(TS_ERR_INVALID_ARG, "null argument");
  (void)hipSetDevice(m->device);
  TS_HIP(hipStreamSynchronize(m->stream));
  std::vector<ts_profile_entry> agg;
  for (const ProfRec& r : m->prof) {
    float ms = 0.f;
    TS_HIP(hipEventElapsedTime(&ms, r.a, r.b));
    size_t i = 0;
    for (; i < agg.size(); ++i)
      if (agg[i].name == r.name || strcmp(agg[i].name, r.name) == 0) break;
    if (i == agg.size()) agg.push_back(ts_profile_entry{r.name, 0, 0.f});
    agg[i].launches += 1;
    agg[i].total_ms += ms;
  }
  *n_entries = (int32_t)agg.size();
  for (int i = 0; i < (int)agg.size() && i < max_entries; ++i) entries[i] = agg[i];
  return TS_OK;
}
