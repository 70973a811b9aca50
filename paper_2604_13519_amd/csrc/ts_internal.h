// Internal declarations shared by the translation units of libtoolspec_hip.so.
// Nothing here is part of the public ABI (see include/toolspec.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "../../include/toolspec.h"

typedef uint16_t bf16_t;   // bfloat16 bit pattern in memory
typedef uint16_t f16_t;    // IEEE half bit pattern in memory

// ---- error plumbing -----------------------------------------------------------
ts_status ts_fail(ts_status code, const char* fmt, ...);
#define TS_HIP(call)                                                                    \
  do {                                                                                  \
    hipError_t e_ = (call);                                                             \
    if (e_ != hipSuccess)                                                               \
      return ts_fail(e_ == hipErrorOutOfMemory ? TS_ERR_OOM : TS_ERR_DEVICE,            \
                     "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
  } while (0)

// ---- geometry constants ---------------------------------------------------------
constexpr int TS_MROWS_PER_BLOCK = 80;  // rows one GEMM pass covers (5 MFMA tiles of 16)
constexpr int TS_GEMM_KC = 128;         // k elements per staged chunk
constexpr int TS_ATTN_KB = 64;          // keys per attention block (4 pages)

// Per-row metadata of one verify pass, structure of arrays in one device buffer.
struct RowMeta {
  int32_t* tok;      // token id
  int32_t* pos;      // absolute position = committed length + depth
  int32_t* seq;      // sequence index within the batch
  int32_t* lrow;     // row index within its sequence (0 = root)
  int32_t* par;      // parent row within its sequence (-1 for the root)
  int32_t* depth;    // depth within its sequence (root 0)
  uint64_t* anc;     // bit i set iff draft node i is this row or one of its ancestors
  float* u;          // stochastic acceptance: the caller's uniform of this row's draft node
};

// Per-sequence descriptor, device-visible.
struct SeqDesc {
  int32_t P;             // committed length
  int32_t M;             // rows of this sequence (n_nodes + 1)
  int32_t row0;          // first row in the concatenated batch
  int32_t n_pages;       // physical pages of the pool the cache's pages live in (the layer stride)
  const int32_t* page_table;   // device, logical page -> physical page
  void* k_pool;          // device, K pages  [L][n_pages][Hkv][16][hd]
  void* v_pool;          // device, V pages  [L][n_pages][Hkv][hd][16]  (transposed in-page)
  int32_t* result;       // device, [0]=accept_len [1]=bonus [2]=best_row, [4..4+64) rows, [68..132) tokens
};
constexpr int TS_RESULT_INTS = 4 + 2 * TS_MAX_NODES;

// Where a row's new K and V go (layer 0, KV head 0): written once per pass, read by every layer's QKV epilogue.
struct RowDst {
  void* k;                 // K page row of the slot: + layer * layer_stride + g * 16 * hd + dim
  void* v;                 // V page column of the slot: + layer * layer_stride + g * hd * 16 + dim * 16
  size_t layer_stride;     // elements per layer of the sequence's pools
};

struct ProfRec { const char* name; hipEvent_t a, b; };

// Physical pages shared by several caches (ts_kv_pool_create)
struct ts_kv_pool {
  ts_model* model;
  int32_t n_pages;
  void* k_pool; void* v_pool;      // device, [L][n_pages][Hkv][16][hd] / [L][n_pages][Hkv][hd][16]
  std::vector<int32_t> free_pages; // stack of free physical pages
  int32_t live;                    // caches drawn from the pool and not yet freed
};

struct ts_kv {
  ts_model* model;
  ts_kv_pool* pool;        // nullptr: the cache owns its pages
  int32_t capacity, page_size, n_pages;
  int32_t pool_pages;      // physical pages of the allocation the pages live in (= n_pages for an own allocation): the layer stride
  int32_t P;               // committed length
  int32_t pending;         // -1 = none
  bool have_result;        // an unapplied verify result exists
  int32_t res_accept_len, res_bonus;
  int32_t res_rows[TS_MAX_NODES];
  int32_t last_M;
  void* k_pool; void* v_pool;      // device
  size_t layer_stride_elems;       // elements per layer in each pool
  int32_t* page_table;             // device
  std::vector<int32_t> page_table_host;
  int32_t* result;                 // device, TS_RESULT_INTS
};

struct LayerW {
  void* wqkv; void* wo; void* wgu; void* wd;   // device; bf16 models: MFMA-tiled IEEE half, f32: row-major [N][K]
  float* norm1; float* norm2;                  // device fp32
};

struct ts_model {
  ts_model_config cfg;
  int device;
  hipStream_t stream;
  int esz;                      // bytes per stored element
  int q_dim, kv_dim, qkv_dim;
  void* embed;                  // device [V][d] in storage dtype, row-major
  void* lm_head;                // device, tiled (bf16) or row-major (f32)
  float* norm_f;
  int* range_flag;              // device; set by the weight re-tiling when a weight does not fit IEEE half
  unsigned long long* sat_count;   // device; projection inputs clamped to half's range since load (bf16 models)
  std::vector<LayerW> layers;
  // workspace, sized for ws_rows rows (multiple of TS_MROWS_PER_BLOCK)
  int ws_rows, ws_seqs;
  float* H;                     // residual stream [rows][d] fp32
  void* Xn;                     // normalised activations [rows][d]; float, or IEEE half for bf16 models
  void* Qb;                     // rotated queries [rows][q_dim]; float, or IEEE half for bf16 models
  void* Ab;                     // attention output [rows][q_dim]; float, or IEEE half for bf16 models
  void* Fb;                     // SwiGLU product [rows][F]; float, or IEEE half for bf16 models
  float* part;                  // split-K partial sums, [S][rows][N] fp32
  size_t part_elems;
  uint16_t* attn_part_o;        // [rows][Hq][splits][hd], IEEE half (each split's normalised output)
  float* attn_part_ml;          // [rows][Hq][splits][2]
  int attn_max_splits;
  float2* rope_cs;              // [rows][hd/2] (cos, sin)
  RowDst* row_dst;              // [rows]
  float* amax_val; int32_t* amax_idx; int amax_parts;   // [rows][parts]
  int amax_used;                // partials per row the last lm_head launch wrote (<= amax_parts)
  float* logits; bool keep_logits; int logits_rows;     // [rows][V] when kept
  float* samp_lse; int32_t* samp_tok;                   // per-row token (greedy arg-max or residual sample); log-sum-exp for sampling
  // per-call metadata (device + pinned host mirror)
  void* meta_dev; void* meta_host; size_t meta_bytes;
  SeqDesc* seq_dev;
  int32_t* res_host;            // pinned, ws_seqs * TS_RESULT_INTS
  // profiling
  bool prof_on;
  std::string prof_filter;      // empty = bracket every kernel kind
  std::vector<ProfRec> prof;
  std::vector<hipEvent_t> ev_pool; size_t ev_used;
  int last_rows;
  int n_cu;
};

// ---- launchers (each defined next to its kernel) ----------------------------------
// misc kernels (ts_kernels_misc.hip)
void launch_repack_tiles(hipStream_t s, const bf16_t* src, f16_t* dst, int N, int K, int n_tile0, int n_tile_stride,
                         int* range_flag);
void launch_embed(ts_model* m, const RowMeta& rm, int R);
void launch_norm(ts_model* m, int R, const float* gain, int n_parts, size_t part_stride, bool first);
void launch_rope_kv(ts_model* m, const RowMeta& rm, int R, int layer, int n_parts, size_t part_stride);
void launch_swiglu(ts_model* m, int R, int n_parts, size_t part_stride);
void launch_plain_read(ts_model* m, const void* src, size_t bytes, uint32_t* sink);
void launch_argmax_rows(ts_model* m, int R);
void launch_walk(ts_model* m, const RowMeta& rm, int R, int n_seqs);
void launch_sample(ts_model* m, const RowMeta& rm, int R, int n_seqs, float temperature, uint64_t seed);
void launch_commit(ts_kv* kv, int accept_len);
void launch_kv_import(ts_kv* kv, int pos0, int n_pos, const void* staged_k, const void* staged_v, int layer);
void launch_kv_export(ts_kv* kv, int pos0, int n_pos, void* staged_k, void* staged_v, int layer);
// fp32 compute path
void launch_gemm_f32(ts_model* m, const float* X, const float* W, float* out, int M, int N, int K);
void launch_attn_f32(ts_model* m, const RowMeta& rm, int R, int n_seqs, int layer, int max_keys);
size_t attn_f32_max_keys();
// bf16 compute path (ts_gemm_bf16.hip / ts_attn_bf16.hip)
struct GemmPlan { int shape; int splits; };   // compiled tile shape id, K splits
// mode: 0 = fp32 partial sums [split][R][N], 1 = fused arg-max (lm_head), 2 = SwiGLU epilogue (gate/up)
GemmPlan gemm_bf16_plan(const ts_model* m, int R, int N, int K, int mode);
int gemm_bf16_cols_per_group(int shape);
int gemm_bf16_chunk(int shape);
void launch_gemm_bf16(ts_model* m, const f16_t* X, const f16_t* Wt, float* out, int R, int N, int K,
                      GemmPlan plan, int mode, float* logits, f16_t* act_out);
// many-row projection (ts_gemm_rows_bf16.hip), reached through gemm_bf16_plan / launch_gemm_bf16 when R > 80
bool gemm_rows_plan(const ts_model* m, int R, int N, int K, int mode, size_t max_part_elems, int* mt, int* cfg, int* splits);
int gemm_rows_chunk(int cfg);
void launch_gemm_rows_bf16(ts_model* m, const f16_t* X, const f16_t* Wt, float* out, int R, int N, int K, int mt, int cfg,
                           int splits, int mode, f16_t* act_out, float* logits);
int attn_bf16_splits(const ts_model* m, int max_keys, int n_seqs, long sum_keys);
void launch_attn_bf16(ts_model* m, const RowMeta& rm, int R, int n_seqs, int layer, int splits, int max_M);
void launch_attn_merge(ts_model* m, int R, int splits);

// profiling bracket
void prof_begin(ts_model* m, const char* name);
void prof_end(ts_model* m);
struct ProfScope {
  ts_model* m;
  bool on;
  ProfScope(ts_model* mm, const char* name) : m(mm) {
    on = m->prof_on && (m->prof_filter.empty() || m->prof_filter == name);
    if (on) prof_begin(m, name);
  }
  ~ProfScope() { if (on) prof_end(m); }
};
