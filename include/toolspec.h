/*
 * toolspec.h - C ABI of the MI355X (gfx950) draft-tree verification library.
 *
 * The library implements the hot step of schema-aware, retrieval-augmented
 * speculative decoding for tool calling: candidate drafts (schema-filled
 * tokens, enumerated alternatives such as tool names, continuations reused from
 * retrieved past invocations) are packed into one flattened sequence with a
 * tree-structured attention mask, the target decoder scores all of them in ONE
 * forward pass over its KV cache, and the longest accepted path is selected
 * and appended (paper Sec. 4.1 "Task Formulation"; App. A.1 "Parallel
 * Verification"; Alg. 1, steps PackDraftsAsTree / Verification /
 * SelectLongestAcceptedPrefix / append).  Drafting itself (FSM, retrieval) is
 * not part of this header: toolspec_draft.h declares host-side drafting calls
 * and the whole loop, built on the functions below.
 *
 * Conventions
 *  - All pointers are HOST pointers unless a parameter says "device".
 *  - Every function returns a ts_status (0 = TS_OK, negative = error) and never
 *    throws; ts_last_error() gives a message for the calling thread's last error.
 *  - Errors leave committed state (cache length, pending token) untouched.
 *  - Handles are not thread-safe.  One HIP stream per model; every call that
 *    returns data to the host has synchronised that stream before returning.
 *  - Matrices handed to ts_model_load are row-major [out][in] (y = x W^T),
 *    element type float (dtype 0) or bfloat16 bit patterns (dtype 1).  The
 *    library copies and re-tiles them on the device; the caller may free its
 *    buffers as soon as ts_model_load returns.
 *
 * Tree conventions (paper App. A.1: all drafts of a step form one sequence that is
 * verified under a tree mask; dynamic trees adapt to each draft's length, so any
 * shape is legal):
 *  - The root of the tree is the PENDING token: the last emitted token, whose
 *    K/V are not in the cache yet.  It is not one of the n_nodes draft nodes.
 *  - parent_idx[i] is -1 (child of the root) or an index in [0, i): parents
 *    precede children.  0 <= n_nodes <= TS_MAX_NODES.  Duplicate sibling
 *    tokens are legal.
 *  - A node sits at position (committed length + depth); it attends to the
 *    whole committed context, to the root, to its ancestors and to itself.
 *  - Acceptance is greedy: a node is accepted iff its parent is accepted (the
 *    root always is) and its token equals the arg-max token of the logits at
 *    its parent.  The deepest accepted node wins; ties go to the lowest node
 *    index, equal logits to the lowest token id.  n_nodes = 0 is plain
 *    autoregressive decoding.
 */
#ifndef TOOLSPEC_H
#define TOOLSPEC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ts_model ts_model; /* opaque; owns device weights, workspace, stream */
typedef struct ts_kv    ts_kv;    /* opaque; owns one sequence's paged K/V          */
typedef struct ts_kv_pool ts_kv_pool; /* opaque; physical K/V pages shared by several caches */
typedef int32_t ts_status;

enum {
  TS_OK = 0,
  TS_ERR_INVALID_ARG  = -1, /* null pointer, bad size, unsupported shape          */
  TS_ERR_INVALID_TREE = -2, /* parent_idx[i] outside [-1, i), n_nodes out of range */
  TS_ERR_TOKEN_RANGE  = -3, /* token id outside [0, vocab)                         */
  TS_ERR_KV_CAPACITY  = -4, /* committed length + tree rows exceed the capacity    */
  TS_ERR_STATE        = -5, /* no pending token; commit without a fresh verify     */
  TS_ERR_OOM          = -6, /* device or host allocation failed                    */
  TS_ERR_DEVICE       = -7  /* a HIP call failed                                   */
};

enum { TS_DTYPE_F32 = 0, TS_DTYPE_BF16 = 1 };
enum { TS_MAX_NODES = 64, TS_PAGE_SIZE = 16 };

/* Decoder shape: pre-norm blocks with RMSNorm, rotary embedding (pair (j, j+hd/2)
 * rotated by pos * rope_theta^(-2j/hd)), grouped-query attention with softmax scale
 * 1/sqrt(head_dim), SwiGLU feed-forward, no biases, untied embedding / lm_head.
 * dtype is the storage type of weights and KV cache.  TS_DTYPE_BF16 computes every
 * matrix product in IEEE half with fp32 accumulation (MFMA): the bf16 weights are
 * re-encoded as half once at load - exact wherever half is normal (it has more
 * significand bits); magnitudes below 2^-14 land on half's subnormal grid (absolute error
 * below 3e-8), and a finite weight beyond half's range (|w| > 65504) makes ts_model_load
 * fail with INVALID_ARG.  An activation that enters a projection is carried as the sum of
 * two halves, hi = half(x) (saturating at 65504) and lo = half(x - hi), about 22
 * significant bits; the rotated Q and the soft-max probabilities are single halves; bf16
 * K/V entries widen to half exactly (same subnormal caveat); soft-max is fp32, and the
 * residual stream and the logits stay fp32.  It needs d_model, n_q_heads*head_dim and d_ffn to be multiples of
 * 128 and head_dim 64 or 128.  TS_DTYPE_F32 computes in fp32. */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_theta, rms_eps;
  int32_t dtype;
} ts_model_config;

/* Host weight pointers.  The per-layer members are arrays of n_layers pointers. */
typedef struct {
  const void* embed;        /* [vocab][d_model]                */
  const void* lm_head;      /* [vocab][d_model]                */
  const void* norm_f;       /* [d_model]                       */
  const void* const* wq;    /* [n_q_heads*head_dim][d_model]   */
  const void* const* wk;    /* [n_kv_heads*head_dim][d_model]  */
  const void* const* wv;    /* [n_kv_heads*head_dim][d_model]  */
  const void* const* wo;    /* [d_model][n_q_heads*head_dim]   */
  const void* const* wg;    /* [d_ffn][d_model]  gate          */
  const void* const* wu;    /* [d_ffn][d_model]  up            */
  const void* const* wd;    /* [d_model][d_ffn]  down          */
  const void* const* norm1; /* [d_model]  pre-attention gain   */
  const void* const* norm2; /* [d_model]  pre-FFN gain         */
} ts_weights;

/* Thread-local description of the last error returned to this thread ("" if none). */
const char* ts_last_error(void);

/* ---- model ------------------------------------------------------------------
 * The target model M of Alg. 1.  Copies all weights to the current HIP device.
 * Errors: INVALID_ARG (null, unsupported shape), OOM, DEVICE. */
ts_status ts_model_load(const ts_model_config* cfg, const ts_weights* host_weights, ts_model** out);
ts_status ts_model_free(ts_model* m);

/* When enabled, ts_verify also stores the full fp32 logits of every row so that
 * ts_get_logits can return them (parity checks); off by default because the
 * arg-max is fused into the lm_head projection and needs no logits in memory. */
ts_status ts_model_keep_logits(ts_model* m, int32_t enable);
/* Logits of rows [row0, row0+n_rows) of the most recent verify on this model
 * (row 0 = root, row i+1 = draft node i; batched calls concatenate sequences).
 * host_logits: n_rows * vocab floats.  STATE if logits were not kept. */
ts_status ts_get_logits(ts_model* m, int32_t row0, int32_t n_rows, float* host_logits);

/* Number of projection inputs (normalised activations, attention outputs, SwiGLU products) whose
 * magnitude exceeded the largest finite half (65504) and were clamped, summed over every pass
 * since ts_model_load.  Non-zero means the model's activations left the range the bf16 path
 * computes in and its results from that pass on are not those of the model; 0 for fp32 models. */
ts_status ts_model_saturations(ts_model* m, uint64_t* count);

/* The token each row of the most recent verify decided on, n_rows int32: after ts_verify /
 * ts_verify_batch the arg-max token of the row's logits as the fused lm_head epilogue found it
 * (lowest id among equal logits) - what the acceptance walk compared the row's children with;
 * after ts_verify_sample the row's residual sample.  Works whether or not logits are kept.
 * STATE before the first verify, INVALID_ARG for rows outside the last pass. */
ts_status ts_get_row_tokens(ts_model* m, int32_t row0, int32_t n_rows, int32_t* host_tokens);

/* Final normalised hidden state (the input of the lm_head) of one row of the most recent
 * verify, d_model floats: for row 0 after ingesting a question this is the last-token
 * representation h_x that retrieval compares with the datastore (Sec. 4.3, Eq. 3).  bf16
 * models hold it in IEEE half (the lm_head's input); it is widened exactly.  STATE if
 * the row is outside the last verify. */
ts_status ts_get_hidden(ts_model* m, int32_t row, float* host_hidden);

/* ---- KV cache ---------------------------------------------------------------
 * One sequence's cache (the K/V of context x and generated output y): pages of
 * page_size (= 16) positions, addressed through a page table.  capacity_tokens
 * must cover the context plus the rows of the largest tree (n_nodes + 1).
 * Starts empty: length 0, no pending token. */
ts_status ts_kv_alloc(ts_model* m, int32_t capacity_tokens, int32_t page_size, ts_kv** out);
/* A cache refers to its model (stream, device): free every cache BEFORE ts_model_free of the
 * model it was allocated on; freeing the model first leaves the cache handle dangling. */
ts_status ts_kv_free(ts_kv* kv);
/* Replace the identity page table by a permutation of [0, n_pages) (n_pages =
 * ceil(capacity/page_size)); only legal while the cache is empty. */
ts_status ts_kv_set_page_table(ts_kv* kv, const int32_t* phys_page, int32_t n_pages);

/* A pool of physical K/V pages (page = 16 positions of every layer and KV head) that several
 * caches of one model draw from, so that requests of different lengths share one allocation
 * (the batched workloads: ragged contexts).  ts_kv_alloc_pooled takes ceil(capacity_tokens / 16)
 * free pages - whichever are free, in no particular order: a cache's pages are scattered over
 * the pool - and ts_kv_free gives them back; the page contents are not cleared (positions beyond
 * a cache's length are never read as data).  Results do not depend on where the pages lie: a
 * pooled cache gives bit for bit what a cache of its own allocation gives.
 * Errors: INVALID_ARG; OOM (device allocation, or fewer free pages than the capacity needs - the
 * pool is then unchanged); STATE (ts_kv_pool_free while caches drawn from the pool are alive;
 * ts_kv_set_page_table on a pooled cache).  Free the pool BEFORE ts_model_free. */
ts_status ts_kv_pool_create(ts_model* m, int32_t n_pages, ts_kv_pool** out);
ts_status ts_kv_pool_free(ts_kv_pool* pool);
ts_status ts_kv_pool_pages_free(const ts_kv_pool* pool, int32_t* n_free_pages);
ts_status ts_kv_alloc_pooled(ts_kv_pool* pool, int32_t capacity_tokens, ts_kv** out);
/* Test/bench helpers: synthetic K/V for contexts whose real prefill the CPU oracle cannot afford.
 * k_host / v_host: [n_layers][n_pos][n_kv_heads][head_dim] in the model dtype,
 * K already rotated.  Import sets the committed length to n_pos. */
ts_status ts_kv_import(ts_kv* kv, int32_t n_pos, const void* k_host, const void* v_host);
ts_status ts_kv_export(ts_kv* kv, int32_t pos0, int32_t n_pos, void* k_host, void* v_host);
/* ts_kv_export for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments, same result, but the
 * per-layer staging slabs that ts_kv_export allocates and frees on every call live in a 2 MiB
 * device array that is part of the library image (every GPU the library runs on holds it until
 * the process ends), so the call allocates and frees nothing.  One layer's K slab and V slab
 * must each fit 1 MiB: n_pos * n_kv_heads * head_dim * element size <= 1048576 (512 positions of
 * the 8B shape); larger requests fail with INVALID_ARG and copy nothing - export in pieces.  All
 * calls on one GPU share the array, so calls that overlap in time on one GPU (two host threads,
 * two models on the same device) race; calls in sequence do not. */
ts_status ts_kv_export_noalloc(ts_kv* kv, int32_t pos0, int32_t n_pos, void* k_host, void* v_host);
ts_status ts_set_pending(ts_kv* kv, int32_t token);   /* root token of the next verify */
ts_status ts_kv_len(const ts_kv* kv, int32_t* committed_len);
/* Roll the committed length back to new_len <= current length (drops later
 * positions, invalidates the last verify result); the caller sets the pending token. */
ts_status ts_kv_truncate(ts_kv* kv, int32_t new_len);

/* Context ingestion (the context x of Alg. 1: prompts and tool documentation, Sec. 4.1) through
 * the verification kernels themselves: the sequence [pending token, if any] + tokens is run in
 * passes of up to 2048 rows, each pass as up to 32 consecutive causal chains of 64 rows (a chain's ancestor
 * set is the causal mask; the chains in front of it are part of its context), every row is kept
 * (the K/V of all but the last token are appended to the cache), the last token becomes the
 * pending token.  No logits are produced; the next ts_verify scores the pending token.  Errors (state unchanged): INVALID_ARG, TOKEN_RANGE,
 * KV_CAPACITY (committed + appended + 1 > capacity), DEVICE. */
ts_status ts_prefill(ts_model* m, ts_kv* kv, const int32_t* tokens, int32_t n_tokens);

/* ---- verification (Alg. 1: Verification + SelectLongestAcceptedPrefix) --------
 * Scores root + n_nodes draft nodes in one forward pass and walks the longest
 * accepted path.  Pure with respect to committed state: it writes only the tree
 * slots [len, len + n_nodes] of the cache and may be repeated.
 *   draft_tokens, parent_idx : n_nodes int32 each (may be NULL when n_nodes = 0)
 *   accept_len      : out, number of accepted draft tokens l
 *   accepted_tokens : out, caller buffer of >= n_nodes ints, first l valid
 *   accepted_nodes  : out, optional (NULL ok), node index of each accepted token
 *   bonus_token     : out, arg-max token after the last accepted node (or the root)
 * Tokens emitted by the step = accepted_tokens[0..l) followed by bonus_token.
 * Errors: INVALID_ARG, INVALID_TREE, TOKEN_RANGE, KV_CAPACITY, STATE (no pending
 * token), DEVICE. */
ts_status ts_verify(ts_model* m, ts_kv* kv,
                    const int32_t* draft_tokens, const int32_t* parent_idx, int32_t n_nodes,
                    int32_t* accept_len, int32_t* accepted_tokens, int32_t* accepted_nodes,
                    int32_t* bonus_token);

/* Stochastic acceptance (the paper's stated acceptance strategy, App. B.2: speculative sampling,
 * Leviathan et al. 2023), for one sequence.  Same pass and same outputs as ts_verify, but at a row
 * with target distribution p = softmax(logits / temperature) the children are tried in node order:
 * child c with token x is accepted with probability p(x) / (1 - mass of its siblings rejected
 * before it), decided by node_uniform[c] < that ratio; a rejected token leaves the distribution; a
 * sibling repeating a rejected token is rejected.  When every child of a row is rejected (or it
 * has none) the step ends with a sample of what is left of p there: bonus_token = arg-max over the
 * remaining tokens of logits / temperature + Gumbel noise, noise(row, token) = -log(-log(u)),
 * u = (top 23 bits of splitmix64(noise_seed + (row << 32 | token)) + 0.5) / 2^23.  The emitted
 * tokens are distributed as the target model's own samples.
 *   node_uniform : n_nodes floats in [0,1), the caller's random draws (one per draft node)
 * Errors as ts_verify, plus INVALID_ARG for temperature <= 0 or a uniform outside [0,1). */
ts_status ts_verify_sample(ts_model* m, ts_kv* kv,
                           const int32_t* draft_tokens, const int32_t* parent_idx, int32_t n_nodes,
                           float temperature, const float* node_uniform, uint64_t noise_seed,
                           int32_t* accept_len, int32_t* accepted_tokens, int32_t* accepted_nodes,
                           int32_t* bonus_token);

/* Same for n_seqs independent sequences in one pass (weights are streamed once).
 * Nodes are concatenated; node_offsets has n_seqs + 1 entries; parent indices are
 * local to their sequence.  accepted_tokens / accepted_nodes use the same offsets.
 * All kvs must belong to m and be distinct. */
ts_status ts_verify_batch(ts_model* m, ts_kv* const* kvs, int32_t n_seqs,
                          const int32_t* draft_tokens, const int32_t* parent_idx,
                          const int32_t* node_offsets,
                          int32_t* accept_len, int32_t* accepted_tokens, int32_t* accepted_nodes,
                          int32_t* bonus_token);

/* ---- commit (Alg. 1: y <- y (+) accepted prefix) ------------------------------
 * Applies the most recent verify on this cache: the root's K/V stay at slot len,
 * the accepted node of depth d moves to slot len + d (all layers, all KV heads,
 * a pure copy since K is stored rotated), len += l + 1, pending <- bonus token.
 * STATE if there is no unapplied verify result. */
ts_status ts_kv_commit(ts_kv* kv);

/* ---- measurement --------------------------------------------------------------
 * With profiling on, every kernel launch of ts_verify is bracketed by HIP events on
 * the model's stream.  ts_profile_read returns, for up to max_entries kernel kinds
 * launched by the most recent verify: name (static string), launches, total ms.
 * It returns the number of kinds through n_entries. */
typedef struct { const char* name; int32_t launches; float total_ms; } ts_profile_entry;
ts_status ts_profile_enable(ts_model* m, int32_t enable);
/* Restrict the bracketing to launches of one kernel kind (e.g. "gemm_gate_up"), so that
 * its timing is not disturbed by events around every other launch; NULL = all kinds.  The
 * kind "verify_pass" brackets nothing but the whole pass of a verify call, from its first
 * launch to the acceptance walk (one record per call; not part of the NULL set). */
ts_status ts_profile_filter(ts_model* m, const char* kind_or_null);
ts_status ts_profile_read(ts_model* m, ts_profile_entry* entries, int32_t max_entries, int32_t* n_entries);
/* Reference point for the projections' bandwidth figures: `launches` launches of a kernel that
 * only reads - launch i streams the fused gate/up weight tensor of layer i mod n_layers, the
 * bytes the largest projection of a step streams - on the model's stream, bracketed like any
 * other kind under the name "plain_read" (profiling must be on, and the filter, if set, must
 * name it).  bf16 models only (INVALID_ARG otherwise).  The records join those of the most recent verify.  Returns after the launches
 * have completed; bytes_per_launch (may be NULL) receives the tensor's size. */
ts_status ts_profile_plain_read(ts_model* m, int32_t launches, uint64_t* bytes_per_launch);

#ifdef __cplusplus
}
#endif
#endif /* TOOLSPEC_H */
