/*
 * toolspec_draft.h - C ABI of the host-side drafting steps around the verification library.
 *
 * One decoding step of the method (paper Alg. 1) is: SuffixMatch against the retrieved
 * historical calls; if nothing matches, SchemaAwareDraft from the finite-state machine of
 * the tool schema; PackDraftsAsTree; Verification + SelectLongestAcceptedPrefix (toolspec.h,
 * on the GPU); append the accepted tokens; update the FSM state.  Everything in this header
 * runs on the host CPU in plain C++ and touches no device memory; its trees go straight into
 * ts_verify as (draft_tokens, parent_idx).
 *
 * All text is handled as token ids: the caller tokenizes the schema strings once.  Token
 * sequences are host int32 arrays; sets of sequences are passed packed (one token array plus
 * n+1 offsets).  Every function returns a ts_status (toolspec.h) and never throws; errors
 * leave the drafter unchanged.  A drafter serves one request at a time and is not thread-safe.
 *
 * FSM (paper Sec. 4.2, F = (Q, Sigma_schema, delta, q0), Fig. 2), at token level:
 *   q_o  "others": free text.  When the output ends with call_open -> q_t.
 *   q_t  tool name: the candidates are  name_prefix (+) tool_name_i (+) name_suffix  (Eq. 2).
 *        Tokens generated since entering the state must stay a prefix of a candidate; when
 *        one is complete -> q_p with that tool selected; when none fits -> q_o.
 *   q_p  parameter name: candidates  param_prefix (+) param_name_j (+) param_suffix  over the
 *        selected tool's fields; complete -> q_v; none fits -> q_o.
 *   q_v  parameter value: unconstrained.  Output ends with call_close -> q_o (call complete);
 *        ends with value_end -> q_p (next parameter).  call_close is tested first.
 *   q0 = q_o.  Schema drafts exist only in q_t and q_p (the structural states); in q_v and q_o
 *   the paper falls back on a general speculative method, which is the caller's business here.
 */
#ifndef TOOLSPEC_DRAFT_H
#define TOOLSPEC_DRAFT_H

#include <stdint.h>

#include "toolspec.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ts_drafter ts_drafter; /* opaque; owns copies of the schema, the retrieved calls, y and q */

enum { TS_Q_OTHERS = 0, TS_Q_TOOL_NAME = 1, TS_Q_PARAM_NAME = 2, TS_Q_PARAM_VALUE = 3 };
enum { TS_DRAFT_NONE = 0, TS_DRAFT_RETRIEVAL = 1, TS_DRAFT_SCHEMA = 2 };

/* Parsed tool schema S (Sec. 4.1: schema tokens, callable tools, parameter fields), as tokens.
 * The drafter copies everything.  Empty sequences (n = 0) are legal except call_open,
 * value_end and call_close, and every tool / parameter name must be non-empty. */
typedef struct {
  const int32_t* call_open;    int32_t n_call_open;    /* e.g. <tool_call>                          */
  const int32_t* name_prefix;  int32_t n_name_prefix;  /* y_prefix of Eq. 2, e.g. {"name": "        */
  const int32_t* name_suffix;  int32_t n_name_suffix;  /* y_suffix of Eq. 2, e.g. ", "parameters": { */
  const int32_t* param_prefix; int32_t n_param_prefix; /* before a parameter name, e.g. "           */
  const int32_t* param_suffix; int32_t n_param_suffix; /* after it, e.g. ": "                       */
  const int32_t* value_end;    int32_t n_value_end;    /* ends a value, next parameter, e.g. ",     */
  const int32_t* call_close;   int32_t n_call_close;   /* ends the call, e.g. "}}                   */
  int32_t n_tools;
  const int32_t* tool_tokens;        /* concatenated tool names                                  */
  const int32_t* tool_offsets;       /* n_tools + 1                                              */
  const int32_t* param_first;        /* n_tools + 1: parameters of tool i are [param_first[i], param_first[i+1]) */
  const int32_t* param_tokens;       /* concatenated parameter names of all tools                */
  const int32_t* param_offsets;      /* param_first[n_tools] + 1                                 */
} ts_schema_desc;

/* Alg. 1, the set-up steps: the schema (already parsed into token sequences) becomes the FSM.  INVALID_ARG on null or
 * inconsistent offsets, OOM. */
ts_status ts_drafter_create(const ts_schema_desc* schema, ts_drafter** out);
ts_status ts_drafter_free(ts_drafter* d);

/* Alg. 1, the retrieval step (Sec. 4.3, Eq. 3): cosine similarity of h_x (dim floats) with
 * the n_entries rows of H (row-major [n_entries][dim]), the k most similar kept in order of
 * decreasing similarity (equal similarity: lower index first; zero vectors have similarity
 * 0).  The tool-call outputs y_j are packed (y_tokens, y_offsets[n_entries + 1]); the drafter
 * copies the retrieved ones.  top_idx (optional) receives min(k, n_entries) indices.
 * k = 10 in the paper.  Replaces the result of an earlier call. */
ts_status ts_drafter_retrieve(ts_drafter* d, const float* h_x, int32_t dim, const float* H, int32_t n_entries,
                              const int32_t* y_tokens, const int32_t* y_offsets, int32_t k, int32_t* top_idx);

/* Start of a request: y <- empty, q <- q0.  The retrieved calls are kept. */
ts_status ts_drafter_reset(ts_drafter* d);

/* y <- y (+) tokens, q <- delta(q, tokens): call it with everything a step emitted (the
 * accepted draft tokens, then the bonus token).  The last token of y is the root of the next
 * tree (the pending token of the cache). */
ts_status ts_drafter_append(ts_drafter* d, const int32_t* tokens, int32_t n_tokens);

/* Current state (TS_Q_*), selected tool (-1 outside q_p / q_v) and length of y. */
ts_status ts_drafter_state(const ts_drafter* d, int32_t* state, int32_t* tool, int32_t* y_len);

/* The draft tree of the next step (Alg. 1: SuffixMatch, else SchemaAwareDraft, then
 * PackDraftsAsTree).
 *  SuffixMatch (Sec. 4.3, App. B.2): suffix lengths L = 7, 6, 5, longest first; for the first
 *  L with any match, the positions m with y'[m-L .. m-1] = y[t-L .. t-1] are taken in order
 *  (retrieved calls in rank order, positions ascending) and the i-th match contributes the
 *  continuation y'[m .. m+n_i-1], n = 32, 16, 8, 8; matches with nothing after them are skipped.
 *  SchemaAwareDraft: the not yet generated remainders of the live candidates of q_t / q_p.
 *  PackDraftsAsTree: the drafts are merged into a trie (one node per distinct prefix), nodes
 *  numbered in creation order - drafts in order, each from its first new token - so parents
 *  precede children; at most max_nodes (<= TS_MAX_NODES) nodes, later ones are dropped.
 * draft_tokens / parent_idx: caller buffers of max_nodes ints.  source: TS_DRAFT_*. */
ts_status ts_drafter_draft(ts_drafter* d, int32_t max_nodes, int32_t* draft_tokens, int32_t* parent_idx,
                           int32_t* n_nodes, int32_t* source);

/* Counters of one ts_generate call. */
typedef struct {
  int32_t steps;             /* target passes (Alg. 1 iterations)                                  */
  int32_t drafted_nodes;     /* draft-tree nodes verified, summed over the steps                   */
  int32_t accepted_tokens;   /* accepted draft tokens (the bonus token of each step not counted)   */
  int32_t retrieval_steps;   /* steps whose tree came from SuffixMatch                             */
  int32_t schema_steps;      /* ... from SchemaAwareDraft                                          */
  int32_t plain_steps;       /* steps with no draft (vanilla decoding)                             */
  int32_t stop_index;        /* index in out_tokens of the first stop_token, -1 if none            */
  double draft_seconds;      /* host time in ts_drafter_draft                                      */
  double verify_seconds;     /* time in ts_verify + ts_kv_commit (device work included)            */
} ts_generate_stats;

/* Alg. 1, the whole loop: repeat { draft tree <- ts_drafter_draft; (l, tokens, bonus) <- ts_verify;
 * ts_kv_commit; y <- y (+) tokens (+) bonus; q <- delta(q, .) } until at least max_new_tokens are
 * out or a step emitted stop_token (stop_token < 0: never).  Before the call the cache holds the
 * context with its last token pending (ts_prefill leaves it so) and the drafter has been reset
 * (and, for retrieval drafts, given its calls).  A step is never cut short: n_out may exceed
 * max_new_tokens by up to TS_MAX_NODES, so out_tokens needs max_new_tokens + TS_MAX_NODES + 1
 * ints; every emitted token is in the cache and in the drafter's y afterwards.  When the cache
 * has no room left for a tree the step falls back to plain decoding (no draft); when it has no
 * room for one more row the call returns KV_CAPACITY with everything emitted so far reported.
 * Greedy acceptance; the emitted stream is the target's own greedy stream (Sec. 5.1).
 * stats may be NULL.  Errors of the calls it makes are returned as they are. */
ts_status ts_generate(ts_model* m, ts_kv* kv, ts_drafter* d, int32_t max_new_tokens, int32_t stop_token,
                      int32_t* out_tokens, int32_t* n_out, ts_generate_stats* stats);

#ifdef __cplusplus
}
#endif
#endif /* TOOLSPEC_DRAFT_H */
