// The method's decoding loop (paper Alg. 1) as one native call: draft (SuffixMatch over the
// retrieved calls, else SchemaAwareDraft, packed as a tree) -> single-pass verification ->
// commit of the longest accepted prefix -> FSM update, until enough tokens are out.  Host code
// on top of the public C ABI only (toolspec.h, toolspec_draft.h); it holds no state of its own.
#include <chrono>

#include "toolspec_draft.h"

ts_status ts_fail(ts_status code, const char* fmt, ...);   // ts_host.hip: sets the thread's last-error text

extern "C" ts_status ts_generate(ts_model* m, ts_kv* kv, ts_drafter* d, int32_t max_new_tokens, int32_t stop_token,
                                 int32_t* out_tokens, int32_t* n_out, ts_generate_stats* stats) {
  if (!m || !kv || !d || !out_tokens || !n_out || max_new_tokens < 0)
    return ts_fail(TS_ERR_INVALID_ARG, "ts_generate: null argument or negative token count");
  typedef std::chrono::steady_clock clk;
  ts_generate_stats st = {0, 0, 0, 0, 0, 0, -1, 0.0, 0.0};
  int32_t toks[TS_MAX_NODES], par[TS_MAX_NODES], acc[TS_MAX_NODES];
  int32_t n = 0;
  *n_out = 0;
  ts_status rc = TS_OK;
  while (n < max_new_tokens && st.stop_index < 0) {
    int32_t nn = 0, src = TS_DRAFT_NONE, l = 0, bonus = -1;
    const clk::time_point t0 = clk::now();
    if ((rc = ts_drafter_draft(d, TS_MAX_NODES, toks, par, &nn, &src))) break;
    const clk::time_point t1 = clk::now();
    rc = ts_verify(m, kv, toks, par, nn, &l, acc, nullptr, &bonus);
    if (rc == TS_ERR_KV_CAPACITY && nn > 0) {          // no room for the tree: a plain decoding step still fits one row
      nn = 0;
      src = TS_DRAFT_NONE;
      rc = ts_verify(m, kv, toks, par, 0, &l, acc, nullptr, &bonus);
    }
    if (rc) break;
    if ((rc = ts_kv_commit(kv))) break;
    const clk::time_point t2 = clk::now();
    for (int32_t i = 0; i <= l; ++i) {
      const int32_t t = i < l ? acc[i] : bonus;
      if (st.stop_index < 0 && stop_token >= 0 && t == stop_token) st.stop_index = n;
      out_tokens[n++] = t;
    }
    if ((rc = ts_drafter_append(d, out_tokens + n - (l + 1), l + 1))) break;
    st.steps += 1;
    st.drafted_nodes += nn;
    st.accepted_tokens += l;
    if (src == TS_DRAFT_RETRIEVAL) st.retrieval_steps += 1;
    else if (src == TS_DRAFT_SCHEMA) st.schema_steps += 1;
    else st.plain_steps += 1;
    st.draft_seconds += std::chrono::duration<double>(t1 - t0).count();
    st.verify_seconds += std::chrono::duration<double>(t2 - t1).count();
  }
  *n_out = n;
  if (stats) *stats = st;
  return rc;
}
