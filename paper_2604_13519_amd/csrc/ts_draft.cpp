// Host-side drafting steps of one decoding step (paper Alg. 1): Top-K retrieval of historical
// calls, SuffixMatch, schema FSM with SchemaAwareDraft, PackDraftsAsTree.  Plain C++, no device
// code; the state is kept incrementally (the FSM advances token by token as the output grows,
// live candidates are narrowed instead of recomputed).
#include <math.h>
#include <stdarg.h>
#include <stddef.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <unordered_map>
#include <vector>

#include "toolspec_draft.h"

ts_status ts_fail(ts_status code, const char* fmt, ...);   // ts_host.hip: sets the thread's last-error text

namespace {

typedef std::vector<int32_t> Seq;

constexpr int kSuffixLengths[3] = {7, 6, 5};          // App. B.2: longest first
constexpr int kContinuation[4] = {32, 16, 8, 8};      // App. B.2: lengths of the extracted continuations

bool ends_with(const Seq& y, const Seq& tail) {
  return y.size() >= tail.size() && std::equal(tail.begin(), tail.end(), y.end() - (ptrdiff_t)tail.size());
}

}  // namespace

struct ts_drafter {
  // schema S
  Seq call_open, name_prefix, name_suffix, param_prefix, param_suffix, value_end, call_close;
  std::vector<Seq> tools;
  std::vector<std::vector<Seq>> params;     // per tool
  // candidates of the structural states, built once: full token sequences
  std::vector<Seq> tool_cands;              // prefix (+) tool_i (+) suffix
  std::vector<std::vector<Seq>> param_cands;
  // retrieved historical calls, in rank order
  std::vector<Seq> calls;
  // request state
  Seq y;
  int state = TS_Q_OTHERS;
  int tool = -1;
  size_t since = 0;                         // tokens generated since the structural state was entered
  size_t in_value = 0;                      // tokens generated inside q_v
  std::vector<int> live;                    // candidates of the current structural state that still fit

  const std::vector<Seq>& cands() const { return state == TS_Q_TOOL_NAME ? tool_cands : param_cands[tool]; }

  void enter_structural(int st) {
    state = st;
    since = 0;
    live.clear();
    const std::vector<Seq>& c = cands();
    for (size_t i = 0; i < c.size(); ++i) live.push_back((int)i);
  }

  // delta for one generated token (already pushed to y)
  void step(int32_t x) {
    if (state == TS_Q_TOOL_NAME || state == TS_Q_PARAM_NAME) {
      const std::vector<Seq>& c = cands();
      std::vector<int> keep;
      int full = -1;
      for (int i : live) {
        if (since < c[i].size() && c[i][since] == x) {
          keep.push_back(i);
          if (full < 0 && c[i].size() == since + 1) full = i;
        }
      }
      since += 1;
      live.swap(keep);
      if (full >= 0) {
        if (state == TS_Q_TOOL_NAME) {
          tool = full;
          enter_structural(TS_Q_PARAM_NAME);
        } else {
          state = TS_Q_PARAM_VALUE;
          in_value = 0;
          live.clear();
        }
      } else if (live.empty()) {
        state = TS_Q_OTHERS;
        tool = -1;
      }
    } else if (state == TS_Q_PARAM_VALUE) {
      in_value += 1;
      if (in_value >= call_close.size() && ends_with(y, call_close)) {
        state = TS_Q_OTHERS;
        tool = -1;
      } else if (in_value >= value_end.size() && ends_with(y, value_end)) {
        enter_structural(TS_Q_PARAM_NAME);
      }
      return;
    }
    if (state == TS_Q_OTHERS && ends_with(y, call_open)) enter_structural(TS_Q_TOOL_NAME);
  }
};

namespace {

bool copy_seq(Seq& dst, const int32_t* p, int32_t n) {
  if (n < 0 || (n > 0 && !p)) return false;
  dst.assign(p, p + n);
  return true;
}

// Trie under construction: (parent node, token) -> node
struct Packer {
  int32_t* toks;
  int32_t* par;
  int max_nodes;
  int n = 0;
  std::unordered_map<uint64_t, int> child;
  Packer(int32_t* t, int32_t* p, int m) : toks(t), par(p), max_nodes(m) {}
  void add(const int32_t* seq, size_t len) {
    int node = -1;
    for (size_t i = 0; i < len; ++i) {
      const uint64_t key = ((uint64_t)(uint32_t)(node + 1) << 32) | (uint32_t)seq[i];
      auto it = child.find(key);
      if (it == child.end()) {
        if (n >= max_nodes) return;
        toks[n] = seq[i];
        par[n] = node;
        it = child.emplace(key, n).first;
        ++n;
      }
      node = it->second;
    }
  }
};

}  // namespace

extern "C" ts_status ts_drafter_create(const ts_schema_desc* s, ts_drafter** out) {
  if (!s || !out) return ts_fail(TS_ERR_INVALID_ARG, "ts_drafter_create: null argument");
  if (s->n_tools < 0 || (s->n_tools > 0 && (!s->tool_offsets || !s->param_first || !s->param_offsets)))
    return ts_fail(TS_ERR_INVALID_ARG, "ts_drafter_create: tool tables missing");
  ts_drafter* d = new (std::nothrow) ts_drafter();
  if (!d) return ts_fail(TS_ERR_OOM, "ts_drafter_create: out of memory");
  bool ok = copy_seq(d->call_open, s->call_open, s->n_call_open) && copy_seq(d->name_prefix, s->name_prefix, s->n_name_prefix) &&
            copy_seq(d->name_suffix, s->name_suffix, s->n_name_suffix) && copy_seq(d->param_prefix, s->param_prefix, s->n_param_prefix) &&
            copy_seq(d->param_suffix, s->param_suffix, s->n_param_suffix) && copy_seq(d->value_end, s->value_end, s->n_value_end) &&
            copy_seq(d->call_close, s->call_close, s->n_call_close);
  ok = ok && !d->call_open.empty() && !d->value_end.empty() && !d->call_close.empty();
  for (int i = 0; ok && i < s->n_tools; ++i) {
    const int a = s->tool_offsets[i], b = s->tool_offsets[i + 1];
    const int pa = s->param_first[i], pb = s->param_first[i + 1];
    if (a < 0 || b <= a || pa < 0 || pb < pa || !s->tool_tokens) { ok = false; break; }
    d->tools.emplace_back(s->tool_tokens + a, s->tool_tokens + b);
    d->params.emplace_back();
    for (int j = pa; j < pb; ++j) {
      const int qa = s->param_offsets[j], qb = s->param_offsets[j + 1];
      if (qa < 0 || qb <= qa || !s->param_tokens) { ok = false; break; }
      d->params.back().emplace_back(s->param_tokens + qa, s->param_tokens + qb);
    }
  }
  if (!ok) {
    delete d;
    return ts_fail(TS_ERR_INVALID_ARG, "ts_drafter_create: empty delimiter or name, or inconsistent offsets");
  }
  auto join = [](const Seq& a, const Seq& b, const Seq& c) {
    Seq r(a);
    r.insert(r.end(), b.begin(), b.end());
    r.insert(r.end(), c.begin(), c.end());
    return r;
  };
  for (size_t i = 0; i < d->tools.size(); ++i) {
    d->tool_cands.push_back(join(d->name_prefix, d->tools[i], d->name_suffix));          // Eq. 2
    d->param_cands.emplace_back();
    for (const Seq& p : d->params[i]) d->param_cands.back().push_back(join(d->param_prefix, p, d->param_suffix));
  }
  *out = d;
  return TS_OK;
}

extern "C" ts_status ts_drafter_free(ts_drafter* d) {
  delete d;
  return TS_OK;
}

extern "C" ts_status ts_drafter_retrieve(ts_drafter* d, const float* h_x, int32_t dim, const float* H, int32_t n_entries,
                                         const int32_t* y_tokens, const int32_t* y_offsets, int32_t k, int32_t* top_idx) {
  if (!d || !h_x || dim <= 0 || n_entries < 0 || k < 0 || (n_entries > 0 && (!H || !y_offsets)))
    return ts_fail(TS_ERR_INVALID_ARG, "ts_drafter_retrieve: bad argument");
  for (int j = 0; j < n_entries; ++j)
    if (y_offsets[j] < 0 || y_offsets[j + 1] < y_offsets[j] || (y_offsets[j + 1] > y_offsets[j] && !y_tokens))
      return ts_fail(TS_ERR_INVALID_ARG, "ts_drafter_retrieve: inconsistent offsets (entry %d)", j);
  double nx = 0.0;
  for (int i = 0; i < dim; ++i) nx += (double)h_x[i] * h_x[i];
  nx = sqrt(nx);
  std::vector<double> sim((size_t)n_entries, 0.0);
  for (int j = 0; j < n_entries; ++j) {
    const float* row = H + (size_t)j * dim;
    double dot = 0.0, nj = 0.0;
    for (int i = 0; i < dim; ++i) { dot += (double)row[i] * h_x[i]; nj += (double)row[i] * row[i]; }
    nj = sqrt(nj);
    sim[j] = (nx > 0.0 && nj > 0.0) ? dot / (nx * nj) : 0.0;
  }
  std::vector<int> order((size_t)n_entries);
  for (int j = 0; j < n_entries; ++j) order[j] = j;
  const int keep = std::min(k, n_entries);
  std::partial_sort(order.begin(), order.begin() + keep, order.end(),
                    [&](int a, int b) { return sim[a] != sim[b] ? sim[a] > sim[b] : a < b; });
  std::vector<Seq> calls;
  for (int r = 0; r < keep; ++r) {
    const int j = order[r];
    calls.emplace_back(y_tokens + y_offsets[j], y_tokens + y_offsets[j + 1]);
    if (top_idx) top_idx[r] = j;
  }
  d->calls.swap(calls);
  return TS_OK;
}

extern "C" ts_status ts_drafter_reset(ts_drafter* d) {
  if (!d) return ts_fail(TS_ERR_INVALID_ARG, "null drafter");
  d->y.clear();
  d->state = TS_Q_OTHERS;
  d->tool = -1;
  d->since = d->in_value = 0;
  d->live.clear();
  return TS_OK;
}

extern "C" ts_status ts_drafter_append(ts_drafter* d, const int32_t* tokens, int32_t n) {
  if (!d || n < 0 || (n > 0 && !tokens)) return ts_fail(TS_ERR_INVALID_ARG, "ts_drafter_append: bad argument");
  for (int i = 0; i < n; ++i) {
    d->y.push_back(tokens[i]);
    d->step(tokens[i]);
  }
  return TS_OK;
}

extern "C" ts_status ts_drafter_state(const ts_drafter* d, int32_t* state, int32_t* tool, int32_t* y_len) {
  if (!d) return ts_fail(TS_ERR_INVALID_ARG, "null drafter");
  if (state) *state = d->state;
  if (tool) *tool = d->tool;
  if (y_len) *y_len = (int32_t)d->y.size();
  return TS_OK;
}

extern "C" ts_status ts_drafter_draft(ts_drafter* d, int32_t max_nodes, int32_t* draft_tokens, int32_t* parent_idx,
                                      int32_t* n_nodes, int32_t* source) {
  if (!d || !n_nodes || max_nodes < 0 || max_nodes > TS_MAX_NODES || (max_nodes > 0 && (!draft_tokens || !parent_idx)))
    return ts_fail(TS_ERR_INVALID_ARG, "ts_drafter_draft: bad argument");
  Packer pk(draft_tokens, parent_idx, max_nodes);
  int src = TS_DRAFT_RETRIEVAL;
  // SuffixMatch: y[t-L .. t-1] = y'[m-L .. m-1], longest L first
  const Seq& y = d->y;
  bool matched = false;
  for (int li = 0; li < 3 && !matched; ++li) {
    const size_t L = (size_t)kSuffixLengths[li];
    if (y.size() < L) continue;
    const int32_t* pat = y.data() + (y.size() - L);
    int taken = 0;
    for (size_t c = 0; c < d->calls.size() && taken < 4; ++c) {
      const Seq& call = d->calls[c];
      for (size_t m = L; m <= call.size() && taken < 4; ++m) {
        if (memcmp(call.data() + (m - L), pat, L * sizeof(int32_t)) != 0) continue;
        const size_t len = std::min((size_t)kContinuation[taken], call.size() - m);
        if (len == 0) continue;                       // nothing follows the match
        pk.add(call.data() + m, len);
        ++taken;
        matched = true;
      }
    }
  }
  if (!matched) {
    src = TS_DRAFT_SCHEMA;
    if (d->state == TS_Q_TOOL_NAME || d->state == TS_Q_PARAM_NAME) {
      const std::vector<Seq>& c = d->cands();
      for (int i : d->live)
        if (c[i].size() > d->since) pk.add(c[i].data() + d->since, c[i].size() - d->since);
    }
  }
  *n_nodes = pk.n;
  if (source) *source = pk.n > 0 ? src : TS_DRAFT_NONE;
  return TS_OK;
}
