"""ctypes binding of libtoolspec_hip.so: argument marshalling only.

Function names mirror include/toolspec.h.  Every step of the verify pass runs
in the library's HIP kernels; nothing here computes.  There is no CPU fallback:
if the library is missing or no GPU is present the calls raise.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtoolspec_hip.so")

TS_OK = 0
TS_ERR_INVALID_ARG, TS_ERR_INVALID_TREE, TS_ERR_TOKEN_RANGE = -1, -2, -3
TS_ERR_KV_CAPACITY, TS_ERR_STATE, TS_ERR_OOM, TS_ERR_DEVICE = -4, -5, -6, -7
TS_DTYPE_F32, TS_DTYPE_BF16 = 0, 1
TS_MAX_NODES, TS_PAGE_SIZE = 64, 16
TS_Q_OTHERS, TS_Q_TOOL_NAME, TS_Q_PARAM_NAME, TS_Q_PARAM_VALUE = 0, 1, 2, 3
TS_DRAFT_NONE, TS_DRAFT_RETRIEVAL, TS_DRAFT_SCHEMA = 0, 1, 2

EXPORTS = ("ts_last_error", "ts_model_load", "ts_model_free", "ts_model_keep_logits", "ts_get_logits", "ts_get_row_tokens", "ts_model_saturations", "ts_get_hidden",
           "ts_kv_alloc", "ts_kv_free", "ts_kv_set_page_table", "ts_kv_pool_create", "ts_kv_pool_free", "ts_kv_pool_pages_free",
           "ts_kv_alloc_pooled", "ts_kv_import", "ts_kv_export", "ts_kv_export_noalloc",
           "ts_set_pending", "ts_kv_len", "ts_kv_truncate", "ts_prefill", "ts_verify", "ts_verify_sample", "ts_verify_batch",
           "ts_kv_commit", "ts_profile_enable", "ts_profile_filter", "ts_profile_read", "ts_profile_plain_read",
           "ts_drafter_create", "ts_drafter_free", "ts_drafter_retrieve", "ts_drafter_reset",
           "ts_drafter_append", "ts_drafter_state", "ts_drafter_draft", "ts_generate")


class TsError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("toolspec status %d: %s" % (status, message))
        self.status = status


class ts_generate_stats(C.Structure):
    _fields_ = [("steps", C.c_int32), ("drafted_nodes", C.c_int32), ("accepted_tokens", C.c_int32),
                ("retrieval_steps", C.c_int32), ("schema_steps", C.c_int32), ("plain_steps", C.c_int32),
                ("stop_index", C.c_int32), ("draft_seconds", C.c_double), ("verify_seconds", C.c_double)]


class ts_model_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float),
                ("dtype", C.c_int32)]


_PP = C.POINTER(C.c_void_p)


class ts_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("norm_f", C.c_void_p),
                ("wq", _PP), ("wk", _PP), ("wv", _PP), ("wo", _PP), ("wg", _PP), ("wu", _PP),
                ("wd", _PP), ("norm1", _PP), ("norm2", _PP)]


_I32P = C.POINTER(C.c_int32)


class ts_schema_desc(C.Structure):
    _fields_ = [("call_open", _I32P), ("n_call_open", C.c_int32), ("name_prefix", _I32P), ("n_name_prefix", C.c_int32),
                ("name_suffix", _I32P), ("n_name_suffix", C.c_int32), ("param_prefix", _I32P), ("n_param_prefix", C.c_int32),
                ("param_suffix", _I32P), ("n_param_suffix", C.c_int32), ("value_end", _I32P), ("n_value_end", C.c_int32),
                ("call_close", _I32P), ("n_call_close", C.c_int32), ("n_tools", C.c_int32),
                ("tool_tokens", _I32P), ("tool_offsets", _I32P), ("param_first", _I32P),
                ("param_tokens", _I32P), ("param_offsets", _I32P)]


class ts_profile_entry(C.Structure):
    _fields_ = [("name", C.c_char_p), ("launches", C.c_int32), ("total_ms", C.c_float)]


_lib = None


def load_library(path=None):
    """Loads the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = path or os.environ.get("TS_LIB_PATH") or LIB_PATH   # TS_LIB_PATH: another build of the same library
    if not os.path.exists(path):
        raise RuntimeError("%s not found: build it with `python -m paper_2604_13519_amd.build`" % path)
    lib = C.CDLL(path)
    i32p = C.POINTER(C.c_int32)
    lib.ts_last_error.restype = C.c_char_p
    lib.ts_last_error.argtypes = []
    sigs = {
        "ts_model_load": [C.POINTER(ts_model_config), C.POINTER(ts_weights), C.POINTER(C.c_void_p)],
        "ts_model_free": [C.c_void_p],
        "ts_model_keep_logits": [C.c_void_p, C.c_int32],
        "ts_get_logits": [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p],
        "ts_get_row_tokens": [C.c_void_p, C.c_int32, C.c_int32, i32p],
        "ts_model_saturations": [C.c_void_p, C.POINTER(C.c_uint64)],
        "ts_get_hidden": [C.c_void_p, C.c_int32, C.c_void_p],
        "ts_kv_alloc": [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_void_p)],
        "ts_kv_free": [C.c_void_p],
        "ts_kv_set_page_table": [C.c_void_p, i32p, C.c_int32],
        "ts_kv_pool_create": [C.c_void_p, C.c_int32, C.POINTER(C.c_void_p)],
        "ts_kv_pool_free": [C.c_void_p],
        "ts_kv_pool_pages_free": [C.c_void_p, C.POINTER(C.c_int32)],
        "ts_kv_alloc_pooled": [C.c_void_p, C.c_int32, C.POINTER(C.c_void_p)],
        "ts_kv_import": [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p],
        "ts_kv_export": [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p],
        "ts_kv_export_noalloc": [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p],
        "ts_set_pending": [C.c_void_p, C.c_int32],
        "ts_kv_len": [C.c_void_p, i32p],
        "ts_kv_truncate": [C.c_void_p, C.c_int32],
        "ts_prefill": [C.c_void_p, C.c_void_p, i32p, C.c_int32],
        "ts_verify": [C.c_void_p, C.c_void_p, i32p, i32p, C.c_int32, i32p, i32p, i32p, i32p],
        "ts_verify_sample": [C.c_void_p, C.c_void_p, i32p, i32p, C.c_int32, C.c_float, C.POINTER(C.c_float), C.c_uint64,
                             i32p, i32p, i32p, i32p],
        "ts_verify_batch": [C.c_void_p, C.POINTER(C.c_void_p), C.c_int32, i32p, i32p, i32p, i32p, i32p, i32p, i32p],
        "ts_kv_commit": [C.c_void_p],
        "ts_profile_enable": [C.c_void_p, C.c_int32],
        "ts_profile_filter": [C.c_void_p, C.c_char_p],
        "ts_profile_read": [C.c_void_p, C.POINTER(ts_profile_entry), C.c_int32, i32p],
        "ts_profile_plain_read": [C.c_void_p, C.c_int32, C.POINTER(C.c_uint64)],
        "ts_drafter_create": [C.POINTER(ts_schema_desc), C.POINTER(C.c_void_p)],
        "ts_drafter_free": [C.c_void_p],
        "ts_drafter_retrieve": [C.c_void_p, C.POINTER(C.c_float), C.c_int32, C.POINTER(C.c_float), C.c_int32, i32p, i32p,
                                C.c_int32, i32p],
        "ts_drafter_reset": [C.c_void_p],
        "ts_drafter_append": [C.c_void_p, i32p, C.c_int32],
        "ts_drafter_state": [C.c_void_p, i32p, i32p, i32p],
        "ts_drafter_draft": [C.c_void_p, C.c_int32, i32p, i32p, i32p, i32p],
        "ts_generate": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, i32p, i32p, C.POINTER(ts_generate_stats)],
    }
    for name, args in sigs.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int32
    _lib = lib
    return lib


def _check(status):
    if status != TS_OK:
        raise TsError(status, load_library().ts_last_error().decode("utf-8", "replace"))


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr_i32(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _np_dtype(dtype):
    return np.float32 if dtype == TS_DTYPE_F32 else np.uint16


# --------------------------------------------------------------------------------------
# thin wrappers, same names as the C ABI
# --------------------------------------------------------------------------------------
def ts_model_load(cfg, weights):
    """cfg: object with the ts_model_config field names; weights: {"embed", "lm_head", "norm_f",
    "layers": [{wq, wk, wv, wo, wg, wu, wd, norm1, norm2}]} of numpy arrays, float32 or uint16
    bf16 bit patterns, row-major [out][in].  Returns an opaque model handle."""
    lib = load_library()
    c = ts_model_config(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                        cfg.d_ffn, cfg.vocab, cfg.rope_theta, cfg.rms_eps, cfg.dtype)
    dt = _np_dtype(cfg.dtype)
    keep = []

    def host(a):
        a = np.ascontiguousarray(a)
        if a.dtype != dt:
            raise TypeError("weight dtype %s does not match the model dtype" % a.dtype)
        keep.append(a)
        return a.ctypes.data

    w = ts_weights()
    w.embed, w.lm_head, w.norm_f = host(weights["embed"]), host(weights["lm_head"]), host(weights["norm_f"])
    L = cfg.n_layers
    for kind in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "norm1", "norm2"):
        arr = (C.c_void_p * L)(*[host(weights["layers"][l][kind]) for l in range(L)])
        keep.append(arr)
        setattr(w, kind, C.cast(arr, _PP))
    out = C.c_void_p()
    _check(lib.ts_model_load(C.byref(c), C.byref(w), C.byref(out)))
    return out


def ts_model_free(model):
    _check(load_library().ts_model_free(model))


def ts_model_keep_logits(model, enable):
    _check(load_library().ts_model_keep_logits(model, int(bool(enable))))


def ts_get_logits(model, row0, n_rows, vocab):
    out = np.empty((n_rows, vocab), dtype=np.float32)
    _check(load_library().ts_get_logits(model, row0, n_rows, out.ctypes.data))
    return out


def ts_model_saturations(model):
    n = C.c_uint64()
    _check(load_library().ts_model_saturations(model, C.byref(n)))
    return int(n.value)


def ts_get_row_tokens(model, row0, n_rows):
    out = np.empty(n_rows, dtype=np.int32)
    _check(load_library().ts_get_row_tokens(model, int(row0), int(n_rows), _ptr_i32(out)))
    return out


def ts_get_hidden(model, row, d_model):
    out = np.empty(d_model, dtype=np.float32)
    _check(load_library().ts_get_hidden(model, row, out.ctypes.data))
    return out


def ts_kv_alloc(model, capacity_tokens, page_size=TS_PAGE_SIZE):
    out = C.c_void_p()
    _check(load_library().ts_kv_alloc(model, capacity_tokens, page_size, C.byref(out)))
    return out


def ts_kv_free(kv):
    _check(load_library().ts_kv_free(kv))


def ts_kv_set_page_table(kv, phys_pages):
    p = _i32(phys_pages)
    _check(load_library().ts_kv_set_page_table(kv, _ptr_i32(p), len(p)))


def ts_kv_pool_create(model, n_pages):
    out = C.c_void_p()
    _check(load_library().ts_kv_pool_create(model, n_pages, C.byref(out)))
    return out


def ts_kv_pool_free(pool):
    _check(load_library().ts_kv_pool_free(pool))


def ts_kv_pool_pages_free(pool):
    n = C.c_int32()
    _check(load_library().ts_kv_pool_pages_free(pool, C.byref(n)))
    return n.value


def ts_kv_alloc_pooled(pool, capacity_tokens):
    out = C.c_void_p()
    _check(load_library().ts_kv_alloc_pooled(pool, capacity_tokens, C.byref(out)))
    return out


def ts_kv_import(kv, k_host, v_host):
    """k_host, v_host: [L][n_pos][Hkv][hd] in the model dtype."""
    k = np.ascontiguousarray(k_host)
    v = np.ascontiguousarray(v_host)
    if k.shape != v.shape or k.dtype != v.dtype:
        raise TypeError("K and V must have the same shape and dtype")
    _check(load_library().ts_kv_import(kv, k.shape[1], k.ctypes.data, v.ctypes.data))


def ts_kv_export(kv, pos0, n_pos, cfg):
    shp = (cfg.n_layers, n_pos, cfg.n_kv_heads, cfg.head_dim)
    k = np.empty(shp, dtype=_np_dtype(cfg.dtype))
    v = np.empty(shp, dtype=_np_dtype(cfg.dtype))
    _check(load_library().ts_kv_export(kv, pos0, n_pos, k.ctypes.data, v.ctypes.data))
    return k, v


def ts_kv_export_noalloc(kv, pos0, n_pos, cfg):
    shp = (cfg.n_layers, n_pos, cfg.n_kv_heads, cfg.head_dim)
    k = np.empty(shp, dtype=_np_dtype(cfg.dtype))
    v = np.empty(shp, dtype=_np_dtype(cfg.dtype))
    _check(load_library().ts_kv_export_noalloc(kv, pos0, n_pos, k.ctypes.data, v.ctypes.data))
    return k, v


def ts_set_pending(kv, token):
    _check(load_library().ts_set_pending(kv, int(token)))


def ts_kv_len(kv):
    n = C.c_int32()
    _check(load_library().ts_kv_len(kv, C.byref(n)))
    return n.value


def ts_kv_truncate(kv, new_len):
    _check(load_library().ts_kv_truncate(kv, int(new_len)))


def ts_prefill(model, kv, tokens):
    t = _i32(tokens)
    _check(load_library().ts_prefill(model, kv, _ptr_i32(t), len(t)))


def ts_verify(model, kv, draft_tokens, parent_idx):
    """Returns (accept_len, accepted_tokens[list], accepted_nodes[list], bonus_token)."""
    t, p = _i32(draft_tokens), _i32(parent_idx)
    n = len(t)
    if len(p) != n:
        raise ValueError("draft_tokens and parent_idx differ in length")
    acc_len, bonus = C.c_int32(), C.c_int32()
    toks = np.zeros(max(n, 1), np.int32)
    nodes = np.zeros(max(n, 1), np.int32)
    _check(load_library().ts_verify(model, kv, _ptr_i32(t), _ptr_i32(p), n, C.byref(acc_len),
                                    _ptr_i32(toks), _ptr_i32(nodes), C.byref(bonus)))
    l = acc_len.value
    return l, toks[:l].tolist(), nodes[:l].tolist(), bonus.value


def ts_verify_sample(model, kv, draft_tokens, parent_idx, temperature, node_uniform, noise_seed):
    """Stochastic acceptance; returns (accept_len, accepted_tokens, accepted_nodes, bonus_token)."""
    t, p = _i32(draft_tokens), _i32(parent_idx)
    u = np.ascontiguousarray(node_uniform, dtype=np.float32)
    n = len(t)
    if len(p) != n or len(u) != n:
        raise ValueError("draft_tokens, parent_idx and node_uniform differ in length")
    acc_len, bonus = C.c_int32(), C.c_int32()
    toks = np.zeros(max(n, 1), np.int32)
    nodes = np.zeros(max(n, 1), np.int32)
    _check(load_library().ts_verify_sample(model, kv, _ptr_i32(t), _ptr_i32(p), n, float(temperature),
                                           u.ctypes.data_as(C.POINTER(C.c_float)), int(noise_seed) & ((1 << 64) - 1),
                                           C.byref(acc_len), _ptr_i32(toks), _ptr_i32(nodes), C.byref(bonus)))
    l = acc_len.value
    return l, toks[:l].tolist(), nodes[:l].tolist(), bonus.value


def ts_verify_batch(model, kvs, trees):
    """trees: list of (draft_tokens, parent_idx) per sequence.  Returns a list of
    (accept_len, accepted_tokens, accepted_nodes, bonus_token)."""
    n_seqs = len(kvs)
    offs = np.zeros(n_seqs + 1, np.int32)
    for i, (t, _) in enumerate(trees):
        offs[i + 1] = offs[i] + len(t)
    tot = int(offs[-1])
    toks = _i32(np.concatenate([_i32(t) for t, _ in trees]) if tot else np.zeros(0, np.int32))
    pars = _i32(np.concatenate([_i32(p) for _, p in trees]) if tot else np.zeros(0, np.int32))
    handles = (C.c_void_p * n_seqs)(*[k.value for k in kvs])
    acc_len = np.zeros(n_seqs, np.int32)
    bonus = np.zeros(n_seqs, np.int32)
    acc_t = np.zeros(max(tot, 1), np.int32)
    acc_n = np.zeros(max(tot, 1), np.int32)
    _check(load_library().ts_verify_batch(model, handles, n_seqs, _ptr_i32(toks), _ptr_i32(pars), _ptr_i32(offs),
                                          _ptr_i32(acc_len), _ptr_i32(acc_t), _ptr_i32(acc_n), _ptr_i32(bonus)))
    out = []
    for i in range(n_seqs):
        l, o = int(acc_len[i]), int(offs[i])
        out.append((l, acc_t[o:o + l].tolist(), acc_n[o:o + l].tolist(), int(bonus[i])))
    return out


def ts_kv_commit(kv):
    _check(load_library().ts_kv_commit(kv))


def ts_profile_enable(model, enable):
    _check(load_library().ts_profile_enable(model, int(bool(enable))))


def ts_profile_filter(model, kind=None):
    _check(load_library().ts_profile_filter(model, kind.encode() if kind else None))


def ts_profile_plain_read(model, launches):
    """Launches the read-only kernel over gate/up weight tensors; returns the bytes one launch reads."""
    n = C.c_uint64()
    _check(load_library().ts_profile_plain_read(model, int(launches), C.byref(n)))
    return int(n.value)


def ts_profile_read(model, max_entries=64):
    """{kernel kind: (launches, total_ms)} of the most recent verify."""
    arr = (ts_profile_entry * max_entries)()
    n = C.c_int32()
    _check(load_library().ts_profile_read(model, arr, max_entries, C.byref(n)))
    return {arr[i].name.decode(): (arr[i].launches, arr[i].total_ms) for i in range(min(n.value, max_entries))}


# --------------------------------------------------------------------------------------
# host drafter (include/toolspec_draft.h): marshalling only
# --------------------------------------------------------------------------------------
def _pack(seqs):
    """List of token sequences -> (concatenated int32 array, offsets int32[n+1])."""
    offs = np.zeros(len(seqs) + 1, np.int32)
    for i, q in enumerate(seqs):
        offs[i + 1] = offs[i] + len(q)
    toks = _i32(np.concatenate([_i32(q) for q in seqs]) if offs[-1] else np.zeros(0, np.int32))
    return toks, offs


def ts_drafter_create(schema):
    """schema: dict with token lists call_open, name_prefix, name_suffix, param_prefix, param_suffix,
    value_end, call_close, tools (list of token lists), params (per tool: list of token lists)."""
    keep = []

    def seq(name):
        a = _i32(schema[name])
        keep.append(a)
        return _ptr_i32(a), len(a)

    d = ts_schema_desc()
    for f in ("call_open", "name_prefix", "name_suffix", "param_prefix", "param_suffix", "value_end", "call_close"):
        p, n = seq(f)
        setattr(d, f, p)
        setattr(d, "n_" + f, n)
    tt, to = _pack(schema["tools"])
    first = np.zeros(len(schema["tools"]) + 1, np.int32)
    flat = []
    for i, ps in enumerate(schema["params"]):
        first[i + 1] = first[i] + len(ps)
        flat += list(ps)
    pt, po = _pack(flat)
    keep += [tt, to, first, pt, po]
    d.n_tools = len(schema["tools"])
    d.tool_tokens, d.tool_offsets, d.param_first = _ptr_i32(tt), _ptr_i32(to), _ptr_i32(first)
    d.param_tokens, d.param_offsets = _ptr_i32(pt), _ptr_i32(po)
    out = C.c_void_p()
    _check(load_library().ts_drafter_create(C.byref(d), C.byref(out)))
    return out


def ts_drafter_free(drafter):
    _check(load_library().ts_drafter_free(drafter))


def ts_drafter_retrieve(drafter, h_x, H, calls, k=10):
    """Returns the retrieved indices (most similar first)."""
    h = np.ascontiguousarray(h_x, np.float32)
    Hm = np.ascontiguousarray(H, np.float32).reshape(-1, h.shape[0])
    yt, yo = _pack(calls)
    top = np.zeros(max(k, 1), np.int32)
    fp = C.POINTER(C.c_float)
    _check(load_library().ts_drafter_retrieve(drafter, h.ctypes.data_as(fp), h.shape[0], Hm.ctypes.data_as(fp), Hm.shape[0],
                                              _ptr_i32(yt), _ptr_i32(yo), k, _ptr_i32(top)))
    return top[:min(k, Hm.shape[0])].tolist()


def ts_drafter_reset(drafter):
    _check(load_library().ts_drafter_reset(drafter))


def ts_drafter_append(drafter, tokens):
    t = _i32(tokens)
    _check(load_library().ts_drafter_append(drafter, _ptr_i32(t), len(t)))


def ts_drafter_state(drafter):
    """(state, tool, len(y))."""
    s, t, n = C.c_int32(), C.c_int32(), C.c_int32()
    _check(load_library().ts_drafter_state(drafter, C.byref(s), C.byref(t), C.byref(n)))
    return s.value, t.value, n.value


def ts_generate(model, kv, drafter, max_new_tokens, stop_token=-1):
    """The decoding loop of the method as one native call.  Returns (tokens, stats dict)."""
    out = np.zeros(max_new_tokens + TS_MAX_NODES + 1, np.int32)
    n = C.c_int32()
    st = ts_generate_stats()
    _check(load_library().ts_generate(model, kv, drafter, max_new_tokens, stop_token, _ptr_i32(out), C.byref(n), C.byref(st)))
    return out[:n.value].tolist(), {f: getattr(st, f) for f, _ in ts_generate_stats._fields_}


def ts_drafter_draft(drafter, max_nodes=TS_MAX_NODES):
    """(draft_tokens, parent_idx, source)."""
    toks = np.zeros(max(max_nodes, 1), np.int32)
    par = np.zeros(max(max_nodes, 1), np.int32)
    n, src = C.c_int32(), C.c_int32()
    _check(load_library().ts_drafter_draft(drafter, max_nodes, _ptr_i32(toks), _ptr_i32(par), C.byref(n), C.byref(src)))
    return toks[:n.value].copy(), par[:n.value].copy(), src.value
