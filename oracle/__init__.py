"""ctypes binding of the C oracle (oracle/step_oracle.c).

TEST INFRASTRUCTURE ONLY.  May be imported by tests/, __graft_entry__.smoke()
and bench.py's cpu_baseline leg; the product package never imports it and it
never imports the product package.

bf16 arrays are numpy uint16 arrays holding the raw bit patterns.
Every function raises OracleError on the conditions the C code reports.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libstep_oracle.so")
_lib = None

ERRORS = {1: "EINVAL", 2: "EPAGE", 3: "ELEN", 4: "EINDEX", 5: "ENAN", 6: "EREFCOUNT"}


class OracleError(RuntimeError):
    def __init__(self, code):
        self.code = code
        self.name = ERRORS.get(code, "E%d" % code)
        super().__init__("oracle error %s" % self.name)


def _load():
    global _lib
    if _lib is not None:
        return _lib
    src = os.path.join(_HERE, "step_oracle.c")
    if not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        import importlib.util
        spec = importlib.util.spec_from_file_location("_oracle_build", os.path.join(_HERE, "build.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        mod.build(force=True)
    _lib = ctypes.CDLL(_LIB_PATH)
    return _lib


def _p(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype)) if a is not None else None


def _chk(a, dtype, name):
    if not (isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"]):
        raise TypeError("%s must be a C-contiguous numpy array of %s" % (name, np.dtype(dtype)))
    return a


def num_threads():
    return int(_load().oracle_num_threads())


def paged_decode_attn(q, k_pages, v_pages, block_tables, seq_lens, scale=None, rows=None, return_lse=False):
    """q [N][Hq][D] u16(bf16); k_pages, v_pages [NP][Hkv][P][D] u16; block_tables [N][MAXB] i32;
    seq_lens [N] i32.  Returns float64 out [N][Hq][D] (or [n_sel][D] when rows=(traces, heads))."""
    lib = _load()
    _chk(q, np.uint16, "q"); _chk(k_pages, np.uint16, "k_pages"); _chk(v_pages, np.uint16, "v_pages")
    _chk(block_tables, np.int32, "block_tables"); _chk(seq_lens, np.int32, "seq_lens")
    N, Hq, D = q.shape
    NP, Hkv, P, D2 = k_pages.shape
    assert D2 == D and v_pages.shape == k_pages.shape
    assert block_tables.shape[0] == N and seq_lens.shape == (N,)
    MAXB = block_tables.shape[1]
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    i32, u16, f64 = ctypes.c_int32, ctypes.c_uint16, ctypes.c_double
    if rows is None:
        out = np.zeros((N, Hq, D), np.float64)
        lse = np.zeros((N, Hq), np.float64)
        rc = lib.oracle_paged_decode_attn(
            N, Hq, Hkv, D, P, MAXB, NP, f64(scale), _p(q, u16), _p(k_pages, u16), _p(v_pages, u16),
            _p(block_tables, i32), _p(seq_lens, i32), _p(out, f64), _p(lse, f64))
    else:
        st = np.ascontiguousarray(rows[0], np.int32)
        sh = np.ascontiguousarray(rows[1], np.int32)
        assert st.shape == sh.shape and st.ndim == 1
        out = np.zeros((st.size, D), np.float64)
        lse = np.zeros((st.size,), np.float64)
        rc = lib.oracle_paged_decode_attn_rows(
            N, Hq, Hkv, D, P, MAXB, NP, f64(scale), _p(q, u16), _p(k_pages, u16), _p(v_pages, u16),
            _p(block_tables, i32), _p(seq_lens, i32), st.size, _p(st, i32), _p(sh, i32), _p(out, f64), _p(lse, f64))
    if rc:
        raise OracleError(rc)
    return (out, lse) if return_lse else out


def step_score(hidden, boundary_idx, W1, b1, W2, b2, act=0):
    """hidden [R][d] u16; boundary_idx [B] i32; W1 [m][d] u16; b1 [m] f32; W2 [m] u16; b2 float.
    Returns (logits, probs) float64 [B]."""
    lib = _load()
    _chk(hidden, np.uint16, "hidden"); _chk(boundary_idx, np.int32, "boundary_idx")
    _chk(W1, np.uint16, "W1"); _chk(b1, np.float32, "b1"); _chk(W2, np.uint16, "W2")
    R, d = hidden.shape
    m, d2 = W1.shape
    assert d2 == d and b1.shape == (m,) and W2.shape == (m,)
    B = boundary_idx.shape[0]
    logits = np.zeros(B, np.float64)
    probs = np.zeros(B, np.float64)
    rc = lib.oracle_step_score(
        R, d, m, B, int(act), _p(hidden, ctypes.c_uint16), _p(boundary_idx, ctypes.c_int32),
        _p(W1, ctypes.c_uint16), _p(b1, ctypes.c_float), _p(W2, ctypes.c_uint16), ctypes.c_float(float(b2)),
        _p(logits, ctypes.c_double), _p(probs, ctypes.c_double))
    if rc:
        raise OracleError(rc)
    return logits, probs


def running_mean(trace_of, probs, score_sum, score_cnt):
    """In-place update of score_sum (f32 [N]) and score_cnt (i32 [N]) with probs (f32 [B]) taken in
    index order; returns scores f32 [N] (+inf where cnt == 0)."""
    lib = _load()
    _chk(trace_of, np.int32, "trace_of"); _chk(probs, np.float32, "probs")
    _chk(score_sum, np.float32, "score_sum"); _chk(score_cnt, np.int32, "score_cnt")
    N = score_sum.shape[0]
    scores = np.zeros(N, np.float32)
    rc = lib.oracle_running_mean(
        trace_of.shape[0], N, _p(trace_of, ctypes.c_int32), _p(probs, ctypes.c_float),
        _p(score_sum, ctypes.c_float), _p(score_cnt, ctypes.c_int32), _p(scores, ctypes.c_float))
    if rc:
        raise OracleError(rc)
    return scores


def prune_free(scores, k, refcounts, block_tables, seq_lens, P=16):
    """In place on refcounts [NP], block_tables [N][MAXB], seq_lens [N] (all i32).
    Returns (pruned [k] i32 in pruning order, freed_pages i32 ascending)."""
    lib = _load()
    _chk(scores, np.float32, "scores"); _chk(refcounts, np.int32, "refcounts")
    _chk(block_tables, np.int32, "block_tables"); _chk(seq_lens, np.int32, "seq_lens")
    N, MAXB = block_tables.shape
    NP = refcounts.shape[0]
    assert scores.shape == (N,) and seq_lens.shape == (N,)
    pruned = np.full(max(k, 0), -1, np.int32)
    freed = np.full(NP, -1, np.int32)
    nf = ctypes.c_int32(0)
    rc = lib.oracle_prune_free(
        N, MAXB, NP, int(P), _p(scores, ctypes.c_float), int(k), _p(refcounts, ctypes.c_int32),
        _p(block_tables, ctypes.c_int32), _p(seq_lens, ctypes.c_int32), _p(pruned, ctypes.c_int32),
        _p(freed, ctypes.c_int32), ctypes.byref(nf))
    if rc:
        raise OracleError(rc)
    return pruned, freed[: nf.value].copy()


def reserve_pages(scores, refcounts, block_tables, seq_lens, P=16):
    """In place on refcounts, block_tables, seq_lens.  Returns (pruned i32 in pruning order,
    new_pages [N] i32: page given to each trace or -1)."""
    lib = _load()
    _chk(scores, np.float32, "scores"); _chk(refcounts, np.int32, "refcounts")
    _chk(block_tables, np.int32, "block_tables"); _chk(seq_lens, np.int32, "seq_lens")
    N, MAXB = block_tables.shape
    NP = refcounts.shape[0]
    pruned = np.full(max(N, 1), -1, np.int32)
    new_pages = np.full(max(N, 1), -1, np.int32)
    n = ctypes.c_int32(0)
    rc = lib.oracle_reserve_pages(
        N, MAXB, NP, int(P), _p(scores, ctypes.c_float), _p(refcounts, ctypes.c_int32),
        _p(block_tables, ctypes.c_int32), _p(seq_lens, ctypes.c_int32), _p(pruned, ctypes.c_int32),
        ctypes.byref(n), _p(new_pages, ctypes.c_int32))
    if rc:
        raise OracleError(rc)
    return pruned[: n.value].copy(), new_pages[:N].copy()


def append_kv(k_new, v_new, k_pages, v_pages, block_tables, refcounts, seq_lens):
    """Writes row L_i of every live trace into its page (in place on k_pages, v_pages) and adds 1 to
    seq_lens.  k_new, v_new: [N][Hkv][D] u16."""
    lib = _load()
    _chk(k_new, np.uint16, "k_new"); _chk(v_new, np.uint16, "v_new")
    _chk(k_pages, np.uint16, "k_pages"); _chk(v_pages, np.uint16, "v_pages")
    _chk(block_tables, np.int32, "block_tables"); _chk(seq_lens, np.int32, "seq_lens")
    if refcounts is not None:
        _chk(refcounts, np.int32, "refcounts")
    N, Hkv, D = k_new.shape
    NP, Hkv2, P, D2 = k_pages.shape
    assert (Hkv2, D2) == (Hkv, D) and v_new.shape == k_new.shape and v_pages.shape == k_pages.shape
    MAXB = block_tables.shape[1]
    u16, i32 = ctypes.c_uint16, ctypes.c_int32
    rc = lib.oracle_append_kv(N, Hkv, D, P, MAXB, NP, _p(k_new, u16), _p(v_new, u16), _p(k_pages, u16),
                              _p(v_pages, u16), _p(block_tables, i32), _p(refcounts, i32), _p(seq_lens, i32))
    if rc:
        raise OracleError(rc)


def weighted_vote(answer, scores):
    """answer [N] i32 (-1: no answer), scores [N] f32.  Returns (winner, weight)."""
    lib = _load()
    _chk(answer, np.int32, "answer"); _chk(scores, np.float32, "scores")
    w = ctypes.c_int32(-1)
    wt = ctypes.c_float(0.0)
    rc = lib.oracle_weighted_vote(answer.shape[0], _p(answer, ctypes.c_int32), _p(scores, ctypes.c_float),
                                  ctypes.byref(w), ctypes.byref(wt))
    if rc:
        raise OracleError(rc)
    return int(w.value), float(wt.value)
