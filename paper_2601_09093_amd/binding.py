"""Thin Python binding of libstep's C ABI (include/step.h): argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used purely as device memory; bf16 arrays may be torch.bfloat16
or their raw bit patterns as torch.int16/uint16.  Every call enqueues on torch's current stream and
returns without synchronising.  There is no CPU fallback: if libstep.so is missing or a tensor is not
on the GPU the call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libstep.so")
_lib = None

STEP_OK = 0
ERROR_NAMES = {
    0: "STEP_OK", 1: "STEP_EINVAL", 2: "STEP_EWORKSPACE", 3: "STEP_ELAUNCH", 16: "STEP_EPAGE",
    17: "STEP_ELEN", 18: "STEP_EINDEX", 19: "STEP_ENAN", 20: "STEP_EREFCOUNT", 21: "STEP_EKLIVE", 22: "STEP_EPLAN",
    23: "STEP_EFREELIST",
}
ACT_RELU, ACT_GELU = 0, 1


class StepError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %s" % (where, ERROR_NAMES.get(code, code)))


class AttnDims(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
                ("P", ctypes.c_int32), ("MAXB", ctypes.c_int32), ("NP", ctypes.c_int32), ("scale", ctypes.c_float)]


class ScoreDims(ctypes.Structure):
    _fields_ = [("R", ctypes.c_int32), ("d", ctypes.c_int32), ("m", ctypes.c_int32), ("B", ctypes.c_int32),
                ("N", ctypes.c_int32), ("act", ctypes.c_int32)]


def lib():
    """Load libstep.so (built in-tree by paper_2601_09093_amd.build); raise if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libstep.so not built: run `python -m paper_2601_09093_amd.build` "
                           "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    L.step_strerror.restype = ctypes.c_char_p
    L.step_strerror.argtypes = [ctypes.c_int]
    L.step_version.restype = ctypes.c_char_p
    L.step_attn_workspace_bytes.restype = sz
    L.step_attn_workspace_bytes.argtypes = [ctypes.POINTER(AttnDims)]
    L.step_attn_waves_per_head.restype = ctypes.c_int32
    L.step_attn_waves_per_head.argtypes = [ctypes.POINTER(AttnDims)]
    L.paged_decode_attn.restype = ctypes.c_int
    L.paged_decode_attn.argtypes = [ctypes.POINTER(AttnDims), vp, vp, vp, vp, vp, vp, vp, sz, vp, vp]
    L.step_attn_plan.restype = ctypes.c_int
    L.step_attn_plan.argtypes = [ctypes.POINTER(AttnDims), vp, vp, vp, sz, vp, vp]
    L.paged_decode_attn_planned.restype = ctypes.c_int
    L.paged_decode_attn_planned.argtypes = [ctypes.POINTER(AttnDims), vp, vp, vp, vp, vp, vp, vp, sz, vp, vp]
    L.step_score_workspace_bytes.restype = sz
    L.step_score_workspace_bytes.argtypes = [ctypes.POINTER(ScoreDims)]
    L.step_score.restype = ctypes.c_int
    L.step_score.argtypes = [ctypes.POINTER(ScoreDims)] + [vp] * 13 + [sz, vp, vp]
    L.step_prune_workspace_bytes.restype = sz
    L.step_prune_workspace_bytes.argtypes = [i32, i32, i32]
    L.prune_free.restype = ctypes.c_int
    L.prune_free.argtypes = [i32, i32, i32, i32, vp, i32] + [vp] * 7 + [sz, vp, vp]
    L.step_prune_static_max_pages.restype = i32
    L.step_prune_static_max_pages.argtypes = []
    L.prune_free_static.restype = ctypes.c_int
    L.prune_free_static.argtypes = [i32, i32, i32, i32, vp, i32] + [vp] * 6 + [vp, vp]
    L.step_reserve_workspace_bytes.restype = sz
    L.step_reserve_workspace_bytes.argtypes = [i32, i32, i32]
    L.step_freelist_rebuild.restype = ctypes.c_int
    L.step_freelist_rebuild.argtypes = [i32, vp, vp, sz, vp]
    L.step_freelist_add.restype = ctypes.c_int
    L.step_freelist_add.argtypes = [i32, vp, vp, i32, vp, sz, vp, vp]
    L.step_reserve_pages.restype = ctypes.c_int
    L.step_reserve_pages.argtypes = [i32, i32, i32, i32] + [vp] * 8 + [sz, vp, vp]
    L.step_append_kv.restype = ctypes.c_int
    L.step_append_kv.argtypes = [ctypes.POINTER(AttnDims)] + [vp] * 9
    L.step_weighted_vote.restype = ctypes.c_int
    L.step_weighted_vote.argtypes = [i32] + [vp] * 6
    L.step_calib_copy.restype = ctypes.c_int
    L.step_calib_copy.argtypes = [vp, vp, sz, vp]
    L.step_read_probe.restype = ctypes.c_int
    L.step_read_probe.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp]
    L.step_profile_begin.restype = ctypes.c_int
    L.step_profile_begin.argtypes = [ctypes.c_int]
    L.step_profile_end.restype = ctypes.c_int
    L.step_profile_end.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float), ctypes.c_int]
    L.step_profile_kernel_name.restype = ctypes.c_char_p
    L.step_profile_kernel_name.argtypes = [ctypes.c_int]
    _lib = L
    return L


_BF16_OK = (torch.bfloat16, torch.int16, torch.uint16)


def _dev(t, dtypes, name, allow_none=False):
    if t is None:
        if allow_none:
            return None
        raise TypeError("%s is required" % name)
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a GPU tensor (libstep has no CPU path)" % name)
    if t.dtype not in dtypes:
        raise TypeError("%s has dtype %s, expected one of %s" % (name, t.dtype, dtypes))
    if not t.is_contiguous():
        raise TypeError("%s must be contiguous" % name)
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def attn_dims(q, k_pages, block_tables, scale=None):
    N, Hq, D = q.shape
    NP, Hkv, P, _ = k_pages.shape
    return AttnDims(N, Hq, Hkv, D, P, block_tables.shape[1], NP, float(scale if scale is not None else D ** -0.5))


def attn_workspace_bytes(dims):
    return int(lib().step_attn_workspace_bytes(ctypes.byref(dims)))


def attn_waves_per_head(dims):
    return int(lib().step_attn_waves_per_head(ctypes.byref(dims)))


def new_workspace(nbytes, device):
    """A 256-byte aligned device buffer (torch's allocator aligns to at least 512 bytes)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def paged_decode_attn(q, k_pages, v_pages, block_tables, seq_lens, out=None, scale=None, workspace=None,
                      status=None):
    """out[N][Hq][D] (bf16) = attention of every trace's newest token over its paged KV cache."""
    dims = attn_dims(q, k_pages, block_tables, scale)
    if v_pages.shape != k_pages.shape or block_tables.shape[0] != dims.N or seq_lens.numel() != dims.N:
        raise ValueError("inconsistent shapes")
    if out is None:
        out = torch.empty_like(q)
    need = attn_workspace_bytes(dims)
    if workspace is None:
        workspace = new_workspace(need, q.device)
    rc = lib().paged_decode_attn(
        ctypes.byref(dims), _dev(q, _BF16_OK, "q"), _dev(k_pages, _BF16_OK, "k_pages"),
        _dev(v_pages, _BF16_OK, "v_pages"), _dev(block_tables, (torch.int32,), "block_tables"),
        _dev(seq_lens, (torch.int32,), "seq_lens"), _dev(out, _BF16_OK, "out"),
        _dev(workspace, (torch.uint8,), "workspace"), workspace.numel(),
        _dev(status, (torch.int32,), "status", True), _stream())
    if rc != STEP_OK:
        raise StepError(rc, "paged_decode_attn")
    return out


def attn_plan(q, k_pages, block_tables, seq_lens, workspace, scale=None, status=None):
    """Find the per-block shared-prefix lengths of one decode step into `workspace` (shared by all layers of the step)."""
    dims = attn_dims(q, k_pages, block_tables, scale)
    rc = lib().step_attn_plan(ctypes.byref(dims), _dev(block_tables, (torch.int32,), "block_tables"),
                              _dev(seq_lens, (torch.int32,), "seq_lens"), _dev(workspace, (torch.uint8,), "workspace"),
                              workspace.numel(), _dev(status, (torch.int32,), "status", True), _stream())
    if rc != STEP_OK:
        raise StepError(rc, "step_attn_plan")
    return dims


def paged_decode_attn_planned(q, k_pages, v_pages, block_tables, seq_lens, out, workspace, scale=None, status=None):
    """paged_decode_attn without the shared-prefix search; `workspace` holds what attn_plan found."""
    dims = attn_dims(q, k_pages, block_tables, scale)
    rc = lib().paged_decode_attn_planned(
        ctypes.byref(dims), _dev(q, _BF16_OK, "q"), _dev(k_pages, _BF16_OK, "k_pages"),
        _dev(v_pages, _BF16_OK, "v_pages"), _dev(block_tables, (torch.int32,), "block_tables"),
        _dev(seq_lens, (torch.int32,), "seq_lens"), _dev(out, _BF16_OK, "out"),
        _dev(workspace, (torch.uint8,), "workspace"), workspace.numel(),
        _dev(status, (torch.int32,), "status", True), _stream())
    if rc != STEP_OK:
        raise StepError(rc, "paged_decode_attn_planned")
    return out


def score_workspace_bytes(dims):
    return int(lib().step_score_workspace_bytes(ctypes.byref(dims)))


def step_score(hidden, boundary_idx, W1, b1, W2, b2, act=ACT_RELU, logits=None, probs=None, trace_of=None,
               score_sum=None, score_cnt=None, scores=None, workspace=None, status=None):
    """logits, probs [B] fp32; with trace_of also updates score_sum/score_cnt and writes scores [N]."""
    R, d = hidden.shape
    m = W1.shape[0]
    B = boundary_idx.numel()
    N = score_sum.numel() if score_sum is not None else 0
    dims = ScoreDims(R, d, m, B, N, int(act))
    dev = hidden.device
    if logits is None:
        logits = torch.empty(B, dtype=torch.float32, device=dev)
    if probs is None:
        probs = torch.empty(B, dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = new_workspace(score_workspace_bytes(dims), dev)
    f32, i32 = (torch.float32,), (torch.int32,)
    rc = lib().step_score(
        ctypes.byref(dims), _dev(hidden, _BF16_OK, "hidden"), _dev(boundary_idx, i32, "boundary_idx"),
        _dev(W1, _BF16_OK, "W1"), _dev(b1, f32, "b1"), _dev(W2, _BF16_OK, "W2"), _dev(b2, f32, "b2"),
        _dev(logits, f32, "logits"), _dev(probs, f32, "probs"), _dev(trace_of, i32, "trace_of", True),
        _dev(score_sum, f32, "score_sum", True), _dev(score_cnt, i32, "score_cnt", True),
        _dev(scores, f32, "scores", True), _dev(workspace, (torch.uint8,), "workspace"), workspace.numel(),
        _dev(status, i32, "status", True), _stream())
    if rc != STEP_OK:
        raise StepError(rc, "step_score")
    return logits, probs


def prune_workspace_bytes(N, MAXB, NP):
    return int(lib().step_prune_workspace_bytes(N, MAXB, NP))


def prune_free(scores, k, refcounts, block_tables, seq_lens, pruned=None, freed_pages=None, n_freed=None,
               workspace=None, status=None, P=16):
    """Prune the k lowest-scoring live traces in place; returns (pruned [k], freed_pages, n_freed [1])."""
    N, MAXB = block_tables.shape
    NP = refcounts.numel()
    dev = scores.device
    i32 = (torch.int32,)
    if pruned is None:
        pruned = torch.empty(max(k, 1), dtype=torch.int32, device=dev)
    if freed_pages is None:
        freed_pages = torch.empty(max(min(NP, max(k, 0) * MAXB), 1), dtype=torch.int32, device=dev)
    if n_freed is None:
        n_freed = torch.empty(1, dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = new_workspace(prune_workspace_bytes(N, MAXB, NP), dev)
    rc = lib().prune_free(
        N, MAXB, NP, int(P), _dev(scores, (torch.float32,), "scores"), int(k), _dev(refcounts, i32, "refcounts"),
        _dev(block_tables, i32, "block_tables"), _dev(seq_lens, i32, "seq_lens"), _dev(pruned, i32, "pruned"),
        _dev(freed_pages, i32, "freed_pages"), _dev(n_freed, i32, "n_freed"),
        _dev(workspace, (torch.uint8,), "workspace"), workspace.numel(), _dev(status, i32, "status", True), _stream())
    if rc != STEP_OK:
        raise StepError(rc, "prune_free")
    return pruned, freed_pages, n_freed


def prune_free_static(scores, k, refcounts, block_tables, seq_lens, pruned, freed_pages, n_freed, status=None, P=16):
    """prune_free with the library's own static scratch: no workspace, nothing allocated (outputs are the caller's)."""
    N, MAXB = block_tables.shape
    NP = refcounts.numel()
    i32 = (torch.int32,)
    rc = lib().prune_free_static(
        N, MAXB, NP, int(P), _dev(scores, (torch.float32,), "scores"), int(k), _dev(refcounts, i32, "refcounts"),
        _dev(block_tables, i32, "block_tables"), _dev(seq_lens, i32, "seq_lens"), _dev(pruned, i32, "pruned"),
        _dev(freed_pages, i32, "freed_pages"), _dev(n_freed, i32, "n_freed"), _dev(status, i32, "status", True),
        _stream())
    if rc != STEP_OK:
        raise StepError(rc, "prune_free_static")
    return pruned, freed_pages, n_freed


def reserve_workspace(refcounts, N=0, MAXB=0):
    """A workspace for reserve_pages with the free list of `refcounts` built in it."""
    ws = new_workspace(int(lib().step_reserve_workspace_bytes(N, MAXB, refcounts.numel())), refcounts.device)
    freelist_rebuild(refcounts, ws)
    return ws


def freelist_rebuild(refcounts, workspace):
    """(Re)build the free list of the reserve workspace from the reference counts."""
    rc = lib().step_freelist_rebuild(refcounts.numel(), _dev(refcounts, (torch.int32,), "refcounts"),
                                     _dev(workspace, (torch.uint8,), "workspace"), workspace.numel(), _stream())
    if rc != STEP_OK:
        raise StepError(rc, "step_freelist_rebuild")


def freelist_add(NP, freed_pages, n_freed, workspace, status=None):
    """Enter the pages a prune_free call freed into the free list of the reserve workspace."""
    i32 = (torch.int32,)
    rc = lib().step_freelist_add(int(NP), _dev(freed_pages, i32, "freed_pages"), _dev(n_freed, i32, "n_freed"),
                                 freed_pages.numel(), _dev(workspace, (torch.uint8,), "workspace"), workspace.numel(),
                                 _dev(status, i32, "status", True), _stream())
    if rc != STEP_OK:
        raise StepError(rc, "step_freelist_add")


def reserve_pages(scores, refcounts, block_tables, seq_lens, pruned=None, n_pruned=None, new_pages=None,
                  workspace=None, status=None, P=16):
    """Memory-triggered pruning + allocation in place; returns (pruned [N], n_pruned [1], new_pages [N]).
    `workspace` holds the free list from call to call (reserve_workspace); without one a fresh free list is
    built from refcounts for this call."""
    N, MAXB = block_tables.shape
    NP = refcounts.numel()
    dev = scores.device
    i32 = (torch.int32,)
    if pruned is None:
        pruned = torch.empty(max(N, 1), dtype=torch.int32, device=dev)
    if n_pruned is None:
        n_pruned = torch.empty(1, dtype=torch.int32, device=dev)
    if new_pages is None:
        new_pages = torch.empty(max(N, 1), dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = reserve_workspace(refcounts, N, MAXB)
    rc = lib().step_reserve_pages(
        N, MAXB, NP, int(P), _dev(scores, (torch.float32,), "scores"), _dev(refcounts, i32, "refcounts"),
        _dev(block_tables, i32, "block_tables"), _dev(seq_lens, i32, "seq_lens"), _dev(pruned, i32, "pruned"),
        _dev(n_pruned, i32, "n_pruned"), _dev(new_pages, i32, "new_pages"),
        _dev(workspace, (torch.uint8,), "workspace"), workspace.numel(), _dev(status, i32, "status", True), _stream())
    if rc != STEP_OK:
        raise StepError(rc, "step_reserve_pages")
    return pruned, n_pruned, new_pages


def append_kv(k_new, v_new, k_pages, v_pages, block_tables, seq_lens, refcounts=None, status=None):
    """Write the newest token's K/V rows of every live trace into its page; seq_lens += 1 (in place)."""
    N, Hkv, D = k_new.shape
    NP, _, P, _ = k_pages.shape
    dims = AttnDims(N, Hkv, Hkv, D, P, block_tables.shape[1], NP, 1.0)
    i32 = (torch.int32,)
    rc = lib().step_append_kv(
        ctypes.byref(dims), _dev(k_new, _BF16_OK, "k_new"), _dev(v_new, _BF16_OK, "v_new"),
        _dev(k_pages, _BF16_OK, "k_pages"), _dev(v_pages, _BF16_OK, "v_pages"),
        _dev(block_tables, i32, "block_tables"), _dev(refcounts, i32, "refcounts", True),
        _dev(seq_lens, i32, "seq_lens"), _dev(status, i32, "status", True), _stream())
    if rc != STEP_OK:
        raise StepError(rc, "step_append_kv")


def weighted_vote(answer, scores, status=None):
    """Returns (winner [1] int32, weight [1] fp32) device tensors."""
    dev = scores.device
    winner = torch.empty(1, dtype=torch.int32, device=dev)
    weight = torch.empty(1, dtype=torch.float32, device=dev)
    rc = lib().step_weighted_vote(
        answer.numel(), _dev(answer, (torch.int32,), "answer"), _dev(scores, (torch.float32,), "scores"),
        _dev(winner, (torch.int32,), "winner"), _dev(weight, (torch.float32,), "weight"),
        _dev(status, (torch.int32,), "status", True), _stream())
    if rc != STEP_OK:
        raise StepError(rc, "step_weighted_vote")
    return winner, weight


def calib_copy(dst, src):
    """dst <- src with libstep's plain copy kernel (profiler byte-counter calibration)."""
    nbytes = src.numel() * src.element_size()
    rc = lib().step_calib_copy(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()), nbytes, _stream())
    if rc != STEP_OK:
        raise StepError(rc, "step_calib_copy")
    return dst


def read_probe(k_pages, v_pages, page_ids, waves, pages_per_wave, pattern, nontemporal, sink):
    """Bare read of the K/V tiles of the listed pages by `waves` x Hkv waves (measurement aid)."""
    NP, Hkv, P, D = k_pages.shape
    if (P, D) != (16, 128) or page_ids.numel() < waves * pages_per_wave:
        raise ValueError("read_probe wants [NP][Hkv][16][128] pools and waves * pages_per_wave page ids")
    rc = lib().step_read_probe(_dev(k_pages, _BF16_OK, "k_pages"), _dev(v_pages, _BF16_OK, "v_pages"),
                               _dev(page_ids, (torch.int32,), "page_ids"), int(waves), int(pages_per_wave), Hkv, NP,
                               int(pattern), int(bool(nontemporal)), _dev(sink, (torch.int32,), "sink"), _stream())
    if rc != STEP_OK:
        raise StepError(rc, "step_read_probe")


def profile_begin(cap):
    """Attach HIP events to each of the next `cap` kernel launches of the library (benchmarks only)."""
    rc = lib().step_profile_begin(int(cap))
    if rc != STEP_OK:
        raise StepError(rc, "step_profile_begin")


def profile_end(cap):
    """[(kernel name, milliseconds)] of the launches timed since profile_begin, in launch order."""
    ids = (ctypes.c_int32 * int(cap))()
    ms = (ctypes.c_float * int(cap))()
    n = lib().step_profile_end(ids, ms, int(cap))
    if n < 0:
        raise StepError(-n, "step_profile_end")
    return [(lib().step_profile_kernel_name(int(ids[i])).decode(), float(ms[i])) for i in range(n)]
