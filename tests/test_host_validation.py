"""Host-side argument checks of the C ABI, exercised without a GPU: every call below is rejected by
the host code before anything is enqueued, so the (fake, never dereferenced) pointers are only ever
compared with NULL and tested for alignment."""
import ctypes

import pytest
import torch

from paper_2601_09093_amd import binding

# With a GPU present a check that wrongly passed would enqueue a kernel on fake pointers: this file is
# for the CPU-only run, where such a regression shows up as STEP_ELAUNCH instead.
pytestmark = pytest.mark.skipif(torch.cuda.is_available(), reason="host-only checks run where no GPU is visible")

OK, EINVAL, EWORKSPACE = 0, 1, 2
A = 0x10000000          # a 256-byte aligned non-NULL address
ODD = A + 2             # misaligned for 16-byte loads


@pytest.fixture(scope="module")
def L():
    return binding.lib()


def vp(x):
    return ctypes.c_void_p(x)


def attn(L, dims, q=A, k=A, v=A, bt=A, sl=A, out=A, ws=A, ws_bytes=1 << 40, fn="paged_decode_attn"):
    return getattr(L, fn)(ctypes.byref(dims), vp(q), vp(k), vp(v), vp(bt), vp(sl), vp(out), vp(ws), ws_bytes, None, None)


def test_attention_rejects_bad_dims_and_pointers(L):
    good = binding.AttnDims(64, 32, 8, 128, 16, 2112, 100000, 0.088)
    need = binding.attn_workspace_bytes(good)
    assert need > 0
    for bad in (binding.AttnDims(64, 32, 8, 96, 16, 2112, 100000, 0.1),      # head dim
                binding.AttnDims(64, 32, 8, 128, 32, 2112, 100000, 0.1),     # page size
                binding.AttnDims(64, 30, 8, 128, 16, 2112, 100000, 0.1),     # Hq % Hkv
                binding.AttnDims(64, 24, 8, 128, 16, 2112, 100000, 0.1),     # group size 3
                binding.AttnDims(4096, 32, 8, 128, 16, 2112, 100000, 0.1),   # more traces than a call takes
                binding.AttnDims(-1, 32, 8, 128, 16, 2112, 100000, 0.1),
                binding.AttnDims(64, 32, 8, 128, 16, -5, 100000, 0.1)):
        assert binding.attn_workspace_bytes(bad) == 0 and binding.attn_waves_per_head(bad) == 0
        for fn in ("paged_decode_attn", "paged_decode_attn_planned"):
            assert attn(L, bad, fn=fn) == EINVAL
        assert L.step_attn_plan(ctypes.byref(bad), vp(A), vp(A), vp(A), 1 << 40, None, None) == EINVAL
    for fn in ("paged_decode_attn", "paged_decode_attn_planned"):
        assert attn(L, good, q=0, fn=fn) == EINVAL
        assert attn(L, good, k=0, fn=fn) == EINVAL
        assert attn(L, good, v=0, fn=fn) == EINVAL
        assert attn(L, good, out=0, fn=fn) == EINVAL
        assert attn(L, good, bt=0, fn=fn) == EINVAL
        assert attn(L, good, sl=0, fn=fn) == EINVAL
        assert attn(L, good, q=ODD, fn=fn) == EINVAL
        assert attn(L, good, k=ODD, fn=fn) == EINVAL
        assert attn(L, good, ws=0, fn=fn) == EWORKSPACE
        assert attn(L, good, ws=A + 16, fn=fn) == EWORKSPACE          # workspace must be 256-byte aligned
        assert attn(L, good, ws_bytes=need - 1, fn=fn) == EWORKSPACE
    assert L.step_attn_plan(ctypes.byref(good), vp(A), vp(A), vp(A), need - 1, None, None) == EWORKSPACE
    assert L.step_attn_plan(ctypes.byref(good), vp(0), vp(A), vp(A), need, None, None) == EINVAL
    # N = 0 is a no-op that needs nothing
    empty = binding.AttnDims(0, 32, 8, 128, 16, 2112, 100000, 0.1)
    assert attn(L, empty, q=0, k=0, v=0, bt=0, sl=0, out=0, ws=0, ws_bytes=0) == OK


def score(L, dims, hidden=A, bidx=A, W1=A, b1=A, W2=A, b2=A, logits=A, probs=A, trace_of=A, ssum=A, cnt=A, scores=A,
          ws=A, ws_bytes=1 << 40):
    return L.step_score(ctypes.byref(dims), vp(hidden), vp(bidx), vp(W1), vp(b1), vp(W2), vp(b2), vp(logits), vp(probs),
                        vp(trace_of), vp(ssum), vp(cnt), vp(scores), vp(ws), ws_bytes, None, None)


def test_scorer_rejects_bad_dims_and_pointers(L):
    good = binding.ScoreDims(64, 4096, 1024, 4, 64, 0)
    need = binding.score_workspace_bytes(good)
    assert need >= 4 * (1024 // 16) * 4
    for bad in (binding.ScoreDims(64, 4000, 1024, 4, 64, 0),      # d % 128
                binding.ScoreDims(64, 4096, 1000, 4, 64, 0),      # m % 16
                binding.ScoreDims(64, 4096, 1024, -1, 64, 0),
                binding.ScoreDims(64, 4096, 1024, 4, 64, 7)):     # unknown activation
        assert binding.score_workspace_bytes(bad) == 0 and score(L, bad) == EINVAL
    assert score(L, good, W1=0) == EINVAL and score(L, good, b2=0) == EINVAL
    assert score(L, good, hidden=0) == EINVAL and score(L, good, logits=0) == EINVAL
    assert score(L, good, hidden=ODD) == EINVAL and score(L, good, W1=ODD) == EINVAL
    assert score(L, good, cnt=0) == EINVAL                        # state needs both arrays
    assert score(L, good, trace_of=0) == EINVAL                   # and the owner of every boundary
    assert score(L, good, ssum=0) == EINVAL                       # no state, but count and scores given
    assert score(L, good, ws=0) == EWORKSPACE and score(L, good, ws=A + 64) == EWORKSPACE
    assert score(L, good, ws_bytes=need - 1) == EWORKSPACE
    assert score(L, binding.ScoreDims(64, 4096, 1024, 4, 0, 0)) == EINVAL   # state arrays with N = 0


def prune(L, N=64, MAXB=100, NP=5000, P=16, scores=A, k=1, rc=A, bt=A, sl=A, pruned=A, freed=A, nf=A, ws=A, ws_bytes=1 << 40):
    return L.prune_free(N, MAXB, NP, P, vp(scores), k, vp(rc), vp(bt), vp(sl), vp(pruned), vp(freed), vp(nf), vp(ws),
                        ws_bytes, None, None)


def test_prune_and_engine_calls_reject_bad_arguments(L):
    need = binding.prune_workspace_bytes(64, 100, 5000)
    assert need >= 256 + 5000 // 8
    assert prune(L, N=-1) == EINVAL and prune(L, N=5000) == EINVAL and prune(L, k=65) == EINVAL and prune(L, k=-1) == EINVAL
    assert prune(L, P=0) == EINVAL and prune(L, NP=-1) == EINVAL and prune(L, nf=0) == EINVAL
    assert prune(L, scores=0) == EINVAL and prune(L, rc=0) == EINVAL and prune(L, pruned=0) == EINVAL
    assert prune(L, ws=0) == EWORKSPACE and prune(L, ws=A + 128) == EWORKSPACE and prune(L, ws_bytes=need - 1) == EWORKSPACE
    rneed = int(L.step_reserve_workspace_bytes(64, 100, 5000))
    assert rneed > 0

    def reserve(N=64, MAXB=100, NP=5000, P=16, scores=A, rc=A, bt=A, sl=A, pruned=A, n_pruned=A, new_pages=A, ws=A,
                ws_bytes=1 << 40):
        return L.step_reserve_pages(N, MAXB, NP, P, vp(scores), vp(rc), vp(bt), vp(sl), vp(pruned), vp(n_pruned),
                                    vp(new_pages), vp(ws), ws_bytes, None, None)
    assert reserve(N=-1) == EINVAL and reserve(N=5000) == EINVAL and reserve(P=0) == EINVAL
    assert reserve(scores=0) == EINVAL and reserve(n_pruned=0) == EINVAL and reserve(new_pages=0) == EINVAL
    assert reserve(ws=0) == EWORKSPACE and reserve(ws_bytes=rneed - 1) == EWORKSPACE

    dims = binding.AttnDims(64, 8, 8, 128, 16, 2112, 100000, 1.0)

    def append(d=dims, kn=A, vn=A, k=A, v=A, bt=A, rc=A, sl=A):
        return L.step_append_kv(ctypes.byref(d), vp(kn), vp(vn), vp(k), vp(v), vp(bt), vp(rc), vp(sl), None, None)
    assert append(d=binding.AttnDims(64, 8, 8, 100, 16, 2112, 100000, 1.0)) == EINVAL      # D must be a multiple of 8
    assert append(d=binding.AttnDims(64, 8, 8, 128, 32, 2112, 100000, 1.0)) == EINVAL      # page size
    assert append(kn=0) == EINVAL and append(v=0) == EINVAL and append(bt=0) == EINVAL and append(sl=0) == EINVAL
    assert append(kn=ODD) == EINVAL and append(k=ODD) == EINVAL
    assert L.step_weighted_vote(-1, vp(A), vp(A), vp(A), vp(A), None, None) == EINVAL
    assert L.step_weighted_vote(8, vp(0), vp(A), vp(A), vp(A), None, None) == EINVAL
    assert L.step_weighted_vote(8, vp(A), vp(A), vp(0), vp(A), None, None) == EINVAL


def test_free_list_static_prune_and_measurement_aids_reject_bad_arguments(L):
    rneed = int(L.step_reserve_workspace_bytes(0, 0, 5000))
    assert rneed >= 256 + 5000 // 8
    assert L.step_freelist_rebuild(-1, vp(A), vp(A), rneed, None) == EINVAL
    assert L.step_freelist_rebuild(5000, vp(0), vp(A), rneed, None) == EINVAL
    assert L.step_freelist_rebuild(5000, vp(A), vp(0), rneed, None) == EWORKSPACE
    assert L.step_freelist_rebuild(5000, vp(A), vp(A + 64), rneed, None) == EWORKSPACE
    assert L.step_freelist_rebuild(5000, vp(A), vp(A), rneed - 1, None) == EWORKSPACE
    assert L.step_freelist_add(5000, vp(A), vp(0), 10, vp(A), rneed, None, None) == EINVAL      # n_freed is required
    assert L.step_freelist_add(5000, vp(0), vp(A), 10, vp(A), rneed, None, None) == EINVAL
    assert L.step_freelist_add(5000, vp(A), vp(A), -1, vp(A), rneed, None, None) == EINVAL
    assert L.step_freelist_add(5000, vp(A), vp(A), 10, vp(A), rneed - 1, None, None) == EWORKSPACE

    def static(N=64, MAXB=100, NP=5000, P=16, scores=A, k=1, rc=A, bt=A, sl=A, pruned=A, freed=A, nf=A):
        return L.prune_free_static(N, MAXB, NP, P, vp(scores), k, vp(rc), vp(bt), vp(sl), vp(pruned), vp(freed), vp(nf),
                                   None, None)
    assert static(N=-1) == EINVAL and static(k=65) == EINVAL and static(nf=0) == EINVAL and static(rc=0) == EINVAL
    assert static(P=0) == EINVAL and static(pruned=0) == EINVAL
    assert static(NP=L.step_prune_static_max_pages() + 1) == EWORKSPACE        # larger than the static bitmap covers

    probe = L.step_read_probe
    assert probe(vp(0), vp(A), vp(A), 128, 10, 8, 1000, 0, 1, vp(A), None) == EINVAL
    assert probe(vp(A), vp(A), vp(0), 128, 10, 8, 1000, 0, 1, vp(A), None) == EINVAL
    assert probe(vp(A), vp(A), vp(A), 0, 10, 8, 1000, 0, 1, vp(A), None) == EINVAL
    assert probe(vp(A), vp(A), vp(A), 128, 10, 8, 1000, 2, 1, vp(A), None) == EINVAL       # unknown load pattern
    assert probe(vp(ODD), vp(A), vp(A), 128, 10, 8, 1000, 0, 1, vp(A), None) == EINVAL
    assert L.step_profile_begin(0) == EINVAL
    ids = (ctypes.c_int32 * 4)(); ms = (ctypes.c_float * 4)()
    assert L.step_profile_end(ids, ms, 4) == -EINVAL                                       # no session open
    assert L.step_profile_kernel_name(2) == b"attn_partial" and L.step_profile_kernel_name(999) == b"unknown"
    assert b"STEP_EFREELIST" in L.step_strerror(23)
    assert binding.score_workspace_bytes(binding.ScoreDims(64, 4096, 16 * 1025, 4, 64, 0)) == 0    # m above 16384

