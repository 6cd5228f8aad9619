"""prune_free_static (the entry point that allocates nothing: its scratch is a device array inside the
library) against prune_free, through the C ABI, bit for bit: two calls in a row on one stream, the
second on a smaller problem, each in the three-kernel path that actually uses the scratch; then a small
problem (single-kernel path) and the size limit."""
import numpy as np
import pytest
import torch

from paper_2601_09093_amd import binding, workloads as wl
from tests.gpu_util import DEV, dev, new_status

pytestmark = pytest.mark.gpu
P = 16


def _case(seed, N, lo, hi, prompt, slack):
    lens = wl.rng_for(seed, 0).integers(lo, hi + 1, N)
    lens[:: 9] = 0
    lay = wl.build_layout(lens, prompt, P, wl.rng_for(seed, 1), slack=slack)
    scores = wl.rng_for(seed, 2).random(N).astype(np.float32)
    scores[3] = scores[5]
    return lay, scores


def _run(fn, lay, scores, k, **kw):
    st = new_status()
    rc, bt, sl = dev(lay.refcounts.copy()), dev(lay.block_tables.copy()), dev(lay.seq_lens.copy())
    pruned = torch.full((max(k, 1),), -7, dtype=torch.int32, device=DEV)
    freed = torch.full((max(min(lay.NP, k * lay.MAXB), 1),), -7, dtype=torch.int32, device=DEV)
    nf = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    fn(dev(scores), k, rc, bt, sl, pruned=pruned, freed_pages=freed, n_freed=nf, status=st, **kw)
    return st, pruned, freed, nf, rc, bt, sl


def _same(a, b, k):
    torch.cuda.synchronize()
    assert int(a[0].item()) == 0 and int(b[0].item()) == 0
    n = int(a[3].item())
    assert n == int(b[3].item()) and n > 0
    assert torch.equal(a[1][:k], b[1][:k]) and torch.equal(a[2][:n], b[2][:n])
    for x, y in zip(a[4:], b[4:]):
        assert torch.equal(x, y)


def test_static_scratch_matches_prune_free_on_two_calls_in_a_row():
    big, big_scores = _case(4100, 200, 3000, 9000, 1024, 1.3)       # k * MAXB far above the one-kernel limit
    small, small_scores = _case(4101, 48, 3400, 4000, 256, 1.1)     # fewer traces, a smaller pool: fewer bitmap words
    assert small.NP < big.NP // 4 and 40 * big.MAXB > 8192 and 36 * small.MAXB > 8192
    assert big.NP <= binding.lib().step_prune_static_max_pages()
    want_big = _run(binding.prune_free, big, big_scores, 40)
    want_small = _run(binding.prune_free, small, small_scores, 36)
    torch.cuda.synchronize()
    mem0 = torch.cuda.memory_allocated()
    got_big = _run(binding.prune_free_static, big, big_scores, 40)   # no synchronisation between the two calls
    got_small = _run(binding.prune_free_static, small, small_scores, 36)
    _same(got_big, want_big, 40)
    _same(got_small, want_small, 36)
    assert torch.cuda.memory_allocated() >= mem0                    # (outputs of _run only; the call itself takes no workspace)
    # and once more the large one after the small one: nothing of the smaller call is left in the way
    _same(_run(binding.prune_free_static, big, big_scores, 40), want_big, 40)


def test_static_scratch_small_problem_and_size_limit():
    lay, scores = _case(4102, 12, 100, 400, 64, 1.2)                # single-kernel path
    _same(_run(binding.prune_free_static, lay, scores, 3), _run(binding.prune_free, lay, scores, 3), 3)
    L = binding.lib()
    too_many = L.step_prune_static_max_pages() + 1
    one = torch.zeros(1, dtype=torch.int32, device=DEV)
    rc = L.prune_free_static(1, 1, too_many, 16, torch.zeros(1, device=DEV).data_ptr(), 0, one.data_ptr(), one.data_ptr(),
                             one.data_ptr(), one.data_ptr(), one.data_ptr(), one.data_ptr(), None, None)
    assert rc == 2                                                  # STEP_EWORKSPACE, nothing enqueued
