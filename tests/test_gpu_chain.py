"""One whole decode step on the GPU -- attention, scorer, running mean, prune -- against the oracle
chain (the memory-saturated pruning step of config 5, scaled down, and the tiny config 1)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_09093_amd import binding, workloads as wl
from tests.gpu_util import DEV, dev, dev_bits, host_f32_of_bf16, new_status

pytestmark = pytest.mark.gpu
P = 16


def gpu_step(w, k):
    lay, s = w.layout, w.scorer
    st = new_status()
    bt, sl, rc = dev(lay.block_tables), dev(lay.seq_lens), dev(lay.refcounts)
    out = binding.paged_decode_attn(dev_bits(w.q), dev_bits(w.k_pages), dev_bits(w.v_pages), bt, sl, status=st)
    ssum, cnt = dev(s.score_sum), dev(s.score_cnt)
    scores = torch.empty(w.shape.N, dtype=torch.float32, device=DEV)
    logits, probs = binding.step_score(dev_bits(s.hidden), dev(s.boundary_idx), dev_bits(s.W1), dev(s.b1),
                                       dev_bits(s.W2), torch.tensor([s.b2], dtype=torch.float32, device=DEV),
                                       act=s.act, trace_of=dev(s.trace_of), score_sum=ssum, score_cnt=cnt,
                                       scores=scores, status=st)
    pruned, freed, nf = binding.prune_free(scores, k, rc, bt, sl, status=st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    return dict(out=host_f32_of_bf16(out), logits=logits.cpu().numpy(), probs=probs.cpu().numpy(),
                scores=scores.cpu().numpy(), sum=ssum.cpu().numpy(), cnt=cnt.cpu().numpy(),
                pruned=pruned.cpu().numpy()[:k], freed=freed.cpu().numpy()[: int(nf.item())],
                rc=rc.cpu().numpy(), bt=bt.cpu().numpy(), sl=sl.cpu().numpy())


def oracle_step(w, k, probs_f32=None):
    lay, s = w.layout, w.scorer
    out = oracle.paged_decode_attn(w.q, w.k_pages, w.v_pages, lay.block_tables, lay.seq_lens)
    logits, probs = oracle.step_score(s.hidden, s.boundary_idx, s.W1, s.b1, s.W2, s.b2, act=s.act)
    ssum, cnt = s.score_sum.copy(), s.score_cnt.copy()
    scores = oracle.running_mean(s.trace_of, probs.astype(np.float32) if probs_f32 is None else probs_f32, ssum, cnt)
    rc, bt, sl = lay.refcounts.copy(), lay.block_tables.copy(), lay.seq_lens.copy()
    pruned, freed = oracle.prune_free(scores, k, rc, bt, sl, P)
    return dict(out=out, logits=logits, probs=probs, scores=scores, sum=ssum, cnt=cnt, pruned=pruned, freed=freed,
                rc=rc, bt=bt, sl=sl)


def compare(g, o_same_bytes, o_indep, k):
    assert np.abs(g["out"] - o_indep["out"]).max() <= 2e-2
    assert np.abs(g["logits"] - o_indep["logits"]).max() <= 1e-3
    # (i) prune parity on identical score bytes: everything integer is bit-exact
    for key in ("scores", "sum", "cnt", "pruned", "freed", "rc", "bt", "sl"):
        assert np.array_equal(g[key], o_same_bytes[key]), key
    # (ii) the fully independent chain picks the same set when the k / k+1 score gap is wide enough
    live = o_indep["sl"] > 0
    order = np.sort(o_indep["scores"][np.isfinite(o_indep["scores"])])
    return order


def test_config1_whole_step():
    w = wl.make_workload(1, poison=True)
    g = gpu_step(w, 1)
    compare(g, oracle_step(w, 1, probs_f32=g["probs"]), oracle_step(w, 1), 1)


def test_scaled_down_config5_whole_step():
    """N = 32 traces over a pool filled to capacity, 1024-token shared prompt, scorer on ~10 % of
    the traces, prior running-mean state, prune the bottom 25 %."""
    w = wl.make_workload(5, N=32, tail=(1100, 2600), poison=True)
    k = w.prune_k
    assert k == 8 and w.layout.NP == w.layout.used_pages
    g = gpu_step(w, k)
    o_same = oracle_step(w, k, probs_f32=g["probs"])
    o_ind = oracle_step(w, k)
    compare(g, o_same, o_ind, k)
    # independent chain: same pruned set unless the boundary scores are closer than the prob tolerance
    s = np.sort(o_ind["scores"])
    if s[k] - s[k - 1] > 4 * 2.5e-4:
        assert sorted(g["pruned"].tolist()) == sorted(o_ind["pruned"].tolist())
        assert np.array_equal(g["freed"], o_ind["freed"]) and np.array_equal(g["rc"], o_ind["rc"])
    assert np.all(g["rc"][w.layout.block_tables[0, :64]] == 32 - k)


def test_every_call_accepts_a_null_status_pointer():
    """status may be NULL: errors are dropped, results are the same, and a data-dependent error (a page id
    out of range) still touches nothing outside the arrays."""
    w = wl.make_workload(1, poison=True)
    lay, s = w.layout, w.scorer
    want = gpu_step(w, 1)
    bt, sl, rc = dev(lay.block_tables), dev(lay.seq_lens), dev(lay.refcounts)
    out = binding.paged_decode_attn(dev_bits(w.q), dev_bits(w.k_pages), dev_bits(w.v_pages), bt, sl)
    ssum, cnt = dev(s.score_sum), dev(s.score_cnt)
    scores = torch.empty(w.shape.N, dtype=torch.float32, device=DEV)
    logits, _ = binding.step_score(dev_bits(s.hidden), dev(s.boundary_idx), dev_bits(s.W1), dev(s.b1), dev_bits(s.W2),
                                   torch.tensor([s.b2], dtype=torch.float32, device=DEV), act=s.act,
                                   trace_of=dev(s.trace_of), score_sum=ssum, score_cnt=cnt, scores=scores)
    pruned, freed, nf = binding.prune_free(scores, 1, rc, bt, sl)
    torch.cuda.synchronize()
    assert np.array_equal(host_f32_of_bf16(out), want["out"]) and np.array_equal(logits.cpu().numpy(), want["logits"])
    assert pruned.cpu().numpy()[:1].tolist() == want["pruned"].tolist() and np.array_equal(rc.cpu().numpy(), want["rc"])
    # errors without a status word
    bad = lay.block_tables.copy(); bad[:, 0] = lay.NP + 7; bad[2, 5] = -3
    tb, tl, trc = dev(bad), dev(lay.seq_lens), dev(lay.refcounts)
    out = binding.paged_decode_attn(dev_bits(w.q), dev_bits(w.k_pages), dev_bits(w.v_pages), tb, tl)
    binding.prune_free(dev(np.array([0.3, 0.1, 0.2, 0.4], np.float32)), 2, trc, tb, tl)
    binding.reserve_pages(dev(np.array([0.3, 0.1, 0.2, 0.4], np.float32)), trc, tb, tl)
    binding.append_kv(dev_bits(w.q[:, :1]), dev_bits(w.q[:, :1]), dev_bits(w.k_pages.copy()), dev_bits(w.v_pages.copy()), tb, tl)
    torch.cuda.synchronize()
    assert out.shape == (w.shape.N, w.shape.Hq, w.shape.D)
