"""GPU parity of the pieces that complete Algorithm 1 around the three hot calls: memory-triggered
pruning + page allocation (Section 4.2), KV append, weighted vote (Section 4.3), and a multi-step
decode loop that runs entirely on the device."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_09093_amd import binding, workloads as wl
from tests.gpu_util import DEV, dev, dev_bits, host_bits, host_f32_of_bf16, new_status

pytestmark = pytest.mark.gpu
P = 16


def gpu_reserve(scores, rc, bt, sl, expect_status=0):
    st = new_status()
    t_rc, t_bt, t_sl = dev(rc.copy()), dev(bt.copy()), dev(sl.copy())
    pruned, n_pruned, new_pages = binding.reserve_pages(dev(scores), t_rc, t_bt, t_sl, status=st)
    torch.cuda.synchronize()
    assert int(st.item()) == expect_status, binding.ERROR_NAMES.get(int(st.item()))
    n = int(n_pruned.item())
    return pruned.cpu().numpy()[:n], new_pages.cpu().numpy()[: sl.size], t_rc.cpu().numpy(), t_bt.cpu().numpy(), t_sl.cpu().numpy()


def check_reserve(scores, rc, bt, sl):
    got = gpu_reserve(scores, rc, bt, sl)
    o_rc, o_bt, o_sl = rc.copy(), bt.copy(), sl.copy()
    o_pruned, o_new = oracle.reserve_pages(scores, o_rc, o_bt, o_sl, P)
    for name, a, b in zip(("pruned", "new_pages", "refcounts", "block_tables", "seq_lens"), got,
                          (o_pruned, o_new, o_rc, o_bt, o_sl)):
        assert np.array_equal(a, b), name
    return got


@pytest.mark.parametrize("seed", range(10))
def test_reserve_pages_random_layouts(seed):
    r = wl.rng_for(700 + seed, 0)
    N = int(r.integers(1, 70))
    lens = 32 + 16 * r.integers(0, 6, N) + np.where(r.random(N) < 0.5, 0, r.integers(1, 16, N))
    lens[r.random(N) < 0.1] = 0
    lay = wl.build_layout(lens, 32, P, wl.rng_for(700 + seed, 1), slack=1.0, maxb=12)
    extra = int(r.integers(0, max(N // 2, 1)))
    rc = np.concatenate([lay.refcounts, np.zeros(extra, np.int32)])
    perm = wl.rng_for(700 + seed, 2).permutation(rc.size)            # scatter the free pages
    rc2 = np.empty_like(rc); rc2[perm] = rc
    bt = np.where(lay.block_tables >= 0, perm[np.maximum(lay.block_tables, 0)], -1).astype(np.int32)
    scores = (r.integers(0, 20, N) / 16.0).astype(np.float32)        # ties
    check_reserve(scores, rc2, bt, lay.seq_lens)


def test_reserve_pages_hand_example_and_no_pressure():
    lay = wl.build_layout(np.array([32, 32, 32, 32]), 0, P, wl.rng_for(2, 1), maxb=4)
    pruned, new, rc, bt, sl = check_reserve(np.array([0.2, 0.7, 0.1, 0.9], np.float32), lay.refcounts,
                                            lay.block_tables, lay.seq_lens)
    assert pruned.tolist() == [2, 0] and sl.tolist() == [0, 32, 0, 32]
    rc_big = np.concatenate([lay.refcounts, np.zeros(10, np.int32)])
    pruned, new, *_ = check_reserve(np.zeros(4, np.float32), rc_big, lay.block_tables, lay.seq_lens)
    assert pruned.size == 0 and new.tolist() == [8, 9, 10, 11]


def test_reserve_pages_config5_scale_saturated_pool():
    """N = 256 traces over a pool filled to capacity: the step that follows needs ~16 pages."""
    w = wl.make_workload(5, kv=False)
    lay = w.layout
    sl = lay.seq_lens.copy()
    sl[::9] = (sl[::9] // P) * P                                      # put some traces on a page boundary
    bt = lay.block_tables.copy()
    rc = lay.refcounts.copy()
    for i in range(0, 256, 9):                                        # drop the pages past the shortened length
        nb_new = sl[i] // P
        extra = bt[i, nb_new:][bt[i, nb_new:] >= 0]
        rc[extra] -= 1
        bt[i, nb_new:] = -1
    scores = (w.scorer.score_sum / w.scorer.score_cnt).astype(np.float32)
    pruned, new, *_ = check_reserve(scores, rc, bt, sl)
    assert (new >= 0).sum() > 0


def test_reserve_pages_most_traces_a_call_takes_under_pressure():
    """N = 4096 traces, a third of them at a page boundary, a pool with only a few free pages: many rounds of
    the trigger (prune the lowest, re-check) before everybody that is left gets a page."""
    r = wl.rng_for(720, 0)
    N = 4096
    lens = 16 + 16 * r.integers(0, 4, N) + np.where(r.random(N) < 0.33, 0, r.integers(1, 16, N))
    lens[r.random(N) < 0.05] = 0
    lay = wl.build_layout(lens, 16, P, wl.rng_for(720, 1), slack=1.0, maxb=6)
    rc = np.concatenate([lay.refcounts, np.zeros(900, np.int32)])
    perm = wl.rng_for(720, 2).permutation(rc.size)
    rc2 = np.empty_like(rc); rc2[perm] = rc
    bt = np.where(lay.block_tables >= 0, perm[np.maximum(lay.block_tables, 0)], -1).astype(np.int32)
    scores = (r.integers(0, 400, N) / 512.0).astype(np.float32)      # many ties
    pruned, new, *_ = check_reserve(scores, rc2, bt, lay.seq_lens)
    assert pruned.size > 50 and (new >= 0).sum() > 900


def test_reserve_pages_errors():
    lay = wl.build_layout(np.array([32, 32]), 0, P, wl.rng_for(4, 1), maxb=2)
    gpu_reserve(np.zeros(2, np.float32), lay.refcounts, lay.block_tables, lay.seq_lens, expect_status=17)
    lay = wl.build_layout(np.array([32, 32]), 0, P, wl.rng_for(5, 1), maxb=4)
    got = gpu_reserve(np.array([np.nan, 0.5], np.float32), lay.refcounts, lay.block_tables, lay.seq_lens,
                      expect_status=19)
    assert np.array_equal(got[2], lay.refcounts) and np.array_equal(got[3], lay.block_tables)


def test_free_list_is_kept_across_prune_free_and_reserve_calls():
    """One workspace through a sequence of calls that free and take pages: reserve (pruning under pressure),
    prune_free followed by step_freelist_add, reserve again.  After every call the state equals the oracle's
    (which scans the reference counts every time), and a workspace without a free list is refused."""
    r = wl.rng_for(1234, 0)
    N = 24
    lens = 32 + 16 * r.integers(1, 5, N)                              # every trace sits on a page boundary
    lay = wl.build_layout(lens, 32, P, wl.rng_for(1234, 1), slack=1.0, maxb=12)
    NP = lay.NP + 5
    rc = np.concatenate([lay.refcounts, np.zeros(5, np.int32)])
    bt, sl = lay.block_tables.copy(), lay.seq_lens.copy()
    scores = r.random(N).astype(np.float32)
    t_rc, t_bt, t_sl, t_sc = dev(rc), dev(bt), dev(sl), dev(scores)
    st = new_status()
    ws = binding.new_workspace(int(binding.lib().step_reserve_workspace_bytes(N, 12, NP)), DEV)
    ws.fill_(0x5A)
    binding.reserve_pages(t_sc, t_rc, t_bt, t_sl, workspace=ws, status=st)
    torch.cuda.synchronize()
    assert binding.ERROR_NAMES[int(st.item())] == "STEP_EFREELIST"
    assert np.array_equal(t_rc.cpu().numpy(), rc) and np.array_equal(t_bt.cpu().numpy(), bt)   # nothing was modified
    st.zero_()
    binding.freelist_rebuild(t_rc, ws)

    def same_state():
        torch.cuda.synchronize()
        assert int(st.item()) == 0, binding.ERROR_NAMES.get(int(st.item()))
        assert np.array_equal(t_rc.cpu().numpy(), rc) and np.array_equal(t_bt.cpu().numpy(), bt)
        assert np.array_equal(t_sl.cpu().numpy(), sl)

    for round_ in range(4):
        pruned, n_pruned, new_pages = binding.reserve_pages(t_sc, t_rc, t_bt, t_sl, workspace=ws, status=st)
        o_pruned, o_new = oracle.reserve_pages(scores, rc, bt, sl, P)
        same_state()
        assert pruned.cpu().numpy()[: int(n_pruned.item())].tolist() == o_pruned.tolist()
        assert np.array_equal(new_pages.cpu().numpy()[:N], o_new)
        live = np.nonzero(sl > 0)[0]
        sl[live] += 16; t_sl.copy_(dev(sl))                           # the traces fill their new page
        if round_ == 1:                                               # a fixed-fraction prune in between
            k = 3
            pr, fr, nf = binding.prune_free(t_sc, k, t_rc, t_bt, t_sl, status=st)
            binding.freelist_add(NP, fr, nf, ws, status=st)
            oracle.prune_free(scores, k, rc, bt, sl, P)
            same_state()
    assert (sl > 0).sum() >= 1


@pytest.mark.parametrize("seq", range(8))
def test_random_sequences_on_one_free_list(seq):
    """Random sequences of calls that free and take pages on one persistent workspace: reserve under pressure,
    prune_free + step_freelist_add, and a change of the reference counts from outside followed by a rebuild; the
    traces grow by random amounts in between.  After every call the state equals the oracle's."""
    r = wl.rng_for(77000 + seq, 0)
    N = int(r.choice([3, 8, 33, 64, 200]))
    MAXB = 40
    lens = 32 + r.integers(1, 200, N)
    lay = wl.build_layout(lens, 32, P, wl.rng_for(77000 + seq, 1), slack=1.0, maxb=MAXB)
    extra = int(r.integers(0, N))
    NP = lay.NP + extra
    perm = r.permutation(NP)
    rc = np.empty(NP, np.int32); rc[perm] = np.concatenate([lay.refcounts, np.zeros(extra, np.int32)])
    bt = np.where(lay.block_tables >= 0, perm[np.maximum(lay.block_tables, 0)], -1).astype(np.int32)
    sl = lay.seq_lens.copy()
    scores = r.random(N).astype(np.float32)
    t_rc, t_bt, t_sl, t_sc = dev(rc), dev(bt), dev(sl), dev(scores)
    st = new_status()
    ws = binding.reserve_workspace(t_rc, N, MAXB)
    for op in range(40):
        live = np.nonzero(sl > 0)[0]
        if live.size == 0:
            break
        kind = r.random()
        if kind < 0.6:
            pruned, n_pruned, new_pages = binding.reserve_pages(t_sc, t_rc, t_bt, t_sl, workspace=ws, status=st)
            o_pruned, o_new = oracle.reserve_pages(scores, rc, bt, sl, P)
            torch.cuda.synchronize()
            assert pruned.cpu().numpy()[: int(n_pruned.item())].tolist() == o_pruned.tolist(), op
            assert np.array_equal(new_pages.cpu().numpy()[:N], o_new), op
            live = np.nonzero(sl > 0)[0]                              # the traces grow inside the pages they own
            room = np.where(sl[live] % P == 0, np.where(o_new[live] >= 0, P, 0), P - sl[live] % P)
            adv = np.minimum(room, r.integers(0, P + 1, live.size))
            adv = np.where(sl[live] + adv > (MAXB - 1) * P, 0, adv)
            sl[live] += adv.astype(np.int32)
            t_sl.copy_(dev(sl))
        elif kind < 0.85 and live.size > 1:
            k = int(r.integers(1, max(2, live.size // 3)))
            _, fr, nf = binding.prune_free(t_sc, k, t_rc, t_bt, t_sl, status=st)
            binding.freelist_add(NP, fr, nf, ws, status=st)
            oracle.prune_free(scores, k, rc, bt, sl, P)
        else:
            free = np.nonzero(rc == 0)[0]
            if free.size:
                rc[free[int(r.integers(0, free.size))]] = 1           # taken by someone else
                t_rc.copy_(dev(rc))
                binding.freelist_rebuild(t_rc, ws)
        torch.cuda.synchronize()
        assert int(st.item()) == 0, (op, binding.ERROR_NAMES.get(int(st.item())))
        assert np.array_equal(t_rc.cpu().numpy(), rc) and np.array_equal(t_bt.cpu().numpy(), bt), op
        assert np.array_equal(t_sl.cpu().numpy(), sl), op


def test_append_kv_bit_exact():
    lay = wl.build_layout(np.array([17, 32, 0, 5, 100, 48]), 0, P, wl.rng_for(6, 1), slack=1.5, maxb=8)
    Hkv, D = 8, 128
    NP = lay.NP + 2
    k = wl.normal_bf16(wl.rng_for(6, 2), (NP, Hkv, P, D)); v = wl.normal_bf16(wl.rng_for(6, 3), k.shape)
    rc = np.concatenate([lay.refcounts, [1, 1]]).astype(np.int32)
    bt = lay.block_tables.copy(); bt[1, 2] = lay.NP; bt[5, 3] = lay.NP + 1
    kn = wl.normal_bf16(wl.rng_for(6, 4), (6, Hkv, D)); vn = wl.normal_bf16(wl.rng_for(6, 5), (6, Hkv, D))
    tk, tv, tsl = dev_bits(k), dev_bits(v), dev(lay.seq_lens.copy())
    st = new_status()
    binding.append_kv(dev_bits(kn), dev_bits(vn), tk, tv, dev(bt), tsl, refcounts=dev(rc), status=st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    sl = lay.seq_lens.copy()
    oracle.append_kv(kn, vn, k, v, bt, rc, sl)
    assert np.array_equal(host_bits(tk), k) and np.array_equal(host_bits(tv), v)
    assert np.array_equal(tsl.cpu().numpy(), sl)


def test_append_kv_errors():
    lay = wl.build_layout(np.array([16, 20]), 0, P, wl.rng_for(8, 1), maxb=2)
    k = np.zeros((lay.NP, 1, P, 64), np.uint16)
    kn = np.ones((2, 1, 64), np.uint16)
    st = new_status()
    tsl = dev(lay.seq_lens.copy())
    binding.append_kv(dev_bits(kn), dev_bits(kn), dev_bits(k), dev_bits(k), dev(lay.block_tables), tsl, status=st)
    torch.cuda.synchronize()
    assert int(st.item()) == 16 and tsl.cpu().numpy().tolist() == [16, 21]     # trace 0 refused, trace 1 appended


def test_weighted_vote_bit_exact():
    r = wl.rng_for(10, 0)
    for N in (1, 6, 64, 257, 1000):
        a = r.integers(-1, 7, N).astype(np.int32)
        s = r.uniform(0, 1, N).astype(np.float32)
        st = new_status()
        w, wt = binding.weighted_vote(dev(a), dev(s), status=st)
        torch.cuda.synchronize()
        ow, owt = oracle.weighted_vote(a, s)
        assert int(st.item()) == 0 and int(w.item()) == ow and np.float32(wt.item()) == np.float32(owt)
    w, _ = binding.weighted_vote(dev(np.full(5, -1, np.int32)), dev(np.ones(5, np.float32)))
    assert int(w.item()) == -1
    # the most traces a call takes, answer ids anywhere in the int32 range, exact ties between answers
    N = 4096
    ids = np.array([0, 1, 17, 2 ** 31 - 2, 2 ** 31 - 1, 123456789, 5, 6], np.int64)
    a = ids[r.integers(0, ids.size, N)].astype(np.int32)
    a[r.random(N) < 0.2] = -1
    s = (r.integers(1, 9, N) / 8.0).astype(np.float32)                # dyadic: sums are exact, ties do happen
    st = new_status()
    w, wt = binding.weighted_vote(dev(a), dev(s), status=st)
    torch.cuda.synchronize()
    ow, owt = oracle.weighted_vote(a, s)
    assert int(st.item()) == 0 and int(w.item()) == ow and np.float32(wt.item()) == np.float32(owt)
    a2 = np.array([2 ** 31 - 1, 7, 2 ** 31 - 1, 7], np.int32); s2 = np.array([0.5, 0.25, 0.25, 0.5], np.float32)
    w, wt = binding.weighted_vote(dev(a2), dev(s2))
    assert (int(w.item()), float(wt.item())) == oracle.weighted_vote(a2, s2) == (7, 0.75)


def _decode_loop(NP):
    """150 decode steps of 8 traces that share a 2-page prompt in a pool of NP pages:
    reserve (memory-triggered pruning + allocation) -> append -> attention -> scorer -> running mean,
    every step on the device; the oracle replays the same steps (fed the GPU's step probabilities,
    so that the scores are the same bytes) and every integer state must match bit for bit.
    Returns (traces pruned by the memory trigger, traces alive at the end)."""
    N, Hq, Hkv, D, d, m = 8, 4, 1, 64, 256, 64
    steps, MAXB = 150, 16
    r = wl.rng_for(77, 0)
    lay = wl.build_layout(np.full(N, 32), 32, P, wl.rng_for(77, 1), slack=1.0, maxb=MAXB)
    rc = np.concatenate([lay.refcounts, np.zeros(NP - lay.NP, np.int32)])
    bt, sl = lay.block_tables.copy(), lay.seq_lens.copy()
    k = wl.normal_bf16(wl.rng_for(77, 2), (NP, Hkv, P, D)); v = wl.normal_bf16(wl.rng_for(77, 3), k.shape)
    sc = wl.build_scorer(77, N, N, d, m, 0, 0)
    ssum, cnt = np.zeros(N, np.float32), np.zeros(N, np.int32)
    scores = np.full(N, np.inf, np.float32)

    t_rc, t_bt, t_sl = dev(rc), dev(bt), dev(sl)
    t_k, t_v = dev_bits(k), dev_bits(v)
    t_sum, t_cnt, t_scores = dev(ssum), dev(cnt), dev(scores)
    t_W1, t_b1, t_W2 = dev_bits(sc.W1), dev(sc.b1), dev_bits(sc.W2)
    t_b2 = torch.tensor([sc.b2], dtype=torch.float32, device=DEV)
    st = new_status()
    ws_res = binding.reserve_workspace(t_rc, N, MAXB)                 # the free list is built once and then kept up
    total_pruned = 0
    for step in range(steps):
        kn = wl.normal_bf16(wl.rng_for(1000 + step, 0), (N, Hkv, D)); vn = wl.normal_bf16(wl.rng_for(1000 + step, 1), (N, Hkv, D))
        q = wl.normal_bf16(wl.rng_for(1000 + step, 2), (N, Hq, D))
        hidden = wl.normal_bf16(wl.rng_for(1000 + step, 3), (N, d))
        live = np.nonzero(sl > 0)[0]
        if live.size == 0:
            break
        bidx = live[wl.rng_for(1000 + step, 4).random(live.size) < 0.3].astype(np.int32)
        # device
        pruned, n_pruned, new_pages = binding.reserve_pages(t_scores, t_rc, t_bt, t_sl, workspace=ws_res, status=st)
        binding.append_kv(dev_bits(kn), dev_bits(vn), t_k, t_v, t_bt, t_sl, refcounts=t_rc, status=st)
        out = binding.paged_decode_attn(dev_bits(q), t_k, t_v, t_bt, t_sl, status=st)
        logits, probs = binding.step_score(dev_bits(hidden), dev(bidx), t_W1, t_b1, t_W2, t_b2, trace_of=dev(bidx),
                                           score_sum=t_sum, score_cnt=t_cnt, scores=t_scores, status=st)
        torch.cuda.synchronize()
        assert int(st.item()) == 0, (step, binding.ERROR_NAMES.get(int(st.item())))
        # oracle replay
        o_pruned, o_new = oracle.reserve_pages(scores, rc, bt, sl, P)
        oracle.append_kv(kn, vn, k, v, bt, rc, sl)
        o_out = oracle.paged_decode_attn(q, k, v, bt, sl)
        o_logits, _ = oracle.step_score(hidden, bidx, sc.W1, sc.b1, sc.W2, sc.b2)
        scores = oracle.running_mean(bidx, probs.cpu().numpy(), ssum, cnt)
        n = int(n_pruned.item())
        total_pruned += n
        assert pruned.cpu().numpy()[:n].tolist() == o_pruned.tolist(), step
        assert np.array_equal(new_pages.cpu().numpy()[:N], o_new), step
        assert np.array_equal(t_rc.cpu().numpy(), rc) and np.array_equal(t_bt.cpu().numpy(), bt), step
        assert np.array_equal(t_sl.cpu().numpy(), sl) and np.array_equal(t_scores.cpu().numpy(), scores), step
        assert np.abs(host_f32_of_bf16(out) - o_out).max() <= 2e-2, step
        if bidx.size:
            assert np.abs(logits.cpu().numpy() - o_logits).max() <= 1e-3, step
    assert np.array_equal(host_bits(t_k), k) and np.array_equal(host_bits(t_v), v)
    assert (sl > 0).sum() >= 1 and np.all(sl[sl > 0] == 32 + steps)   # no step failed to allocate: survivors never waited
    # the survivors vote
    answers = np.where(sl > 0, np.arange(N) % 3, -1).astype(np.int32)
    w, wt = binding.weighted_vote(dev(answers), t_scores)
    o_w, o_wt = oracle.weighted_vote(answers, scores)
    assert int(w.item()) == o_w and np.float32(wt.item()) == np.float32(o_wt)
    return total_pruned, int((sl > 0).sum())


def test_multi_step_decode_loop_on_device():
    pruned, alive = _decode_loop(44)                          # a pool too small for all eight traces
    assert pruned >= 3 and alive == 8 - pruned


def test_memory_budget_sweep_prunes_fewer_traces_with_more_memory():
    """The shape of the paper's memory-budget sweep (Table 4) on synthetic traces: the same 150-step
    run in pools of growing size prunes fewer and fewer traces and none once everything fits
    (8 traces x 10 private pages + 2 prompt pages = 82 pages at the end); in every pool each
    surviving trace got its page at every boundary."""
    counts = [_decode_loop(NP)[0] for NP in (30, 60, 90)]
    assert counts[0] >= counts[1] >= counts[2] == 0 and counts[0] > counts[1]
