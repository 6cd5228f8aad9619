"""GPU parity of prune_free against the oracle: pruned list, freed-page list, refcounts, block
tables and lengths must be bit-identical on identical score bytes."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_09093_amd import binding, workloads as wl
from tests.gpu_util import DEV, dev, new_status

pytestmark = pytest.mark.gpu
P = 16


def run_gpu(scores, k, rc, bt, sl, expect_status=0):
    st = new_status()
    t_rc, t_bt, t_sl = dev(rc.copy()), dev(bt.copy()), dev(sl.copy())
    pruned, freed, nf = binding.prune_free(dev(scores), k, t_rc, t_bt, t_sl, status=st)
    torch.cuda.synchronize()
    assert int(st.item()) == expect_status, binding.ERROR_NAMES.get(int(st.item()))
    n = int(nf.item())
    return pruned.cpu().numpy()[:k], freed.cpu().numpy()[:n], t_rc.cpu().numpy(), t_bt.cpu().numpy(), t_sl.cpu().numpy()


def check(scores, k, lay):
    got = run_gpu(scores, k, lay.refcounts, lay.block_tables, lay.seq_lens)
    rc, bt, sl = lay.refcounts.copy(), lay.block_tables.copy(), lay.seq_lens.copy()
    pruned, freed = oracle.prune_free(scores, k, rc, bt, sl, P)
    for name, a, b in zip(("pruned", "freed", "refcounts", "block_tables", "seq_lens"), got, (pruned, freed, rc, bt, sl)):
        assert a.dtype == b.dtype and np.array_equal(a, b), name
    return got


def _layout(seed, N, prompt, lo, hi, slack=1.2):
    lens = wl.rng_for(seed, 0).integers(lo, hi + 1, N)
    return wl.build_layout(lens, prompt, P, wl.rng_for(seed, 1), slack=slack)


def test_config1_bottom_one_of_four():
    w = wl.make_workload(1, kv=False)
    scores = np.array([0.6, 0.2, 0.9, 0.4], np.float32)
    pruned, freed, rc, *_ = check(scores, 1, w.layout)
    assert pruned.tolist() == [1] and np.all(rc[w.layout.block_tables[0, :4]] == 3)


def test_hand_cases_from_golden_file():
    import json, os
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "bottomk_hand.json")))
    for c in g["cases"]:
        scores = np.array([float(x) for x in c["scores"]], np.float32)
        live = np.array(c["live"])
        lens = np.where(live == 1, 20 + np.arange(scores.size), 0)
        lay = wl.build_layout(lens, 0, P, wl.rng_for(1, 1))
        pruned, *_ = check(scores, c["k"], lay)
        assert pruned.tolist() == c["pruned"]


@pytest.mark.parametrize("N,k", [(1, 1), (2, 1), (5, 0), (5, 5), (63, 17), (64, 64), (65, 3), (256, 64), (1000, 333),
                                 (4096, 1024)])
def test_sizes_with_ties_and_dead_traces(N, k):
    lay = _layout(300 + N, N, 32, 33, 400)
    r = wl.rng_for(300 + N, 2)
    scores = (r.integers(0, max(N // 3, 2), N) / 64.0).astype(np.float32)      # many ties
    scores[r.integers(0, N, max(N // 10, 1))] = np.inf                          # unscored traces
    dead = r.integers(0, N, N // 8)
    for t in dead:                                                              # kill some traces consistently
        if lay.seq_lens[t] > 0:
            pages = lay.block_tables[t][lay.block_tables[t] >= 0]
            lay.refcounts[pages] -= 1
            lay.block_tables[t] = -1
            lay.seq_lens[t] = 0
    scores[dead[: dead.size // 2]] = np.nan                                     # NaN on dead traces is ignored
    k = min(k, int((lay.seq_lens > 0).sum()))
    check(scores, k, lay)


def test_scaled_down_config5_saturated_pool():
    w = wl.make_workload(5, kv=False, N=32, tail=(1100, 3000))
    assert w.layout.NP == w.layout.used_pages and w.prune_k == 8
    scores = wl.rng_for(5, 3).uniform(0.2, 0.8, 32).astype(np.float32)
    pruned, freed, rc, bt, sl = check(scores, 8, w.layout)
    assert np.all(rc[w.layout.block_tables[0, :64]] == 24)                      # prompt pages 32 -> 24


def test_full_config5_prune_quarter():
    w = wl.make_workload(5, kv=False)
    s = w.scorer
    scores = (s.score_sum / s.score_cnt).astype(np.float32)
    pruned, freed, rc, bt, sl = check(scores, 64, w.layout)
    assert np.all(rc[w.layout.block_tables[0, :64]] == 192) and freed.size > 20000


def test_two_rounds_equal_one_round_on_device():
    lay = _layout(41, 40, 64, 65, 700)
    scores = wl.rng_for(41, 2).uniform(0, 1, 40).astype(np.float32)
    one = run_gpu(scores, 9, lay.refcounts, lay.block_tables, lay.seq_lens)
    a = run_gpu(scores, 4, lay.refcounts, lay.block_tables, lay.seq_lens)
    b = run_gpu(scores, 5, a[2], a[3], a[4])
    assert np.concatenate([a[0], b[0]]).tolist() == one[0].tolist()
    assert sorted(np.concatenate([a[1], b[1]]).tolist()) == one[1].tolist()
    for x, y in zip(b[2:], one[2:]):
        assert np.array_equal(x, y)


def test_device_reported_errors_leave_selection_state_untouched():
    lay = _layout(42, 8, 32, 33, 200)
    scores = wl.rng_for(42, 2).uniform(0, 1, 8).astype(np.float32)
    bad = scores.copy(); bad[3] = np.nan
    got = run_gpu(bad, 2, lay.refcounts, lay.block_tables, lay.seq_lens, expect_status=19)      # STEP_ENAN
    assert got[1].size == 0 and np.array_equal(got[2], lay.refcounts) and np.array_equal(got[3], lay.block_tables)
    sl = lay.seq_lens.copy(); sl[:6] = 0
    got = run_gpu(scores, 3, lay.refcounts, lay.block_tables, sl, expect_status=21)             # STEP_EKLIVE
    assert np.array_equal(got[4], sl) and np.array_equal(got[2], lay.refcounts)
    sl = lay.seq_lens.copy(); sl[1] = lay.MAXB * P + 1
    run_gpu(scores, 1, lay.refcounts, lay.block_tables, sl, expect_status=17)                   # STEP_ELEN
    t = int(np.argmin(scores))
    bt = lay.block_tables.copy(); bt[t, 1] = lay.NP
    run_gpu(scores, 1, lay.refcounts, bt, lay.seq_lens, expect_status=16)                       # STEP_EPAGE
    rc = lay.refcounts.copy(); rc[lay.block_tables[t, 3]] = 0
    got = run_gpu(scores, 1, rc, lay.block_tables, lay.seq_lens, expect_status=20)              # STEP_EREFCOUNT
    assert got[2][lay.block_tables[t, 3]] == 0                                                  # not driven negative


@pytest.mark.parametrize("big", [False, True])
def test_documented_post_state_after_a_bad_page_id_or_reference_count(big):
    """An error met while releasing (a page id outside the pool, a reference count that is already 0) is
    reported and that one entry skipped; everything else of the call is carried out.  The oracle, by its own
    convention, changes nothing on any error: the two are compared on what both define -- which traces are
    pruned -- and the GPU's post-state is checked against the rule the header documents.  Both kernel paths:
    the one-workgroup path (small) and the three-kernel path (k * row width above its limit)."""
    N, k = (40, 24) if big else (10, 3)
    lay = _layout(48 if big else 47, N, 32, 6000 if big else 100, 8000 if big else 300)
    assert (k * lay.MAXB > 8192) == big
    scores = wl.rng_for(47, 2).uniform(0, 1, N).astype(np.float32)
    order = np.argsort(scores, kind="stable")[:k]
    t_bad_page, t_bad_rc = int(order[0]), int(order[1])
    bt = lay.block_tables.copy(); rc = lay.refcounts.copy()
    lost = int(bt[t_bad_page, 3])                                  # a private page whose entry is overwritten
    bt[t_bad_page, 3] = lay.NP + 11
    zero_page = int(bt[t_bad_rc, 4])
    rc[zero_page] = 0
    st = new_status()
    t_rc, t_bt, t_sl = dev(rc), dev(bt), dev(lay.seq_lens.copy())
    pruned, freed, nf = binding.prune_free(dev(scores), k, t_rc, t_bt, t_sl, status=st)
    torch.cuda.synchronize()
    assert binding.ERROR_NAMES[int(st.item())] in ("STEP_EPAGE", "STEP_EREFCOUNT")
    g_rc, g_bt, g_sl = t_rc.cpu().numpy(), t_bt.cpu().numpy(), t_sl.cpu().numpy()
    g_pruned = pruned.cpu().numpy()[:k]; g_freed = freed.cpu().numpy()[: int(nf.item())]
    assert g_pruned.tolist() == order.tolist()                        # the selection is unaffected
    surv = np.setdiff1d(np.arange(N), order)
    assert np.array_equal(g_bt[surv], bt[surv]) and np.array_equal(g_sl[surv], lay.seq_lens[surv])   # survivors untouched
    assert np.all(g_bt[order] == -1) and np.all(g_sl[order] == 0)     # pruned rows cleared all the same
    want = rc.copy()
    for t in order:
        for j in range((lay.seq_lens[t] + P - 1) // P):
            pg = bt[t, j]
            if 0 <= pg < lay.NP and want[pg] > 0:
                want[pg] -= 1
    assert np.array_equal(g_rc, want) and g_rc.min() >= 0             # every valid entry released once, none negative
    assert g_rc[lost] == 1 and g_rc[zero_page] == 0                   # the page behind the bad entry stays referenced
    assert np.all(np.diff(g_freed) > 0)                               # still ascending, and exactly the pages that reached 0
    assert np.array_equal(g_freed, np.nonzero((want == 0) & (rc > 0))[0])
    with pytest.raises(oracle.OracleError):
        o_rc, o_bt, o_sl = rc.copy(), bt.copy(), lay.seq_lens.copy()
        oracle.prune_free(scores, k, o_rc, o_bt, o_sl, P)
    assert np.array_equal(o_rc, rc) and np.array_equal(o_bt, bt)      # the oracle's convention: nothing modified


def test_stale_entries_behind_the_last_page_in_use_are_cleared_and_release_nothing():
    """The hand case of the oracle's pins (the whole row becomes -1, entries behind ceil(L / P) release nothing),
    and the same on a layout large enough for the three-launch path, with stale valid page ids behind every row."""
    bt = np.array([[2, 0, 3, 1], [1, 4, -1, -1]], np.int32)
    sl = np.array([20, 30], np.int32)
    rc = np.array([1, 1, 1, 7, 1], np.int32)
    pruned, freed, rc1, bt1, sl1 = run_gpu(np.array([0.1, 0.9], np.float32), 1, rc, bt, sl)
    assert pruned.tolist() == [0] and freed.tolist() == [0, 2]
    assert bt1.tolist() == [[-1, -1, -1, -1], [1, 4, -1, -1]] and sl1.tolist() == [0, 30] and rc1.tolist() == [0, 1, 0, 7, 1]
    lay = _layout(91, 96, 64, 200, 4000)
    r = wl.rng_for(91, 5)
    for i in range(96):
        nb = (lay.seq_lens[i] + P - 1) // P
        lay.block_tables[i, nb:] = r.integers(0, lay.NP, lay.MAXB - nb)
    check(wl.rng_for(91, 2).uniform(0, 1, 96).astype(np.float32), 40, lay)


@pytest.mark.parametrize("NP", [262143, 262144, 262145, 300000])
def test_pool_sizes_around_the_single_launch_limit(NP):
    """The single-launch path keeps the freed-page bitmap on chip for pools of up to 262144 pages; one page more
    goes to the three-launch path.  A small batch scattered over such a pool, its last page included."""
    lay = _layout(93, 40, 32, 100, 900)
    r = wl.rng_for(93, 7)
    spread = r.choice(NP - 1, lay.NP, replace=False).astype(np.int32)
    spread[lay.block_tables[0, 3]] = NP - 1                  # a private page of trace 0, which is pruned first
    rc = np.zeros(NP, np.int32); rc[spread] = lay.refcounts
    bt = np.where(lay.block_tables >= 0, spread[np.maximum(lay.block_tables, 0)], -1).astype(np.int32)
    scores = wl.rng_for(93, 2).uniform(0, 1, 40).astype(np.float32)
    scores[0] = -1.0
    got = run_gpu(scores, 9, rc, bt, lay.seq_lens)
    rc2, bt2, sl2 = rc.copy(), bt.copy(), lay.seq_lens.copy()
    pruned, freed = oracle.prune_free(scores, 9, rc2, bt2, sl2, P)
    assert pruned[0] == 0 and freed[-1] == NP - 1
    for name, a, b in zip(("pruned", "freed", "refcounts", "block_tables", "seq_lens"), got, (pruned, freed, rc2, bt2, sl2)):
        assert np.array_equal(a, b), name


def test_host_reported_errors():
    lay = _layout(43, 4, 0, 20, 60)
    scores = dev(np.zeros(4, np.float32))
    with pytest.raises(binding.StepError) as e:
        binding.prune_free(scores, 5, dev(lay.refcounts), dev(lay.block_tables), dev(lay.seq_lens))   # k > N
    assert e.value.code == 1
    with pytest.raises(binding.StepError) as e:
        binding.prune_free(scores, 1, dev(lay.refcounts), dev(lay.block_tables), dev(lay.seq_lens),
                           workspace=torch.zeros(256, dtype=torch.uint8, device=DEV))
    assert e.value.code == 2


def test_fused_and_three_kernel_paths_agree():
    """Small problems take the single-launch path, large ones three launches; both must give the
    oracle's result.  The three-launch path is forced in a child process through its switch."""
    import os, subprocess, sys, json
    code = (
        "import numpy as np, torch, json, sys\n"
        "sys.path.insert(0, %r)\n"
        "from paper_2601_09093_amd import binding, workloads as wl\n"
        "lens = wl.rng_for(55, 0).integers(40, 600, 48)\n"
        "lay = wl.build_layout(lens, 32, 16, wl.rng_for(55, 1), slack=1.2)\n"
        "scores = wl.rng_for(55, 2).uniform(0, 1, 48).astype(np.float32)\n"
        "d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to('cuda:0')\n"
        "rc, bt, sl = d(lay.refcounts), d(lay.block_tables), d(lay.seq_lens)\n"
        "st = torch.zeros(1, dtype=torch.int32, device='cuda:0')\n"
        "pr, fr, nf = binding.prune_free(d(scores), 5, rc, bt, sl, status=st)\n"
        "torch.cuda.synchronize()\n"
        "print(json.dumps(dict(status=int(st.item()), pruned=pr.cpu().tolist()[:5], freed=fr.cpu().tolist()[:int(nf.item())],"
        " rc=rc.cpu().tolist(), sl=sl.cpu().tolist(), bt=int(bt.cpu().numpy().astype(np.int64).sum()))))\n"
    ) % os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    outs = []
    for multi in (False, True):
        env = dict(os.environ)
        env.pop("STEP_PRUNE_MULTI", None)
        if multi:
            env["STEP_PRUNE_MULTI"] = "1"
        res = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=300)
        assert res.returncode == 0, res.stderr[-2000:]
        outs.append(json.loads(res.stdout.strip().splitlines()[-1]))
    assert outs[0] == outs[1] and outs[0]["status"] == 0
    lens = wl.rng_for(55, 0).integers(40, 600, 48)
    lay = wl.build_layout(lens, 32, P, wl.rng_for(55, 1), slack=1.2)
    scores = wl.rng_for(55, 2).uniform(0, 1, 48).astype(np.float32)
    rc, bt, sl = lay.refcounts.copy(), lay.block_tables.copy(), lay.seq_lens.copy()
    pruned, freed = oracle.prune_free(scores, 5, rc, bt, sl, P)
    assert outs[0]["pruned"] == pruned.tolist() and outs[0]["freed"] == freed.tolist()
    assert outs[0]["rc"] == rc.tolist() and outs[0]["sl"] == sl.tolist()
