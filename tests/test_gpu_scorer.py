"""GPU parity of step_score (MFMA projection + running mean) against the float64 oracle.
Bar: max-abs 1e-3 on logits; the running-mean state is compared on identical prob bytes."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_09093_amd import binding, workloads as wl
from tests.gpu_util import DEV, dev, dev_bits, new_status

pytestmark = pytest.mark.gpu
TOL = 1e-3


def run_gpu(s, N, with_state=True, expect_status=0):
    st = new_status()
    ssum = dev(s.score_sum.copy()); cnt = dev(s.score_cnt.copy())
    scores = torch.empty(N, dtype=torch.float32, device=DEV)
    b2 = torch.tensor([s.b2], dtype=torch.float32, device=DEV)
    kw = dict(trace_of=dev(s.trace_of), score_sum=ssum, score_cnt=cnt, scores=scores) if with_state else {}
    logits, probs = binding.step_score(dev_bits(s.hidden), dev(s.boundary_idx), dev_bits(s.W1), dev(s.b1),
                                       dev_bits(s.W2), b2, act=s.act, status=st, **kw)
    torch.cuda.synchronize()
    assert int(st.item()) == expect_status
    return logits.cpu().numpy(), probs.cpu().numpy(), ssum.cpu().numpy(), cnt.cpu().numpy(), scores.cpu().numpy()


def check(s, N):
    lo, pr, ssum, cnt, scores = run_gpu(s, N)
    want_lo, want_pr = oracle.step_score(s.hidden, s.boundary_idx, s.W1, s.b1, s.W2, s.b2, act=s.act)
    assert np.abs(lo - want_lo).max() <= TOL, float(np.abs(lo - want_lo).max())
    assert np.abs(pr - want_pr).max() <= 2.5e-4
    # running mean: exact on the GPU's own prob bytes (fp32 sequential sums, IEEE divide)
    o_sum = s.score_sum.copy(); o_cnt = s.score_cnt.copy()
    o_scores = oracle.running_mean(s.trace_of, pr, o_sum, o_cnt)
    assert np.array_equal(ssum, o_sum) and np.array_equal(cnt, o_cnt) and np.array_equal(scores, o_scores)
    # and close to the fully independent chain
    i_sum = s.score_sum.copy(); i_cnt = s.score_cnt.copy()
    i_scores = oracle.running_mean(s.trace_of, want_pr.astype(np.float32), i_sum, i_cnt)
    fin = np.isfinite(i_scores)
    assert np.array_equal(fin, np.isfinite(scores))
    assert np.abs(scores[fin] - i_scores[fin]).max(initial=0) <= 2.5e-4
    return lo


def test_config1_gelu_8_boundaries_over_4_traces():
    s = wl.make_workload(1, kv=False).scorer
    assert s.act == 1 and s.boundary_idx.size == 8 and s.trace_of.tolist() == [0, 1, 2, 3, 0, 1, 2, 3]
    check(s, 4)


@pytest.mark.parametrize("act", [0, 1])
@pytest.mark.parametrize("d,m,B", [(4096, 1024, 4), (4096, 512, 4), (2560, 512, 13), (5120, 512, 26),
                                   (4096, 1024, 26), (256, 64, 1), (128, 16, 33), (4096, 512, 70)])
def test_scorer_shapes(d, m, B, act):
    N = max(B, 4)
    s = wl.build_scorer(500 + d + m + B + act, N, N, d, m, B, act, prior_state=True)
    check(s, N)


@pytest.mark.parametrize("d,m,B,N,R", [(256, 64, 2500, 3000, 400), (256, 64, 1025, 2049, 64), (128, 16384, 3, 4, 3),
                                       (128, 16384, 40, 7, 40)])
def test_sizes_beyond_what_is_staged_on_chip(d, m, B, N, R):
    """More boundaries than the finishing workgroup stages at a time (1024), more traces than it keeps the running
    state on chip for (2048), several boundaries per trace across those stages (the order of the fp32 sums must
    survive), and the widest hidden layer the call takes (m = 16384: 1024 row tiles)."""
    s = wl.build_scorer(600 + B + m, N, R, d, m, B, 0, prior_state=True, distinct_rows=False)
    s.trace_of = wl.rng_for(600 + B, 50).integers(0, min(N, 97), B).astype(np.int32)   # many boundaries per trace
    s.trace_of[-1] = N - 1
    check(s, N)


def test_duplicate_rows_and_repeated_traces_in_order():
    s = wl.build_scorer(77, 6, 10, 256, 64, 40, 0, distinct_rows=False)
    s.trace_of = (wl.rng_for(77, 50).integers(0, 6, 40)).astype(np.int32)
    lo = check(s, 6)
    same = s.boundary_idx == s.boundary_idx[0]
    assert np.all(lo[same] == lo[0])


def test_no_boundaries_still_refreshes_scores():
    s = wl.build_scorer(78, 5, 5, 256, 64, 0, 0, prior_state=True)
    s.score_cnt[2] = 0
    lo, pr, ssum, cnt, scores = run_gpu(s, 5)
    assert lo.size == 0
    want = oracle.running_mean(s.trace_of, np.zeros(0, np.float32), s.score_sum.copy(), s.score_cnt.copy())
    assert np.array_equal(scores, want) and np.isposinf(scores[2])


def test_running_mean_division_is_the_correctly_rounded_quotient():
    """The hand cases of tests/golden/running_mean_hand.json that have no boundaries (B = 0) through step_score:
    their quotients (41/41, 20.5/41, 21/7 ...) are exact, and a reciprocal-then-multiply evaluation would miss them
    by one unit in the last place (Section 4.3 equation).  Then one with boundaries whose step score is exactly
    0.5 (W1 = 0, b1 = 0, b2 = 0): 20 + 0.5 over 41 steps is 0.5."""
    import json, os
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "running_mean_hand.json")))
    ran = 0
    for c in g["cases"]:
        if c["probs"]:
            continue
        N = c["N"]
        s = wl.build_scorer(82, N, N, 256, 64, 0, 0)
        s.score_sum = np.array(c["sum0"], np.float32); s.score_cnt = np.array(c["cnt0"], np.int32)
        _, _, ssum, cnt, scores = run_gpu(s, N)
        want = np.array([np.inf if x == "inf" else x for x in c["scores"]], np.float32)
        assert np.array_equal(scores, want), (scores, want)
        assert np.array_equal(ssum, np.array(c["sum"], np.float32)) and np.array_equal(cnt, np.array(c["cnt"], np.int32))
        ran += 1
    assert ran >= 2
    s = wl.build_scorer(83, 3, 3, 256, 64, 3, 0)
    s.W1[:] = 0; s.b1[:] = 0; s.b2 = 0.0
    s.trace_of = np.array([0, 1, 2], np.int32)
    s.score_sum = np.array([20.0, 23.0, 27.0], np.float32); s.score_cnt = np.array([40, 46, 54], np.int32)
    lo, pr, ssum, cnt, scores = run_gpu(s, 3)
    assert np.all(lo == 0) and np.all(pr == np.float32(0.5))
    assert np.array_equal(ssum, np.array([20.5, 23.5, 27.5], np.float32)) and cnt.tolist() == [41, 47, 55]
    assert np.array_equal(scores, np.full(3, 0.5, np.float32))


def test_calls_in_flight_on_several_streams_do_not_disturb_each_other():
    """step_score hands sums from workgroup to workgroup through arrival counters that belong to the library, one
    set of counters per workspace address.  Twelve calls of three different shapes, each with its own workspace,
    are enqueued on twelve streams without waiting in between, six times over; every result equals, bit for bit,
    the one the same call gives alone.  Then one call goes through seventy workspaces in turn -- more than the
    library keeps sets for, so sets change hands -- with the same result every time."""
    shapes = [(4096, 1024, 4, 0), (4096, 512, 26, 0), (2560, 512, 13, 1)]
    cases = []
    for i in range(12):
        d, m, B, act = shapes[i % 3]
        N = max(B, 4)
        sc = wl.build_scorer(9000 + i, N, N, d, m, B, act, prior_state=True)
        t = dict(hidden=dev_bits(sc.hidden), bidx=dev(sc.boundary_idx), W1=dev_bits(sc.W1), b1=dev(sc.b1), W2=dev_bits(sc.W2),
                 b2=torch.tensor([sc.b2], dtype=torch.float32, device=DEV), trace_of=dev(sc.trace_of), act=act, N=N,
                 sum0=dev(sc.score_sum), cnt0=dev(sc.score_cnt))
        t["ws"] = binding.new_workspace(binding.score_workspace_bytes(binding.ScoreDims(N, d, m, B, N, act)), DEV)
        cases.append(t)

    def run(t, st):
        ssum, cnt = t["sum0"].clone(), t["cnt0"].clone()
        scores = torch.empty(t["N"], dtype=torch.float32, device=DEV)
        lo, pr = binding.step_score(t["hidden"], t["bidx"], t["W1"], t["b1"], t["W2"], t["b2"], act=t["act"],
                                    trace_of=t["trace_of"], score_sum=ssum, score_cnt=cnt, scores=scores,
                                    workspace=t["ws"], status=st)
        return lo, pr, ssum, cnt, scores

    st = new_status()
    alone = []
    for t in cases:
        alone.append(run(t, st))
        torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in cases]
    for _ in range(6):
        torch.cuda.synchronize()
        got = []
        for t, s in zip(cases, streams):
            with torch.cuda.stream(s):
                got.append(run(t, st))
        torch.cuda.synchronize()
        assert int(st.item()) == 0
        for a, b in zip(alone, got):
            for x, y in zip(a, b):
                assert torch.equal(x.view(torch.int32), y.view(torch.int32))
    t = dict(cases[1])
    nbytes = binding.score_workspace_bytes(binding.ScoreDims(t["N"], 4096, 512, 26, t["N"], 0))
    arena = binding.new_workspace(70 * ((nbytes + 255) // 256 * 256), DEV)
    for i in range(70):
        off = i * ((nbytes + 255) // 256 * 256)
        t["ws"] = arena[off:off + nbytes]
        for x, y in zip(alone[1], run(t, st)):
            assert torch.equal(x.view(torch.int32), y.view(torch.int32))
    assert int(st.item()) == 0


def test_logits_only_without_state():
    s = wl.build_scorer(79, 4, 4, 512, 64, 3, 1)
    lo, pr, *_ = run_gpu(s, 4, with_state=False)
    want_lo, _ = oracle.step_score(s.hidden, s.boundary_idx, s.W1, s.b1, s.W2, s.b2, act=1)
    assert np.abs(lo - want_lo).max() <= TOL


def test_device_reported_index_errors():
    s = wl.build_scorer(80, 4, 4, 256, 64, 3, 0)
    s.boundary_idx[1] = 4
    run_gpu(s, 4, expect_status=18)
    s = wl.build_scorer(80, 4, 4, 256, 64, 3, 0)
    s.trace_of[2] = -1
    run_gpu(s, 4, expect_status=18)


def test_host_reported_errors():
    s = wl.build_scorer(81, 4, 4, 256, 64, 3, 0)
    b2 = torch.zeros(1, dtype=torch.float32, device=DEV)
    with pytest.raises(binding.StepError) as e:                   # d not a multiple of 128
        binding.step_score(dev_bits(s.hidden[:, :200].copy()), dev(s.boundary_idx), dev_bits(s.W1[:, :200].copy()),
                           dev(s.b1), dev_bits(s.W2), b2, workspace=torch.zeros(4096, dtype=torch.uint8, device=DEV))
    assert e.value.code == 1
    with pytest.raises(binding.StepError) as e:                   # unknown activation
        binding.step_score(dev_bits(s.hidden), dev(s.boundary_idx), dev_bits(s.W1), dev(s.b1), dev_bits(s.W2), b2,
                           act=7, workspace=torch.zeros(4096, dtype=torch.uint8, device=DEV))
    assert e.value.code == 1
