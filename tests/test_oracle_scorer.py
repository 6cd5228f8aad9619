"""Pins of the step-scorer and running-mean oracles (Section 4.1 equation, Table 5 shape,
Section 4.3 running average, Appendix D operation count)."""
import json
import os

import numpy as np
import pytest
from scipy.special import erf, expit

import oracle
from paper_2601_09093_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")
bits = wl.f32_to_bf16_bits
f32 = wl.bf16_bits_to_f32


def _inf(v):
    return [float(x) for x in v]


def test_hand_worked_two_by_two():
    g = json.load(open(os.path.join(GOLD, "scorer_hand.json")))
    hidden = bits(np.array([[9.0, 9.0], g["h"]], np.float32))      # row 1 is the boundary row
    W1 = bits(np.array(g["W1"], np.float32)); W2 = bits(np.array(g["W2"], np.float32))
    b1 = np.array(g["b1"], np.float32)
    for c in g["cases"]:
        lo, pr = oracle.step_score(hidden, np.array([1], np.int32), W1, b1, W2, c["b2"], act=c["act"])
        assert lo[0] == pytest.approx(c["logit"], abs=1e-14)
        assert pr[0] == pytest.approx(c["prob"], abs=1e-14)


def _inputs(seed, R=6, d=48, m=20, B=5, act=0):
    return wl.build_scorer(seed, N=R, R=R, d=d, m=m, B=B, act=act, distinct_rows=False)


@pytest.mark.parametrize("act", [0, 1])
def test_library_float64_linear_act_linear(act):
    s = _inputs(21, act=act)
    lo, pr = oracle.step_score(s.hidden, s.boundary_idx, s.W1, s.b1, s.W2, s.b2, act=act)
    X = f32(s.hidden).astype(np.float64)[s.boundary_idx]          # [B][d]
    Z = X @ f32(s.W1).astype(np.float64).T + s.b1.astype(np.float64)
    A = np.maximum(Z, 0) if act == 0 else 0.5 * Z * (1 + erf(Z / np.sqrt(2)))
    want = A @ f32(s.W2).astype(np.float64) + np.float64(np.float32(s.b2))
    np.testing.assert_allclose(lo, want, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(pr, expit(want), rtol=1e-12)


def test_library_on_config1_shape_gelu():
    w = wl.make_workload(1, kv=False)
    s = w.scorer
    assert s.hidden.shape == (8, 256) and s.W1.shape == (64, 256) and s.act == 1 and s.boundary_idx.size == 8
    lo, _ = oracle.step_score(s.hidden, s.boundary_idx, s.W1, s.b1, s.W2, s.b2, act=1)
    Z = f32(s.hidden).astype(np.float64)[s.boundary_idx] @ f32(s.W1).astype(np.float64).T + s.b1
    want = (0.5 * Z * (1 + erf(Z / np.sqrt(2)))) @ f32(s.W2).astype(np.float64) + np.float64(np.float32(s.b2))
    np.testing.assert_allclose(lo, want, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("act", [0, 1])
def test_zero_W1_closed_form(act):
    s = _inputs(22, act=act)
    W1 = np.zeros_like(s.W1)
    lo, _ = oracle.step_score(s.hidden, s.boundary_idx, W1, s.b1, s.W2, s.b2, act=act)
    z = s.b1.astype(np.float64)
    a = np.maximum(z, 0) if act == 0 else 0.5 * z * (1 + erf(z / np.sqrt(2)))
    want = np.float64(np.float32(s.b2)) + np.dot(f32(s.W2).astype(np.float64), a)
    np.testing.assert_allclose(lo, np.full(5, want), rtol=1e-13)


def test_zero_W2_gives_sigmoid_of_b2():
    s = _inputs(23)
    lo, pr = oracle.step_score(s.hidden, s.boundary_idx, s.W1, s.b1, np.zeros_like(s.W2), 0.75)
    assert np.all(lo == 0.75)
    np.testing.assert_allclose(pr, 1 / (1 + np.exp(-0.75)), rtol=1e-15)


def test_relu_is_positively_homogeneous():
    s = _inputs(24)
    lo1, _ = oracle.step_score(s.hidden, s.boundary_idx, s.W1, s.b1, s.W2, 0.125)
    h4 = bits(4.0 * f32(s.hidden))                                 # exact: power-of-two factor
    lo4, _ = oracle.step_score(h4, s.boundary_idx, s.W1, 4 * s.b1, s.W2, 0.125)
    np.testing.assert_allclose(lo4 - 0.125, 4 * (lo1 - 0.125), rtol=1e-12, atol=1e-15)


def test_W1_is_m_by_d_not_transposed():
    # unit j responds to input coordinate j only when W1[j][j] = 1: a transposed read would differ
    d, m = 3, 2
    hidden = bits(np.array([[1.0, 2.0, 4.0]], np.float32))
    W1 = bits(np.array([[0, 1, 0], [0, 0, 1]], np.float32))         # z = [h1, h2] = [2, 4]
    W2 = bits(np.array([1.0, 0.5], np.float32))
    lo, _ = oracle.step_score(hidden, np.array([0], np.int32), W1, np.zeros(m, np.float32), W2, 0.0)
    assert lo[0] == 2.0 + 0.5 * 4.0


def test_duplicate_and_permuted_boundaries():
    s = _inputs(25)
    idx = np.array([3, 3, 0, 5, 3], np.int32)
    lo, _ = oracle.step_score(s.hidden, idx, s.W1, s.b1, s.W2, s.b2)
    assert lo[0] == lo[1] == lo[4]
    lo2, _ = oracle.step_score(s.hidden, idx[::-1].copy(), s.W1, s.b1, s.W2, s.b2)
    assert np.array_equal(lo2, lo[::-1])


def test_operation_count_matches_appendix_d():
    """Appendix D prices the scorer at 2m(d+1) operations per step: m(d+1) multiply-adds, i.e.
    m*d products in W1 h plus m products in W2 a.  Count them via linearity: with all-ones
    weights and inputs and ReLU, logit - b2 = m * (d + b1) exactly."""
    d, m = 37, 11
    one = bits(np.ones((1, d), np.float32))
    lo, _ = oracle.step_score(one, np.array([0], np.int32), bits(np.ones((m, d), np.float32)),
                              np.zeros(m, np.float32), bits(np.ones(m, np.float32)), 0.0)
    assert lo[0] == m * d                       # m*d first-layer products, m second-layer products
    assert 2 * (m * d + m) == 2 * m * (d + 1)


def test_boundary_index_errors():
    s = _inputs(26)
    for bad in (-1, 6):
        with pytest.raises(oracle.OracleError) as e:
            oracle.step_score(s.hidden, np.array([0, bad], np.int32), s.W1, s.b1, s.W2, s.b2)
        assert e.value.name == "EINDEX"
    lo, pr = oracle.step_score(s.hidden, np.zeros(0, np.int32), s.W1, s.b1, s.W2, s.b2)
    assert lo.size == 0 and pr.size == 0
    for act in (-1, 2):                                     # only the two named activations exist
        with pytest.raises(oracle.OracleError) as e:
            oracle.step_score(s.hidden, np.array([0], np.int32), s.W1, s.b1, s.W2, s.b2, act=act)
        assert e.value.name == "EINVAL"
    for bad in (-1, 3):                                     # a boundary of a trace that does not exist
        sm, cn = np.ones(3, np.float32), np.ones(3, np.int32)
        with pytest.raises(oracle.OracleError) as e:
            oracle.running_mean(np.array([1, bad], np.int32), np.array([0.5, 0.5], np.float32), sm, cn)
        assert e.value.name == "EINDEX" and sm.tolist() == [1, 1, 1] and cn.tolist() == [1, 1, 1]


def test_running_mean_hand_cases():
    g = json.load(open(os.path.join(GOLD, "running_mean_hand.json")))
    for c in g["cases"]:
        ssum = np.array(c["sum0"], np.float32); cnt = np.array(c["cnt0"], np.int32)
        sc = oracle.running_mean(np.array(c["trace_of"], np.int32), np.array(c["probs"], np.float32), ssum, cnt)
        assert np.array_equal(ssum, np.array(c["sum"], np.float32))
        assert np.array_equal(cnt, np.array(c["cnt"], np.int32))
        assert np.array_equal(sc, np.array(_inf(c["scores"]), np.float32))


def test_running_mean_is_fp32_sequential_in_index_order():
    # 1 + 2^-24 + 2^-24: sequential fp32 addition rounds each step back to 1 (ties to even);
    # any pairwise / higher-precision sum would give 1 + 2^-23.
    t = np.zeros(3, np.int32)
    probs = np.array([1.0, 2.0 ** -24, 2.0 ** -24], np.float32)
    ssum = np.zeros(1, np.float32); cnt = np.zeros(1, np.int32)
    sc = oracle.running_mean(t, probs, ssum, cnt)
    assert ssum[0] == np.float32(1.0) and cnt[0] == 3
    assert sc[0] == np.float32(1.0) / np.float32(3.0)
    # and the other order does reach the larger sum
    ssum[:] = 0; cnt[:] = 0
    oracle.running_mean(t, probs[::-1].copy(), ssum, cnt)
    assert ssum[0] == np.float32(1.0 + 2.0 ** -23)


def test_running_mean_matches_mean_of_all_probs():
    r = wl.rng_for(27, 0)
    N, B = 5, 40
    t = r.integers(0, N, B).astype(np.int32)
    p = (r.integers(0, 257, B) / 256.0).astype(np.float32)          # dyadic: exact in fp32
    ssum = np.zeros(N, np.float32); cnt = np.zeros(N, np.int32)
    sc = oracle.running_mean(t, p, ssum, cnt)
    for i in range(N):
        if (t == i).any():
            assert sc[i] == np.float32(np.float32(p[t == i].astype(np.float64).sum()) / np.float32((t == i).sum()))
        else:
            assert np.isposinf(sc[i])
    with pytest.raises(oracle.OracleError):
        oracle.running_mean(np.array([N], np.int32), p[:1].copy(), ssum, cnt)
