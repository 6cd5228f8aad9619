"""Pins of the attention oracle against things other than itself: library brute force, closed
forms and invariants.  The paper gives no formula or worked example for the attention inside
NextToken (Algorithm 1); the definition pinned here is textbook softmax attention."""
import numpy as np
import pytest

import oracle
from paper_2601_09093_amd import workloads as wl
from tests.helpers import dense_attention

P = 16


def _tiny(seed, N=3, Hq=4, Hkv=2, D=8, lens=(5, 16, 37), prompt=0, slack=1.5, permute=True):
    r = wl.rng_for(seed, 100)
    lay = wl.build_layout(np.array(lens), prompt, P, r, slack=slack, permute=permute)
    q = wl.normal_bf16(wl.rng_for(seed, 101), (N, Hq, D))
    k = wl.normal_bf16(wl.rng_for(seed, 102), (lay.NP, Hkv, P, D))
    v = wl.normal_bf16(wl.rng_for(seed, 103), (lay.NP, Hkv, P, D))
    return lay, q, k, v


@pytest.mark.parametrize("seed,Hq,Hkv,D", [(1, 4, 2, 8), (2, 4, 1, 64), (3, 8, 2, 16), (4, 6, 6, 8)])
def test_brute_force_dense_softmax(seed, Hq, Hkv, D):
    lay, q, k, v = _tiny(seed, Hq=Hq, Hkv=Hkv, D=D)
    scale = 1.0 / np.sqrt(D)
    got = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens, scale)
    want = dense_attention(q, k, v, lay.block_tables, lay.seq_lens, scale)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_brute_force_with_shared_prompt_config1():
    w = wl.make_workload(1)
    got = oracle.paged_decode_attn(w.q, w.k_pages, w.v_pages, w.layout.block_tables, w.layout.seq_lens)
    want = dense_attention(w.q, w.k_pages, w.v_pages, w.layout.block_tables, w.layout.seq_lens, 1 / 8.0)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    assert np.all(w.layout.refcounts[w.layout.block_tables[0, :4]] == 4)  # prompt's 4 pages shared by all


def test_default_scale_is_inverse_sqrt_D():
    lay, q, k, v = _tiny(5, D=16)
    a = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens)
    b = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens, 0.25)
    assert np.array_equal(a, b)


def test_all_equal_keys_give_mean_of_v():
    lay, q, k, v = _tiny(6)
    k[:] = k[0, 0, 0]  # every key row identical, every head
    got = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens)
    vf = wl.bf16_bits_to_f32(v).astype(np.float64)
    for i, L in enumerate(lay.seq_lens):
        for h in range(4):
            rows = [vf[lay.block_tables[i, t // P], h // 2, t % P] for t in range(L)]
            np.testing.assert_allclose(got[i, h], np.mean(rows, axis=0), rtol=1e-13, atol=1e-14)


def test_single_token_returns_its_value_row_exactly():
    lay, q, k, v = _tiny(7, lens=(1, 1, 1))
    got = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens)
    vf = wl.bf16_bits_to_f32(v).astype(np.float64)
    for i in range(3):
        for h in range(4):
            assert np.array_equal(got[i, h], vf[lay.block_tables[i, 0], h // 2, 0])


def test_zero_length_trace_gives_zero_row():
    lay, q, k, v = _tiny(8, lens=(0, 20, 0))
    got, lse = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens, return_lse=True)
    assert np.all(got[0] == 0) and np.all(got[2] == 0) and np.all(np.isneginf(lse[0]))
    assert np.any(got[1] != 0)


def test_page_permutation_is_bit_identical():
    lay, q, k, v = _tiny(9)
    a = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens)
    perm = wl.rng_for(9, 7).permutation(lay.NP)          # new id of old page p is perm[p]
    k2 = np.empty_like(k); v2 = np.empty_like(v)
    k2[perm] = k; v2[perm] = v
    bt2 = np.where(lay.block_tables >= 0, perm[np.maximum(lay.block_tables, 0)], -1).astype(np.int32)
    b = oracle.paged_decode_attn(q, k2, v2, bt2, lay.seq_lens)
    assert np.array_equal(a, b)


def test_shared_prefix_equals_private_copies_bitwise():
    lens = np.array([48, 70, 33])
    lay = wl.build_layout(lens, 32, P, wl.rng_for(10, 0), slack=1.0)
    q = wl.normal_bf16(wl.rng_for(10, 1), (3, 4, 8))
    k = wl.normal_bf16(wl.rng_for(10, 2), (lay.NP, 2, P, 8))
    v = wl.normal_bf16(wl.rng_for(10, 3), (lay.NP, 2, P, 8))
    a = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens)
    # give traces 1 and 2 private copies of the two prompt pages
    extra = 4
    k2 = np.concatenate([k, np.zeros((extra,) + k.shape[1:], np.uint16)])
    v2 = np.concatenate([v, np.zeros((extra,) + v.shape[1:], np.uint16)])
    bt2 = lay.block_tables.copy()
    nxt = lay.NP
    for i in (1, 2):
        for j in range(2):
            k2[nxt] = k[lay.block_tables[i, j]]; v2[nxt] = v[lay.block_tables[i, j]]
            bt2[i, j] = nxt; nxt += 1
    b = oracle.paged_decode_attn(q, k2, v2, bt2, lay.seq_lens)
    assert np.array_equal(a, b)


def test_dominant_key_selects_its_value():
    lay, q, k, v = _tiny(11, D=8, lens=(9, 30, 40))
    qf = wl.bf16_bits_to_f32(q)
    vf = wl.bf16_bits_to_f32(v).astype(np.float64)
    tok = {0: 3, 1: 17, 2: 39}
    for i, t in tok.items():
        # key of token t in KV head 0 := 64 * q[i, head 0]  (exact in bf16: power-of-two factor)
        k[lay.block_tables[i, t // P], 0, t % P] = wl.f32_to_bf16_bits(64.0 * qf[i, 0])
    got = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens, 1.0)
    for i, t in tok.items():
        np.testing.assert_allclose(got[i, 0], vf[lay.block_tables[i, t // P], 0, t % P], atol=1e-9)


def test_split_and_merge_identity():
    """Attention over [0, L) equals the lse-weighted merge of attention over [0, a) and [a, L)."""
    lay, q, k, v = _tiny(12, lens=(64, 45, 37))
    full, lse = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens, return_lse=True)
    a = 32  # two pages
    l1 = np.minimum(lay.seq_lens, a).astype(np.int32)
    o1, s1 = oracle.paged_decode_attn(q, k, v, lay.block_tables, l1, return_lse=True)
    bt2 = np.full_like(lay.block_tables, -1)
    bt2[:, :-2] = lay.block_tables[:, 2:]
    l2 = (lay.seq_lens - l1).astype(np.int32)
    o2, s2 = oracle.paged_decode_attn(q, k, v, bt2, l2, return_lse=True)
    w1 = np.exp(s1 - lse)[..., None]
    w2 = np.exp(s2 - lse)[..., None]
    np.testing.assert_allclose(w1 * o1 + w2 * o2, full, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(np.exp(s1 - lse) + np.exp(s2 - lse), 1.0, rtol=1e-12)


def test_lse_matches_library_logsumexp():
    from scipy.special import logsumexp
    from tests.helpers import gather_dense
    lay, q, k, v = _tiny(13)
    _, lse = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens, 0.5, return_lse=True)
    qf = wl.bf16_bits_to_f32(q).astype(np.float64)
    for i, L in enumerate(lay.seq_lens):
        K = gather_dense(k, lay.block_tables[i], int(L), 1, P)
        np.testing.assert_allclose(lse[i, 3], logsumexp(0.5 * (K @ qf[i, 3])), rtol=1e-13)


def test_nan_in_unowned_slots_is_never_read():
    w = wl.make_workload(1)
    a = oracle.paged_decode_attn(w.q, w.k_pages, w.v_pages, w.layout.block_tables, w.layout.seq_lens)
    k2 = w.k_pages.copy(); v2 = w.v_pages.copy()
    wl.poison_unused(k2, v2, w.layout, P)
    assert np.isnan(wl.bf16_bits_to_f32(k2)).any()
    b = oracle.paged_decode_attn(w.q, k2, v2, w.layout.block_tables, w.layout.seq_lens)
    assert np.all(np.isfinite(b)) and np.array_equal(a, b)


def test_scaling_q_by_two_equals_doubling_scale():
    lay, q, k, v = _tiny(14)
    q2 = wl.f32_to_bf16_bits(2.0 * wl.bf16_bits_to_f32(q))
    a = oracle.paged_decode_attn(q2, k, v, lay.block_tables, lay.seq_lens, 0.25)
    b = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens, 0.5)
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-15)


def test_selected_rows_match_full():
    lay, q, k, v = _tiny(15)
    full = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens)
    rows = (np.array([2, 0, 1, 2]), np.array([3, 0, 2, 1]))
    sel = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens, rows=rows)
    for r in range(4):
        assert np.array_equal(sel[r], full[rows[0][r], rows[1][r]])


def test_errors():
    lay, q, k, v = _tiny(16)
    bt = lay.block_tables.copy(); bt[1, 0] = lay.NP
    with pytest.raises(oracle.OracleError) as e:
        oracle.paged_decode_attn(q, k, v, bt, lay.seq_lens)
    assert e.value.name == "EPAGE"
    bt[1, 0] = -1
    with pytest.raises(oracle.OracleError):
        oracle.paged_decode_attn(q, k, v, bt, lay.seq_lens)
    sl = lay.seq_lens.copy(); sl[2] = lay.MAXB * P + 1
    with pytest.raises(oracle.OracleError) as e:
        oracle.paged_decode_attn(q, k, v, lay.block_tables, sl)
    assert e.value.name == "ELEN"
    with pytest.raises(oracle.OracleError):   # Hq not a multiple of Hkv
        oracle.paged_decode_attn(q[:, :3].copy(), k, v, lay.block_tables, lay.seq_lens)
    # two different mistakes: the one in the earlier (trace, head) row is the one reported
    bt = lay.block_tables.copy(); bt[2, 0] = lay.NP
    sl = lay.seq_lens.copy(); sl[0] = -1
    with pytest.raises(oracle.OracleError) as e:
        oracle.paged_decode_attn(q, k, v, bt, sl)
    assert e.value.name == "ELEN"
    sl = lay.seq_lens.copy(); sl[2] = -1
    bt = lay.block_tables.copy(); bt[0, 0] = lay.NP
    with pytest.raises(oracle.OracleError) as e:
        oracle.paged_decode_attn(q, k, v, bt, sl)
    assert e.value.name == "EPAGE"
