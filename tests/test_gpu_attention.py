"""GPU parity of paged_decode_attn (through the C ABI) against the float64 oracle, element by element
on the same seeded bytes.  Bar: max-abs 2e-2 on bf16 outputs (fp32 accumulation)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_09093_amd import binding, workloads as wl
from tests.gpu_util import DEV, dev, dev_bits, host_f32_of_bf16, host_bits, new_status

pytestmark = pytest.mark.gpu
TOL = 2e-2
P = 16


def run_gpu(q, k, v, bt, sl, scale=None, expect_status=0):
    st = new_status()
    out = binding.paged_decode_attn(dev_bits(q), dev_bits(k), dev_bits(v), dev(bt), dev(sl), scale=scale, status=st)
    torch.cuda.synchronize()
    assert int(st.item()) == expect_status, binding.ERROR_NAMES.get(int(st.item()))
    return host_f32_of_bf16(out)


def check(q, k, v, bt, sl, scale=None, tol=TOL):
    got = run_gpu(q, k, v, bt, sl, scale)
    want = oracle.paged_decode_attn(q, k, v, bt, sl, scale)
    assert np.all(np.isfinite(got))
    err = np.abs(got - want)
    # bf16 rounding of the output (2^-9 relative) plus fp32 accumulation noise
    assert np.all(err <= 2.0 ** -8 * np.abs(want) + 4e-3), float(err.max())
    assert err.max() <= tol
    return got, want


def build(seed, lens, Hq, Hkv, D, prompt=0, slack=1.3, poison=True, qstd=1.0):
    lay = wl.build_layout(np.asarray(lens), prompt, P, wl.rng_for(seed, 0), slack=slack)
    N = len(lens)
    q = wl.normal_bf16(wl.rng_for(seed, 1), (N, Hq, D), qstd)
    k = wl.normal_bf16(wl.rng_for(seed, 2), (lay.NP, Hkv, P, D))
    v = wl.normal_bf16(wl.rng_for(seed, 3), (lay.NP, Hkv, P, D))
    if poison:
        wl.poison_unused(k, v, lay, P)
    return lay, q, k, v


def test_config1_tiny_decode_step():
    w = wl.make_workload(1, poison=True)
    check(w.q, w.k_pages, w.v_pages, w.layout.block_tables, w.layout.seq_lens)
    w2 = wl.make_workload(1, poison=True, permute=False)
    check(w2.q, w2.k_pages, w2.v_pages, w2.layout.block_tables, w2.layout.seq_lens)


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_all_head_shapes(D, G):
    Hkv = 2
    lens = [1, 15, 16, 17, 100, 333, 512, 513, 1100]
    lay, q, k, v = build(100 + D + G, lens, G * Hkv, Hkv, D)
    check(q, k, v, lay.block_tables, lay.seq_lens)


def test_forty_query_heads_over_ten_kv_heads():
    """The 14B model of Section 5.1 has 40 query heads over 10 KV heads (the other two 32 over 8)."""
    lens = 64 + wl.rng_for(140, 5).integers(1, 2500, 24)
    lay, q, k, v = build(140, lens, 40, 10, 128, prompt=64)
    check(q, k, v, lay.block_tables, lay.seq_lens)


def test_ragged_edges_around_page_and_chunk_boundaries():
    lens = [0, 1, 2, 15, 16, 17, 31, 32, 33, 511, 512, 513, 527, 528, 529, 1023, 1024, 1025, 1537, 0, 2049]
    lay, q, k, v = build(7, lens, 8, 2, 128)
    got, _ = check(q, k, v, lay.block_tables, lay.seq_lens)
    assert np.all(got[0] == 0) and np.all(got[19] == 0)          # dead traces give zero rows
    vf = wl.bf16_bits_to_f32(v)
    assert np.array_equal(got[1, 5], vf[lay.block_tables[1, 0], 1, 0])   # L = 1: exactly v_0


def test_scaled_down_config2_shared_prompt():
    w = wl.make_workload(2, N=6, tail=(100, 2500), poison=True)
    assert w.shape.Hq == 32 and w.shape.Hkv == 8 and w.shape.D == 128
    check(w.q, w.k_pages, w.v_pages, w.layout.block_tables, w.layout.seq_lens)


def test_scaled_down_config3_fragmented_pool():
    w = wl.make_workload(3, N=8, tail=(700, 3000), poison=True)
    assert w.layout.NP > w.layout.used_pages                      # pool has holes
    assert np.all(w.layout.refcounts[w.layout.block_tables[0, :64]] == 8)
    check(w.q, w.k_pages, w.v_pages, w.layout.block_tables, w.layout.seq_lens)


def test_page_permutation_is_bit_identical_and_private_prefix_copies_agree():
    lens = [700, 1300, 64 + 5]
    lay, q, k, v = build(8, lens, 8, 2, 128, prompt=64, slack=1.0, poison=False)
    a = run_gpu(q, k, v, lay.block_tables, lay.seq_lens)
    perm = wl.rng_for(8, 9).permutation(lay.NP)
    k2 = np.empty_like(k); v2 = np.empty_like(v)
    k2[perm] = k; v2[perm] = v
    bt2 = np.where(lay.block_tables >= 0, perm[np.maximum(lay.block_tables, 0)], -1).astype(np.int32)
    assert np.array_equal(a, run_gpu(q, k2, v2, bt2, lay.seq_lens))
    # private copies of the 4 prompt pages for traces 1 and 2
    k3 = np.concatenate([k, np.zeros((8,) + k.shape[1:], np.uint16)])
    v3 = np.concatenate([v, np.zeros((8,) + v.shape[1:], np.uint16)])
    bt3 = lay.block_tables.copy(); nxt = lay.NP
    for i in (1, 2):
        for j in range(4):
            k3[nxt] = k[lay.block_tables[i, j]]; v3[nxt] = v[lay.block_tables[i, j]]
            bt3[i, j] = nxt; nxt += 1
    # a shared prefix is computed on the matrix cores, private copies by the streaming kernel: the
    # same mathematical result through two summation orders
    b, want = check(q, k3, v3, bt3, lay.seq_lens)
    assert np.all(np.abs(a - b) <= 2.0 ** -7 * np.abs(want) + 4e-3)
    assert np.abs(a - want).max() <= TOL


@pytest.mark.parametrize("switches", [{"STEP_ATTN_PREFIX": "0"}, {"STEP_ATTN_G4_MFMA": "1"},
                                      {"STEP_ATTN_PREFIX": "0", "STEP_ATTN_G4_MFMA": "1"},
                                      {"STEP_ATTN_WAVES_PER_CU": "8"}, {"STEP_ATTN_WAVES_PER_CU": "1"}])
def test_alternative_kernel_routes_meet_the_same_bar(switches):
    """STEP_ATTN_PREFIX=0 keeps the shared prefix in the streaming kernels, STEP_ATTN_G4_MFMA=1 sends
    group size 4 to the matrix-core streaming kernel, STEP_ATTN_WAVES_PER_CU changes into how many runs the
    private pages are cut (8 per unit: a second round of waves, and with one KV head the most runs a call
    takes; 1: a quarter of the usual) -- all read once per process, hence the child process; every route
    meets the same bar."""
    import json, os, subprocess, sys
    code = (
        "import sys, json; sys.path.insert(0, %r)\n"
        "import numpy as np, torch, oracle\n"
        "from paper_2601_09093_amd import binding, workloads as wl\n"
        "from tests.gpu_util import dev, dev_bits, host_f32_of_bf16, new_status\n"
        "errs = []\n"
        "for D, Hq, Hkv, prompt in ((128, 8, 2, 272), (64, 4, 1, 64), (128, 16, 2, 1024), (128, 2, 2, 48), (64, 8, 4, 0), (128, 32, 8, 16)):\n"
        "    lens = prompt + wl.rng_for(61, D).integers(1, 900, 20)\n"
        "    lay = wl.build_layout(lens, prompt, 16, wl.rng_for(61, 1), slack=1.2)\n"
        "    q = wl.normal_bf16(wl.rng_for(61, 2), (20, Hq, D))\n"
        "    k = wl.normal_bf16(wl.rng_for(61, 3), (lay.NP, Hkv, 16, D)); v = wl.normal_bf16(wl.rng_for(61, 4), k.shape)\n"
        "    wl.poison_unused(k, v, lay, 16)\n"
        "    st = new_status()\n"
        "    out = binding.paged_decode_attn(dev_bits(q), dev_bits(k), dev_bits(v), dev(lay.block_tables), dev(lay.seq_lens), status=st)\n"
        "    torch.cuda.synchronize()\n"
        "    want = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens)\n"
        "    errs.append([int(st.item()), float(np.abs(host_f32_of_bf16(out) - want).max())])\n"
        "print(json.dumps(errs))\n"
    ) % os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ)
    env.update(switches)
    res = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stderr[-2000:]
    for status, err in json.loads(res.stdout.strip().splitlines()[-1]):
        assert status == 0 and err <= TOL


def test_large_logits_and_dominant_key():
    lens = [300, 900, 40]
    lay, q, k, v = build(9, lens, 8, 2, 128, qstd=6.0)          # logits ~ N(0, 6^2): running max moves a lot
    check(q, k, v, lay.block_tables, lay.seq_lens)
    qf = wl.bf16_bits_to_f32(q)
    k[lay.block_tables[1, 20], 0, 3] = wl.f32_to_bf16_bits(8.0 * qf[1, 0])
    got, want = check(q, k, v, lay.block_tables, lay.seq_lens, scale=1.0)
    np.testing.assert_allclose(got[1, 0], wl.bf16_bits_to_f32(v)[lay.block_tables[1, 20], 0, 3], atol=1e-6)


def test_all_equal_keys_give_mean_of_v():
    lay, q, k, v = build(10, [777, 16, 3], 4, 1, 64, poison=False)
    k[:] = k[0, 0, 0]
    check(q, k, v, lay.block_tables, lay.seq_lens)


def test_device_reported_errors():
    lay, q, k, v = build(11, [100, 200], 4, 1, 64, poison=False)
    bt = lay.block_tables.copy(); bt[1, 2] = lay.NP
    run_gpu(q, k, v, bt, lay.seq_lens, expect_status=16)          # STEP_EPAGE
    bt[1, 2] = -1
    run_gpu(q, k, v, bt, lay.seq_lens, expect_status=16)
    sl = lay.seq_lens.copy(); sl[0] = lay.MAXB * P + 1
    run_gpu(q, k, v, lay.block_tables, sl, expect_status=17)      # STEP_ELEN
    sl[0] = -5
    run_gpu(q, k, v, lay.block_tables, sl, expect_status=17)
    # a page id out of range inside the shared prefix (same bad id in every row) is reported as well
    lay2, q2, k2, v2 = build(13, [64 + 40, 64 + 300, 64 + 7], 4, 1, 64, prompt=64, poison=False)
    bt2 = lay2.block_tables.copy(); bt2[:, 1] = lay2.NP + 3
    run_gpu(q2, k2, v2, bt2, lay2.seq_lens, expect_status=16)
    bt2[:, 1] = -1
    run_gpu(q2, k2, v2, bt2, lay2.seq_lens, expect_status=16)
    # garbage in unused block-table entries is ignored
    bt = lay.block_tables.copy(); bt[0, 7:] = 123456789
    got = run_gpu(q, k, v, bt, lay.seq_lens)
    assert np.array_equal(got, run_gpu(q, k, v, lay.block_tables, lay.seq_lens))


def test_host_reported_errors():
    lay, q, k, v = build(12, [100], 4, 1, 64, poison=False)
    tq, tk, tv, tb, tl = dev_bits(q), dev_bits(k), dev_bits(v), dev(lay.block_tables), dev(lay.seq_lens)
    with pytest.raises(binding.StepError) as e:                   # workspace too small
        binding.paged_decode_attn(tq, tk, tv, tb, tl, workspace=torch.zeros(256, dtype=torch.uint8, device=DEV))
    assert e.value.code == 2
    bad = torch.zeros(1, 4, 96, dtype=torch.int16, device=DEV)    # head_dim 96 unsupported
    kb = torch.zeros(2, 1, 16, 96, dtype=torch.int16, device=DEV)
    with pytest.raises(binding.StepError) as e:
        binding.paged_decode_attn(bad, kb, kb, tb, tl, workspace=torch.zeros(1 << 20, dtype=torch.uint8, device=DEV))
    assert e.value.code == 1
    for shape_q, shape_k in (((2049, 4, 64), (2, 1, 16, 64)),      # more traces than a call takes
                             ((1, 6, 64), (2, 2, 16, 64)),         # group size 3
                             ((1, 5, 64), (2, 2, 16, 64))):        # Hq not a multiple of Hkv
        bq = torch.zeros(shape_q, dtype=torch.int16, device=DEV)
        bk = torch.zeros(shape_k, dtype=torch.int16, device=DEV)
        with pytest.raises(binding.StepError) as e:
            binding.paged_decode_attn(bq, bk, bk, torch.zeros((shape_q[0], 2), dtype=torch.int32, device=DEV),
                                      torch.ones(shape_q[0], dtype=torch.int32, device=DEV),
                                      workspace=torch.zeros(1 << 20, dtype=torch.uint8, device=DEV))
        assert e.value.code == 1
    # N = 0 is a valid no-op
    binding.paged_decode_attn(tq[:0], tk, tv, tb[:0], tl[:0])
    torch.cuda.synchronize()


@pytest.mark.parametrize("case", ["many_short", "more_traces_than_waves", "single_trace", "all_shared",
                                  "long_prefix", "prefix_beyond_search_cap", "prefix_ends_ragged",
                                  "most_traces_a_call_takes", "two_traces"])
def test_corner_cases_of_the_cut(case):
    """Shapes that push the way a call is cut: shared-prefix detection, sub-chunking, runs that span many
    traces, more live traces than waves per KV head, traces that lie entirely inside the prefix."""
    r = wl.rng_for(900, 0)
    D, Hq, Hkv = 128, 8, 2
    if case == "many_short":
        lens = r.integers(1, 40, 300); lens[::7] = 0
        lay = wl.build_layout(lens, 0, P, wl.rng_for(901, 0), slack=1.2)
    elif case == "more_traces_than_waves":
        lens = 32 + r.integers(1, 200, 1500)                 # 1500 live traces, 2 shared pages
        lay = wl.build_layout(lens, 32, P, wl.rng_for(902, 0), slack=1.0)
        Hq, Hkv = 32, 8
    elif case == "single_trace":
        lay = wl.build_layout(np.array([0, 0, 5000, 0]), 0, P, wl.rng_for(903, 0))
    elif case == "all_shared":
        lay = wl.build_layout(np.array([160, 160, 160]), 160, P, wl.rng_for(904, 0))   # nothing private
    elif case == "long_prefix":
        lens = 300 * 16 + r.integers(1, 900, 5)              # 300 shared pages: two column blocks of the search
        lay = wl.build_layout(lens, 300 * 16, P, wl.rng_for(905, 0))
    elif case == "prefix_beyond_search_cap":
        lens = 1100 * 16 + r.integers(1, 500, 3)             # 1100 shared pages, above the 1024-page cap
        lay = wl.build_layout(lens, 1100 * 16, P, wl.rng_for(909, 0))
    elif case == "prefix_ends_ragged":
        lens = np.array([64 + 9, 64 + 9, 64 + 700])
        lay = wl.build_layout(lens, 64, P, wl.rng_for(906, 0))
        lay.block_tables[1, 4] = lay.block_tables[0, 4]      # traces 0 and 1 also share their ragged last page
    elif case == "most_traces_a_call_takes":
        lens = 64 + r.integers(1, 120, 2048); lens[5::97] = 0   # N = 2048, four shared pages
        lay = wl.build_layout(lens, 64, P, wl.rng_for(910, 0), slack=1.0)
        Hq, Hkv = 4, 1                                           # one KV head: 1024 waves on it
    else:
        lens = np.array([4000, 17])
        lay = wl.build_layout(lens, 16, P, wl.rng_for(907, 0))
    N = lay.seq_lens.size
    q = wl.normal_bf16(wl.rng_for(908, 1), (N, Hq, D))
    k = wl.normal_bf16(wl.rng_for(908, 2), (lay.NP, Hkv, P, D))
    v = wl.normal_bf16(wl.rng_for(908, 3), (lay.NP, Hkv, P, D))
    wl.poison_unused(k, v, lay, P)
    check(q, k, v, lay.block_tables, lay.seq_lens)


@pytest.mark.parametrize("G,D,Hkv,rep", [(4, 128, 2, 1), (1, 64, 2, 1), (8, 128, 2, 1), (2, 128, 2, 1), (8, 128, 8, 2),
                                         (8, 64, 8, 2)])
def test_blocks_of_traces_with_different_shared_prefixes(G, D, Hkv, rep):
    """Shared prefixes are found per block of 16 * QT / G consecutive traces.  Here groups of traces share
    different prompts of different lengths (two prompts in one batch), some blocks hold a single live trace or
    none, one trace ends inside its group's prompt pages, and the groups do not line up with the blocks.
    The last two shapes (104 traces of 8 query heads per KV head, 8 KV heads) have more blocks than a KV head's
    waves serve four sub-chunks each, so the shared-prefix kernel takes two query tiles per wave there."""
    r = wl.rng_for(4400 + G + D, 0)
    groups = [(11, 20), (7, 0), (9, 130), (5, 3), (13, 64), (1, 9), (6, 257)] * rep  # (traces, prompt pages)
    lens, prompts = [], []
    for n, pp in groups:
        for _ in range(n):
            lens.append(pp * P + int(r.integers(0 if pp else 1, 700)))
            prompts.append(pp)
    lens = np.array(lens)
    lens[3] = 0; lens[12] = 0; lens[30:34] = 0
    lens[20] = 130 * P                                             # ends exactly at its group's prompt
    N = lens.size
    nb = (lens + P - 1) // P
    MAXB = int(nb.max()) + 3
    bt = np.full((N, MAXB), -1, np.int32)
    nxt, i0 = 0, 0
    for n, pp in groups:                                           # prompt pages of a group, then private pages
        shared = np.arange(nxt, nxt + pp); nxt += pp
        for i in range(i0, i0 + n):
            if lens[i] == 0:
                continue
            bt[i, :pp] = shared
            bt[i, pp:nb[i]] = np.arange(nxt, nxt + nb[i] - pp); nxt += nb[i] - pp
        i0 += n
    perm = wl.rng_for(4400, 1).permutation(nxt + 17).astype(np.int32)
    bt = np.where(bt >= 0, perm[np.maximum(bt, 0)], -1).astype(np.int32)
    NP = nxt + 17
    sl = lens.astype(np.int32)
    lay = wl.PagedLayout(sl, bt, np.zeros(NP, np.int32), NP, MAXB, 0, nxt, 0, int(lens.sum()))
    q = wl.normal_bf16(wl.rng_for(4400, 2), (N, G * Hkv, D))
    k = wl.normal_bf16(wl.rng_for(4400, 3), (NP, Hkv, P, D))
    v = wl.normal_bf16(wl.rng_for(4400, 4), (NP, Hkv, P, D))
    wl.poison_unused(k, v, lay, P)
    got, _ = check(q, k, v, bt, sl)
    assert np.all(got[lens == 0] == 0)


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_and_length_mixes(seed):
    """Seeded sweep over head shapes (KV-head counts that do not divide the chip evenly included),
    trace counts, dead traces, shared-prefix lengths, pool slack and row widths wider than needed."""
    r = wl.rng_for(7000 + seed, 0)
    D = int(r.choice([64, 128]))
    G = int(r.choice([1, 2, 4, 4, 4, 8]))
    Hkv = int(r.choice([1, 2, 3, 5, 8, 10]))
    N = int(r.integers(1, 48))
    prompt = int(r.choice([0, 0, 16, 48, 272])) if seed % 2 else int(r.choice([0, 1024]))
    kind = r.integers(0, 4, N)
    lens = np.where(kind == 0, r.integers(1, 20, N),
                    np.where(kind == 1, r.integers(1, 600, N), r.integers(1, 3000, N))) + prompt
    lens[r.random(N) < 0.15] = 0
    nb_max = max(int((lens.max() + P - 1) // P), 1)
    lay = wl.build_layout(lens, prompt, P, wl.rng_for(7000 + seed, 1), slack=float(r.choice([1.0, 1.3, 2.0])),
                          maxb=nb_max + int(r.integers(0, 9)))
    q = wl.normal_bf16(wl.rng_for(7000 + seed, 2), (N, G * Hkv, D), float(r.choice([0.5, 1.0, 2.0])))
    k = wl.normal_bf16(wl.rng_for(7000 + seed, 3), (lay.NP, Hkv, P, D))
    v = wl.normal_bf16(wl.rng_for(7000 + seed, 4), (lay.NP, Hkv, P, D))
    wl.poison_unused(k, v, lay, P)
    bt = lay.block_tables.copy()
    nb = (lay.seq_lens.astype(np.int64) + P - 1) // P
    for i in range(N):                                            # unused entries hold garbage, not -1
        bt[i, nb[i]:] = r.integers(-5, 1 << 30, lay.MAXB - nb[i])
    got, want = check(q, k, v, bt, lay.seq_lens)
    assert np.all(got[lay.seq_lens == 0] == 0)


@pytest.mark.parametrize("seed", range(24))
def test_random_trace_counts_and_prefix_lengths(seed):
    """A second seeded sweep, wider in the number of traces (1 to 600) and in the shared prefix (0 to 300
    pages, around the 128-column trips of the shared-prefix search), with traces that end exactly at the
    prefix, many dead traces and short tails."""
    r = wl.rng_for(90000 + seed, 0)
    D = int(r.choice([64, 128, 128]))
    G = int(r.choice([1, 2, 4, 4, 4, 8]))
    Hkv = int(r.choice([1, 2, 3, 4, 5, 8, 10]))
    N = int(r.choice([1, 2, 3, 7, 16, 33, 64, 100, 257, 600]))
    prompt_pages = int(r.choice([0, 0, 1, 2, 3, 5, 17, 64, 255, 256, 257, 300]))
    if N >= 257:
        prompt_pages = min(prompt_pages, 17)
    prompt = prompt_pages * P
    maxtail = int(r.choice([20, 200, 1500, 4000])) if N <= 64 else int(r.choice([20, 200]))
    lens = r.integers(0 if prompt else 1, maxtail + 1, N) + prompt
    if prompt and r.random() < 0.5:
        lens[r.integers(0, N)] = prompt                           # a trace with nothing private
    lens[r.random(N) < r.choice([0.0, 0.1, 0.5])] = 0
    if not np.any(lens > 0):
        lens[0] = max(prompt, 1)
    nb_max = max(int((lens.max() + P - 1) // P), 1)
    lay = wl.build_layout(lens, prompt, P, wl.rng_for(90000 + seed, 1), slack=float(r.choice([1.0, 1.5])),
                          maxb=nb_max + int(r.integers(0, 5)))
    q = wl.normal_bf16(wl.rng_for(90000 + seed, 2), (N, G * Hkv, D), float(r.choice([0.5, 1.0, 3.0])))
    k = wl.normal_bf16(wl.rng_for(90000 + seed, 3), (lay.NP, Hkv, P, D))
    v = wl.normal_bf16(wl.rng_for(90000 + seed, 4), (lay.NP, Hkv, P, D))
    wl.poison_unused(k, v, lay, P)
    got = run_gpu(q, k, v, lay.block_tables, lay.seq_lens)
    want = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens)
    err = np.abs(got - want)
    # short traces of large values: the bf16 rounding of the output alone is 2^-9 |out|
    assert np.all(np.isfinite(got)) and np.all(err <= 2.0 ** -8 * np.abs(want) + 6e-3), float(err.max())
    assert err.max() <= TOL and np.all(got[lay.seq_lens == 0] == 0)


def test_full_config2():
    w = wl.make_workload(2)
    check(w.q, w.k_pages, w.v_pages, w.layout.block_tables, w.layout.seq_lens)


def _device_kv(NP, Hkv, D, seed):
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    k = torch.empty((NP, Hkv, P, D), dtype=torch.bfloat16, device=DEV).normal_(generator=g)
    v = torch.empty((NP, Hkv, P, D), dtype=torch.bfloat16, device=DEV).normal_(generator=g)
    return k, v


def test_full_config3_every_row():
    """Config 3 (the headline workload) at full size, in the launch configuration bench.py times: K/V
    are drawn on the device (about 6.5 GB), read back, and every one of the 64 x 32 output rows is
    compared with the float64 oracle, element by element.  (Config 5 at full size: tests/test_gpu_chain.py;
    config 4: tests/test_gpu_a_config4_sweep.py.)"""
    w = wl.make_workload(3, kv=False)
    lay, s = w.layout, w.shape
    k, v = _device_kv(lay.NP, s.Hkv, s.D, w.seed)
    st = new_status()
    out = binding.paged_decode_attn(dev_bits(w.q), k, v, dev(lay.block_tables), dev(lay.seq_lens), status=st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    got = host_f32_of_bf16(out)
    kh, vh = host_bits(k), host_bits(v)
    del k, v
    want = oracle.paged_decode_attn(w.q, kh, vh, lay.block_tables, lay.seq_lens)
    err = np.abs(got - want)
    assert np.all(np.isfinite(got)) and err.max() <= TOL, float(err.max())
    assert np.all(err <= 2.0 ** -8 * np.abs(want) + 4e-3), float(err.max())
    torch.cuda.empty_cache()


def test_one_plan_shared_by_several_layers():
    """Config 4's structure, scaled down: lognormal lengths, one plan per step, every layer's
    attention (own K/V pool, own q, same block tables) reuses it."""
    w = wl.make_workload(4, kv=False, N=12)
    lay, s = w.layout, w.shape
    layers = 3
    ws = binding.new_workspace(binding.attn_workspace_bytes(
        binding.AttnDims(s.N, s.Hq, s.Hkv, s.D, P, lay.MAXB, lay.NP, s.D ** -0.5)), DEV)
    bt, sl = dev(lay.block_tables), dev(lay.seq_lens)
    st = new_status()
    qs = [wl.normal_bf16(wl.rng_for(40 + l, 1), (s.N, s.Hq, s.D)) for l in range(layers)]
    ks = [wl.normal_bf16(wl.rng_for(40 + l, 2), (lay.NP, s.Hkv, P, s.D)) for l in range(layers)]
    vs = [wl.normal_bf16(wl.rng_for(40 + l, 3), (lay.NP, s.Hkv, P, s.D)) for l in range(layers)]
    tq, tk, tv = [dev_bits(x) for x in qs], [dev_bits(x) for x in ks], [dev_bits(x) for x in vs]
    binding.attn_plan(tq[0], tk[0], bt, sl, ws, status=st)
    outs = []
    for l in range(layers):
        out = torch.empty_like(tq[l])
        binding.paged_decode_attn_planned(tq[l], tk[l], tv[l], bt, sl, out, ws, status=st)
        outs.append(out)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    for l in range(layers):
        want = oracle.paged_decode_attn(qs[l], ks[l], vs[l], lay.block_tables, lay.seq_lens)
        got = host_f32_of_bf16(outs[l])
        assert np.abs(got - want).max() <= TOL
        # and bit-identical to the one-call form
        one = binding.paged_decode_attn(tq[l], tk[l], tv[l], bt, sl, status=st)
        torch.cuda.synchronize()
        assert np.array_equal(host_bits(one), host_bits(outs[l]))


@pytest.mark.parametrize("D,Hq,Hkv,N", [(64, 2, 2, 12), (64, 64, 8, 100), (128, 4, 2, 20), (128, 64, 8, 100)])
def test_planned_form_on_every_kernel_variant(D, Hq, Hkv, N):
    """The planned form (prefix lengths read from the workspace instead of searched) on the shapes the one-plan test
    does not reach: head dimension 64, one and two query tiles per wave of the shared-prefix kernel (two where the
    blocks of 16 query rows outnumber a third of a KV head's waves: 100 traces of 8 heads per KV head, 8 KV
    heads), the matrix-core streaming kernel.  Same bar as the one-call form and the same bits."""
    r = wl.rng_for(7700 + D + N, 0)
    lens = 96 + r.integers(1, 700, N); lens[3] = 0
    lay, q, k, v = build(7700 + D + N, lens, Hq, Hkv, D, prompt=96)
    tq, tk, tv, bt, sl = dev_bits(q), dev_bits(k), dev_bits(v), dev(lay.block_tables), dev(lay.seq_lens)
    ws = binding.new_workspace(binding.attn_workspace_bytes(
        binding.AttnDims(N, Hq, Hkv, D, P, lay.MAXB, lay.NP, D ** -0.5)), DEV)
    st = new_status()
    binding.attn_plan(tq, tk, bt, sl, ws, status=st)
    out = torch.empty_like(tq)
    binding.paged_decode_attn_planned(tq, tk, tv, bt, sl, out, ws, status=st)
    one = binding.paged_decode_attn(tq, tk, tv, bt, sl, status=st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    want = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens)
    assert np.abs(host_f32_of_bf16(out) - want).max() <= TOL
    assert np.array_equal(host_bits(one), host_bits(out))


@pytest.mark.parametrize("fill", [0, 0x7F, "other_dims"])
def test_attend_without_a_matching_plan_is_reported_not_followed(fill):
    """paged_decode_attn_planned on a workspace that holds no plan for these dims (cleared, garbage,
    or planned for another block-table width) reports STEP_EPLAN and reads nothing the records name."""
    lens = [40, 700, 33, 512, 90, 1500]
    lay, q, k, v = build(77, lens, 8, 2, 128)
    tq, tk, tv, bt, sl = dev_bits(q), dev_bits(k), dev_bits(v), dev(lay.block_tables), dev(lay.seq_lens)
    nbytes = binding.attn_workspace_bytes(binding.AttnDims(len(lens), 8, 2, 128, P, lay.MAXB, lay.NP, 128 ** -0.5))
    st = new_status()
    if fill == "other_dims":
        wide = np.concatenate([lay.block_tables, np.zeros_like(lay.block_tables)], axis=1)
        nb2 = binding.attn_workspace_bytes(binding.AttnDims(len(lens), 8, 2, 128, P, wide.shape[1], lay.NP, 128 ** -0.5))
        ws = binding.new_workspace(max(nbytes, nb2), DEV)
        binding.attn_plan(tq, tk, dev(np.ascontiguousarray(wide)), sl, ws, status=st)
        torch.cuda.synchronize()
        assert int(st.item()) == 0
    else:
        ws = torch.full((nbytes,), fill, dtype=torch.uint8, device=DEV)
    out = torch.empty_like(tq)
    binding.paged_decode_attn_planned(tq, tk, tv, bt, sl, out, ws, status=st)
    torch.cuda.synchronize()
    assert binding.ERROR_NAMES[int(st.item())] == "STEP_EPLAN"
    # the same workspace is good again once it has been planned for these dims
    st.zero_()
    binding.attn_plan(tq, tk, bt, sl, ws, status=st)
    binding.paged_decode_attn_planned(tq, tk, tv, bt, sl, out, ws, status=st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    want = oracle.paged_decode_attn(q, k, v, lay.block_tables, lay.seq_lens)
    assert np.abs(host_f32_of_bf16(out) - want).max() <= TOL
