"""Config 4 at full size through the C ABI: the 36-layer sweep with one plan per decode step.

This is the heaviest GPU test (about 210 GB of KV are drawn and swept); the file name makes pytest
collect it first, so that the lighter tests, not a benchmark started right after the suite, follow it."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_09093_amd import binding, workloads as wl
from tests.gpu_util import DEV, dev, host_f32_of_bf16, host_bits, new_status

pytestmark = pytest.mark.gpu
TOL = 2e-2
P = 16


def test_config4_full_sweep_sampled_layers():
    """Config 4 at full size: 36 layers, N = 128 traces with lognormal lengths, ~210 GB of bf16 KV
    drawn on the device, one plan for the step, 36 attention calls; parity on layers 0, 17 and 35
    for sampled (trace, head) rows.  Skipped when the device does not have the memory free."""
    w = wl.make_workload(4, kv=False)
    lay, s = w.layout, w.shape
    layers = w.layers
    need = 2 * layers * lay.NP * s.Hkv * P * s.D * 2
    free_b, _ = torch.cuda.mem_get_info()
    if need > free_b - (12 << 30):
        pytest.skip("needs %.0f GB of device memory, %.0f GB free" % (need / 1e9, free_b / 1e9))
    g = torch.Generator(device=DEV); g.manual_seed(w.seed)
    shape = (lay.NP, s.Hkv, P, s.D)
    ks = [torch.empty(shape, dtype=torch.bfloat16, device=DEV).normal_(generator=g) for _ in range(layers)]
    vs = [torch.empty(shape, dtype=torch.bfloat16, device=DEV).normal_(generator=g) for _ in range(layers)]
    qs = [torch.empty((s.N, s.Hq, s.D), dtype=torch.bfloat16, device=DEV).normal_(generator=g) for _ in range(layers)]
    bt, sl = dev(lay.block_tables), dev(lay.seq_lens)
    st = new_status()
    ws = binding.new_workspace(binding.attn_workspace_bytes(binding.attn_dims(qs[0], ks[0], bt)), DEV)
    outs = [torch.empty_like(qs[0]) for _ in range(layers)]
    binding.attn_plan(qs[0], ks[0], bt, sl, ws, status=st)
    for l in range(layers):
        binding.paged_decode_attn_planned(qs[l], ks[l], vs[l], bt, sl, outs[l], ws, status=st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    order = np.argsort(lay.seq_lens)
    traces = np.unique([order[0], order[-1], order[len(order) // 2]])
    heads = np.arange(s.Hkv) * (s.Hq // s.Hkv) + (np.arange(s.Hkv) % (s.Hq // s.Hkv))
    pages = np.unique(np.concatenate([lay.block_tables[t][: (lay.seq_lens[t] + P - 1) // P] for t in traces]))
    remap = -np.ones(lay.NP, np.int64); remap[pages] = np.arange(pages.size)
    idx = torch.from_numpy(pages).to(DEV)
    btr = np.where(lay.block_tables[traces] >= 0, remap[np.maximum(lay.block_tables[traces], 0)], -1).astype(np.int32)
    slr = lay.seq_lens[traces].copy()
    rows = (np.repeat(np.arange(traces.size), heads.size).astype(np.int32), np.tile(heads, traces.size).astype(np.int32))
    for l in (0, 17, 35):
        got = host_f32_of_bf16(outs[l])
        assert np.all(np.isfinite(got))
        kh = host_bits(ks[l].index_select(0, idx)); vh = host_bits(vs[l].index_select(0, idx))
        qh = np.ascontiguousarray(host_bits(qs[l])[traces])
        want = oracle.paged_decode_attn(qh, kh, vh, btr, slr, rows=rows)
        err = np.abs(got[traces][rows[0], rows[1]] - want)
        assert err.max() <= TOL, (l, float(err.max()))
    del ks, vs
    torch.cuda.empty_cache()
