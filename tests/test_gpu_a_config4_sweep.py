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


def test_config4_full_sweep_three_layers_every_row():
    """Config 4 at full size: 36 layers, N = 128 traces with lognormal lengths, ~210 GB of bf16 KV
    drawn on the device, one plan for the step, 36 attention calls; parity on layers 0, 17 and 35
    for every (trace, head) row (that layer's K/V pool is read back for the oracle).  Skipped when
    the device does not have the memory free."""
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
    for l in (0, 17, 35):
        print("config 4: oracle on layer %d, all %d x %d rows" % (l, s.N, s.Hq), flush=True)
        got = host_f32_of_bf16(outs[l])
        want = oracle.paged_decode_attn(host_bits(qs[l]), host_bits(ks[l]), host_bits(vs[l]), lay.block_tables,
                                        lay.seq_lens)
        err = np.abs(got - want)
        assert np.all(np.isfinite(got)) and err.max() <= TOL, (l, float(err.max()))
        assert np.all(err <= 2.0 ** -8 * np.abs(want) + 4e-3), (l, float(err.max()))
    for l in range(layers):    # the other layers: finite, inside the value range of a convex combination
        got = host_f32_of_bf16(outs[l])
        assert np.all(np.isfinite(got)) and np.abs(got).max() < 6.0, l
    del ks, vs
    torch.cuda.empty_cache()
