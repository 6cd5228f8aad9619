"""The measurement aids of the library on the GPU: the plain copy kernel the byte counters are calibrated on, the
bare read probe, and the per-launch event timing the bench's roofline figures come from."""
import numpy as np
import pytest
import torch

from paper_2601_09093_amd import binding, workloads as wl
from tests.gpu_util import DEV, dev, dev_bits, new_status

pytestmark = pytest.mark.gpu
P = 16


def test_calibration_copy_copies():
    src = torch.arange(0, 1 << 20, dtype=torch.int32, device=DEV)
    dst = torch.zeros_like(src)
    binding.calib_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    odd = torch.arange(0, 4 * 37, dtype=torch.int32, device=DEV)     # not a multiple of a workgroup's share
    out = torch.zeros_like(odd)
    binding.calib_copy(out, odd)
    torch.cuda.synchronize()
    assert torch.equal(out, odd)


@pytest.mark.parametrize("pattern", [0, 1])
@pytest.mark.parametrize("nontemporal", [False, True])
def test_read_probe_runs_on_listed_pages_and_leaves_them_alone(pattern, nontemporal):
    NP, Hkv, D = 300, 2, 128
    k = wl.normal_bf16(wl.rng_for(61, 0), (NP, Hkv, P, D)); v = wl.normal_bf16(wl.rng_for(61, 1), (NP, Hkv, P, D))
    tk, tv = dev_bits(k), dev_bits(v)
    waves, per = 24, 11                                        # an odd number of pages per wave
    ids = wl.rng_for(61, 2).integers(0, NP, waves * per).astype(np.int32)
    ids[5] = NP + 7; ids[6] = -1                               # ids outside the pool are read as page 0
    sink = torch.zeros(1, dtype=torch.int32, device=DEV)
    binding.read_probe(tk, tv, dev(ids), waves, per, pattern, nontemporal, sink)
    torch.cuda.synchronize()
    assert int(sink.item()) in (0, 1)
    assert np.array_equal(tk.cpu().numpy().view(np.uint16), k) and np.array_equal(tv.cpu().numpy().view(np.uint16), v)


def test_per_launch_timing_names_the_kernels_of_a_call_in_order():
    lens = 64 + wl.rng_for(62, 0).integers(1, 900, 9)
    lay = wl.build_layout(lens, 64, P, wl.rng_for(62, 1), slack=1.2)
    q = wl.normal_bf16(wl.rng_for(62, 2), (9, 8, 128))
    k = wl.normal_bf16(wl.rng_for(62, 3), (lay.NP, 2, P, 128)); v = wl.normal_bf16(wl.rng_for(62, 4), (lay.NP, 2, P, 128))
    tq, tk, tv, bt, sl = dev_bits(q), dev_bits(k), dev_bits(v), dev(lay.block_tables), dev(lay.seq_lens)
    st = new_status()
    ref = binding.paged_decode_attn(tq, tk, tv, bt, sl, status=st)
    torch.cuda.synchronize()
    binding.profile_begin(8)
    out = binding.paged_decode_attn(tq, tk, tv, bt, sl, status=st)
    scores = dev(np.linspace(0.1, 0.9, 9).astype(np.float32))
    binding.prune_free(scores, 1, dev(lay.refcounts), bt.clone(), sl.clone(), status=st)
    timed = binding.profile_end(8)
    torch.cuda.synchronize()
    assert [n for n, _ in timed] == ["attn_front", "attn_partial", "attn_merge", "prune_fused"]
    assert all(0.0 < ms < 50.0 for _, ms in timed)
    assert int(st.item()) == 0 and torch.equal(out.view(torch.int16), ref.view(torch.int16))   # timing changes nothing
    with pytest.raises(binding.StepError):                     # nothing is being timed any more
        binding.profile_end(8)
