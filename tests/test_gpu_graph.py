"""One decode step of Algorithm 1 (reserve pages with memory-triggered pruning -> KV append -> paged
attention -> step scorer + running mean) captured once as a HIP graph and replayed step after step on
an evolving state.  Every entry point only enqueues kernels on the caller's stream (no allocation, no
memset, no synchronisation, all control flow on the device), so the replayed steps must equal the
eagerly launched ones bit for bit; the eager path itself is checked against the oracle in
test_gpu_engine.py."""
import numpy as np
import pytest
import torch

from paper_2601_09093_amd import binding, workloads as wl
from tests.gpu_util import DEV, dev, dev_bits, new_status

pytestmark = pytest.mark.gpu
P = 16


def test_decode_step_replayed_as_hip_graph_matches_eager():
    N, Hq, Hkv, D, d, m, B = 8, 8, 2, 128, 256, 64, 3
    steps, NP, MAXB = 60, 24, 16
    lay = wl.build_layout(np.full(N, 32), 32, P, wl.rng_for(91, 1), slack=1.0, maxb=MAXB)
    rc0 = np.concatenate([lay.refcounts, np.zeros(NP - lay.NP, np.int32)])
    k0 = wl.normal_bf16(wl.rng_for(91, 2), (NP, Hkv, P, D))
    v0 = wl.normal_bf16(wl.rng_for(91, 3), k0.shape)
    sc = wl.build_scorer(91, N, N, d, m, 0, 0)
    init = dict(rc=dev(rc0), bt=dev(lay.block_tables), sl=dev(lay.seq_lens), k=dev_bits(k0), v=dev_bits(v0),
                sum=dev(np.zeros(N, np.float32)), cnt=dev(np.zeros(N, np.int32)),
                scores=dev(np.full(N, np.inf, np.float32)))
    S = {name: t.clone() for name, t in init.items()}                 # the evolving state
    W1, b1, W2 = dev_bits(sc.W1), dev(sc.b1), dev_bits(sc.W2)
    b2 = torch.tensor([sc.b2], dtype=torch.float32, device=DEV)
    # static step inputs and outputs (a graph replays fixed addresses)
    kn = torch.zeros(N, Hkv, D, dtype=torch.int16, device=DEV); vn = torch.zeros_like(kn)
    q = torch.zeros(N, Hq, D, dtype=torch.int16, device=DEV)
    hidden = torch.zeros(N, d, dtype=torch.int16, device=DEV)
    bidx = torch.zeros(B, dtype=torch.int32, device=DEV)
    out = torch.zeros_like(q)
    logits = torch.zeros(B, dtype=torch.float32, device=DEV); probs = torch.zeros_like(logits)
    pruned = torch.zeros(N, dtype=torch.int32, device=DEV); new_pages = torch.zeros_like(pruned)
    n_pruned = torch.zeros(1, dtype=torch.int32, device=DEV)
    st = new_status()
    ws_attn = binding.new_workspace(binding.attn_workspace_bytes(
        binding.AttnDims(N, Hq, Hkv, D, P, MAXB, NP, D ** -0.5)), DEV)
    ws_score = binding.new_workspace(binding.score_workspace_bytes(binding.ScoreDims(N, d, m, B, N, 0)), DEV)
    ws_res = binding.new_workspace(int(binding.lib().step_reserve_workspace_bytes(N, MAXB, NP)), DEV)

    def one_step():
        binding.reserve_pages(S["scores"], S["rc"], S["bt"], S["sl"], pruned=pruned, n_pruned=n_pruned,
                              new_pages=new_pages, workspace=ws_res, status=st)
        binding.append_kv(kn, vn, S["k"], S["v"], S["bt"], S["sl"], refcounts=S["rc"], status=st)
        binding.paged_decode_attn(q, S["k"], S["v"], S["bt"], S["sl"], out=out, workspace=ws_attn, status=st)
        binding.step_score(hidden, bidx, W1, b1, W2, b2, logits=logits, probs=probs, trace_of=bidx,
                           score_sum=S["sum"], score_cnt=S["cnt"], scores=S["scores"], workspace=ws_score, status=st)

    def feed(step):
        kn.copy_(dev_bits(wl.normal_bf16(wl.rng_for(3000 + step, 0), (N, Hkv, D))))
        vn.copy_(dev_bits(wl.normal_bf16(wl.rng_for(3000 + step, 1), (N, Hkv, D))))
        q.copy_(dev_bits(wl.normal_bf16(wl.rng_for(3000 + step, 2), (N, Hq, D))))
        hidden.copy_(dev_bits(wl.normal_bf16(wl.rng_for(3000 + step, 3), (N, d))))
        bidx.copy_(dev(wl.rng_for(3000 + step, 4).integers(0, N, B).astype(np.int32)))

    def snapshot():
        torch.cuda.synchronize()
        assert int(st.item()) == 0, binding.ERROR_NAMES.get(int(st.item()))
        return [t.clone() for t in (out, logits, probs, pruned[: int(n_pruned.item())], new_pages, n_pruned,
                                    S["rc"], S["bt"], S["sl"], S["scores"], S["sum"], S["cnt"])]

    binding.freelist_rebuild(S["rc"], ws_res)                         # the free list lives in ws_res from here on
    eager = []
    for step in range(steps):
        feed(step)
        one_step()
        eager.append(snapshot())
    final_eager = {name: t.clone() for name, t in S.items()}
    assert sum(int(e[5].item()) for e in eager) >= 2                 # the small pool forced pruning along the way

    for name, t in init.items():
        S[name].copy_(t)
    binding.freelist_rebuild(S["rc"], ws_res)
    feed(0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_step()
    for name, t in init.items():                                      # capture launches nothing, but be explicit
        S[name].copy_(t)
    binding.freelist_rebuild(S["rc"], ws_res)                         # the reference counts were reset: so is the list
    for step in range(steps):
        feed(step)
        graph.replay()
        got = snapshot()
        for a, b in zip(got, eager[step]):
            assert a.shape == b.shape and torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a,
                                                      b.view(torch.int32) if b.dtype == torch.float32 else b), step
    for name, t in final_eager.items():
        assert torch.equal(S[name], t), name
