#!/usr/bin/env python3
"""bench.py -- one decode step of the STEP hot path on one MI355X, timed end to end.

A "step" is one pass of the whole path over N parallel traces of one prompt:
    paged_decode_attn  ->  step_score (+ running-mean update)  ->  prune_free
on synthetic inputs shaped like the paper's N = 64 workload (workload config 3: 32 query /
8 KV heads, head_dim 128, 16-token pages, a shared 1024-token prompt and tails of 8k-32k tokens in
a fragmented page pool; scorer 4096 -> 1024 -> 1 on 4 boundary hidden states; Algorithm 1's prune
of the single lowest-scoring trace).  Inputs are resident in HBM before the timed region.
Every step gets its own copy of the (small) mutable state so that pruning does not shrink the
next step's work.

Prints ONE JSON line: metric, value, unit, ms_per_step, config, plus
  "roofline"        the dominant kernel (attention stage 1) against the HBM peak, from HIP events attached
                    to that kernel's launches, live in this run;
  "attention"       the whole paged_decode_attn call (all its kernels, all its bytes) against the same peak;
  "step_breakdown"  microseconds per step of every kernel of the step (same events);
  "cpu_baseline"    the oracle on the host cores.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5], help="workload config, 1-based (3: the N = 64 headline)")
    ap.add_argument("--layers", type=int, default=None, help="layers per step (default: the config's; config 4: 36)")
    ap.add_argument("--prune-k", type=int, default=None, help="traces pruned per step (default 1; config 5: 64)")
    ap.add_argument("--heads", default=None, metavar="HQ/HKV", help="another head shape on the config's lengths, e.g. 32/4")
    ap.add_argument("--head-dim", type=int, default=None, choices=[64, 128], help="another head dimension on the config's lengths")
    ap.add_argument("--scorer", default=None, metavar="D,M,B", help="another scorer shape, e.g. 4096,512,26 (the paper's width is 512)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle baseline sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mode", choices=["step", "loop"], default="step",
                    help="step: attention + scorer + prune_free(k) on a fresh copy of the state every step (default); "
                         "loop: Algorithm 1's decode loop on one evolving state: reserve pages (memory-triggered "
                         "pruning) + KV append + attention + scorer")
    ap.add_argument("--free-pages", type=int, default=16,
                    help="loop mode: free pages left in the pool at the start (the rest is marked occupied)")
    ap.add_argument("--graph", action="store_true", help="record the K timed steps as one HIP graph and time its replay")
    ap.add_argument("--calib-copy", type=int, default=0, metavar="MIB",
                    help="only run libstep's plain copy kernel on MIB MiB (profiler byte-counter calibration)")
    ap.add_argument("--launch-floor", action="store_true",
                    help="also time a 16-byte copy kernel launched right after every attention call of the profiled "
                         "steps: the duration of a kernel that does nothing, in the state the step's small kernels "
                         "start in (reported as launch_floor_us)")
    ap.add_argument("--read-probe", action="store_true",
                    help="only run the bare tile-read probe on the config's pool and private pages (what HBM delivers "
                         "to the streaming kernel's access pattern with no arithmetic behind it)")
    return ap.parse_args()


def kernel_source_hash():
    """sha256 over the HIP sources: a committed counter summary is quoted only for the code it was measured on."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2601_09093_amd", "csrc")
    for f in sorted(os.listdir(csrc)):
        if f.endswith((".hip", ".h")):
            h.update(f.encode())
            h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()[:16]


def traffic_from_profiles(kernel, workload):
    """(bytes per launch, source note): HBM bytes measured with rocprofv3 --pmc, taken from the committed summary
    only if that summary was made from the kernel sources of this tree; otherwise (None, why)."""
    rel = os.path.join("profiles", "%s_%s_pmc.txt" % (kernel, workload))
    val = sha = None
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic_bytes_per_launch:"):
                val = float(line.split(":", 1)[1])
            if line.startswith("source_sha256:"):
                sha = line.split(":", 1)[1].strip()
    except OSError:
        return None, "no counter summary for this workload under profiles/"
    if val is None:
        return None, "%s holds no traffic figure" % rel
    if sha != kernel_source_hash():
        return None, "%s was measured on other kernel sources (%s): not quoted" % (rel, sha)
    return val, "%s (two rocprofv3 --pmc runs of this command on these kernel sources, %s)" % (rel, sha)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not "
              "supported." % args.gpus, file=sys.stderr)
        sys.exit(2)
    if int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: WORLD_SIZE > 1 is not supported (one GPU only)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2601_09093_amd import binding, build as hip_build, workloads as wl
    hip_build.ensure_built()  # builds only a tree that has never been built

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; libstep has no CPU path", file=sys.stderr)
        sys.exit(3)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    binding.lib()

    if args.calib_copy:
        n = args.calib_copy << 20
        src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            binding.calib_copy(dst, src)
        torch.cuda.synchronize()
        print(json.dumps({"calib_copy_bytes": n, "launches": 5}))
        return

    K, W = args.steps, args.warmup
    heads = tuple(int(x) for x in args.heads.split("/")) if args.heads else None
    w = wl.make_workload(args.config, kv=False, heads=heads, head_dim=args.head_dim)
    lay, s, sc = w.layout, w.shape, w.scorer
    if args.scorer:
        d_, m_, B_ = (int(x) for x in args.scorer.split(","))
        sc = wl.build_scorer(w.seed, s.N, s.N, d_, m_, B_, 0, prior_state=(args.config == 5))
    prune_k = args.prune_k if args.prune_k is not None else (w.prune_k if args.config == 5 else 1)

    def bits(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(dev)

    def t(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    # ---- resident inputs -------------------------------------------------------------------
    layers = args.layers if args.layers is not None else w.layers
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    kv_shape = (lay.NP, s.Hkv, s.P, s.D)
    need = 2 * layers * lay.NP * s.Hkv * s.P * s.D * 2
    free_b, _ = torch.cuda.mem_get_info()
    if need > free_b - (8 << 30):
        print("bench.py: config %d with %d layers needs %.1f GB of KV, %.1f GB free" % (
            args.config, layers, need / 1e9, free_b / 1e9), file=sys.stderr)
        sys.exit(4)
    k_layers, v_layers = [], []
    step_pages = max(1, (1 << 29) // (s.Hkv * s.P * s.D))           # draw in 1 GiB pieces
    for _ in range(layers):
        pair = []
        for _kv in range(2):
            arr = torch.empty(kv_shape, dtype=torch.bfloat16, device=dev)
            for p0 in range(0, lay.NP, step_pages):
                p1 = min(lay.NP, p0 + step_pages)
                arr[p0:p1].normal_(generator=gen)
            pair.append(arr)
        k_layers.append(pair[0])
        v_layers.append(pair[1])
    k_pages, v_pages = k_layers[0], v_layers[0]
    G = s.Hq // s.Hkv
    nb = (lay.seq_lens.astype(np.int64) + s.P - 1) // s.P
    workload = "config%d" % args.config + ("-loop" if args.mode == "loop" else "")
    if heads or args.head_dim:
        workload += "-%dq%dkv-d%d" % (s.Hq, s.Hkv, s.D)

    if args.read_probe:
        read_probe(args, binding, torch, np, w, k_pages, v_pages, workload)
        return

    q = bits(w.q)
    out = torch.empty_like(q)
    q_layers = [q] + [torch.randn(q.shape, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
                      for _ in range(layers - 1)]
    hidden, W1, W2 = bits(sc.hidden), bits(sc.W1), bits(sc.W2)
    b1 = t(sc.b1)
    b2 = torch.tensor([sc.b2], dtype=torch.float32, device=dev)
    bidx, trace_of = t(sc.boundary_idx), t(sc.trace_of)
    B = int(sc.boundary_idx.size)
    logits = torch.empty(max(B, 1), dtype=torch.float32, device=dev)[:B]
    probs = torch.empty(max(B, 1), dtype=torch.float32, device=dev)[:B]
    scores = torch.empty(s.N, dtype=torch.float32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    # prior running-mean state so that every trace has a score (Algorithm 1 prunes scored traces)
    st = wl.rng_for(w.seed, 99)
    cnt0 = st.integers(1, 41, s.N).astype(np.int32)
    sum0 = (cnt0 * st.uniform(0.2, 0.8, s.N)).astype(np.float32)
    nsteps = 2 * K + W
    bt_s = t(np.broadcast_to(lay.block_tables, (nsteps,) + lay.block_tables.shape).copy())
    sl_s = t(np.broadcast_to(lay.seq_lens, (nsteps, s.N)).copy())
    rc_s = t(np.broadcast_to(lay.refcounts, (nsteps, lay.NP)).copy())
    sum_s = t(np.broadcast_to(sum0, (nsteps, s.N)).copy())
    cnt_s = t(np.broadcast_to(cnt0, (nsteps, s.N)).copy())
    pruned = torch.empty(max(prune_k, 1), dtype=torch.int32, device=dev)
    freed = torch.empty(max(min(lay.NP, prune_k * lay.MAXB), 1), dtype=torch.int32, device=dev)
    n_freed = torch.zeros(1, dtype=torch.int32, device=dev)

    adims = binding.attn_dims(q, k_pages, bt_s[0])
    ws_attn = binding.new_workspace(binding.attn_workspace_bytes(adims), dev)
    ws_score = binding.new_workspace(binding.score_workspace_bytes(
        binding.ScoreDims(sc.hidden.shape[0], sc.hidden.shape[1], sc.W1.shape[0], B, s.N, sc.act)), dev)
    ws_prune = binding.new_workspace(binding.prune_workspace_bytes(s.N, lay.MAXB, lay.NP), dev)

    floor_src = torch.zeros(16, dtype=torch.uint8, device=dev)
    floor_dst = torch.zeros(16, dtype=torch.uint8, device=dev)
    floor_on = [False]

    def step(i):
        if layers == 1:
            binding.paged_decode_attn(q, k_pages, v_pages, bt_s[i], sl_s[i], out=out, workspace=ws_attn, status=status)
            if floor_on[0]:
                binding.calib_copy(floor_dst, floor_src)
        else:  # the per-block shared-prefix lengths are found once per step and shared by every layer's attention
            binding.attn_plan(q, k_pages, bt_s[i], sl_s[i], ws_attn, status=status)
            for l in range(layers):
                binding.paged_decode_attn_planned(q_layers[l], k_layers[l], v_layers[l], bt_s[i], sl_s[i], out,
                                                  ws_attn, status=status)
        binding.step_score(hidden, bidx, W1, b1, W2, b2, act=sc.act, logits=logits, probs=probs, trace_of=trace_of,
                           score_sum=sum_s[i], score_cnt=cnt_s[i], scores=scores, workspace=ws_score, status=status)
        binding.prune_free(scores, prune_k, rc_s[i], bt_s[i], sl_s[i], pruned=pruned, freed_pages=freed,
                           n_freed=n_freed, workspace=ws_prune, status=status)

    if args.mode == "loop":
        # one evolving state; the pool is nearly full so that the memory trigger fires inside the run
        rc_np = lay.refcounts.copy()
        free_ids = np.nonzero(rc_np == 0)[0]
        rc_np[free_ids[args.free_pages:]] = 1                       # occupied by someone else
        # the rows get a few spare entries: a trace that sits at the config's length cap still grows
        bt_np = np.pad(lay.block_tables, ((0, 0), (0, (2 * K + W) // s.P + 2)), constant_values=-1)
        rc_l, bt_l, sl_l = t(rc_np), t(bt_np), t(lay.seq_lens)
        sum_l, cnt_l = t(sum0), t(cnt0)
        scores.copy_(t((sum0 / cnt0).astype(np.float32)))
        k_new = torch.randn((s.N, s.Hkv, s.D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        v_new = torch.randn((s.N, s.Hkv, s.D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        pruned_l = torch.empty(s.N, dtype=torch.int32, device=dev)
        n_pruned_l = torch.zeros(1, dtype=torch.int32, device=dev)
        new_pages_l = torch.empty(s.N, dtype=torch.int32, device=dev)
        ws_res = binding.reserve_workspace(rc_l, s.N, bt_np.shape[1])   # the free list is built once, then kept up
        live_at_start = int((lay.seq_lens > 0).sum())
        adims = binding.attn_dims(q, k_pages, bt_l)
        ws_attn = binding.new_workspace(binding.attn_workspace_bytes(adims), dev)

        def step(i):  # noqa: F811  (replaces the per-copy step above)
            binding.reserve_pages(scores, rc_l, bt_l, sl_l, pruned=pruned_l, n_pruned=n_pruned_l,
                                  new_pages=new_pages_l, workspace=ws_res, status=status)
            binding.append_kv(k_new, v_new, k_pages, v_pages, bt_l, sl_l, refcounts=rc_l, status=status)
            binding.paged_decode_attn(q, k_pages, v_pages, bt_l, sl_l, out=out, workspace=ws_attn, status=status)
            binding.step_score(hidden, bidx, W1, b1, W2, b2, act=sc.act, logits=logits, probs=probs,
                               trace_of=trace_of, score_sum=sum_l, score_cnt=cnt_l, scores=scores,
                               workspace=ws_score, status=status)
        n_freed.fill_(1)

    # state copies: W warm-up steps, K timed steps, K more steps with every kernel bracketed by events
    for i in range(W):
        step(i)
    graph = None
    if args.graph:
        # the K timed steps recorded once as a HIP graph (every entry point only enqueues kernels);
        # the timed region replays it
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(W, W + K):
                step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graph is not None:
        graph.replay()
    else:
        for i in range(W, W + K):
            step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # the same K steps again with HIP events attached to every kernel launch (the event records cost a few
    # microseconds each, so they stay out of the step time above)
    cap = K * (3 * layers + 12)
    floor_on[0] = args.launch_floor
    binding.profile_begin(cap)
    for i in range(W + K, W + 2 * K):
        step(i)
    torch.cuda.synchronize()
    timed = binding.profile_end(cap)
    assert int(status.item()) == 0, binding.ERROR_NAMES.get(int(status.item()))
    assert int(n_freed.item()) > 0 or prune_k == 0
    per_kernel = {}
    for name, ms in timed:
        per_kernel.setdefault(name, []).append(ms)
    stage1_ms = per_kernel["attn_partial"]
    assert len(stage1_ms) == K * layers
    breakdown = {name: round(1e3 * float(np.sum(v)) / K, 2) for name, v in per_kernel.items()}   # us per step
    floor_ms = per_kernel.pop("calib_copy", None)
    breakdown.pop("calib_copy", None)
    launches_per_step = (len(timed) - (len(floor_ms) if floor_ms else 0)) / K

    ms_per_step = (t1 - t0) * 1e3 / K
    value = s.N / (ms_per_step * 1e-3)                              # trace-tokens per second

    # ---- roofline of the dominant kernel (attention stage 1) --------------------------------
    hdr = ws_attn[:64].view(torch.int32).cpu().tolist()              # figures of the cut left by the streaming kernel
    pieces, private_pages, quota, prefix_slots, shared_pages = hdr[1], hdr[2], hdr[3], hdr[4], hdr[5]
    lens_now = sl_l.cpu().numpy() if args.mode == "loop" else lay.seq_lens
    nb_now = (lens_now.astype(np.int64) + s.P - 1) // s.P
    n_live = int((lens_now > 0).sum())
    assert private_pages == int(nb_now.sum()) - n_live * shared_pages, "per-block shared prefixes differ: not this workload"
    # the shared prompt runs on the matrix cores (attn_front); stage 1 streams the private pages only
    stage1_tokens = int(lens_now.sum()) - n_live * shared_pages * s.P
    part_bytes = s.Hkv * G * (s.D + 2) * 4                          # one partial slot: (m, l, acc) of every query head
    alg_bytes = (stage1_tokens * s.kv_bytes_per_token               # every KV byte stage 1 is responsible for, once
                 + private_pages * 4                                # block-table entries
                 + s.N * s.Hq * s.D * 2                             # q
                 + pieces * part_bytes)                             # split-K partials written by stage 1
    # the "requested" variant counts every trace's own view of its context (the shared prompt N times)
    req_bytes = alg_bytes + n_live * shared_pages * s.P * s.kv_bytes_per_token
    avg_ms = float(np.mean(stage1_ms))
    achieved = alg_bytes / (avg_ms * 1e-3) / 1e9
    traffic, traffic_source = traffic_from_profiles("attn_partial", workload)
    roofline = {
        "kernel": "attn_partial", "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_source,
        "algorithmic_bytes": int(alg_bytes), "requested_bytes": int(req_bytes), "avg_kernel_ms": round(avg_ms, 4),
        "median_kernel_ms": round(float(np.median(stage1_ms)), 4),
        "min_kernel_ms": round(float(np.min(stage1_ms)), 4), "launches": len(stage1_ms),
    }
    # ---- the whole attention call: every byte it has to move, every kernel it launches --------
    unique_tokens = stage1_tokens + (shared_pages * s.P if n_live else 0)
    attn_bytes = (unique_tokens * s.kv_bytes_per_token               # every resident referenced K/V byte once
                  + int(nb_now.sum()) * 4                            # block-table entries
                  + 2 * s.N * s.Hq * s.D * 2                         # q in, out
                  + 2 * (pieces + prefix_slots) * part_bytes)        # partials written, then read by the merge
    attn_us = sum(breakdown.get(kname, 0.0) for kname in ("attn_front", "attn_plan_blocks", "attn_partial", "attn_merge")) / layers
    attn_gbs = attn_bytes / (attn_us * 1e-6) / 1e9
    attention = {
        "bytes": int(attn_bytes), "us": round(attn_us, 2), "achieved": round(attn_gbs, 1), "unit": "GB/s",
        "frac": round(attn_gbs / HBM_PEAK_GBS, 4),
        "whole_step_frac": round(attn_bytes * layers / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "note": "all kernels of one paged_decode_attn call (per layer) over all its bytes; whole_step_frac divides the "
                "same bytes by ms_per_step (scorer and pruning included in the time)",
    }

    result = {
        "metric": "paged decode-attn HBM GB/s (%% of peak) + trace-tokens/s per step at N=%d" % s.N,
        "value": round(value, 1), "unit": "trace-tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": workload, "N": s.N, "Hq": s.Hq, "Hkv": s.Hkv, "D": s.D, "page_tokens": s.P,
                   "layers": layers, "prompt_tokens": lay.prompt_len, "context_tokens_total": lay.requested_tokens,
                   "unique_kv_tokens": lay.unique_tokens, "pool_pages": lay.NP, "scorer": "%d->%d->1 %s, B=%d" % (
                       sc.hidden.shape[1], sc.W1.shape[0], "ReLU" if sc.act == 0 else "GELU", B),
                   "prune_k": prune_k, "attn_waves_per_kv_head": binding.attn_waves_per_head(adims),
                   "attn_records": pieces, "attn_pages_per_wave": quota, "shared_prefix_pages_on_mfma": shared_pages,
                   "mode": args.mode, "launch": "hip-graph" if args.graph else "stream",
                   "kernel_launches_per_step": round(launches_per_step, 2)},
        "stage1_hbm_gbs": round(achieved, 1), "stage1_pct_of_peak": round(100 * achieved / HBM_PEAK_GBS, 2),
        "attn_hbm_gbs": round(attn_gbs, 1), "attn_pct_of_peak": round(100 * attn_gbs / HBM_PEAK_GBS, 2),
        "roofline": roofline, "attention": attention, "step_breakdown": breakdown,
    }

    if floor_ms:
        result["launch_floor_us"] = {"avg": round(1e3 * float(np.mean(floor_ms)), 2), "min": round(1e3 * float(np.min(floor_ms)), 2),
                                     "what": "a 16-byte copy kernel (one workgroup) right after each attention call"}
    if args.mode == "loop":
        # nothing else ends a trace in this loop, so the difference is what the memory trigger pruned
        result["config"]["traces_pruned_by_memory_trigger"] = live_at_start - int((sl_l > 0).sum().item())
        result["config"]["live_traces_at_end"] = int((sl_l > 0).sum().item())
        result["config"]["free_pages_at_start"] = args.free_pages
    if not args.no_cpu_baseline and args.mode == "step":
        result["cpu_baseline"] = cpu_baseline(args, w, sc, k_layers, v_layers, q_layers, sum0, cnt0, prune_k, layers)
    print(json.dumps(result))


def read_probe(args, binding, torch, np, w, k_pages, v_pages, workload):
    """Bare tile reads over the workload's pool: what the memory system delivers with no arithmetic behind it."""
    lay, s = w.layout, w.shape
    if s.D != 128:
        print("bench.py --read-probe: 4096-byte tiles (head_dim 128) only", file=sys.stderr)
        sys.exit(2)
    dev = k_pages.device
    pp = lay.prompt_len // s.P
    nb = (lay.seq_lens.astype(np.int64) + s.P - 1) // s.P
    private = np.concatenate([lay.block_tables[i, pp:nb[i]] for i in range(s.N) if nb[i] > pp]).astype(np.int32)
    adims = binding.AttnDims(s.N, s.Hq, s.Hkv, s.D, s.P, lay.MAXB, lay.NP, 1.0)
    waves = binding.attn_waves_per_head(adims)
    ppw = (private.size // waves) & ~1
    orders = {"random (the workload's private pages in trace order)": private[: waves * ppw],
              "sequential (the same number of pages, ascending ids)": np.arange(waves * ppw, dtype=np.int32) % lay.NP}
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    rows = []
    for oname, ids in orders.items():
        ids_d = torch.from_numpy(np.ascontiguousarray(ids)).to(dev)
        for pattern, pname in ((0, "1 KB per load"), (1, "matrix-core operand pattern")):
            for nt in (0, 1):
                for _ in range(3):
                    binding.read_probe(k_pages, v_pages, ids_d, waves, ppw, pattern, nt, sink)
                binding.profile_begin(args.steps)
                for _ in range(args.steps):
                    binding.read_probe(k_pages, v_pages, ids_d, waves, ppw, pattern, nt, sink)
                torch.cuda.synchronize()
                ms = [m for _, m in binding.profile_end(args.steps)]
                nbytes = waves * ppw * s.Hkv * 8192
                rows.append({"order": oname, "loads": pname, "nontemporal": bool(nt), "bytes": nbytes,
                             "avg_ms": round(float(np.mean(ms)), 4), "min_ms": round(float(np.min(ms)), 4),
                             "GB/s": round(nbytes / (float(np.mean(ms)) * 1e-3) / 1e9, 1)})
    print(json.dumps({"read_probe": workload, "waves_per_kv_head": waves, "pages_per_wave": ppw, "launches": args.steps,
                      "peak_GB/s": HBM_PEAK_GBS, "rows": rows}))


def cpu_baseline(args, w, sc, k_layers, v_layers, q_layers, sum0, cnt0, prune_k, layers=1):
    """The oracle, as it stands, on the host cores: the whole step on a bounded sample of traces."""
    import numpy as np
    import torch

    import oracle

    lay, s = w.layout, w.shape
    P = s.P
    threads = oracle.num_threads()

    def sample_inputs(traces, layer):
        pages = np.unique(np.concatenate([lay.block_tables[t][: (lay.seq_lens[t] + P - 1) // P] for t in traces]))
        remap = -np.ones(lay.NP, np.int64)
        remap[pages] = np.arange(pages.size)
        idx = torch.from_numpy(pages).to(k_layers[layer].device)
        ks = k_layers[layer].index_select(0, idx).view(torch.int16).cpu().numpy().view(np.uint16)
        vs = v_layers[layer].index_select(0, idx).view(torch.int16).cpu().numpy().view(np.uint16)
        bt = np.where(lay.block_tables[traces] >= 0, remap[np.maximum(lay.block_tables[traces], 0)], -1).astype(np.int32)
        qh = q_layers[layer].view(torch.int16).cpu().numpy().view(np.uint16)
        return np.ascontiguousarray(qh[traces]), ks, vs, bt, lay.seq_lens[traces].copy()

    # several layers (config 4): the oracle is timed on the first, the middle and the last layer and the sum is
    # scaled to all of them
    timed_layers = [0] if layers == 1 else sorted({0, layers // 2 - (1 if layers % 2 == 0 else 0), layers - 1})
    order = np.argsort(-lay.seq_lens.astype(np.int64))             # a length-stratified sample
    probe = np.sort(order[[len(order) // 2]])
    qs, ks, vs, bt, sl = sample_inputs(probe, 0)
    t0 = time.perf_counter()
    oracle.paged_decode_attn(qs, ks, vs, bt, sl)
    per_token = (time.perf_counter() - t0) / float(sl.sum())
    budget_tokens = args.cpu_seconds / per_token / len(timed_layers)
    stride_pick = order[:: max(1, int(np.ceil(lay.requested_tokens / budget_tokens)))]
    traces = np.sort(stride_pick)
    t_attn = 0.0
    for layer in timed_layers:
        qs, ks, vs, bt, sl = sample_inputs(traces, layer)
        t0 = time.perf_counter()
        oracle.paged_decode_attn(qs, ks, vs, bt, sl)
        t_attn += time.perf_counter() - t0
    t0 = time.perf_counter()
    _, probs = oracle.step_score(sc.hidden, sc.boundary_idx, sc.W1, sc.b1, sc.W2, sc.b2, act=sc.act)
    ssum, cnt = sum0.copy(), cnt0.copy()
    scores = oracle.running_mean(sc.trace_of, probs.astype(np.float32), ssum, cnt)
    oracle.prune_free(scores, prune_k, lay.refcounts.copy(), lay.block_tables.copy(), lay.seq_lens.copy(), P)
    t_rest = time.perf_counter() - t0
    scale = layers / len(timed_layers)
    total = t_attn * scale + t_rest
    how = "" if layers == 1 else " on layers %s, x%g: extrapolated to %d layers" % (timed_layers, scale, layers)
    return {
        "value": round(traces.size / total, 3), "unit": "trace-tokens/s", "cores": threads, "kind": "oracle",
        "sample": "oracle attention on %d of %d traces (every %d-th by length, %d context tokens)%s, plus the full "
                  "scorer (B=%d), running mean and prune_free(k=%d); %.2f s attention measured + %.3f s rest" % (
                      traces.size, s.N, max(1, len(order) // max(traces.size, 1)), int(sl.sum()), how,
                      sc.boundary_idx.size, prune_k, t_attn, t_rest),
        "seconds": round(total, 3),
    }


if __name__ == "__main__":
    main()
