"""Seeded synthetic inputs for the decode-step hot path (numpy only).

This module holds NO arithmetic of the method: it draws lengths, page tables,
reference counts and random tensors shaped like the workloads of STEP's
evaluation (N parallel traces of one prompt, tens of thousands of tokens each;
the 8B model's hidden size 4096) and hands the same bytes to both the CPU
oracle and the HIP library.  bf16 tensors are numpy uint16 arrays holding raw
bit patterns.

Recipe (per config c = 1..5, seed 0x5EED0000 + c, one independent stream per
array, keyed by a fixed stream id):
  lengths     L_i = prompt + U{tail_lo..tail_hi}          (configs 1, 2, 3)
              L_i = clip(round(exp(N(ln 12288, 0.3^2))), prompt+1, 32768)  (config 4)
              L_i = U{2048..16384}, prompt included       (config 5)
  pages       the prompt's pages are shared by every trace (refcount N), every
              tail page is private (refcount 1); physical ids are a random
              permutation of a pool of ceil(slack * used) pages
  q, K, V     N(0,1) rounded to bf16 (round-to-nearest-even)
  scorer      hidden N(0,1) bf16; W1, W2 ~ N(0, 0.02) bf16; b1, b2 ~ N(0, 0.02) fp32
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

P_TOKENS = 16
BF16_NAN = np.uint16(0x7FC0)

# stream ids: one generator per array, fixed order
_S_LENS, _S_PERM, _S_Q, _S_K, _S_V, _S_HID, _S_W1, _S_B1, _S_W2, _S_B2, _S_ROWS, _S_STATE = range(12)


def rng_for(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even) and return the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(rng: np.random.Generator, shape, std: float = 1.0, chunk: int = 1 << 24) -> np.ndarray:
    """N(0, std) rounded to bf16, generated in chunks to bound peak memory."""
    n = int(np.prod(shape))
    out = np.empty(n, np.uint16)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        x = rng.standard_normal(e - s, dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        out[s:e] = f32_to_bf16_bits(x)
    return out.reshape(shape)


@dataclass
class AttnShape:
    N: int
    Hq: int
    Hkv: int
    D: int
    P: int = P_TOKENS

    @property
    def kv_bytes_per_token(self) -> int:  # K and V, all KV heads, bf16
        return 2 * self.Hkv * self.D * 2


@dataclass
class PagedLayout:
    """Lengths, block tables and reference counts of N traces sharing a prompt."""
    seq_lens: np.ndarray        # [N] i32
    block_tables: np.ndarray    # [N][MAXB] i32, -1 padded
    refcounts: np.ndarray       # [NP] i32
    NP: int
    MAXB: int
    prompt_len: int
    used_pages: int             # distinct referenced pages
    unique_tokens: int          # tokens resident in referenced pages, prompt counted once
    requested_tokens: int       # sum of seq_lens


def build_layout(lens, prompt_len: int, P: int, rng: np.random.Generator, *, slack: float = 1.0,
                 permute: bool = True, maxb: Optional[int] = None) -> PagedLayout:
    lens = np.asarray(lens, np.int64)
    N = lens.size
    assert prompt_len % P == 0, "shared prefix is whole pages only"
    assert np.all((lens == 0) | (lens >= prompt_len))
    nb = (lens + P - 1) // P
    pp = prompt_len // P
    tail_pages = np.where(lens > 0, nb - pp, 0)
    used = int(pp * (1 if np.any(lens > 0) else 0) + tail_pages.sum())
    NP = max(int(np.ceil(slack * used)), used, 1)
    ids = rng.permutation(NP)[:used] if permute else np.arange(used)
    ids = ids.astype(np.int32)
    MAXB = int(maxb if maxb is not None else max(int(nb.max()) if N else 0, 1))
    assert MAXB >= (int(nb.max()) if N else 0)
    bt = np.full((N, MAXB), -1, np.int32)
    rc = np.zeros(NP, np.int32)
    prompt_ids = ids[:pp]
    cur = pp
    for i in range(N):
        if lens[i] == 0:
            continue
        bt[i, :pp] = prompt_ids
        rc[prompt_ids] += 1
        n_t = int(tail_pages[i])
        bt[i, pp:pp + n_t] = ids[cur:cur + n_t]
        rc[ids[cur:cur + n_t]] += 1
        cur += n_t
    assert cur == used
    live = lens > 0
    unique_tokens = int((prompt_len if np.any(live) else 0) + (lens[live] - prompt_len).sum())
    return PagedLayout(lens.astype(np.int32), bt, rc, NP, MAXB, prompt_len, used, unique_tokens, int(lens.sum()))


def poison_unused(k_pages: np.ndarray, v_pages: np.ndarray, layout: PagedLayout, P: int) -> None:
    """Fill every slot no trace owns (unreferenced pages, slots past a trace's last token) with NaN."""
    NP = k_pages.shape[0]
    valid = np.zeros((NP, P), bool)
    for i in range(layout.seq_lens.size):
        L = int(layout.seq_lens[i])
        if L == 0:
            continue
        nb = (L + P - 1) // P
        pages = layout.block_tables[i, :nb]
        valid[pages[:-1], :] = True
        last = L - (nb - 1) * P
        valid[pages[-1], :last] = True
    mask = ~valid  # [NP][P]
    k_pages[np.broadcast_to(mask[:, None, :, None], k_pages.shape)] = BF16_NAN
    v_pages[np.broadcast_to(mask[:, None, :, None], v_pages.shape)] = BF16_NAN


@dataclass
class ScorerInputs:
    hidden: np.ndarray          # [R][d] u16
    boundary_idx: np.ndarray    # [B] i32 rows of hidden
    trace_of: np.ndarray        # [B] i32 trace owning each boundary
    W1: np.ndarray              # [m][d] u16
    b1: np.ndarray              # [m] f32
    W2: np.ndarray              # [m] u16
    b2: float
    act: int                    # 0 ReLU, 1 GELU-erf
    score_sum: np.ndarray       # [N] f32 prior state
    score_cnt: np.ndarray       # [N] i32 prior state


def build_scorer(seed: int, N: int, R: int, d: int, m: int, B: int, act: int, *, trace_of=None,
                 distinct_rows: bool = True, prior_state: bool = False) -> ScorerInputs:
    hidden = normal_bf16(rng_for(seed, _S_HID), (R, d))
    W1 = normal_bf16(rng_for(seed, _S_W1), (m, d), 0.02)
    b1 = (rng_for(seed, _S_B1).standard_normal(m, dtype=np.float32) * np.float32(0.02)).astype(np.float32)
    W2 = normal_bf16(rng_for(seed, _S_W2), (m,), 0.02)
    b2 = float(np.float32(rng_for(seed, _S_B2).standard_normal(1, dtype=np.float32)[0] * np.float32(0.02)))
    r = rng_for(seed, _S_ROWS)
    if distinct_rows:
        assert B <= R
        rows = np.sort(r.permutation(R)[:B]).astype(np.int32)
    else:
        rows = r.integers(0, R, B).astype(np.int32)
    if trace_of is None:
        trace_of = (rows % N).astype(np.int32)
    st = rng_for(seed, _S_STATE)
    if prior_state:
        cnt = st.integers(1, 41, N).astype(np.int32)
        ssum = (cnt.astype(np.float32) * st.uniform(0.2, 0.8, N).astype(np.float32)).astype(np.float32)
    else:
        cnt = np.zeros(N, np.int32)
        ssum = np.zeros(N, np.float32)
    return ScorerInputs(hidden, rows, np.ascontiguousarray(trace_of, np.int32), W1, b1, W2, b2, act, ssum, cnt)


@dataclass
class Workload:
    name: str
    seed: int
    shape: AttnShape
    layout: PagedLayout
    q: np.ndarray                         # [N][Hq][D] u16
    k_pages: Optional[np.ndarray]         # [NP][Hkv][P][D] u16 or None (generate on device)
    v_pages: Optional[np.ndarray]
    scorer: Optional[ScorerInputs]
    prune_k: int
    layers: int = 1
    notes: dict = field(default_factory=dict)


_CFG = {
    # name: N, Hq, Hkv, D, prompt, (tail_lo, tail_hi), slack, scorer (d, m, B, act), prune_k, layers
    1: dict(N=4, Hq=4, Hkv=1, D=64, prompt=64, tail=(64, 256), slack=1.0, scorer=(256, 64, 8, 1), k=1, layers=1),
    2: dict(N=16, Hq=32, Hkv=8, D=128, prompt=512, tail=(4096, 16384), slack=1.0, scorer=(4096, 1024, 4, 0), k=0, layers=1),
    3: dict(N=64, Hq=32, Hkv=8, D=128, prompt=1024, tail=(8192, 32768), slack=1.25, scorer=(4096, 1024, 4, 0), k=0, layers=1),
    4: dict(N=128, Hq=32, Hkv=8, D=128, prompt=1024, tail=None, slack=1.0, scorer=(4096, 1024, 13, 0), k=0, layers=36),
    # config 5's scorer inputs have a seed of their own, re-drawn (0x5EED0005 + 0x100 j, j = 0, 1, ...) until the
    # independent float64 chain leaves a gap above 4e-3 between the 64th and 65th lowest trace score, so that
    # the pruned set does not hinge on the scorer's last bits; tests/golden/pick_config5_scorer_seed.py finds j = 5
    5: dict(N=256, Hq=32, Hkv=8, D=128, prompt=1024, tail=None, slack=1.0, scorer=(4096, 1024, 26, 0), k=64, layers=1,
            scorer_seed=0x5EED0505),
}


def config_lens(cfg: int, seed: int, *, N: Optional[int] = None, tail=None) -> np.ndarray:
    c = _CFG[cfg]
    N = c["N"] if N is None else N
    r = rng_for(seed, _S_LENS)
    if cfg in (1, 2, 3):
        lo, hi = c["tail"] if tail is None else tail
        return (c["prompt"] + r.integers(lo, hi + 1, N)).astype(np.int64)
    if cfg == 4:
        x = np.exp(r.normal(np.log(12288.0), 0.3, N))
        return np.clip(np.rint(x), c["prompt"] + 1, 32768).astype(np.int64)
    lo, hi = (2048, 16384) if tail is None else tail
    return r.integers(lo, hi + 1, N).astype(np.int64)


def make_workload(cfg: int, *, kv: bool = True, poison: bool = False, permute: bool = True,
                  N: Optional[int] = None, tail=None, seed: Optional[int] = None,
                  full_maxb: bool = True, heads=None, head_dim: Optional[int] = None) -> Workload:
    """Build config `cfg` (1..5).  kv=False leaves k_pages/v_pages None (large pools are drawn on
    the device by the caller).  N / tail shrink a config for fast CPU tests, same structure;
    heads = (Hq, Hkv) / head_dim put another head shape on the config's lengths and layout."""
    c = _CFG[cfg]
    seed = (0x5EED0000 + cfg) if seed is None else seed
    Nn = c["N"] if N is None else N
    Hq, Hkv = heads if heads is not None else (c["Hq"], c["Hkv"])
    shape = AttnShape(Nn, Hq, Hkv, head_dim if head_dim is not None else c["D"])
    lens = config_lens(cfg, seed, N=Nn, tail=tail)
    P = shape.P
    maxb = None
    if full_maxb and tail is None:
        cap = {1: 64 + 256, 2: 512 + 16384, 3: 1024 + 32768, 4: 32768, 5: 16384}[cfg]
        maxb = cap // P
    layout = build_layout(lens, c["prompt"], P, rng_for(seed, _S_PERM), slack=c["slack"], permute=permute, maxb=maxb)
    q = normal_bf16(rng_for(seed, _S_Q), (Nn, shape.Hq, shape.D))
    k_pages = v_pages = None
    if kv:
        k_pages = normal_bf16(rng_for(seed, _S_K), (layout.NP, shape.Hkv, P, shape.D))
        v_pages = normal_bf16(rng_for(seed, _S_V), (layout.NP, shape.Hkv, P, shape.D))
        if poison:
            poison_unused(k_pages, v_pages, layout, P)
    d, m, B, act = c["scorer"]
    if cfg == 1:
        sc = build_scorer(seed, Nn, 8, d, m, 8, act, trace_of=np.arange(8, dtype=np.int32) % Nn)
    else:
        B = min(B, Nn) if N is not None else B
        sc = build_scorer(c.get("scorer_seed", seed) if seed == 0x5EED0000 + cfg else seed, Nn, Nn, d, m, B, act,
                          prior_state=(cfg == 5))
    k = c["k"] if N is None else (c["k"] * Nn) // c["N"]
    return Workload("config%d" % cfg, seed, shape, layout, q, k_pages, v_pages, sc, k, c["layers"])
