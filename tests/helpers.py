"""Independent numpy helpers for the oracle pins (no code shared with oracle/ or the HIP path)."""
import numpy as np
from scipy.special import softmax

from paper_2601_09093_amd.workloads import bf16_bits_to_f32


def gather_dense(pages, block_table, L, g, P):
    """Rows of one KV head of one trace as a dense float64 [L][D] matrix."""
    rows = []
    for t in range(L):
        rows.append(bf16_bits_to_f32(pages[block_table[t // P], g, t % P]).astype(np.float64))
    return np.stack(rows) if rows else np.zeros((0, pages.shape[-1]))


def dense_attention(q, k_pages, v_pages, block_tables, seq_lens, scale):
    """softmax(q K^T scale) V with library float64 routines on gathered dense matrices."""
    N, Hq, D = q.shape
    _, Hkv, P, _ = k_pages.shape
    G = Hq // Hkv
    out = np.zeros((N, Hq, D))
    qf = bf16_bits_to_f32(q).astype(np.float64)
    for i in range(N):
        L = int(seq_lens[i])
        if L == 0:
            continue
        for h in range(Hq):
            K = gather_dense(k_pages, block_tables[i], L, h // G, P)
            V = gather_dense(v_pages, block_tables[i], L, h // G, P)
            w = softmax(scale * (K @ qf[i, h]))
            out[i, h] = w @ V
    return out
