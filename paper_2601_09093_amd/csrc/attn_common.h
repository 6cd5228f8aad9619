// Declarations shared by the attention translation units (attn*.hip): the kernel argument block, the
// way the work of one call is cut (decided on the device, by every wave for itself, from seq_lens and the
// per-block shared-prefix lengths), and the host-side launchers of each stage.
//
// How one call is cut
//   Blocks.   The traces are taken in blocks of TB = 16 * QT / G consecutive indices (the traces whose G
//             query heads fill QT 16-column query tiles of the matrix cores).  S_b, the shared prefix of
//             block b, is the number of leading block-table entries that are identical in every live trace
//             of the block and lie below every such trace's last full page (the prompt's pages; 0 when the
//             block has fewer than two live traces).  It is found by one wave from the block's TB rows.
//   Prefix.   The S_b shared pages of a block are cut into parts_b sub-chunks of sc_b pages (prefix_split);
//             sub-chunk p of trace t is partial slot prefix_base + p * N + t (attn_front computes these).
//   Private.  Trace t keeps priv_t = pages_t - S_b(t) private pages.  The private pages of all traces,
//             concatenated in trace order, are cut into Wh runs of Q = ceil(total / Wh) pages, one per
//             streaming wave of a KV head; the piece of trace t inside the run of wave wh is one record,
//             partial slot priv_base + base_t + (wh - first wave of t), base_t = pieces of the traces before t.
//   Every wave derives its own run from seq_lens and S_b with two prefix sums (plan_build): there is no
//   planning kernel and no record array.
#pragma once
#include "common.h"

namespace step {
namespace attn {

constexpr float kMinusBig = -1.0e30f;  // finite "no token seen yet" running max (keeps exp2 NaN-free)

constexpr int kMaxParts = 8;      // a shared prefix is cut into at most this many sub-chunks per trace
constexpr int kMaxPlanN = 2048;   // traces per call
constexpr int kMaxWh = 2048;      // streaming waves per KV head
constexpr int kMaxShared = 1024;  // pages of common prefix looked for per block (16384 tokens)

struct PlanHeader {   // 256 bytes at the start of the workspace
    int32_t stamp;    // hash of the dims the per-block prefix lengths were found for (AttnArgs::stamp), never 0
    // written by the streaming kernel for measurement only (never read by a kernel):
    int32_t pieces;   // records of private pages in this call
    int32_t private_pages;  // pages streamed per KV head
    int32_t quota;    // Q: pages per streaming wave
    int32_t prefix_slots;   // shared-prefix partial slots written (sum over live traces of parts_b)
    int32_t shared_max;     // largest S_b
    int32_t pad[58];
};

struct AttnArgs {
    const uint16_t *q, *k_pages, *v_pages;
    const int32_t *block_tables, *seq_lens;
    PlanHeader *hdr;
    int32_t *blk_shared;  // [nblk] S_b
    int32_t *first2;      // [N] first private-page slot of the trace (written by the streaming kernel, read by the merge)
    int32_t *cnt2;        // [N] number of such slots
    float *part_acc;      // [slots * Hkv][G][D]   index = slot * Hkv + kv head
    float *part_ml;       // [slots * Hkv][G][2]   (running max in log2 units, weight sum)
    uint16_t *out;
    int32_t *status;
    int N, Hq, Hkv, MAXB, NP, Wh;
    int TB, nblk;         // traces per block, number of blocks
    int pmax;             // sub-chunks of a shared prefix per trace at most
    int priv_base;        // first partial slot of the private-page records (N + Wh of them at most)
    int prefix_base;      // first partial slot of the shared-prefix sub-chunks (N * pmax of them)
    int max_slots;        // partial slots the workspace holds: N * pmax + N + Wh
    int stamp;            // what hdr->stamp must hold when the per-block prefix lengths are taken from the workspace
    int prefix_qt;        // 16-row query tiles per wave of attn_front (1 or 2); 0: shared prefixes are not looked for
    float scale_log2;     // scale * log2(e)
};

// Wave-uniform reads of data that no kernel of the same launch writes (block-table entries, lengths):
// through the constant address space they become scalar loads, which have a counter of their own and
// so do not queue behind the vector loads of the tile stream.
__device__ __forceinline__ int32_t scalar_read(const int32_t *p)
{
    typedef const __attribute__((address_space(4))) int32_t *ConstPtr;
    return *reinterpret_cast<ConstPtr>(reinterpret_cast<uintptr_t>(p));
}

// A single wave's LDS operations retire in order; this also keeps the compiler from moving LDS reads and
// writes across the point where lanes exchange data through LDS (no instructions are emitted).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// pages of a trace of L tokens; 0 for a dead trace or a length outside the block-table row
__device__ __forceinline__ int pages_of(int L, int MAXB)
{
    return (L > 0 && (long long)L <= (long long)MAXB * kPageTokens) ? (L + kPageTokens - 1) / kPageTokens : 0;
}

// What one wave finds out about block b of the traces.
struct BlockPrefix {
    unsigned live;     // bit r: trace b * TB + r has pages
    int S;             // S_b: leading block-table entries common to every live trace of the block, below each
                       // one's last full page, at most kMaxShared (0 with fewer than two live traces)
    bool have_ids;     // ids_a / ids_b are valid
    int ids_a, ids_b;  // per lane: entries `lane` and `64 + lane` of the first live trace's row (exact below S_b)
};

// Every lane of the wave calls; the results are wave-uniform (ids_a / ids_b are per lane).  detect = false only
// looks at the lengths (S comes back 0).  The search takes 128 columns per trip with the loads of up to 8 rows
// in flight together; for a block of at most 8 traces the first trip's loads are requested together with the
// lengths (columns clamped to the row, compared only below the cap the lengths give).
__device__ __forceinline__ BlockPrefix block_prefix(const AttnArgs &a, int b, int lane, bool detect)
{
    BlockPrefix r;
    r.S = 0;
    r.have_ids = false;
    r.ids_a = r.ids_b = 0;
    const int t0 = b * a.TB, nt = min(a.TB, a.N - t0);
    const int32_t *rows = a.block_tables + (size_t)t0 * a.MAXB;
    const bool spec = detect && nt <= 8 && a.MAXB > 0;
    int L = 0;
    if (lane < nt) L = a.seq_lens[t0 + lane];
    int xa[8], xb[8];
    if (spec) {
        const int ca = min(lane, a.MAXB - 1), cb = min(64 + lane, a.MAXB - 1);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int rr = min(u, nt - 1);
            xa[u] = rows[(size_t)rr * a.MAXB + ca];
            xb[u] = rows[(size_t)rr * a.MAXB + cb];
        }
    }
    const bool ok = pages_of(L, a.MAXB) > 0;
    int mf = ok ? L / kPageTokens : 0x7fffffff;
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) mf = min(mf, __shfl_xor(mf, off));
    const int minfull = __builtin_amdgcn_readfirstlane(mf);
    const unsigned live = (unsigned)__ballot(ok);
    r.live = live;
    if (!detect || __popc(live) < 2) return r;
    const int cap = min(min(kMaxShared, minfull), a.MAXB);
    if (cap <= 0) return r;
    const int f = __ffs(live) - 1;
    const int32_t *row_f = rows + (size_t)f * a.MAXB;
    for (int c0 = 0; c0 < cap; c0 += 128) {
        int ref_a, ref_b;
        bool diff_a = false, diff_b = false;
        if (c0 == 0 && spec) {
            ref_a = xa[0];
            ref_b = xb[0];
#pragma unroll
            for (int u = 1; u < 8; ++u)
                if (f == u) {
                    ref_a = xa[u];
                    ref_b = xb[u];
                }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const bool is_live = (live >> min(u, nt - 1)) & 1u;
                diff_a |= is_live && xa[u] != ref_a;
                diff_b |= is_live && xb[u] != ref_b;
            }
            diff_a &= lane < cap;
            diff_b &= 64 + lane < cap;
        } else {
            const int ca = min(c0 + lane, cap - 1), cb = min(c0 + 64 + lane, cap - 1);  // clamped: a repeat of the last column
            ref_a = row_f[ca];
            ref_b = row_f[cb];
            for (int r0 = 0; r0 < nt; r0 += 8) {
                int ya[8], yb[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int rr = min(r0 + u, nt - 1);
                    ya[u] = rows[(size_t)rr * a.MAXB + ca];
                    yb[u] = rows[(size_t)rr * a.MAXB + cb];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const bool is_live = (live >> min(r0 + u, nt - 1)) & 1u;
                    diff_a |= is_live && ya[u] != ref_a;
                    diff_b |= is_live && yb[u] != ref_b;
                }
            }
        }
        if (c0 == 0) {
            r.have_ids = true;
            r.ids_a = ref_a;
            r.ids_b = ref_b;
        }
        const unsigned long long da = __ballot(diff_a), db = __ballot(diff_b);
        if (da) {
            r.S = min(cap, c0 + (int)__ffsll(da) - 1);
            return r;
        }
        if (db) {
            r.S = min(cap, c0 + 64 + (int)__ffsll(db) - 1);
            return r;
        }
    }
    r.S = cap;
    return r;
}

// Sub-chunks of a shared prefix of S pages: about one wave per SIMD over the blocks of a KV head, whole page
// pairs per sub-chunk, at most pmax.  parts = 0 when there is nothing shared.
__device__ __forceinline__ void prefix_split(const AttnArgs &a, int S, int &parts, int &sc)
{
    parts = 0;
    sc = 0;
    if (S <= 0 || a.prefix_qt == 0) return;
    parts = max(1, min(min(a.pmax, (S + 1) / 2), (a.Wh + a.nblk - 1) / a.nblk));
    sc = (S + parts - 1) / parts;
    sc += sc & 1;
    parts = (S + sc - 1) / sc;
}

// S_b as the streaming kernels and the merge take it from the workspace, clamped to what the trace can hold
// (`raw` = blk_shared[t / TB]; nb = pages of the trace)
__device__ __forceinline__ int clamp_shared(const AttnArgs &a, int raw, int nb)
{
    if (a.prefix_qt == 0 || nb <= 0) return 0;
    return min(max(raw, 0), min(nb, kMaxShared));
}

// ---------------------------------------------------------------------------------------------
// The run of one streaming wave, derived by the wave itself.
//   P_s[t]    private pages of the traces before t (P_s[N] = total), base_s[t] = pieces of the traces before t
// Both arrays live in the wave's LDS.  All lanes call plan_build; results are wave-uniform.
// ---------------------------------------------------------------------------------------------
struct WavePlan {
    int total;   // private pages of all traces (per KV head)
    int Q;       // pages per wave
    int pieces;  // records of all traces
};

__device__ __forceinline__ int wave_incl_scan(int v, int lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(v, off);
        if (lane >= off) v += y;
    }
    return v;
}

__device__ __forceinline__ WavePlan plan_build(const AttnArgs &a, int lane, int *P_s, int *base_s, bool report_errors)
{
    WavePlan w;
    // private pages per trace, exclusive prefix sum; four groups of 64 lengths are requested together
    int carry = 0;
    bool bad_len = false;
    for (int c0 = 0; c0 < a.N; c0 += 256) {
        int L[4], Sraw[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = c0 + u * 64 + lane;
            L[u] = t < a.N ? a.seq_lens[t] : 0;
            Sraw[u] = t < a.N ? a.blk_shared[t / a.TB] : 0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = c0 + u * 64 + lane;
            if (c0 + u * 64 >= a.N) break;  // uniform
            const int nb = pages_of(L[u], a.MAXB);
            bad_len |= (L[u] != 0 && nb == 0);
            const int priv = nb - clamp_shared(a, Sraw[u], nb);
            const int inc = wave_incl_scan(priv, lane);
            if (t < a.N) P_s[t] = carry + inc - priv;
            carry += __shfl(inc, 63);
        }
    }
    if (lane == 0) P_s[a.N] = carry;
    w.total = carry;
    w.Q = max(1, (carry + a.Wh - 1) / a.Wh);
    wave_lds_sync();
    // pieces per trace: the waves its private pages touch
    int pc = 0;
    for (int c0 = 0; c0 < a.N; c0 += 64) {
        const int t = c0 + lane;
        int pieces = 0;
        if (t < a.N) {
            const int p0 = P_s[t], p1 = P_s[t + 1];
            if (p1 > p0) pieces = (p1 - 1) / w.Q - p0 / w.Q + 1;
        }
        const int inc = wave_incl_scan(pieces, lane);
        if (t < a.N) base_s[t] = pc + inc - pieces;
        pc += __shfl(inc, 63);
    }
    if (lane == 0) base_s[a.N] = pc;
    w.pieces = pc;
    wave_lds_sync();
    if (report_errors && __any(bad_len) && lane == 0) report(a.status, STEP_ELEN);
    return w;
}

// The streaming wave 0 of KV head 0 leaves, for the merge, where each trace's private-page partials are,
// and a few figures of the cut for measurement.
__device__ __forceinline__ void publish_plan(const AttnArgs &a, const WavePlan &w, int lane, const int *P_s, const int *base_s)
{
    int slots = 0, smax = 0;
    for (int t = lane; t < a.N; t += 64) {
        a.first2[t] = a.priv_base + base_s[t];
        a.cnt2[t] = base_s[t + 1] - base_s[t];
        const int nb = pages_of(a.seq_lens[t], a.MAXB);
        const int S = nb - (P_s[t + 1] - P_s[t]);
        int parts, sc;
        prefix_split(a, S, parts, sc);
        slots += nb > 0 ? parts : 0;
        smax = max(smax, S);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        slots += __shfl_xor(slots, off);
        smax = max(smax, __shfl_xor(smax, off));
    }
    if (lane == 0) {
        a.hdr->pieces = w.pieces;
        a.hdr->private_pages = w.total;
        a.hdr->quota = w.Q;
        a.hdr->prefix_slots = slots;
        a.hdr->shared_max = smax;
    }
}

// One record of a streaming wave: the pages [first, first + n) of trace i (block-table row coordinates),
// ntok tokens in the last of them, partial slot `slot`.
struct Record {
    int32_t i, first, n, ntok, slot;
};

// Walks the records of wave wh: the traces its run [wh * Q, (wh + 1) * Q) of the concatenated private pages touches.
struct RunWalker {
    const AttnArgs &a;
    const int *P_s, *base_s;
    int Q, wh, end;  // the run ends at `end` (exclusive)
    int t, pos;      // next record starts at private page `pos`, inside trace t; t < 0: none left

    __device__ __forceinline__ RunWalker(const AttnArgs &a_, const WavePlan &w, const int *P, const int *B, int wh_)
        : a(a_), P_s(P), base_s(B), Q(w.Q), wh(wh_)
    {
        const long long start = (long long)wh * w.Q;
        end = (int)min((long long)w.total, start + w.Q);
        t = -1;
        pos = 0;
        if (start < end) {
            pos = (int)start;
            int lo = 0, hi = a.N;  // invariant: P_s[lo] <= pos < P_s[hi]
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (P_s[mid] <= pos) lo = mid; else hi = mid;
            }
            t = lo;
        }
    }
    __device__ __forceinline__ bool more() const { return t >= 0; }
    // the record at the cursor; then the cursor moves to the next trace of the run that has private pages
    __device__ __forceinline__ Record take()
    {
        Record r;
        const int p0 = P_s[t], p1 = P_s[t + 1];
        const int stop = min(end, p1);
        const int L = scalar_read(a.seq_lens + t);
        const int nb = pages_of(L, a.MAXB);
        const int S = nb - (p1 - p0);  // the pages of the trace that are not private are its block's shared prefix
        r.i = t;
        r.first = S + (pos - p0);
        r.n = stop - pos;
        r.ntok = (r.first + r.n == nb) ? L - (nb - 1) * kPageTokens : kPageTokens;
        r.slot = a.priv_base + base_s[t] + (wh - p0 / Q);
        pos = stop;
        if (pos >= end) {
            t = -1;
        } else {
            int nt = t + 1;
            while (nt < a.N && P_s[nt + 1] <= pos) ++nt;  // skip traces without private pages
            t = nt < a.N ? nt : -1;
        }
        return r;
    }
};

// Host-side launchers, one per translation unit.  D is the head dimension (64 or 128).
void launch_front(const AttnArgs &a, int D, bool detect, hipStream_t s);                    // attn_front.hip
void launch_plan_blocks(const AttnArgs &a, hipStream_t s);                                  // attn_front.hip
void launch_stream_mfma(const AttnArgs &a, int D, hipStream_t s);                           // attn_mfma.hip
void launch_stream_g4(const AttnArgs &a, hipStream_t s);                                    // attn_g4.hip (D = 128, G = 4)
int stream_g4_waves_per_cu();                                                               // attn_g4.hip
void launch_merge(const AttnArgs &a, int D, hipStream_t s);                                 // attn_merge.hip

}  // namespace attn
}  // namespace step
