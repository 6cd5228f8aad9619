// attn_plan: the device-side planner of paged_decode_attn (one workgroup per call).
#include "attn_common.h"

namespace step {
namespace attn {
namespace {

// ---------------------------------------------------------------------------------------------
// plan: cut the work into records so that every one of the Wh waves of a KV head streams the same
// number of pages (Q, give or take one).
//   1. S = number of leading block-table entries that are identical in every live trace and lie
//      below every live trace's last full page (the prompt's pages).  Those pages are cut into
//      `parts` sub-chunks and sub-chunk p of the trace of rank rk is record p * N_live + rk.  With
//      attn_prefix the sub-chunks are sized for its waves (whole page pairs, about one wave per SIMD)
//      and stage 1 never sees these records.  Without it (testing aid) record s goes to wave s mod Wh
//      ahead of that wave's private pages: all waves start on the shared pages at the same time, so
//      N reads of each shared tile become one HBM read plus L2 hits.
//   2. The private pages of all traces, concatenated trace by trace, are cut into Wh consecutive
//      runs whose lengths top every wave up to Q pages; a run is one record per trace it touches.
// ---------------------------------------------------------------------------------------------
constexpr int kPlanThreads = 1024;
static_assert(kPlanThreads == 1024, "block_excl_scan works on 1024-thread workgroups");
static_assert(kMaxShared <= kPlanThreads, "one thread copies one entry of the first live row");

// in-place exclusive scan of arr[0..n), n <= 2 * kPlanThreads; returns the total
__device__ int array_excl_scan(int *arr, int n, int *scratch)
{
    const int tid = threadIdx.x;
    const int a0 = 2 * tid < n ? arr[2 * tid] : 0;
    const int a1 = 2 * tid + 1 < n ? arr[2 * tid + 1] : 0;
    int total;
    const int e = block_excl_scan(a0 + a1, scratch, &total);
    if (2 * tid < n) arr[2 * tid] = e;
    if (2 * tid + 1 < n) arr[2 * tid + 1] = e + a0;
    __syncthreads();
    return total;
}

__global__ __launch_bounds__(kPlanThreads) void attn_plan(const AttnArgs a)
{
    __shared__ int nb_s[kMaxPlanN];      // pages of trace t (0: dead or invalid)
    __shared__ int len_s[kMaxPlanN];     // tokens of trace t
    __shared__ int live_list[kMaxPlanN]; // rank -> trace
    __shared__ int P_s[kMaxPlanN + 1];   // private pages before trace t in the concatenation
    __shared__ int wq[kMaxWh + 1];       // per wave: private-page quota, then its start position
    __shared__ int wcnt[kMaxWh + 1];     // per wave: record count, then record offset
    __shared__ int scratch[32];
    __shared__ int S_s, minfull_s;
    const int tid = threadIdx.x;
    const int N = a.N, Wh = a.Wh;

    if (tid == 0) { S_s = kMaxShared; minfull_s = 0x7fffffff; }
    __syncthreads();
    // lengths, live ranks
    for (int t = tid; t < 2 * kPlanThreads; t += kPlanThreads) {
        int nb = 0, L = 0;
        if (t < N) {
            L = a.seq_lens[t];
            if (L < 0 || (long long)L > (long long)a.MAXB * kPageTokens) report(a.status, STEP_ELEN);
            else nb = (L + kPageTokens - 1) / kPageTokens;
            a.cnt2[t] = 0;
            a.first2[t] = 0;
        }
        // fewest full pages of a live trace (the shared prefix is whole pages that every live trace
        // attends to completely): one LDS atomic per wave
        int mn = nb > 0 ? L / kPageTokens : 0x7fffffff;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mn = min(mn, __shfl_xor(mn, off));
        if ((tid & 63) == 0 && mn != 0x7fffffff) atomicMin(&minfull_s, mn);
        if (t < kMaxPlanN) { nb_s[t] = nb; len_s[t] = L; P_s[t] = nb > 0 ? 1 : 0; }
    }
    __syncthreads();
    const int n_live = array_excl_scan(P_s, N, scratch);   // P_s[t] = rank of trace t
    for (int t = tid; t < N; t += kPlanThreads) {
        a.rank[t] = P_s[t];
        if (nb_s[t] > 0) {
            live_list[P_s[t]] = t;
            a.live[P_s[t]] = t;
        }
    }
    __syncthreads();
    // shared prefix: compare every live row with the first live row.  The first live row's leading
    // entries are also what attn_prefix walks: fetched here, next to the compare loads, stored below
    const bool copies_row0 = a.prefix_qt > 0 && n_live >= 2 && tid < min(kMaxShared, a.MAXB);
    int row0_entry = -1;
    if (copies_row0) row0_entry = a.block_tables[(size_t)live_list[0] * a.MAXB + tid];
    int S = 0;
    if (n_live >= 2) {
        const int cap = min(kMaxShared, minfull_s);
        if (tid == 0) S_s = cap;
        __syncthreads();
        const int32_t *row0 = a.block_tables + (size_t)live_list[0] * a.MAXB;
        // the columns are searched kSearchCols at a time and the search stops at the first block that
        // holds a difference: a prompt of a few dozen pages costs one block however long the traces are
        constexpr int kSearchCols = 256;
        for (int c0 = 0; c0 < cap; c0 += kSearchCols) {
            const int w = min(kSearchCols, cap - c0);
            int first_diff = cap;  // smallest page index at which some live row differs from the first live row
            // consecutive lanes compare consecutive entries of one row (coalesced); the planner runs
            // right after gigabytes were streamed through every cache, so all of a thread's loads are
            // issued before the first compare (16 pairs in flight per thread)
            constexpr int kBatch = 16;
            const int work = (n_live - 1) * w;
            for (int base = 0; base < work; base += kBatch * kPlanThreads) {
                int x[kBatch], y[kBatch], jj[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int idx = min(base + u * kPlanThreads + tid, work - 1);
                    const int rk = 1 + idx / w;
                    jj[u] = c0 + idx % w;
                    x[u] = a.block_tables[(size_t)live_list[rk] * a.MAXB + jj[u]];
                    y[u] = row0[jj[u]];
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u)
                    if (x[u] != y[u]) first_diff = min(first_diff, jj[u]);
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) first_diff = min(first_diff, __shfl_xor(first_diff, off));
            if ((tid & 63) == 0 && first_diff < cap) atomicMin(&S_s, first_diff);
            __syncthreads();
            // a later block can only lower S_s to a column at or beyond its own start, so every thread
            // takes the same decision here whenever it reads S_s
            if (S_s < c0 + w) break;
        }
        S = S_s;
    }
    int parts = 0, sc = 0;
    const bool mfma = a.prefix_qt > 0 && S > 0;
    if (mfma) {
        // attn_prefix runs one wave per (KV head, block of 16 * qt query rows, sub-chunk): enough
        // sub-chunks for about one wave per SIMD, whole page pairs per sub-chunk
        const int G = a.Hq / a.Hkv;
        const int nqb = (n_live * G + 16 * a.prefix_qt - 1) / (16 * a.prefix_qt);
        parts = max(1, min(min(kMaxParts, (S + 1) / 2), (Wh + nqb - 1) / nqb));
        parts = min(parts, 1 + 4 * Wh / n_live);  // n_live * parts <= 4 Wh + n_live records (workspace bound)
        sc = (S + parts - 1) / parts;
        sc += sc & 1;
        parts = (S + sc - 1) / sc;
    } else if (S > 0) {
        parts = max(1, min(min(kMaxParts, S), Wh / n_live));
        sc = (S + parts - 1) / parts;
        parts = (S + sc - 1) / sc;
    }
    if (copies_row0) a.shared_pages[tid] = row0_entry;  // entries [0, S) are the shared pages
    const int N1 = n_live * parts;  // shared-prefix records
    // private pages: prefix over traces
    __syncthreads();
    for (int t = tid; t < N; t += kPlanThreads) P_s[t] = nb_s[t] > 0 ? nb_s[t] - S : 0;
    __syncthreads();
    const int T2 = array_excl_scan(P_s, N, scratch);
    if (tid == 0) P_s[N] = T2;
    const long long T_all = (long long)T2 + (mfma ? 0 : (long long)n_live * S);
    const int Q = (int)((T_all + Wh - 1) / Wh);
    // per wave: pages of its shared-prefix records, private quota
    auto part_pages = [&](int p) { return min(sc, S - p * sc); };
    for (int wh = tid; wh < Wh; wh += kPlanThreads) {
        int a_wh = 0;
        if (!mfma)
            for (int s = wh; s < N1; s += Wh) a_wh += part_pages(s / n_live);
        wq[wh] = max(Q - a_wh, 0);
    }
    __syncthreads();
    array_excl_scan(wq, Wh, scratch);                        // wq[wh] = start of the wave's run
    if (tid == 0) wq[Wh] = 0x7fffffff;
    __syncthreads();
    // first trace of a run: largest t with P_s[t] <= pos
    auto trace_at = [&](int pos) {
        int lo = 0, hi = N;  // invariant: P_s[lo] <= pos < P_s[hi] (P_s[N] = T2 > pos)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (P_s[mid] <= pos) lo = mid; else hi = mid;
        }
        return lo;
    };
    for (int wh = tid; wh < Wh; wh += kPlanThreads) {
        int cnt = 0;
        int pos = wq[wh];
        const int end = min(wq[wh + 1], T2);
        if (pos < end) {
            int t = trace_at(pos);
            while (pos < end) {
                const int te = P_s[t + 1];
                if (te > pos) { ++cnt; pos = min(end, te); }
                ++t;
            }
        }
        wcnt[wh] = cnt;
    }
    __syncthreads();
    const int total2 = array_excl_scan(wcnt, Wh, scratch);  // wcnt[wh] = first private record of the wave
    if (tid == 0) wcnt[Wh] = total2;
    __syncthreads();
    for (int wh = tid; wh <= Wh; wh += kPlanThreads) a.off2[wh] = wcnt[wh];
    auto emit = [&](int rec, int t, int first, int n) {
        const int nb = nb_s[t];
        Record r;
        r.i = t; r.first = first; r.n = n;
        r.ntok = (first + n == nb) ? len_s[t] - (nb - 1) * kPageTokens : kPageTokens;
        a.records[rec] = r;
    };
    for (int wh = tid; wh < Wh; wh += kPlanThreads) {
        if (!mfma)  // attn_prefix takes its sub-chunks from the header and the live list, not from records
            for (int s = wh; s < N1; s += Wh) {
                const int p = s / n_live;
                emit(s, live_list[s % n_live], p * sc, part_pages(p));
            }
        int rec = N1 + wcnt[wh];
        int pos = wq[wh];
        const int end = min(wq[wh + 1], T2);
        if (pos < end) {
            int t = trace_at(pos);
            while (pos < end) {
                const int tb = P_s[t], te = P_s[t + 1];
                if (te > pos) {
                    const int stop = min(end, te);
                    emit(rec, t, S + pos - tb, stop - pos);
                    if (pos == tb) a.first2[t] = rec;
                    atomicAdd(&a.cnt2[t], 1);
                    ++rec;
                    pos = stop;
                }
                ++t;
            }
        }
    }
    if (tid == 0) {
        a.hdr->total = N1 + total2;
        a.hdr->n1 = N1;
        a.hdr->n_live = n_live;
        a.hdr->parts = parts;
        a.hdr->shared = S;
        a.hdr->quota = Q;
        a.hdr->part_pages = sc;
        a.hdr->prefix_mfma = mfma ? 1 : 0;
        a.hdr->stamp = a.stamp;
    }
}

}  // namespace

void launch_plan(const AttnArgs &a, hipStream_t s)
{
    hipLaunchKernelGGL(attn_plan, dim3(1), dim3(kPlanThreads), 0, s, a);
}

}  // namespace attn
}  // namespace step
