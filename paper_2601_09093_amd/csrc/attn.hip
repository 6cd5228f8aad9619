// paged_decode_attn: split-K (flash-decoding) grouped-query decode attention over a paged bf16
// KV cache -- the attention inside NextToken(t) of Algorithm 1 (the paper gives no formula; this
// is softmax(q K^T scale) V for the newest token of every live trace).
//
// Four kernels per call:
//   attn_plan    one workgroup.  Validates the lengths, finds the leading pages that every live trace
//                shares (the prompt), and cuts the work into records (trace, first page, page count,
//                tokens in the last page): the shared pages into sub-chunks, the private pages of all
//                traces, concatenated, into one equal run per resident wave.
//   attn_prefix  the shared pages on the matrix cores: for one KV head the query rows of all live
//                traces form a dense matrix, so logits and output are two MFMA products and every
//                shared tile is read once per block of query rows instead of once per trace.
//   stage 1      the HBM-streaming kernels over the private pages: persistent single-wave workgroups,
//                one per resident wave slot, each walking its own list of records with the loads of the
//                next pages (and of the next record) in flight.
//                attn_partial_g4 (G == 4, D == 128): a (page, head) tile is P*D bf16 contiguous; the wave reads
//                it with 16-byte loads, lane l taking bytes [j*1024 + 16 l, +16) on load j.  A row of D
//                values lives in LPR = D/8 neighbouring lanes and each group of LPR lanes ("row group"
//                r) sees the tokens r, r+TPI, ... of every page: TPI = 64/LPR independent online-softmax
//                streams per wave, merged once per record; the 4 query heads share every K and V
//                register (bf16 dot2 on the vector ALUs).
//                attn_partial_mfma (every other shape): the two products on the matrix cores with the G
//                query heads of the trace in the columns, so the arithmetic per byte does not grow with G.
//   attn_merge   stage 2: per (trace, query head) combine the record partials (m, l, acc), round to
//                bf16.
#include <hip/hip_ext.h>

#include "common.h"

namespace step {
namespace {

constexpr float kMinusBig = -1.0e30f;  // finite "no token seen yet" running max (keeps exp2 NaN-free)

struct Record {       // 16 bytes, read with one scalar load
    int32_t i;        // trace
    int32_t first;    // first page (index into the trace's block-table row)
    int32_t n;        // pages, >= 1
    int32_t ntok;     // tokens in the record's last page, 1 .. 16
};

constexpr int kMaxParts = 8;     // a shared prefix is cut into at most this many sub-chunks per trace
constexpr int kMaxPlanN = 2048;  // traces the planner handles
constexpr int kMaxWh = 2048;     // waves per KV head the planner handles
constexpr int kMaxShared = 1024; // pages of common prefix looked for (16384 tokens); <= kPlanThreads

struct PlanHeader {   // 256 bytes
    int32_t total;    // records: [0, n1) cover the shared prefix, [n1, total) the private pages
    int32_t n1;       // n_live * parts
    int32_t n_live;   // traces with seq_len > 0
    int32_t parts;    // sub-chunks of the shared prefix per trace (0 when nothing is shared)
    int32_t shared;   // S: leading pages common to every live trace
    int32_t quota;    // Q: pages per wave
    int32_t stamp;    // hash of the dims the plan was made for (AttnArgs::stamp), never 0
    int32_t part_pages; // pages per sub-chunk of the shared prefix (the last one may hold fewer)
    int32_t prefix_mfma; // 1: the shared-prefix records are computed by attn_prefix, stage 1 skips them
    int32_t pad[55];
};

struct AttnArgs {
    const uint16_t *q, *k_pages, *v_pages;
    const int32_t *block_tables, *seq_lens;
    PlanHeader *hdr;
    int32_t *off2;        // [Wh + 1] private-page records of wave wh are n1 + [off2[wh], off2[wh+1])
    Record *records;      // [max_records]; shared-prefix record s = p * n_live + rank belongs to wave s % Wh
    int32_t *rank;        // [N] rank of a live trace among the live traces
    int32_t *first2;      // [N] first record of the trace's private pages (they are consecutive)
    int32_t *cnt2;        // [N] number of such records
    int32_t *live;        // [N] rank -> trace (the live traces in index order)
    int32_t *shared_pages; // [kMaxShared] page ids of the shared prefix (read by attn_prefix)
    float *part_acc;      // [records * Hkv][G][D]   slot = record * Hkv + kv head
    float *part_ml;       // [records * Hkv][G][2]   (running max in log2 units, weight sum)
    uint16_t *out;
    int32_t *status;
    int N, Hq, Hkv, MAXB, NP, Wh, max_records;
    int stamp;            // what hdr->stamp must hold for this call's dims
    int prefix_qt;        // 16-row query tiles per wave of attn_prefix (1 or 2); 0: no attn_prefix
    float scale_log2;     // scale * log2(e)
};

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
static_assert(kMaxShared <= kPlanThreads, "one thread copies one entry of the first live row");

// exclusive scan of one int per thread over the workgroup (wave shuffles + 16 wave totals)
__device__ int block_excl_scan(int v, int *scratch /*[32]*/, int *total)
{
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    int x = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(x, off);
        if (lane >= off) x += y;
    }
    if (lane == 63) scratch[wid] = x;
    __syncthreads();
    if (wid == 0) {
        int t = lane < 16 ? scratch[lane] : 0;
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) {
            const int y = __shfl_up(t, off);
            if (lane >= off) t += y;
        }
        if (lane < 16) scratch[16 + lane] = t;
    }
    __syncthreads();
    const int base = wid > 0 ? scratch[16 + wid - 1] : 0;
    *total = scratch[31];
    __syncthreads();
    return base + x - v;
}

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

// A plan is trusted only if it was made for the same dims: the stamp guards against a workspace
// that was never planned or was planned for another shape (garbage records would index out of the
// block tables).  Returns false, and reports, when the plan in the workspace cannot be used.
__device__ __forceinline__ bool plan_usable(const AttnArgs &a)
{
    const PlanHeader *h = a.hdr;
    const bool ok = h->stamp == a.stamp && h->n1 >= 0 && h->total >= h->n1 && h->total <= a.max_records &&
                    h->n_live >= 0 && h->n_live <= a.N && h->parts >= 0 && h->parts <= kMaxParts &&
                    h->n1 == h->n_live * h->parts && h->shared >= 0 && h->shared <= a.MAXB && h->part_pages >= 0 &&
                    (long long)h->parts * h->part_pages >= h->shared;
    if (!ok && threadIdx.x == 0) report(a.status, STEP_EPLAN);
    return ok;
}

// max without the NaN-quieting pass (inputs here are never signalling NaNs that matter)
__device__ __forceinline__ float max_nc(float x, float y) { return __builtin_amdgcn_fmed3f(x, y, INFINITY); }

// ---------------------------------------------------------------------------------------------
// The matrix-core form of one page pair, shared by attn_prefix and attn_partial_mfma.
// Operand layouts (lane = 16 * gr + c; a lane holds 8 contraction slots, and slot e of lane group gr
// of A meets slot e of lane group gr of B):
//   logits  S^T = K Q^T   A = K tile: row = token c, slots = d in [32 kb + 8 gr, +8)   (16-byte load)
//                         B = Q:      column = query row c, the same d                  (16-byte load)
//                         result: lane holds tokens 4 gr + j (j < 4) of query column c
//   output  O^T = V^T P^T B = P^T:    column = query c; slots 0..3 = the lane's own 4 weights of the
//                                     pair's first page, 4..7 = of its second page (no data movement)
//                         A = V^T:    tile j, row c <-> d = DB c + j; slots as for P^T.  The lane
//                                     loads, for its 8 tokens, the DB consecutive values d in
//                                     [DB c, DB c + DB) (16 bytes at D = 128) and transposes the
//                                     8 x DB block in registers with v_perm_b32.
//                         result: tile j, lane holds d = DB (4 gr + jj) + j: over the DB tiles, the 4 DB
//                                 consecutive values d in [4 DB gr, 4 DB gr + 4 DB) of query column c
// ---------------------------------------------------------------------------------------------
template <int D>
struct MfmaPair {
    static constexpr int KB = D / 32;  // contraction blocks of the logits
    static constexpr int DB = D / 16;  // output tiles
    static constexpr int VW = DB / 2;  // dwords of one V row a lane holds
    typedef u32 VRow __attribute__((ext_vector_type(VW)));

    // V^T operands of a pair from the lane's 8 V rows (rows 0..3: tokens 4 gr + e of the first page,
    // 4..7: of the second).  ntok0 / ntok1 = tokens of the two pages that belong to the trace: rows
    // past them may hold anything (NaN included) and are cleared before they meet a zero weight.
    static __device__ __forceinline__ void v_operands(VRow (&vr)[8], int ntok0, int ntok1, int gr, uint4 (&vf)[DB])
    {
        if (ntok0 < kPageTokens || ntok1 < kPageTokens) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (4 * gr + e >= ntok0) vr[e] = VRow(0);
                if (4 * gr + e >= ntok1) vr[4 + e] = VRow(0);
            }
        }
#pragma unroll
        for (int jt = 0; jt < DB; ++jt) {
            const u32 sel = (jt & 1) ? 0x07060302u : 0x05040100u;
            u32 w[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) w[k] = __builtin_amdgcn_perm(vr[2 * k + 1][jt / 2], vr[2 * k][jt / 2], sel);
            vf[jt] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }

    // logits of one 16-column query tile against the pair, online softmax per column (running max m,
    // this lane group's share l of the weight sum), weights rounded to bf16 straight into the second
    // product; the weight sum is taken from the rounded weights, the accumulators are rescaled only
    // when some column's maximum moved
    static __device__ __forceinline__ void attend(const uint4 (&kf)[2][KB], const uint4 (&qf)[KB], const uint4 (&vf)[DB],
                                                  int ntok0, int ntok1, int gr, float scale_log2, float &m, float &l,
                                                  f32x4 (&o)[DB])
    {
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[0][kb]),
                                                         __builtin_bit_cast(bf16x8, qf[kb]), s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[1][kb]),
                                                         __builtin_bit_cast(bf16x8, qf[kb]), s1, 0, 0, 0);
        }
        float x[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[e] = s0[e] * scale_log2;
            x[4 + e] = s1[e] * scale_log2;
        }
        if (ntok0 < kPageTokens || ntok1 < kPageTokens) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (4 * gr + e >= ntok0) x[e] = -INFINITY;
                if (4 * gr + e >= ntok1) x[4 + e] = -INFINITY;
            }
        }
        float mx = x[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) mx = max_nc(mx, x[e]);
        mx = max_nc(mx, __shfl_xor(mx, 16));
        mx = max_nc(mx, __shfl_xor(mx, 32));
        const float m_new = max_nc(m, mx);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        u32 pw[4];
        float lsum = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bf16x2 pk = {(__bf16)__builtin_amdgcn_exp2f(x[2 * k] - m_new),
                               (__bf16)__builtin_amdgcn_exp2f(x[2 * k + 1] - m_new)};
            pw[k] = __builtin_bit_cast(u32, pk);
            lsum += bf16_lo(pw[k]) + bf16_hi(pw[k]);  // the weights as V sees them
        }
        l = fmaf(l, alpha, lsum);
        const bf16x8 pt = __builtin_bit_cast(bf16x8, make_uint4(pw[0], pw[1], pw[2], pw[3]));
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int jt = 0; jt < DB; ++jt) o[jt] *= alpha;
        }
#pragma unroll
        for (int jt = 0; jt < DB; ++jt)
            o[jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf[jt]), pt, o[jt], 0, 0, 0);
    }

    // the finished accumulators of query column c as the partial of (slot, head): lane (gr, c) holds d
    // in [4 DB gr, 4 DB gr + 4 DB); l is this lane group's share of the weight sum
    static __device__ __forceinline__ void store_partial(const AttnArgs &a, size_t slot, int G, int head, int gr, bool write,
                                                         float m, float l, const f32x4 (&o)[DB])
    {
        float ls = l;
        ls += __shfl_xor(ls, 16);
        ls += __shfl_xor(ls, 32);
        if (!write) return;
        float *pacc = a.part_acc + slot * ((size_t)G * D) + (size_t)head * D + 4 * DB * gr;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int j4 = 0; j4 < DB; j4 += 4)
                *reinterpret_cast<float4 *>(pacc + DB * jj + j4) =
                    make_float4(o[j4][jj], o[j4 + 1][jj], o[j4 + 2][jj], o[j4 + 3][jj]);
        if (gr == 0) {
            float *pml = a.part_ml + slot * ((size_t)G * 2) + head * 2;
            pml[0] = m;
            pml[1] = ls;
        }
    }
};

// ---------------------------------------------------------------------------------------------
// shared prefix on the matrix cores.  The S leading pages are the same physical pages for every live
// trace, so for one KV head the n_live * G query rows that attend to them form a dense matrix: the
// logits are K Q^T and the output V^T P^T, both v_mfma_f32_16x16x32_bf16, and every shared tile is
// read once per block of query rows instead of once per trace.  One wave per (KV head, block of
// 16 * QT query rows, sub-chunk p of the prefix); it writes the partial (m, l, acc) of the shared-prefix
// records p * n_live + rank, exactly what stage 1 would have written for them, so the merge does
// not change.
//
// (operand layouts: MfmaPair above)
// These units are a launch of their own, ahead of stage 1.  Run inside the stage-1 launch, next to
// the streaming waves (both fit on a SIMD), they were measured to cost more than they do alone: every
// streaming wave owns the same share of pages, so the wave that shares its SIMD longest sets the
// kernel's end.
template <int D, int QT>
__global__ __launch_bounds__(64) void attn_prefix(const AttnArgs a)
{
    typedef MfmaPair<D> MP;
    constexpr int KB = MP::KB, DB = MP::DB;
    typedef typename MP::VRow VRow;
    const int lane = threadIdx.x, c = lane & 15, gr = lane >> 4;
    if (!plan_usable(a)) return;
    const PlanHeader *hd = a.hdr;
    if (!hd->prefix_mfma) return;
    const int S = hd->shared, parts = hd->parts, n_live = hd->n_live, sc = hd->part_pages;
    const int G = a.Hq / a.Hkv;
    const int rows = n_live * G;
    const int nqb = (a.N * G + 16 * QT - 1) / (16 * QT);
    int u = blockIdx.x;
    const int g = u % a.Hkv;
    u /= a.Hkv;
    const int qb = u % nqb, p = u / nqb;
    if (p >= parts || qb * 16 * QT >= rows) return;
    const int first = p * sc, n = min(sc, S - first);
    if (n < 1 || S > kMaxShared || a.NP <= 0) {
        if (lane == 0) report(a.status, a.NP <= 0 ? STEP_EPAGE : STEP_EPLAN);
        return;
    }

    bool bad_plan = false, bad_page = false;
    auto trace_of_rank = [&](int rk) {
        const int t = a.live[rk];
        const bool ok = (u32)t < (u32)a.N;
        bad_plan |= !ok;
        return ok ? t : 0;
    };
    const int32_t *bt = a.shared_pages + first;  // first + n <= S <= kMaxShared
    auto page_at = [&](int j) {
        const int pg = __builtin_amdgcn_readfirstlane(bt[min(j, n - 1)]);  // the same for every lane: keep it scalar
        const bool ok = (u32)pg < (u32)a.NP;
        bad_page |= !ok;
        return ok ? pg : 0;
    };

    // query rows of this block: row = rank * G + head-in-group
    uint4 qf[QT][KB];
    int rank_of[QT], hh_of[QT];
    bool valid[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int row = (qb * QT + qt) * 16 + c;
        valid[qt] = row < rows;
        const int rw = valid[qt] ? row : 0;
        rank_of[qt] = rw / G;
        hh_of[qt] = rw % G;
        const uint16_t *qrow = a.q + ((size_t)trace_of_rank(rank_of[qt]) * a.Hq + g * G + hh_of[qt]) * D;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const uint4 x = *reinterpret_cast<const uint4 *>(qrow + kb * 32 + gr * 8);
            qf[qt][kb] = valid[qt] ? x : make_uint4(0, 0, 0, 0);
        }
    }

    // a tile's address is a wave-uniform base (page id from a scalar load) plus a 32-bit lane offset
    // plus a constant: one scalar multiply per page, no per-lane 64-bit arithmetic
    const size_t tile_bytes = (size_t)kPageTokens * D * 2;
    const u32 k_lane = (u32)(c * D + gr * 8) * 2;
    const u32 v_lane = (u32)(4 * gr * D + DB * c) * 2;
    auto load_pair = [&](int j, uint4 (&kf)[2][KB], VRow (&vr)[8]) {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
            const size_t base = ((size_t)page_at(j + pg) * a.Hkv + g) * tile_bytes;
            const char *kt = reinterpret_cast<const char *>(a.k_pages) + base;
            const char *vt = reinterpret_cast<const char *>(a.v_pages) + base;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) kf[pg][kb] = *reinterpret_cast<const uint4 *>(kt + k_lane + kb * 64);
#pragma unroll
            for (int e = 0; e < 4; ++e) vr[pg * 4 + e] = *reinterpret_cast<const VRow *>(vt + v_lane + e * D * 2);
        }
    };

    f32x4 o[QT][DB];
    float m[QT], l[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        m[qt] = kMinusBig;
        l[qt] = 0.f;
#pragma unroll
        for (int j = 0; j < DB; ++j) o[qt][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // one page pair against the QT query tiles; an odd sub-chunk ends on half a pair, whose second page
    // gets no weight
    auto attend_pair = [&](const uint4 (&kf)[2][KB], VRow (&vr)[8], bool second) {
        const int ntok1 = second ? kPageTokens : 0;
        uint4 vf[DB];
        MP::v_operands(vr, kPageTokens, ntok1, gr, vf);
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
            MP::attend(kf, qf[qt], vf, kPageTokens, ntok1, gr, a.scale_log2, m[qt], l[qt], o[qt]);
    };

    // NBUF pair buffers in rotation: the loads of the next NBUF - 1 pairs are in flight while a pair is
    // used (a sub-chunk is a handful of pairs, so most of its tiles are requested at once)
    constexpr int NBUF = QT == 1 ? 3 : 2;
    uint4 kf[NBUF][2][KB];
    VRow vr[NBUF][8];
    // the units that share this sub-chunk (same KV head, other query blocks) walk its pairs in
    // rotated orders, so that they do not all ask the L2 for the same lines at the same moment
    const int np = (n + 1) / 2;
    const int rot = qb % np;
    auto pair_at = [&](int t) { return 2 * ((t + rot) % np); };  // first page of the t-th pair visited
#pragma unroll
    for (int b = 0; b < NBUF; ++b)
        if (b < np) load_pair(pair_at(b), kf[b], vr[b]);
    for (int t0 = 0; t0 < np; t0 += NBUF) {
#pragma unroll
        for (int b = 0; b < NBUF; ++b) {
            const int t = t0 + b;
            if (t < np) {
                // an odd sub-chunk ends on half a pair: that pair's second page gets no weight
                attend_pair(kf[b], vr[b], pair_at(t) + 1 < n);
                if (t + NBUF < np) load_pair(pair_at(t + NBUF), kf[b], vr[b]);
            }
        }
    }

    // partials of the records p * n_live + rank
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
        MP::store_partial(a, ((size_t)p * n_live + rank_of[qt]) * a.Hkv + g, G, hh_of[qt], gr, valid[qt], m[qt], l[qt], o[qt]);
    if (bad_plan && lane == 0) report(a.status, STEP_EPLAN);
    if (bad_page && lane == 0) report(a.status, STEP_EPAGE);
}

// ---------------------------------------------------------------------------------------------
// stage 1 on the matrix cores, any group size: the persistent streaming kernel for G != 4.
// The same two products as attn_prefix with the G query heads of ONE trace in the columns (the other
// 16 - G columns are zero and never stored), over the private pages of the wave's records, pair of
// pages by pair of pages.  The operand loads (K: 16 rows x 64 bytes per instruction, V: 4 rows x
// 256 bytes) stream a fragmented pool as fast as the 1 KB-per-instruction loads of the G == 4 kernel
// (measured on a bare read probe: 6.79 against 6.81 TB/s), and the arithmetic per byte no longer grows
// with G.  Page ids, records and tiles are requested ahead of their use across record boundaries:
// the wave's page pairs form one sequence, a load cursor runs kBufs pairs ahead of the compute cursor.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(64) void attn_partial_mfma(const AttnArgs a)
{
    typedef MfmaPair<D> MP;
    constexpr int KB = MP::KB, DB = MP::DB;
    constexpr int kBufs = 3;
    typedef typename MP::VRow VRow;
    typedef u32 u32x4 __attribute__((ext_vector_type(4)));
    const int lane = threadIdx.x, c = lane & 15, gr = lane >> 4;
    const int g = blockIdx.x % a.Hkv;
    const int wh = blockIdx.x / a.Hkv;
    if (!plan_usable(a)) return;
    const int G = a.Hq / a.Hkv;
    const int n1 = a.hdr->n1;
    const int p2_begin = n1 + a.off2[wh], p2_end = n1 + a.off2[wh + 1];
    if (p2_begin < n1 || p2_end < p2_begin || p2_end > a.hdr->total) {
        if (lane == 0) report(a.status, STEP_EPLAN);
        return;
    }
    auto next_record = [&](int id) {  // id of the record after `id` in this wave's list, -1 at the end
        int nx;
        if (id < n1) {
            nx = id + a.Wh;
            if (nx >= n1) nx = p2_begin;
        } else {
            nx = id + 1;
        }
        return nx < p2_end ? nx : -1;
    };
    const int first_id = (wh < n1 && !a.hdr->prefix_mfma) ? wh : (p2_begin < p2_end ? p2_begin : -1);
    if (first_id < 0) return;
    if (a.NP <= 0) {
        if (lane == 0) report(a.status, STEP_EPAGE);
        return;
    }

    bool bad_plan = false, bad_page = false;
    auto record_at = [&](int id) {  // a record that points outside the block tables is replaced and reported
        Record x = a.records[id];
        const bool ok = (u32)x.i < (u32)a.N && x.first >= 0 && x.n >= 1 && (long long)x.first + x.n <= a.MAXB &&
                        x.ntok >= 1 && x.ntok <= kPageTokens;
        bad_plan |= !ok;
        if (!ok) x = Record{0, 0, 1, 1};
        return x;
    };

    // a position in the wave's sequence of page pairs: pages j and j + 1 of record id
    struct Cursor {
        int id;      // < 0: past the end
        int next_id; // the record after it
        Record rec, next_rec;
        int j;
    };
    auto enter = [&](int id, const Record &rec) {  // first pair of record id; its successor is fetched now, used later
        Cursor x;
        x.id = id;
        x.rec = rec;
        x.j = 0;
        x.next_id = id >= 0 ? next_record(id) : -1;
        x.next_rec = x.next_id >= 0 ? record_at(x.next_id) : Record{0, 0, 1, 1};
        return x;
    };
    auto advance = [&](Cursor &x) {
        x.j += 2;
        if (x.j >= x.rec.n) x = enter(x.next_id, x.next_rec);
    };
    auto page_ids = [&](const Cursor &x, int &p0, int &p1) {  // second page of an odd record's last pair: the last page again
        const int32_t *row = a.block_tables + (size_t)x.rec.i * a.MAXB + x.rec.first;
        p0 = row[x.j];
        p1 = row[min(x.j + 1, x.rec.n - 1)];
    };

    const size_t tile_bytes = (size_t)kPageTokens * D * 2;
    const u32 k_lane = (u32)(c * D + gr * 8) * 2;
    const u32 v_lane = (u32)(4 * gr * D + DB * c) * 2;
    auto tile_of = [&](int page) {
        const int pg = __builtin_amdgcn_readfirstlane(page);
        const bool ok = (u32)pg < (u32)a.NP;
        bad_page |= !ok;
        return ((size_t)(ok ? pg : 0) * a.Hkv + g) * tile_bytes;
    };
    // KV tiles are read once: non-temporal loads (streaming cache policy)
    auto load_pair = [&](int p0, int p1, uint4 (&kf)[2][KB], VRow (&vr)[8]) {
        const int pgs[2] = {p0, p1};
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
            const size_t base = tile_of(pgs[pg]);
            const char *kt = reinterpret_cast<const char *>(a.k_pages) + base;
            const char *vt = reinterpret_cast<const char *>(a.v_pages) + base;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(kt + k_lane + kb * 64));
                kf[pg][kb] = make_uint4(t.x, t.y, t.z, t.w);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
                vr[pg * 4 + e] = __builtin_nontemporal_load(reinterpret_cast<const VRow *>(vt + v_lane + e * D * 2));
        }
    };
    auto load_q = [&](int trace, uint4 (&qf)[KB]) {  // column c = query head g * G + c of the trace, zero beyond G
        const uint16_t *qrow = a.q + ((size_t)trace * a.Hq + g * G + min(c, G - 1)) * D;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const uint4 x = *reinterpret_cast<const uint4 *>(qrow + kb * 32 + gr * 8);
            qf[kb] = c < G ? x : make_uint4(0, 0, 0, 0);
        }
    };

    // per record: running max, weight sum (this lane group's tokens) and output tiles of column c
    f32x4 o[DB];
    float m = kMinusBig, l = 0.f;
    uint4 qf[KB];

    auto attend_pair = [&](const uint4 (&kf)[2][KB], VRow (&vr)[8], int ntok0, int ntok1) {
        uint4 vf[DB];
        MP::v_operands(vr, ntok0, ntok1, gr, vf);
        MP::attend(kf, qf, vf, ntok0, ntok1, gr, a.scale_log2, m, l, o);
    };

    // pair buffers: tiles, the cursor they belong to and, for the first pair of a record, its queries
    uint4 kf[kBufs][2][KB];
    VRow vr[kBufs][8];
    uint4 qslot[kBufs][KB];
    Cursor at[kBufs];

    Cursor cur = enter(first_id, record_at(first_id));  // load cursor
    int id0, id1;                                       // page ids of the load cursor's pair
    page_ids(cur, id0, id1);
    auto fill = [&](uint4 (&kfb)[2][KB], VRow (&vrb)[8], uint4 (&qb)[KB], Cursor &slot) {
        slot = cur;
        if (cur.id < 0) return;
        load_pair(id0, id1, kfb, vrb);
        if (cur.j == 0) load_q(cur.rec.i, qb);
        advance(cur);
        if (cur.id >= 0) page_ids(cur, id0, id1);  // used one refill later
    };
#pragma unroll
    for (int b = 0; b < kBufs; ++b) fill(kf[b], vr[b], qslot[b], at[b]);

    bool done = false;
    while (!done) {
#pragma unroll
        for (int b = 0; b < kBufs; ++b) {
            if (done) continue;
            const Cursor x = at[b];
            if (x.id < 0) {
                done = true;
                continue;
            }
            if (x.j == 0) {  // a new record starts
                m = kMinusBig;
                l = 0.f;
#pragma unroll
                for (int jt = 0; jt < DB; ++jt) o[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) qf[kb] = qslot[b][kb];
            }
            const int n = x.rec.n;
            auto tokens_of = [&](int jj) { return jj < n - 1 ? kPageTokens : (jj == n - 1 ? x.rec.ntok : 0); };
            attend_pair(kf[b], vr[b], tokens_of(x.j), tokens_of(x.j + 1));
            const bool last = x.j + 2 >= n;
            fill(kf[b], vr[b], qslot[b], at[b]);  // the buffer is free: request the pair kBufs ahead
            if (last) MP::store_partial(a, (size_t)x.id * a.Hkv + g, G, min(c, G - 1), gr, c < G, m, l, o);
        }
    }
    if (bad_plan && lane == 0) report(a.status, STEP_EPLAN);
    if (bad_page && lane == 0) report(a.status, STEP_EPAGE);
}

// ---------------------------------------------------------------------------------------------
// stage 1, G == 4 and D == 128 (the shape of all three models of the paper): persistent, software-pipelined.
//   phase A(page) : logits of the page (bf16 dot2), transposing reduction that leaves each lane
//                   with one (token, head) logit, running max, p = 2^(x - m), rounded to bf16 and
//                   packed in token pairs, handed to the row group through LDS.
//   phase B(page) : acc += P V with bf16 dot2 on (token pair) x (head), fp32 accumulation.
// A(page j+1) and B(page j) are independent and sit in ONE basic block, so the scheduler overlaps
// the cross-lane / LDS / exp latencies of A with the dot2 stream of B.  The rescale of acc by
// 2^(m_old - m_new), needed only when a page raises the running max, follows B.
// The weight sum l is accumulated from the same bf16-rounded weights that multiply V, so the result
// is an exact weighted average of V rows with weights perturbed by <= 2^-9 relative.
// ---------------------------------------------------------------------------------------------
template <int BIT>
__device__ __forceinline__ float partner(float v)
{
    if constexpr (BIT == 3) return dpp<kDppRowMirror>(v);
    else if constexpr (BIT == 2) return dpp<kDppHalfMirror>(v);
    else if constexpr (BIT == 1) return dpp<kDppXor2>(v);
    else return dpp<kDppXor1>(v);
}

// One stage of the transposing reduction: lanes whose bit BIT of c differ pair up, each keeps the
// half of its NCUR values whose index has that bit equal to its own and adds the partner's copy.
template <int BIT, int NCUR, int NV>
__device__ __forceinline__ void bfly_stage(float (&val)[NV], int c)
{
    const bool up = (c >> BIT) & 1;
#pragma unroll
    for (int t = 0; t < NCUR / 2; ++t) {
        const float lo = val[t], hi = val[t + NCUR / 2];
        const float keep = up ? hi : lo;
        const float send = up ? lo : hi;
        val[t] = keep + partner<BIT>(send);
    }
}

template <int D>
__global__ __launch_bounds__(64, 2) void attn_partial_g4(const AttnArgs a)
{
    constexpr int G = 4;
    constexpr int LPR = D / 8, TPI = 64 / LPR, IPP = kPageTokens / TPI, NV = IPP * G;
    static_assert(D == 128 && NV == LPR, "a row is 16 lanes wide: one logit per lane after the transposing reduction");
    constexpr int NPAIR = IPP / 2;  // token pairs per lane per page
    __shared__ u32 pbuf[2][64];

    const int lane = threadIdx.x;
    const int r = lane / LPR, c = lane % LPR;
    // gridDim == Wh * Hkv: wave (wh, g) serves KV head g only.  Consecutive workgroups land on
    // consecutive XCDs, so with Hkv == 8 every XCD streams (and caches) the tiles of one KV head.
    // Its records: the shared-prefix records wh, wh + Wh, ... below n1, then the private-page
    // records n1 + [off2[wh], off2[wh + 1]).
    const int g = blockIdx.x % a.Hkv;
    const int wh = blockIdx.x / a.Hkv;
    if (!plan_usable(a)) return;
    const int n1 = a.hdr->n1;
    const int p2_begin = n1 + a.off2[wh], p2_end = n1 + a.off2[wh + 1];
    if (p2_begin < n1 || p2_end < p2_begin || p2_end > a.hdr->total) {
        if (lane == 0) report(a.status, STEP_EPLAN);
        return;
    }
    auto next_record = [&](int id) {  // id of the record after `id` in this wave's list, -1 at the end
        int nx;
        if (id < n1) {
            nx = id + a.Wh;
            if (nx >= n1) nx = p2_begin;
        } else {
            nx = id + 1;
        }
        return nx < p2_end ? nx : -1;
    };
    // (with attn_prefix the shared-prefix records are not this kernel's)
    int rec_id = (wh < n1 && !a.hdr->prefix_mfma) ? wh : (p2_begin < p2_end ? p2_begin : -1);
    if (rec_id < 0) return;
    if (a.NP <= 0) {
        if (lane == 0) report(a.status, STEP_EPAGE);
        return;
    }

    const size_t tile_u4 = (size_t)kPageTokens * D / 8;  // uint4 units per (page, head) tile
    const uint4 *kbase = reinterpret_cast<const uint4 *>(a.k_pages);
    const uint4 *vbase = reinterpret_cast<const uint4 *>(a.v_pages);
    bool bad_page = false;
    auto tile_at = [&](int page) -> size_t {
        const bool ok = (u32)page < (u32)a.NP;
        bad_page |= !ok;
        return ((size_t)(ok ? page : 0) * a.Hkv + g) * tile_u4 + lane;
    };
    // KV tiles are read once and never again by this wave: non-temporal loads (streaming cache
    // policy) keep them from displacing each other in the caches; measured +10 % on a bare tile
    // stream, and the shared prompt tiles are still served from L2
    auto load4 = [&](const uint4 *base, size_t off, uint4 (&x)[IPP]) {
        typedef u32 u32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int j = 0; j < IPP; ++j) {
            const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(base + off + j * 64));
            x[j] = make_uint4(t.x, t.y, t.z, t.w);
        }
    };

    uint4 qv[G];
    auto load_q = [&](int i) {
#pragma unroll
        for (int h = 0; h < G; ++h)
            qv[h] = *reinterpret_cast<const uint4 *>(a.q + ((size_t)i * a.Hq + (size_t)g * G + h) * D + c * 8);
    };

    float m[G], acc[G][8];
    float m_own, l_own, mx_pending;

    auto phaseA = [&](const uint4 (&k)[IPP], int slot, int ntok) {
        float val[NV];
#pragma unroll
        for (int j = 0; j < IPP; ++j)
#pragma unroll
            for (int h = 0; h < G; ++h) {
                float s = dot2_bf16(k[j].x, qv[h].x, 0.f);
                s = dot2_bf16(k[j].y, qv[h].y, s);
                s = dot2_bf16(k[j].z, qv[h].z, s);
                s = dot2_bf16(k[j].w, qv[h].w, s);
                val[j * G + h] = s;
            }
        bfly_stage<3, 16, NV>(val, c);
        bfly_stage<2, 8, NV>(val, c);
        bfly_stage<1, 4, NV>(val, c);
        bfly_stage<0, 2, NV>(val, c);
        // this lane owns the logit of (slot (c/G)*TPI + r, head c % G); slots >= ntok are not tokens
        float x = val[0] * a.scale_log2;
        x = ((c / G) * TPI + r < ntok) ? x : -INFINITY;
        float mx = x;
        mx = max_nc(mx, dpp<kDppRowRor4>(mx));
        mx = max_nc(mx, dpp<kDppRowRor8>(mx));
        const float m_new = max_nc(m_own, mx);
        const float alpha_own = __builtin_amdgcn_exp2f(m_own - m_new);
        m_own = m_new;
        mx_pending = mx;
        const float p = __builtin_amdgcn_exp2f(x - m_new);
        // lane c + 4 of the row group holds the same head's weight for the next token row
        const float p_next = dpp<0x12C>(p);  // row_ror:12 = value of lane (c + 4) % 16
        const bf16x2 pk = {(__bf16)p, (__bf16)p_next};
        const u32 w = __builtin_bit_cast(u32, pk);
        l_own = fmaf(l_own, alpha_own, bf16_lo(w));
        pbuf[slot][lane] = w;
    };

    auto pv_pairs = [&](const uint4 (&v)[IPP], int slot) {
        const uint4 *pb = reinterpret_cast<const uint4 *>(&pbuf[slot][r * LPR]);
#pragma unroll
        for (int pr = 0; pr < NPAIR; ++pr) {
            const uint4 pp = pb[2 * pr];  // words 8 pr .. 8 pr + 3: heads 0..3 of token pair pr
            const u32 ph[4] = {pp.x, pp.y, pp.z, pp.w};
            const u32 w0[4] = {v[2 * pr].x, v[2 * pr].y, v[2 * pr].z, v[2 * pr].w};
            const u32 w1[4] = {v[2 * pr + 1].x, v[2 * pr + 1].y, v[2 * pr + 1].z, v[2 * pr + 1].w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const u32 lo = __builtin_amdgcn_perm(w1[t], w0[t], 0x05040100u);  // (row0[2t],   row1[2t])
                const u32 hi = __builtin_amdgcn_perm(w1[t], w0[t], 0x07060302u);  // (row0[2t+1], row1[2t+1])
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    acc[h][2 * t] = dot2_bf16(lo, ph[h], acc[h][2 * t]);
                    acc[h][2 * t + 1] = dot2_bf16(hi, ph[h], acc[h][2 * t + 1]);
                }
            }
        }
    };

    auto rescale = [&]() {
        float mq[G];
        mq[0] = max_nc(m[0], dpp<STEP_DPP_QUAD_BCAST(0)>(mx_pending));
        mq[1] = max_nc(m[1], dpp<STEP_DPP_QUAD_BCAST(1)>(mx_pending));
        mq[2] = max_nc(m[2], dpp<STEP_DPP_QUAD_BCAST(2)>(mx_pending));
        mq[3] = max_nc(m[3], dpp<STEP_DPP_QUAD_BCAST(3)>(mx_pending));
        const bool grow = (mq[0] > m[0]) | (mq[1] > m[1]) | (mq[2] > m[2]) | (mq[3] > m[3]);
        if (__any(grow)) {
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const float alpha = __builtin_amdgcn_exp2f(m[h] - mq[h]);
                m[h] = mq[h];
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[h][e] *= alpha;
            }
        }
    };
    // rows past the trace's last token may hold anything (NaN included): clear them before they
    // meet a zero weight
    auto clear_tail = [&](uint4 (&v)[IPP], int ntok) {
#pragma unroll
        for (int jj = 0; jj < IPP; ++jj)
            if (jj * TPI + r >= ntok) v[jj] = make_uint4(0, 0, 0, 0);
    };

    // a record that points outside the block tables (a workspace overwritten after planning) is
    // replaced by a one-token record of trace 0 and reported; nothing is read out of bounds
    bool bad_plan = false;
    auto record_at = [&](int id) {
        Record x = a.records[id];
        const bool ok = (u32)x.i < (u32)a.N && x.first >= 0 && x.n >= 1 && (long long)x.first + x.n <= a.MAXB &&
                        x.ntok >= 1 && x.ntok <= kPageTokens;
        bad_plan |= !ok;
        if (!ok) x = Record{0, 0, 1, 1};
        return x;
    };

    uint4 k0[IPP], v0[IPP], k1[IPP], v1[IPP];
    Record rec = record_at(rec_id);
    {
        const int32_t *bt0 = a.block_tables + (size_t)rec.i * a.MAXB + rec.first;
        const size_t t0 = tile_at(bt0[0]), t1 = tile_at(bt0[rec.n > 1 ? 1 : 0]);
        load4(kbase, t0, k0);
        load4(vbase, t0, v0);
        load4(kbase, t1, k1);
        load4(vbase, t1, v1);
        load_q(rec.i);
    }

    for (;;) {
        const int next_id = next_record(rec_id);
        const bool has_next = next_id >= 0;
        // the next record and the ids of its first two pages are fetched now and consumed after this
        // record's pages
        const Record nrec = record_at(has_next ? next_id : rec_id);
        const int32_t *nbt = a.block_tables + (size_t)nrec.i * a.MAXB + nrec.first;
        const int npage0 = nbt[0], npage1 = nbt[nrec.n > 1 ? 1 : 0];

        const int n = rec.n;
        const int32_t *bt = a.block_tables + (size_t)rec.i * a.MAXB + rec.first;
        // page ids are fetched one loop trip (two pages) ahead of the tile loads that need them; the
        // index is clamped so the pipeline can run past the end without a branch (the surplus load
        // re-reads the last tile, which is then not used)
        auto page_id = [&](int j) { return bt[min(j, n - 1)]; };
        auto ntok_of = [&](int j) { return j == n - 1 ? rec.ntok : kPageTokens; };

        m_own = kMinusBig; l_own = 0.f; mx_pending = kMinusBig;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            m[h] = kMinusBig;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
        }

        int pid2 = page_id(2), pid3 = page_id(3);
        phaseA(k0, 0, ntok_of(0));
        rescale();
        int j = 0;
        for (; j + 2 <= n - 1; j += 2) {
            const size_t t2 = tile_at(pid2), t3 = tile_at(pid3);
            pid2 = page_id(j + 4);
            pid3 = page_id(j + 5);
            load4(kbase, t2, k0);
            phaseA(k1, 1, kPageTokens);
            pv_pairs(v0, 0);
            load4(vbase, t2, v0);
            rescale();
            load4(kbase, t3, k1);
            phaseA(k0, 0, ntok_of(j + 2));
            pv_pairs(v1, 1);
            load4(vbase, t3, v1);
            rescale();
        }
        if (j + 1 <= n - 1) {
            phaseA(k1, 1, ntok_of(j + 1));
            pv_pairs(v0, 0);
            rescale();
            clear_tail(v1, ntok_of(j + 1));
            pv_pairs(v1, 1);
        } else {
            clear_tail(v0, ntok_of(j));
            pv_pairs(v0, 0);
        }

        // all four tile buffers are dead: start the next record before reducing this one
        if (has_next) {
            const size_t t0 = tile_at(npage0), t1 = tile_at(npage1);
            load4(kbase, t0, k0);
            load4(vbase, t0, v0);
            load4(kbase, t1, k1);
            load4(vbase, t1, v1);
            load_q(nrec.i);
        }

        // ---- merge the TPI row-group streams of this wave, write the record's partial ----
        float ls = l_own;
        ls += dpp<kDppRowRor4>(ls);
        ls += dpp<kDppRowRor8>(ls);
        float lh[G];
        lh[0] = dpp<STEP_DPP_QUAD_BCAST(0)>(ls);
        lh[1] = dpp<STEP_DPP_QUAD_BCAST(1)>(ls);
        lh[2] = dpp<STEP_DPP_QUAD_BCAST(2)>(ls);
        lh[3] = dpp<STEP_DPP_QUAD_BCAST(3)>(ls);
        const size_t slot = (size_t)rec_id * a.Hkv + g;
        float *pacc = a.part_acc + slot * (G * D);
        float *pml = a.part_ml + slot * (G * 2);
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float M = m[h];
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) M = max_nc(M, __shfl_xor(M, off));
            const float f = __builtin_amdgcn_exp2f(m[h] - M);
            float l = lh[h] * f;
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) l += __shfl_xor(l, off);
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float x = acc[h][e] * f;
#pragma unroll
                for (int off = LPR; off < 64; off <<= 1) x += __shfl_xor(x, off);
                o[e] = x;
            }
            if (r == 0) {
                float4 *dst = reinterpret_cast<float4 *>(pacc + h * D + c * 8);
                dst[0] = make_float4(o[0], o[1], o[2], o[3]);
                dst[1] = make_float4(o[4], o[5], o[6], o[7]);
                if (c == 0) {
                    pml[h * 2 + 0] = M;
                    pml[h * 2 + 1] = l;
                }
            }
        }
        if (!has_next) break;
        rec = nrec;
        rec_id = next_id;
    }
    if (bad_plan && lane == 0) report(a.status, STEP_EPLAN);
    if (bad_page && lane == 0) report(a.status, STEP_EPAGE);
}

// ---------------------------------------------------------------------------------------------
// stage 2: out[i][h][:] = sum_c 2^(m_c - M) acc_c / sum_c 2^(m_c - M) l_c, rounded to bf16
// ---------------------------------------------------------------------------------------------
template <int D, int G>
__global__ __launch_bounds__(64) void attn_merge(const AttnArgs a)
{
    constexpr int DPT = D / 64;
    const int lane = threadIdx.x;
    const int i = blockIdx.x / a.Hq, h = blockIdx.x % a.Hq;
    const int g = h / G, hh = h % G;
    uint16_t *orow = a.out + ((size_t)i * a.Hq + h) * D;
    const int L = a.seq_lens[i];
    // the trace's records: `parts` shared-prefix sub-chunks, then cnt2 consecutive private ones
    const bool usable = plan_usable(a);
    const int parts = a.hdr->parts, n_live = a.hdr->n_live;
    const int rk = a.rank[i], f2 = a.first2[i];
    int nch = parts + a.cnt2[i];
    if (L <= 0 || (long long)L > (long long)a.MAXB * kPageTokens || !usable) nch = 0;
    if (nch > 0 && ((u32)rk >= (u32)n_live || f2 < 0 || a.cnt2[i] < 0 || f2 + a.cnt2[i] > a.hdr->total)) {
        if (lane == 0) report(a.status, STEP_EPLAN);
        nch = 0;
    }
    auto slot_of = [&](int ch) { return (size_t)(ch < parts ? ch * n_live + rk : f2 + (ch - parts)) * a.Hkv + g; };

    float o[DPT];
#pragma unroll
    for (int t = 0; t < DPT; ++t) o[t] = 0.f;
    float M = kMinusBig, den = 0.f;
    // 64 pieces at a time: lane p holds (m, l) of piece base + p, the wave agrees on the maximum,
    // then the piece accumulators are added with four loads in flight
    for (int base = 0; base < nch; base += 64) {
        const int cnt = min(64, nch - base);
        float mp = kMinusBig, lp = 0.f;
        if (lane < cnt) {
            const float *ml = a.part_ml + slot_of(base + lane) * (G * 2) + hh * 2;
            mp = ml[0];
            lp = ml[1];
        }
        float Mn = mp;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) Mn = fmaxf(Mn, __shfl_xor(Mn, off));
        Mn = fmaxf(Mn, M);
        const float resc = __builtin_amdgcn_exp2f(M - Mn);
        M = Mn;
        den *= resc;
#pragma unroll
        for (int t = 0; t < DPT; ++t) o[t] *= resc;
        const float fp = __builtin_amdgcn_exp2f(mp - M);  // 0 for lanes without a piece
        float lsum = fp * lp;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) lsum += __shfl_xor(lsum, off);
        den += lsum;
        int p = 0;
        for (; p + 3 < cnt; p += 4) {
            float v[4][DPT], f[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float *pa = a.part_acc + slot_of(base + p + u) * (G * D) + hh * D;
                f[u] = __shfl(fp, p + u);
#pragma unroll
                for (int t = 0; t < DPT; ++t) v[u][t] = pa[lane * DPT + t];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int t = 0; t < DPT; ++t) o[t] = fmaf(f[u], v[u][t], o[t]);
        }
        for (; p < cnt; ++p) {
            const float *pa = a.part_acc + slot_of(base + p) * (G * D) + hh * D;
            const float f = __shfl(fp, p);
#pragma unroll
            for (int t = 0; t < DPT; ++t) o[t] = fmaf(f, pa[lane * DPT + t], o[t]);
        }
    }
    const float inv = den > 0.f ? 1.0f / den : 0.f;
    if constexpr (DPT == 2) {
        const u32 w = f32_to_bf16_bits(o[0] * inv) | (f32_to_bf16_bits(o[1] * inv) << 16);
        reinterpret_cast<u32 *>(orow)[lane] = w;
    } else {
        orow[lane] = (uint16_t)f32_to_bf16_bits(o[0] * inv);
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
bool dims_ok(const step_attn_dims *d)
{
    if (!d) return false;
    if (d->N < 0 || d->Hq <= 0 || d->Hkv <= 0 || d->MAXB < 0 || d->NP < 0) return false;
    if (d->P != kPageTokens || (d->D != 64 && d->D != 128)) return false;
    if (d->Hq % d->Hkv) return false;
    const int G = d->Hq / d->Hkv;
    if (G != 1 && G != 2 && G != 4 && G != 8) return false;
    if (d->N > kMaxPlanN) return false;
    return true;
}

// waves per KV head: (CUs x waves of the stage-1 kernel that fit on one CU) / Hkv.  The environment
// variable STEP_ATTN_WAVES_PER_CU, read once, overrides the occupancy query (tuning aid).
int waves_per_head(const step_attn_dims *d)
{
    static const int cus = [] {
        int dev = 0, n = 256;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            n = prop.multiProcessorCount;
        return n;
    }();
    static const int per_cu_env = [] {
        const char *s = getenv("STEP_ATTN_WAVES_PER_CU");
        return s ? atoi(s) : 0;
    }();
    static const int per_cu_128 = [] {
        int nblk = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nblk, attn_partial_g4<128>, 64, 0) != hipSuccess || nblk <= 0)
            nblk = 8;
        return nblk < 4 ? nblk : 4;  // measured: one wave per SIMD streams fastest (no ALU contention between waves)
    }();
    const int per_cu = per_cu_env > 0 ? per_cu_env : per_cu_128;
    int wh = cus * per_cu / d->Hkv;
    if (wh < 1) wh = 1;
    if (wh > kMaxWh) wh = kMaxWh;
    return wh;
}

// The shared prefix goes to the matrix cores (attn_prefix) unless the environment variable
// STEP_ATTN_PREFIX is "0" (read once; testing aid: stage 1 then streams the prefix per trace).
bool prefix_enabled()
{
    static const bool on = [] {
        const char *s = getenv("STEP_ATTN_PREFIX");
        return !(s && s[0] == '0');
    }();
    return on;
}

struct Layout {  // byte offsets into the workspace, all multiples of 256
    size_t off2, records, rank, first2, cnt2, live, shared_pages, ml, acc, total;
    int Wh, max_records;
};

size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

Layout layout_for(const step_attn_dims *d)
{
    Layout l;
    l.Wh = waves_per_head(d);
    // private pages: at most Wh + N records; shared prefix: at most 4 Wh + N (attn_prefix), Wh + N otherwise
    l.max_records = 6 * l.Wh + 2 * d->N;
    const size_t R = (size_t)l.max_records, G = d->Hq / d->Hkv, N = d->N;
    l.off2 = 256;
    l.records = l.off2 + up256((size_t)(l.Wh + 1) * sizeof(int32_t));
    l.rank = l.records + up256(R * sizeof(Record));
    l.first2 = l.rank + up256(N * sizeof(int32_t));
    l.cnt2 = l.first2 + up256(N * sizeof(int32_t));
    l.live = l.cnt2 + up256(N * sizeof(int32_t));
    l.shared_pages = l.live + up256(N * sizeof(int32_t));
    l.ml = l.shared_pages + up256(kMaxShared * sizeof(int32_t));
    l.acc = l.ml + up256(R * d->Hkv * G * 2 * sizeof(float));
    l.total = l.acc + up256(R * d->Hkv * G * d->D * sizeof(float));
    return l;
}

// optional per-call event pairs around stage 1 (benchmarks only)
struct Profile {
    hipEvent_t *ev = nullptr;  // 2 * cap events
    int cap = 0, used = 0;
} g_prof;

enum : int { kDoPlan = 1, kDoAttend = 2 };

template <int D, int G>
int launch(const AttnArgs &a, hipStream_t s, int what)
{
    if (what & kDoPlan) hipLaunchKernelGGL(attn_plan, dim3(1), dim3(kPlanThreads), 0, s, a);
    const int prefix_units = a.prefix_qt ? a.Hkv * ((a.N * G + 16 * a.prefix_qt - 1) / (16 * a.prefix_qt)) * kMaxParts : 0;
    if ((what & kDoAttend) && prefix_units) {
        const dim3 grid((u32)prefix_units);
        if (a.prefix_qt == 2) hipLaunchKernelGGL((attn_prefix<D, 2>), grid, dim3(64), 0, s, a);
        else hipLaunchKernelGGL((attn_prefix<D, 1>), grid, dim3(64), 0, s, a);
    }
    if (what & kDoAttend) {
        // when profiling, the stage-1 launch carries its own start/stop events: they take the
        // kernel's begin and end timestamps, with no marker processing inside the interval
        const bool timed = g_prof.ev && g_prof.used < g_prof.cap;
        hipEvent_t e0 = timed ? g_prof.ev[2 * g_prof.used] : nullptr;
        hipEvent_t e1 = timed ? g_prof.ev[2 * g_prof.used + 1] : nullptr;
        if (timed) ++g_prof.used;
        // G == 4, D == 128: the dot2 kernel (about 1 % ahead of the matrix-core kernel at that shape; at
        // D == 64 the matrix-core kernel is the faster one, 6.2 against 5.5 TB/s);
        // STEP_ATTN_G4_MFMA=1, read once, sends that shape to the matrix-core kernel too (testing aid)
        static const bool g4_mfma = [] {
            const char *e = getenv("STEP_ATTN_G4_MFMA");
            return e && e[0] == '1';
        }();
        const dim3 grid((u32)(a.Wh * a.Hkv));
        bool launched = false;
        if constexpr (G == 4 && D == 128) {
            if (!g4_mfma) {
                if (timed) hipExtLaunchKernelGGL((attn_partial_g4<D>), grid, dim3(64), 0, s, e0, e1, 0, a);
                else hipLaunchKernelGGL((attn_partial_g4<D>), grid, dim3(64), 0, s, a);
                launched = true;
            }
        }
        if (!launched) {
            if (timed) hipExtLaunchKernelGGL((attn_partial_mfma<D>), grid, dim3(64), 0, s, e0, e1, 0, a);
            else hipLaunchKernelGGL((attn_partial_mfma<D>), grid, dim3(64), 0, s, a);
        }
        hipLaunchKernelGGL((attn_merge<D, G>), dim3((u32)(a.N * a.Hq)), dim3(64), 0, s, a);
    }
    return launch_status();
}

int run(const step_attn_dims *d, const uint16_t *q, const uint16_t *k_pages, const uint16_t *v_pages,
        const int32_t *block_tables, const int32_t *seq_lens, uint16_t *out, void *workspace,
        size_t workspace_bytes, int32_t *status, void *stream, int what)
{
    if (!dims_ok(d)) return STEP_EINVAL;
    if (d->N == 0) return STEP_OK;
    if (!block_tables || !seq_lens) return STEP_EINVAL;
    if (what & kDoAttend) {
        if (!q || !k_pages || !v_pages || !out) return STEP_EINVAL;
        if (!aligned(q, 16) || !aligned(k_pages, 16) || !aligned(v_pages, 16) || !aligned(out, 4)) return STEP_EINVAL;
    }
    const Layout l = layout_for(d);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < l.total) return STEP_EWORKSPACE;

    char *ws = reinterpret_cast<char *>(workspace);
    AttnArgs a;
    a.q = q; a.k_pages = k_pages; a.v_pages = v_pages;
    a.block_tables = block_tables; a.seq_lens = seq_lens;
    a.hdr = reinterpret_cast<PlanHeader *>(ws);
    a.off2 = reinterpret_cast<int32_t *>(ws + l.off2);
    a.records = reinterpret_cast<Record *>(ws + l.records);
    a.rank = reinterpret_cast<int32_t *>(ws + l.rank);
    a.first2 = reinterpret_cast<int32_t *>(ws + l.first2);
    a.cnt2 = reinterpret_cast<int32_t *>(ws + l.cnt2);
    a.live = reinterpret_cast<int32_t *>(ws + l.live);
    a.shared_pages = reinterpret_cast<int32_t *>(ws + l.shared_pages);
    a.part_ml = reinterpret_cast<float *>(ws + l.ml);
    a.part_acc = reinterpret_cast<float *>(ws + l.acc);
    a.out = out; a.status = status;
    a.N = d->N; a.Hq = d->Hq; a.Hkv = d->Hkv; a.MAXB = d->MAXB; a.NP = d->NP;
    a.Wh = l.Wh; a.max_records = l.max_records;
    // query tiles per prefix wave: 2 once there are enough query rows to fill the chip that way
    a.prefix_qt = !prefix_enabled() ? 0 : ((long long)d->N * (d->Hq / d->Hkv) >= 256) ? 2 : 1;
    // never 0, so a cleared workspace never passes for a plan
    a.stamp = (int)((0x5157u ^ ((u32)d->N * 2654435761u) ^ ((u32)d->MAXB * 40503u) ^ ((u32)d->NP * 2246822519u) ^
                     ((u32)d->Hkv << 24) ^ ((u32)l.Wh << 12) ^ ((u32)a.prefix_qt << 8)) | 1u);
    a.scale_log2 = d->scale * 1.4426950408889634f;

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const int key = d->D * 16 + d->Hq / d->Hkv;
    switch (key) {
        case 64 * 16 + 1: return launch<64, 1>(a, s, what);
        case 64 * 16 + 2: return launch<64, 2>(a, s, what);
        case 64 * 16 + 4: return launch<64, 4>(a, s, what);
        case 64 * 16 + 8: return launch<64, 8>(a, s, what);
        case 128 * 16 + 1: return launch<128, 1>(a, s, what);
        case 128 * 16 + 2: return launch<128, 2>(a, s, what);
        case 128 * 16 + 4: return launch<128, 4>(a, s, what);
        case 128 * 16 + 8: return launch<128, 8>(a, s, what);
    }
    return STEP_EINVAL;
}

}  // namespace
}  // namespace step

using namespace step;

extern "C" int32_t step_attn_waves_per_head(const step_attn_dims *d)
{
    return dims_ok(d) ? waves_per_head(d) : 0;
}

extern "C" size_t step_attn_workspace_bytes(const step_attn_dims *d)
{
    if (!dims_ok(d)) return 0;
    return layout_for(d).total;
}

extern "C" int paged_decode_attn(const step_attn_dims *d, const uint16_t *q, const uint16_t *k_pages,
                                 const uint16_t *v_pages, const int32_t *block_tables, const int32_t *seq_lens,
                                 uint16_t *out, void *workspace, size_t workspace_bytes, int32_t *status,
                                 void *stream)
{
    return run(d, q, k_pages, v_pages, block_tables, seq_lens, out, workspace, workspace_bytes, status, stream,
               kDoPlan | kDoAttend);
}

extern "C" int step_attn_plan(const step_attn_dims *d, const int32_t *block_tables, const int32_t *seq_lens,
                              void *workspace, size_t workspace_bytes, int32_t *status, void *stream)
{
    return run(d, nullptr, nullptr, nullptr, block_tables, seq_lens, nullptr, workspace, workspace_bytes, status,
               stream, kDoPlan);
}

extern "C" int paged_decode_attn_planned(const step_attn_dims *d, const uint16_t *q, const uint16_t *k_pages,
                                         const uint16_t *v_pages, const int32_t *block_tables,
                                         const int32_t *seq_lens, uint16_t *out, void *workspace,
                                         size_t workspace_bytes, int32_t *status, void *stream)
{
    return run(d, q, k_pages, v_pages, block_tables, seq_lens, out, workspace, workspace_bytes, status, stream,
               kDoAttend);
}

extern "C" int step_attn_profile_begin(int cap)
{
    if (cap <= 0 || g_prof.ev) return STEP_EINVAL;
    g_prof.ev = new hipEvent_t[2 * (size_t)cap];
    for (int i = 0; i < 2 * cap; ++i)
        if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) return STEP_ELAUNCH;
    g_prof.cap = cap;
    g_prof.used = 0;
    return STEP_OK;
}

extern "C" int step_attn_profile_end(float *ms, int cap)
{
    if (!g_prof.ev || !ms || cap < g_prof.used) return -STEP_EINVAL;
    const int n = g_prof.used;
    for (int i = 0; i < n; ++i) {
        (void)hipEventSynchronize(g_prof.ev[2 * i + 1]);
        if (hipEventElapsedTime(&ms[i], g_prof.ev[2 * i], g_prof.ev[2 * i + 1]) != hipSuccess) ms[i] = -1.f;
    }
    for (int i = 0; i < 2 * g_prof.cap; ++i) (void)hipEventDestroy(g_prof.ev[i]);
    delete[] g_prof.ev;
    g_prof = Profile();
    return n;
}
