// The matrix-core kernels of paged_decode_attn: attn_front (the pages shared by the live traces of a block
// of traces, and the per-block shared-prefix lengths the rest of the call is cut by) and attn_partial_mfma
// (stage 1 over private pages for every shape but G = 4, D = 128).
#include "attn_common.h"

namespace step {
namespace attn {
namespace {

// ---------------------------------------------------------------------------------------------
// The matrix-core form of one page pair, shared by attn_front and attn_partial_mfma.
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
        mx = max_rows(mx);
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
        ls = sum_rows(ls);
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
// attn_front: shared prefixes on the matrix cores, one wave per (KV head g, block b of TB traces, sub-chunk p).
// The S_b leading pages of block b are the same physical pages for every live trace of the block, so for
// one KV head the TB * G query rows that attend to them form a dense 16 * QT-row matrix: the logits are
// K Q^T and the output V^T P^T, both v_mfma_f32_16x16x32_bf16, and every shared tile is read once per block
// instead of once per trace.  The wave finds S_b itself from the block's block-table rows (DETECT; every
// unit of a block computes the same value, unit (0, b, 0) stores it for the streaming kernel and the merge),
// or takes it from the workspace (a plan made earlier by step_attn_plan), works out the sub-chunks
// (prefix_split) and, if p is one of them, writes the partial (m, l, acc) of slot p * N + t for every live
// trace t of the block -- exactly what a streaming wave writes for a record, so the merge treats both alike.
// (operand layouts: MfmaPair above)
// ---------------------------------------------------------------------------------------------
template <int D, int QT, bool DETECT>
__global__ __launch_bounds__(64) void attn_front(const AttnArgs a)
{
    typedef MfmaPair<D> MP;
    constexpr int KB = MP::KB, DB = MP::DB;
    typedef typename MP::VRow VRow;
    const int lane = threadIdx.x, c = lane & 15, gr = lane >> 4;
    const int G = a.Hq / a.Hkv;
    int u = blockIdx.x;
    const int g = u % a.Hkv;
    u /= a.Hkv;
    const int b = u % a.nblk, p = u / a.nblk;
    const int t0 = b * a.TB;

    // query rows of this block: row = (trace - t0) * G + head-in-group.  Requested first (they depend on nothing
    // the wave still has to find out; rows of dead traces are zeroed below)
    uint4 qf[QT][KB];
    int trace_of[QT], hh_of[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int row = qt * 16 + c;
        trace_of[qt] = min(t0 + row / G, a.N - 1);
        hh_of[qt] = row % G;
        const uint16_t *qrow = a.q + ((size_t)trace_of[qt] * a.Hq + g * G + hh_of[qt]) * D;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) qf[qt][kb] = *reinterpret_cast<const uint4 *>(qrow + kb * 32 + gr * 8);
    }

    const BlockPrefix bp = block_prefix(a, b, lane, DETECT);
    const unsigned live = bp.live;
    int S = bp.S;
    if constexpr (DETECT) {
        if (p == 0 && g == 0 && lane == 0) {
            a.blk_shared[b] = S;
            if (b == 0) a.hdr->stamp = a.stamp;
        }
    } else {
        // lengths made for other dims (or none at all) are reported; the clamp keeps every access inside
        // the block tables whatever the workspace holds
        if (a.hdr->stamp != a.stamp && lane == 0) report(a.status, STEP_EPLAN);
        int minfull = 0x7fffffff;
        for (unsigned m = live; m; m &= m - 1) minfull = min(minfull, scalar_read(a.seq_lens + t0 + __ffs(m) - 1) / kPageTokens);
        S = __popc(live) >= 2 ? min(max(scalar_read(a.blk_shared + b), 0), min(min(kMaxShared, minfull), a.MAXB)) : 0;
    }
    int parts, sc;
    prefix_split(a, S, parts, sc);
    if (p >= parts) return;
    const int first = p * sc, n = min(sc, S - first);
    if (n < 1) return;
    if (a.NP <= 0) {
        if (lane == 0) report(a.status, STEP_EPAGE);
        return;
    }

    bool bad_page = false;
    const int32_t *bt = a.block_tables + (size_t)(t0 + __ffs(live) - 1) * a.MAXB;  // first + n <= S <= MAXB
    auto page_at = [&](int j) {
        const int col = first + min(j, n - 1);  // the same for every lane
        int pg;
        if (bp.have_ids && col < 128)  // the search has already fetched the row's first 128 entries
            pg = col < 64 ? __builtin_amdgcn_readlane(bp.ids_a, col) : __builtin_amdgcn_readlane(bp.ids_b, col - 64);
        else
            pg = scalar_read(bt + col);
        const bool ok = (u32)pg < (u32)a.NP;
        bad_page |= !ok;
        return ok ? pg : 0;
    };

    bool valid[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int r = (qt * 16 + c) / G;
        valid[qt] = r < a.TB && ((live >> r) & 1u);
        if (!valid[qt]) {
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) qf[qt][kb] = make_uint4(0, 0, 0, 0);
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
    // the units that share this sub-chunk (same KV head, other blocks with the same prompt) walk its pairs
    // in rotated orders, so that they do not all ask the L2 for the same lines at the same moment
    const int np = (n + 1) / 2;
    const int rot = b % np;
    auto pair_at = [&](int t) { return 2 * ((t + rot) % np); };  // first page of the t-th pair visited
#pragma unroll
    for (int bf = 0; bf < NBUF; ++bf)
        if (bf < np) load_pair(pair_at(bf), kf[bf], vr[bf]);
    for (int i0 = 0; i0 < np; i0 += NBUF) {
#pragma unroll
        for (int bf = 0; bf < NBUF; ++bf) {
            const int t = i0 + bf;
            if (t < np) {
                attend_pair(kf[bf], vr[bf], pair_at(t) + 1 < n);
                if (t + NBUF < np) load_pair(pair_at(t + NBUF), kf[bf], vr[bf]);
            }
        }
    }

    // partials of the slots p * N + trace
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
        MP::store_partial(a, ((size_t)a.prefix_base + (size_t)p * a.N + trace_of[qt]) * a.Hkv + g, G, hh_of[qt], gr, valid[qt], m[qt], l[qt], o[qt]);
    if (bad_page && lane == 0) report(a.status, STEP_EPAGE);
}

// step_attn_plan: the per-block shared-prefix lengths alone (one wave per block), for a decode step whose
// layers all see the same block tables; also reports lengths outside the block-table row.
__global__ __launch_bounds__(64) void attn_plan_blocks(const AttnArgs a)
{
    const int lane = threadIdx.x, b = blockIdx.x;
    const int t0 = b * a.TB, nt = min(a.TB, a.N - t0);
    const BlockPrefix bp = block_prefix(a, b, lane, a.prefix_qt != 0);
    const int L = lane < nt ? a.seq_lens[t0 + lane] : 0;
    if (__any(L != 0 && pages_of(L, a.MAXB) == 0) && lane == 0) report(a.status, STEP_ELEN);
    const int S = bp.S;
    if (lane == 0) {
        a.blk_shared[b] = S;
        if (b == 0) a.hdr->stamp = a.stamp;
    }
}

// ---------------------------------------------------------------------------------------------
// stage 1 on the matrix cores, any group size: the persistent streaming kernel for G != 4.
// The same two products as attn_front with the G query heads of ONE trace in the columns (the other
// 16 - G columns are zero and never stored), over the private pages of the wave's records, pair of
// pages by pair of pages.  The operand loads (K: 16 rows x 64 bytes per instruction, V: 4 rows x
// 256 bytes) stream a fragmented pool as fast as the 1 KB-per-instruction loads of the G == 4 kernel,
// and the arithmetic per byte no longer grows with G.  Page ids, records and tiles are requested ahead of
// their use across record boundaries: the wave's page pairs form one sequence, a load cursor runs kBufs
// pairs ahead of the compute cursor.
// ---------------------------------------------------------------------------------------------
template <int D>  // (one wave per SIMD, enforced: see attn_partial_g4)
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_partial_mfma(const AttnArgs a)
{
    typedef MfmaPair<D> MP;
    constexpr int KB = MP::KB, DB = MP::DB;
    constexpr int kBufs = 2;
    typedef typename MP::VRow VRow;
    typedef u32 u32x4 __attribute__((ext_vector_type(4)));
    __shared__ int P_s[kMaxPlanN + 1], base_s[kMaxPlanN + 1];
    const int lane = threadIdx.x, c = lane & 15, gr = lane >> 4;
    const int g = blockIdx.x % a.Hkv;
    const int wh = blockIdx.x / a.Hkv;
    const int G = a.Hq / a.Hkv;
    const WavePlan wp = plan_build(a, lane, P_s, base_s, blockIdx.x == 0);
    if (blockIdx.x == 0) publish_plan(a, wp, lane, P_s, base_s);
    RunWalker walk(a, wp, P_s, base_s, wh);
    if (!walk.more()) return;
    if (a.NP <= 0) {
        if (lane == 0) report(a.status, STEP_EPAGE);
        return;
    }

    bool bad_page = false;
    // a position in the wave's sequence of page pairs: pages j and j + 1 of record rec
    struct Cursor {
        bool valid;
        Record rec;
        int j;
    };
    auto next_record = [&]() {
        Cursor x;
        x.valid = walk.more();
        x.j = 0;
        x.rec = x.valid ? walk.take() : Record{0, 0, 1, 1, 0};
        return x;
    };
    Cursor cur = next_record();   // load cursor
    Cursor after = next_record(); // the record after the load cursor's, worked out one record early
    auto advance = [&]() {
        cur.j += 2;
        if (cur.j >= cur.rec.n) {
            cur = after;
            if (cur.valid) after = next_record();
        }
    };
    auto page_ids = [&](const Cursor &x, int &p0, int &p1) {  // second page of an odd record's last pair: the last page again
        const int32_t *row = a.block_tables + (size_t)x.rec.i * a.MAXB + x.rec.first;
        p0 = scalar_read(row + x.j);
        p1 = scalar_read(row + min(x.j + 1, x.rec.n - 1));
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

    int id0, id1;  // page ids of the load cursor's pair
    page_ids(cur, id0, id1);
    auto fill = [&](uint4 (&kfb)[2][KB], VRow (&vrb)[8], uint4 (&qb)[KB], Cursor &slot) {
        slot = cur;
        if (!cur.valid) return;
        load_pair(id0, id1, kfb, vrb);
        if (cur.j == 0) load_q(cur.rec.i, qb);
        advance();
        if (cur.valid) page_ids(cur, id0, id1);  // scalar loads, used one refill later
    };
#pragma unroll
    for (int bf = 0; bf < kBufs; ++bf) fill(kf[bf], vr[bf], qslot[bf], at[bf]);

    bool done = false;
    while (!done) {
#pragma unroll
        for (int bf = 0; bf < kBufs; ++bf) {
            if (done) continue;
            const Cursor x = at[bf];
            if (!x.valid) {
                done = true;
                continue;
            }
            if (x.j == 0) {  // a new record starts
                m = kMinusBig;
                l = 0.f;
#pragma unroll
                for (int jt = 0; jt < DB; ++jt) o[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) qf[kb] = qslot[bf][kb];
            }
            const int n = x.rec.n;
            auto tokens_of = [&](int jj) { return jj < n - 1 ? kPageTokens : (jj == n - 1 ? x.rec.ntok : 0); };
            attend_pair(kf[bf], vr[bf], tokens_of(x.j), tokens_of(x.j + 1));
            const bool last = x.j + 2 >= n;
            fill(kf[bf], vr[bf], qslot[bf], at[bf]);  // the buffer is free: request the pair kBufs ahead
            if (last) MP::store_partial(a, (size_t)x.rec.slot * a.Hkv + g, G, min(c, G - 1), gr, c < G, m, l, o);
        }
    }
    if (bad_page && lane == 0) report(a.status, STEP_EPAGE);
}

}  // namespace

void launch_front(const AttnArgs &a, int D, bool detect, hipStream_t s)
{
    if (!a.prefix_qt) return;
    const dim3 grid((u32)(a.Hkv * a.nblk * a.pmax));  // units beyond a block's sub-chunks exit once they know S_b
    void (*kernel)(AttnArgs);
    if (D == 128) {
        if (a.prefix_qt == 2) kernel = detect ? attn_front<128, 2, true> : attn_front<128, 2, false>;
        else kernel = detect ? attn_front<128, 1, true> : attn_front<128, 1, false>;
    } else {
        if (a.prefix_qt == 2) kernel = detect ? attn_front<64, 2, true> : attn_front<64, 2, false>;
        else kernel = detect ? attn_front<64, 1, true> : attn_front<64, 1, false>;
    }
    launch_kernel(kKernFront, kernel, grid, dim3(64), s, a);
}

void launch_plan_blocks(const AttnArgs &a, hipStream_t s)
{
    launch_kernel(kKernPlanBlocks, attn_plan_blocks, dim3((u32)a.nblk), dim3(64), s, a);
}

void launch_stream_mfma(const AttnArgs &a, int D, hipStream_t s)
{
    const dim3 grid((u32)(a.Wh * a.Hkv));
    if (D == 128) launch_kernel(kKernStage1, attn_partial_mfma<128>, grid, dim3(64), s, a);
    else launch_kernel(kKernStage1, attn_partial_mfma<64>, grid, dim3(64), s, a);
}

}  // namespace attn
}  // namespace step
