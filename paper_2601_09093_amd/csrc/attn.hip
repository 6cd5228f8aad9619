// paged_decode_attn: split-K (flash-decoding) grouped-query decode attention over a paged bf16
// KV cache -- the attention inside NextToken(t) of Algorithm 1 (the paper gives no formula; this
// is softmax(q K^T scale) V for the newest token of every live trace).
//
// Three kernels per call (how the work is cut: attn_common.h):
//   attn_front   the pages shared by the live traces of a block of traces (the prompt) on the matrix cores:
//                for one KV head the query rows of the block form a dense matrix, so logits and output are
//                two MFMA products and every shared tile is read once per block instead of once per trace.
//                Each wave finds its block's shared-prefix length S_b by itself and stores it.
//   stage 1      the HBM-streaming kernels over the private pages: persistent single-wave workgroups,
//                one per resident wave slot.  Every wave works out, from seq_lens and the S_b, the equal
//                share of the concatenated private pages that is its own (no planning kernel, no record
//                array) and walks it with the loads of the next pages (and of the next record) in flight.
//                attn_partial_g4 (G == 4, D == 128): a (page, head) tile is P*D bf16 contiguous; the
//                wave reads it with 16-byte loads, lane l taking bytes [j*1024 + 16 l, +16) on load j.  A row of D
//                values lives in LPR = D/8 neighbouring lanes and each group of LPR lanes ("row group"
//                r) sees the tokens r, r+TPI, ... of every page: TPI = 64/LPR independent online-softmax
//                streams per wave, merged once per record; the 4 query heads share every K and V
//                register (bf16 dot2 on the vector ALUs).
//                attn_partial_mfma (every other shape): the two products on the matrix cores with the G
//                query heads of the trace in the columns, so the arithmetic per byte does not grow with G.
//   attn_merge   stage 2: per (trace, query head) combine the partials (m, l, acc) of its shared-prefix
//                sub-chunks and of its private-page records, round to bf16.
// Files: attn_common.h (argument struct, the cut, launcher declarations), attn_mfma.hip (attn_front,
// attn_partial_mfma), attn_g4.hip (attn_partial_g4), attn_merge.hip, and this file: argument checks, the
// workspace layout, the launch sequence and the C entry points.
#include "attn_common.h"

namespace step {
namespace attn {
namespace {

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
    if ((long long)d->N * d->MAXB >= (1ll << 30)) return false;  // page counts are summed in 32 bits
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
        const int nblk = stream_g4_waves_per_cu();
        return nblk < 4 ? nblk : 4;  // measured: one wave per SIMD streams fastest (no ALU contention between waves)
    }();
    const int per_cu = per_cu_env > 0 ? per_cu_env : per_cu_128;
    int wh = cus * per_cu / d->Hkv;
    if (wh < 1) wh = 1;
    if (wh > kMaxWh) wh = kMaxWh;
    return wh;
}

// Shared prefixes go to the matrix cores (attn_front) unless the environment variable
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
    size_t blk_shared, first2, cnt2, ml, acc, total;
    int Wh, TB, nblk, pmax, max_slots, prefix_qt;
};

size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

Layout layout_for(const step_attn_dims *d)
{
    Layout l;
    const int G = d->Hq / d->Hkv;
    l.Wh = waves_per_head(d);
    // query tiles per wave of attn_front: one, as long as that leaves a shared prefix at least four sub-chunks per
    // block (waves per KV head / blocks of 16 query rows); with more blocks than that, two tiles per wave halve
    // the number of blocks.  Measured on eight shapes (N * G from 256 to 2048, 2 and 8 KV heads): each is faster
    // on the side this rule puts it.
    const int nblk1 = (int)(((long long)d->N * G + 15) / 16);
    l.prefix_qt = !prefix_enabled() ? 0 : (nblk1 <= 0 || (l.Wh + nblk1 - 1) / nblk1 >= 4) ? 1 : 2;
    l.TB = 16 * (l.prefix_qt ? l.prefix_qt : 1) / G;
    l.nblk = (d->N + l.TB - 1) / l.TB;
    // sub-chunks of a shared prefix per trace: never more than prefix_split can ask for (about one wave per
    // SIMD over the blocks of a KV head), at most kMaxParts, and N * pmax <= 4096 partial slots
    l.pmax = 4096 / (d->N > 0 ? d->N : 1);
    if (l.pmax > kMaxParts) l.pmax = kMaxParts;
    if (l.nblk > 0 && l.pmax > (l.Wh + l.nblk - 1) / l.nblk) l.pmax = (l.Wh + l.nblk - 1) / l.nblk;
    if (l.pmax < 1) l.pmax = 1;
    l.max_slots = d->N * l.pmax + d->N + l.Wh;  // private pages: at most one record per trace and one more per wave
    const size_t R = (size_t)l.max_slots, N = d->N;
    l.blk_shared = 256;
    l.first2 = l.blk_shared + up256((size_t)(l.nblk > 0 ? l.nblk : 1) * sizeof(int32_t));
    l.cnt2 = l.first2 + up256(N * sizeof(int32_t));
    l.ml = l.cnt2 + up256(N * sizeof(int32_t));
    l.acc = l.ml + up256(R * d->Hkv * G * 2 * sizeof(float));
    l.total = l.acc + up256(R * d->Hkv * G * d->D * sizeof(float));
    return l;
}

enum : int { kDoPlan = 1, kDoAttend = 2 };

int launch(const AttnArgs &a, int D, hipStream_t s, int what)
{
    if (what == kDoPlan) launch_plan_blocks(a, s);
    if (what & kDoAttend) {
        // one call: every wave of attn_front finds its block's shared prefix itself; planned: they are in the workspace
        launch_front(a, D, (what & kDoPlan) != 0, s);
        // G == 4, D == 128: the dot2 kernel (about 1 % ahead of the matrix-core kernel at that shape; at
        // D == 64 the matrix-core kernel is the faster one, 6.2 against 5.5 TB/s);
        // STEP_ATTN_G4_MFMA=1, read once, sends that shape to the matrix-core kernel too (testing aid)
        static const bool g4_mfma = [] {
            const char *e = getenv("STEP_ATTN_G4_MFMA");
            return e && e[0] == '1';
        }();
        if (a.Hq / a.Hkv == 4 && D == 128 && !g4_mfma) launch_stream_g4(a, s);
        else launch_stream_mfma(a, D, s);
        launch_merge(a, D, s);
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
    a.blk_shared = reinterpret_cast<int32_t *>(ws + l.blk_shared);
    a.first2 = reinterpret_cast<int32_t *>(ws + l.first2);
    a.cnt2 = reinterpret_cast<int32_t *>(ws + l.cnt2);
    a.part_ml = reinterpret_cast<float *>(ws + l.ml);
    a.part_acc = reinterpret_cast<float *>(ws + l.acc);
    a.out = out; a.status = status;
    a.N = d->N; a.Hq = d->Hq; a.Hkv = d->Hkv; a.MAXB = d->MAXB; a.NP = d->NP;
    a.Wh = l.Wh; a.TB = l.TB; a.nblk = l.nblk; a.pmax = l.pmax; a.max_slots = l.max_slots;
    a.prefix_base = 0;
    a.priv_base = d->N * l.pmax;
    a.prefix_qt = l.prefix_qt;
    // never 0, so a cleared workspace never passes for a plan
    a.stamp = (int)((0x5157u ^ ((u32)d->N * 2654435761u) ^ ((u32)d->MAXB * 40503u) ^ ((u32)d->NP * 2246822519u) ^
                     ((u32)d->Hkv << 24) ^ ((u32)l.Wh << 12) ^ ((u32)a.prefix_qt << 8) ^ ((u32)d->Hq << 4)) | 1u);
    a.scale_log2 = d->scale * 1.4426950408889634f;

    return launch(a, d->D, reinterpret_cast<hipStream_t>(stream), what);
}

}  // namespace
}  // namespace attn
}  // namespace step

using namespace step;
using namespace step::attn;

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
