// Declarations shared by the attention translation units (attn*.hip): the plan that attn_plan writes
// into the workspace, the kernel argument block, and the host-side launchers of each stage.
#pragma once
#include <hip/hip_ext.h>

#include "common.h"

namespace step {
namespace attn {

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

// Wave-uniform reads of data that no kernel of the same launch writes (records, block-table entries):
// through the constant address space they become scalar loads, which have a counter of their own and
// so do not queue behind the vector loads of the tile stream.
__device__ __forceinline__ int32_t scalar_read(const int32_t *p)
{
    typedef const __attribute__((address_space(4))) int32_t *ConstPtr;
    return *reinterpret_cast<ConstPtr>(reinterpret_cast<uintptr_t>(p));
}
__device__ __forceinline__ Record scalar_read(const Record *p)
{
    typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(4))) i32x4 *ConstPtr;
    const i32x4 v = *reinterpret_cast<ConstPtr>(reinterpret_cast<uintptr_t>(p));
    return Record{v.x, v.y, v.z, v.w};
}

// Host-side launchers, one per translation unit.  D is the head dimension (64 or 128); e0 / e1, when
// not null, are recorded at the start and the end of the stage-1 kernel (benchmarks only).
void launch_plan(const AttnArgs &a, hipStream_t s);                                         // attn_plan.hip
void launch_prefix(const AttnArgs &a, int D, hipStream_t s);                                // attn_mfma.hip
void launch_stream_mfma(const AttnArgs &a, int D, hipStream_t s, hipEvent_t e0, hipEvent_t e1);  // attn_mfma.hip
void launch_stream_g4(const AttnArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1);      // attn_g4.hip (D = 128, G = 4)
int stream_g4_waves_per_cu();                                                               // attn_g4.hip
void launch_merge(const AttnArgs &a, int D, hipStream_t s);                                 // attn_merge.hip

}  // namespace attn
}  // namespace step
