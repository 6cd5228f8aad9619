// step_score: the step scorer y = sigma(W2 act(W1 h + b1) + b2) of Section 4.1 ("Model
// Architecture"; Table 5 fixes act = ReLU, hidden width 512) on the hidden states of the traces at a
// step boundary, followed by the running-average trace score of Section 4.3 ("Update score_t" in
// Algorithm 1).
//
// One kernel, score_hidden, grid (m / 16 row tiles, chunks of the contraction over d, tiles of 32 boundaries):
//   1. a workgroup of four waves owns 16 rows of W1 (one MFMA tile of hidden units), one chunk of d and up to
//      32 boundaries; its waves split the chunk, 128 values per iteration (v_mfma_f32_16x16x32_bf16), the gather
//      hidden[boundary_idx[b]] fused into the B-operand loads, and are summed through LDS.  With one chunk
//      the workgroup goes straight to step 3 with its sums in LDS; otherwise it stores them.
//   2. the last workgroup of a row tile to arrive (a ticket per tile) adds the chunks in chunk order,
//   3. applies bias and activation, multiplies by the 16 matching entries of W2 and stores one partial logit
//      per boundary.
//   4. the last workgroup of the launch to arrive adds the partial logits in tile order, applies the sigmoid,
//      then updates (sum, count) per trace with the trace's boundaries in index order -- fp32 addition is not
//      associative and a trace may own several boundaries, so the order is part of the result; different traces
//      do not meet and are replayed by different threads -- and the scores are refreshed.
// The split over d puts at least 256 workgroups on the W1 stream whatever m is (the paper's m = 512 gives only
// 32 row tiles); every sum is taken in a fixed order, so the result does not depend on which workgroup arrives last.
// The tickets are library-owned device words that start at zero and are put back to zero by the workgroup that
// finds itself last.  Calls that may be in flight together already have to use different workspaces (the chunk
// sums live there), so a ticket set is kept per workspace address: such calls never meet, whether they are
// issued directly or replayed from a recorded graph, unless more than kTicketSets workspaces are in use.
#include <mutex>

#include "common.h"

namespace step {
namespace {

constexpr int kWaves = 4;          // the chunk of d is split over the waves of a workgroup
constexpr int kBT = 2;             // boundary tiles (of 16) per workgroup
constexpr int kMaxRowTiles = 1024; // m <= 16384
constexpr int kTicketSets = 64;
constexpr int kTicketsPerSet = 2 * kMaxRowTiles + 1;  // a row-tile ticket per (tile of 32 boundaries <= 2, row tile), one for the launch

__device__ int32_t score_tickets[kTicketSets][kTicketsPerSet];

struct ScoreArgs {
    const uint16_t *hidden, *W1, *W2;
    const int32_t *boundary_idx, *trace_of;
    const float *b1, *b2;
    float *logits, *probs, *score_sum, *scores;
    float *partial;  // [chunks][row tiles][B][16] sums of one chunk of d (only with more than one chunk)
    float *plogit;   // [row tiles][B] partial logits
    int32_t *score_cnt, *status;
    int R, d, m, B, N, act;
    int nchunk, chunk_iters;  // chunks of d, iterations (128 values) per chunk
    int set;                  // ticket set of this call
};

__device__ __forceinline__ float activate(float z, int act)
{
    if (act == STEP_ACT_RELU) return fmaxf(z, 0.f);
    return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
}

constexpr int kFinishChunk = 1024;  // boundaries whose (trace, prob) are staged in LDS at a time
constexpr int kStateMax = 2048;     // traces whose (sum, count) state is staged in LDS
constexpr int kThreads = 64 * kWaves;

// Words that workgroups of one launch hand to each other are stored and loaded at device scope (the
// compute dies have caches of their own, which these accesses go past), so no cache has to be written back
// or invalidated as a whole, which is what a device-wide fence would do.
__device__ __forceinline__ void st_dev(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_dev(const float *p)
{
    return __hip_atomic_load(const_cast<float *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// two neighbouring floats (8-byte aligned) as one access
typedef unsigned long long u64;
__device__ __forceinline__ void st_dev2(float *p, float x, float y)
{
    const u64 v = (u64)__float_as_uint(x) | ((u64)__float_as_uint(y) << 32);
    __hip_atomic_store(reinterpret_cast<u64 *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ld_dev2(const float *p, float &x, float &y)
{
    const u64 v = __hip_atomic_load(reinterpret_cast<u64 *>(const_cast<float *>(p)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    x = __uint_as_float((u32)v);
    y = __uint_as_float((u32)(v >> 32));
}

// true in every thread of the workgroup that is the last of `expected` to take the ticket; that workgroup
// puts the ticket back to zero.  Every thread first waits until its own device-scope stores have been
// acknowledged, then the workgroup meets, then one thread takes the ticket: whoever is last therefore finds
// the words of all earlier arrivals when it loads them at device scope.
__device__ __forceinline__ bool last_to_arrive(int32_t *ticket, int expected, int *flag_s)
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const int old = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = old == expected - 1;
        if (last) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag_s = last ? 1 : 0;
    }
    __syncthreads();
    return *flag_s != 0;
}

// Logits and probabilities of the boundaries base + bb0 .. + KB4 (one wave): lane l adds the row tiles l, l + 64, ...
// in ascending order, then the lanes are added by wave_sum -- the same order whatever KB4 is.
template <int KB4>
__device__ __forceinline__ void partial_logits(const ScoreArgs &a, int base, int nbd, int bb0, int lane, int mt, float b2,
                                               float *prob_s)
{
    float acc[KB4];
#pragma unroll
    for (int u = 0; u < KB4; ++u) acc[u] = 0.f;
    for (int t0 = 0; t0 < mt; t0 += 64 * 4) {
        float v[4][KB4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int u = 0; u < KB4; ++u) {
                const int t = t0 + r * 64 + lane, bb = bb0 + u;
                v[r][u] = (t < mt && bb < nbd) ? ld_dev(&a.plogit[(size_t)t * a.B + base + bb]) : 0.f;
            }
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int u = 0; u < KB4; ++u) acc[u] += v[r][u];
    }
#pragma unroll
    for (int u = 0; u < KB4; ++u) {
        const float x = wave_sum(acc[u]);
        const int bb = bb0 + u;
        if (lane == 0 && bb < nbd) {
            const float logit = b2 + x;
            const float prob = 1.0f / (1.0f + expf(-logit));
            a.logits[base + bb] = logit;
            a.probs[base + bb] = prob;
            prob_s[bb] = prob;
        }
    }
}

// step 4 (also the whole kernel when B == 0): logits, probabilities, running mean, scores
// What the finishing workgroup needs and nothing in the launch changes before it: the running-mean state (when it
// is staged on chip), the traces of the first kFinishChunk boundaries and the output bias.  Every workgroup requests them when it
// starts -- it may turn out to be the last -- so these cold loads are not on the path behind the last ticket.
constexpr int kPer = kStateMax / kThreads;
constexpr int kTrPer = kFinishChunk / kThreads;
struct FinishInputs {
    float b2;
    float rs[kPer];
    int rc[kPer];
    int tr[kTrPer];
};

__device__ __forceinline__ void request_finish_inputs(const ScoreArgs &a, FinishInputs &f)
{
    const int tid = threadIdx.x;
    const bool state = a.score_sum != nullptr;
    const bool staged = state && a.N <= kStateMax;
    f.b2 = a.b2[0];
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
        const int t = tid + u * kThreads;
        f.rs[u] = (staged && t < a.N) ? a.score_sum[t] : 0.f;
        f.rc[u] = (staged && t < a.N) ? a.score_cnt[t] : 0;
    }
#pragma unroll
    for (int u = 0; u < kTrPer; ++u) {
        const int bb = tid + u * kThreads;
        f.tr[u] = (state && bb < a.B) ? a.trace_of[bb] : -1;
    }
}

__device__ void score_finish(const ScoreArgs &a, const FinishInputs &f, float *prob_s, int *trace_s, float *sum_s, int *cnt_s)
{
    const int tid = threadIdx.x;
    const int mt = a.m / 16;
    const float b2 = f.b2;
    const bool state = a.score_sum != nullptr;
    const bool staged = state && a.N <= kStateMax;  // keep the replay off global memory
    bool parked = false;
    auto park_state = [&]() {
        if (staged && !parked) {
#pragma unroll
            for (int u = 0; u < kPer; ++u) {
                const int t = tid + u * kThreads;
                if (t < a.N) {
                    sum_s[t] = f.rs[u];
                    cnt_s[t] = f.rc[u];
                }
            }
        }
        parked = true;
    };
    const int lane = tid & 63, wv = tid >> 6;
    for (int base = 0; base < a.B; base += kFinishChunk) {
        const int nbd = min(kFinishChunk, a.B - base);
        // logit of a boundary = b2 + sum over the row tiles of its partial logits, in a fixed order (partial_logits);
        // a wave takes four boundaries at a time, eight when there are more than 16, so that their loads are in
        // flight together and the boundaries of a call take one round
        if (nbd > 16) {
            for (int bb0 = wv * 8; bb0 < nbd; bb0 += kWaves * 8) partial_logits<8>(a, base, nbd, bb0, lane, mt, b2, prob_s);
        } else {
            for (int bb0 = wv * 4; bb0 < nbd; bb0 += kWaves * 4) partial_logits<4>(a, base, nbd, bb0, lane, mt, b2, prob_s);
        }
        // the boundaries' traces, padded with -1 to a multiple of four (they are read four at a time below)
#pragma unroll
        for (int u = 0; u < kTrPer; ++u) {
            const int bb = tid + u * kThreads;
            if (bb < ((nbd + 3) & ~3)) {
                int t = -1;
                if (state && bb < nbd) {
                    t = base == 0 ? f.tr[u] : a.trace_of[base + bb];
                    if ((u32)t >= (u32)a.N) {
                        report(a.status, STEP_EINDEX);
                        t = -1;
                    }
                }
                trace_s[bb] = t;
            }
        }
        if (!state) continue;  // uniform
        park_state();
        __syncthreads();
        // A trace's sum takes its boundaries in index order: fp32 addition is not associative and a trace may own
        // several.  Different traces do not meet, so with the state on chip every thread replays, for its own
        // traces, the whole list (LDS broadcasts); otherwise one thread walks the list once.
        if (staged) {
            const int4 *tr4 = reinterpret_cast<const int4 *>(trace_s);
            for (int t = tid; t < a.N; t += kThreads) {
                float sm = sum_s[t];
                int n = cnt_s[t];
                for (int q4 = 0; q4 < (nbd + 3) / 4; ++q4) {
                    const int4 tt = tr4[q4];
                    if (tt.x == t) { sm = sm + prob_s[4 * q4 + 0]; ++n; }
                    if (tt.y == t) { sm = sm + prob_s[4 * q4 + 1]; ++n; }
                    if (tt.z == t) { sm = sm + prob_s[4 * q4 + 2]; ++n; }
                    if (tt.w == t) { sm = sm + prob_s[4 * q4 + 3]; ++n; }
                }
                sum_s[t] = sm;
                cnt_s[t] = n;
            }
        } else if (tid == 0) {
            for (int bb = 0; bb < nbd; ++bb) {
                const int t = trace_s[bb];
                if (t < 0) continue;
                a.score_sum[t] = a.score_sum[t] + prob_s[bb];
                a.score_cnt[t] = a.score_cnt[t] + 1;
            }
        }
        __syncthreads();
    }
    if (!state) return;
    park_state();  // (no boundaries: nothing above has done it)
    __threadfence_block();
    __syncthreads();
    for (int t = tid; t < a.N; t += kThreads) {
        float sm;
        int n;
        if (staged) {
            sm = sum_s[t];
            n = cnt_s[t];
            a.score_sum[t] = sm;
            a.score_cnt[t] = n;
        } else {
            sm = a.score_sum[t];
            n = a.score_cnt[t];
        }
        if (a.scores) a.scores[t] = n > 0 ? sm / (float)n : INFINITY;
    }
}

__global__ __launch_bounds__(kThreads) void score_hidden(const ScoreArgs a)
{
    __shared__ float red[kWaves][kBT][4][64];
    __shared__ float prob_s[kFinishChunk];
    __shared__ __attribute__((aligned(16))) int trace_s[kFinishChunk];  // read four at a time
    __shared__ float sum_s[kStateMax];
    __shared__ int cnt_s[kStateMax];
    __shared__ int flag_s;
    FinishInputs fin;
    request_finish_inputs(a, fin);
    if (a.B == 0) {  // nothing to score: the scores are refreshed from the state
        score_finish(a, fin, prob_s, trace_s, sum_s, cnt_s);
        return;
    }
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int row16 = lane & 15, kg = lane >> 4;
    const int mt = blockIdx.x, MT = gridDim.x, chunk = blockIdx.y, bz = blockIdx.z;
    const int m0 = mt * 16;
    const int b0 = bz * (16 * kBT);

    // Requested before anything they do not depend on: this wave's first 64 bytes of W1 per lane, and the bias and
    // output weights of the workgroup's 16 hidden units (used only after the sums are complete).
    const uint16_t *wrow = a.W1 + (size_t)(m0 + row16) * a.d;
    const int it0 = chunk * a.chunk_iters, it1 = min(it0 + a.chunk_iters, a.d / 128);
    uint4 av[4];
    if (it0 + w < it1) {
        const uint4 *wp = reinterpret_cast<const uint4 *>(wrow + (it0 + w) * 128 + kg * 32);
#pragma unroll
        for (int s = 0; s < 4; ++s) av[s] = wp[s];
    }
    float b1v[4], w2v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        b1v[i] = a.b1[m0 + kg * 4 + i];
        w2v[i] = bf16_lo((u32)a.W2[m0 + kg * 4 + i]);
    }

    // rows of `hidden` feeding the B operand of each boundary tile (column = lane % 16)
    const uint16_t *xrow[kBT];
#pragma unroll
    for (int t = 0; t < kBT; ++t) {
        const int b = b0 + t * 16 + row16;
        int rix = 0;
        if (b < a.B) {
            rix = a.boundary_idx[b];
            if ((u32)rix >= (u32)a.R) {
                if (mt == 0 && chunk == 0 && kg == 0 && w == 0) report(a.status, STEP_EINDEX);
                rix = 0;
            }
        }
        xrow[t] = a.hidden + (size_t)rix * a.d;
    }
    const bool tile1 = (b0 + 16 < a.B);  // wave-uniform: second boundary tile in use

    f32x4 c0 = {0.f, 0.f, 0.f, 0.f}, c1 = {0.f, 0.f, 0.f, 0.f};
    for (int it = it0 + w; it < it1; it += kWaves) {
        // the contraction index is permuted identically for both operands: lane group kg takes the
        // 32 consecutive values kbase + 32 kg .. +32, eight per MFMA, so a lane reads 64 contiguous
        // bytes per iteration and the four groups cover 256 contiguous bytes of the row
        const int kbase = it * 128 + kg * 32;
        const uint4 *x0 = reinterpret_cast<const uint4 *>(xrow[0] + kbase);
        const uint4 *x1 = reinterpret_cast<const uint4 *>(xrow[1] + kbase);
        uint4 bv0[4], bv1[4];
        if (it != it0 + w) {  // (the first iteration's W1 is already on its way)
            const uint4 *wp = reinterpret_cast<const uint4 *>(wrow + kbase);
#pragma unroll
            for (int s = 0; s < 4; ++s) av[s] = wp[s];
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) bv0[s] = x0[s];
        if (tile1) {
#pragma unroll
            for (int s = 0; s < 4; ++s) bv1[s] = x1[s];
        }
#pragma unroll
        for (int s = 0; s < 4; ++s)
            c0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av[s]),
                                                         __builtin_bit_cast(bf16x8, bv0[s]), c0, 0, 0, 0);
        if (tile1) {
#pragma unroll
            for (int s = 0; s < 4; ++s)
                c1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, av[s]),
                                                             __builtin_bit_cast(bf16x8, bv1[s]), c1, 0, 0, 0);
        }
    }
    // accumulator layout: lane holds column (boundary) lane % 16, rows (hidden units) 4*(lane/16)+i
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        red[w][0][i][lane] = c0[i];
        red[w][1][i][lane] = c1[i];
    }
    __syncthreads();
    // this workgroup's sums of its chunk: wave t < kBT takes boundary tile t; z[i] belongs to hidden unit
    // m0 + 4 kg + i and boundary b
    const int b = b0 + w * 16 + row16;
    float z[4] = {0.f, 0.f, 0.f, 0.f};
    if (w < kBT) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int ww = 0; ww < kWaves; ++ww) z[i] += red[ww][w][i][lane];
    }
    int32_t *tickets = score_tickets[a.set];
    if (a.nchunk > 1) {
        // step 1 -> 2: store the chunk's sums; the tile's last chunk to arrive adds all of them in chunk order
        if (w < kBT && b < a.B) {
            float *dst = a.partial + (((size_t)chunk * MT + mt) * a.B + b) * 16 + kg * 4;
            st_dev2(dst, z[0], z[1]);
            st_dev2(dst + 2, z[2], z[3]);
        }
        if (!last_to_arrive(&tickets[bz * MT + mt], a.nchunk, &flag_s)) return;
        if (w < kBT && b < a.B) {
#pragma unroll
            for (int i = 0; i < 4; ++i) z[i] = 0.f;
            for (int ch0 = 0; ch0 < a.nchunk; ch0 += 8) {  // eight chunks requested together, added in chunk order
                float v[8][4];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int ch = min(ch0 + u, a.nchunk - 1);
                    const float *src = a.partial + (((size_t)ch * MT + mt) * a.B + b) * 16 + kg * 4;
                    ld_dev2(src, v[u][0], v[u][1]);
                    ld_dev2(src + 2, v[u][2], v[u][3]);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (ch0 + u < a.nchunk) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) z[i] += v[u][i];
                    }
            }
        }
    }
    // step 3
    if (w < kBT) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) s = fmaf(w2v[i], activate(z[i] + b1v[i], a.act), s);
        s = sum_rows(s);
        if (kg == 0 && b < a.B) st_dev(&a.plogit[(size_t)mt * a.B + b], s);
    }
    // step 4
    if (!last_to_arrive(&tickets[kTicketsPerSet - 1], (int)(MT * gridDim.z), &flag_s)) return;
    score_finish(a, fin, prob_s, trace_s, sum_s, cnt_s);
}

// ticket set of a workspace; with more than kTicketSets workspaces the one unused for longest gives up its set
std::mutex g_set_mutex;
struct SetSlot {
    const void *workspace;
    unsigned long long last_use;
};
SetSlot g_set_slots[kTicketSets];
unsigned long long g_set_clock = 0;

int ticket_set_of(const void *workspace)
{
    std::lock_guard<std::mutex> lock(g_set_mutex);
    int oldest = 0;
    for (int i = 0; i < kTicketSets; ++i) {
        if (g_set_slots[i].workspace == workspace) {
            g_set_slots[i].last_use = ++g_set_clock;
            return i;
        }
        if (g_set_slots[i].last_use < g_set_slots[oldest].last_use) oldest = i;
    }
    g_set_slots[oldest].workspace = workspace;
    g_set_slots[oldest].last_use = ++g_set_clock;
    return oldest;
}

// chunks of the contraction over d: enough workgroups to stream W1 from the whole chip when there are few
// row tiles and few boundaries
void chunking(const step_score_dims *d, int &nchunk, int &chunk_iters)
{
    const int iters = d->d / 128, MT = d->m / 16;
    const int nbz = d->B > 0 ? (d->B + 16 * kBT - 1) / (16 * kBT) : 1;
    int want = 1;
    if (nbz <= 2 && MT * nbz < 256) want = (256 + MT * nbz - 1) / (MT * nbz);
    if (want > iters) want = iters;
    chunk_iters = (iters + want - 1) / want;
    nchunk = (iters + chunk_iters - 1) / chunk_iters;
}

bool dims_ok(const step_score_dims *d)
{
    if (!d) return false;
    if (d->R < 0 || d->d <= 0 || d->m <= 0 || d->B < 0 || d->N < 0) return false;
    if (d->d % 128 || d->m % 16 || d->m / 16 > kMaxRowTiles) return false;
    if (d->act != STEP_ACT_RELU && d->act != STEP_ACT_GELU) return false;
    if (d->B > 0 && d->R == 0) return false;
    if (d->B > (1 << 20)) return false;
    return true;
}

}  // namespace
}  // namespace step

using namespace step;

extern "C" size_t step_score_workspace_bytes(const step_score_dims *d)
{
    if (!dims_ok(d)) return 0;
    int nchunk, chunk_iters;
    chunking(d, nchunk, chunk_iters);
    const size_t B = d->B > 0 ? d->B : 1, MT = d->m / 16;
    const size_t plogit = (MT * B * sizeof(float) + 255) & ~(size_t)255;
    const size_t partial = nchunk > 1 ? (((size_t)nchunk * MT * B * 16 * sizeof(float)) + 255) & ~(size_t)255 : 0;
    return plogit + partial;
}

extern "C" int step_score(const step_score_dims *d, const uint16_t *hidden, const int32_t *boundary_idx,
                          const uint16_t *W1, const float *b1, const uint16_t *W2, const float *b2,
                          float *logits, float *probs, const int32_t *trace_of, float *score_sum,
                          int32_t *score_cnt, float *scores, void *workspace, size_t workspace_bytes,
                          int32_t *status, void *stream)
{
    if (!dims_ok(d)) return STEP_EINVAL;
    if (!W1 || !b1 || !W2 || !b2) return STEP_EINVAL;
    if (d->B > 0 && (!hidden || !boundary_idx || !logits || !probs)) return STEP_EINVAL;
    if (!aligned(hidden, 16) || !aligned(W1, 16)) return STEP_EINVAL;
    const bool state = score_sum != nullptr;
    if (state && (!score_cnt || d->N <= 0 || (d->B > 0 && !trace_of))) return STEP_EINVAL;
    if (!state && (score_cnt || scores)) return STEP_EINVAL;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < step_score_workspace_bytes(d))
        return STEP_EWORKSPACE;

    ScoreArgs a;
    a.hidden = hidden; a.W1 = W1; a.W2 = W2; a.boundary_idx = boundary_idx; a.trace_of = trace_of;
    a.b1 = b1; a.b2 = b2; a.logits = logits; a.probs = probs; a.score_sum = score_sum; a.scores = scores;
    a.score_cnt = score_cnt; a.status = status;
    a.R = d->R; a.d = d->d; a.m = d->m; a.B = d->B; a.N = d->N; a.act = d->act;
    chunking(d, a.nchunk, a.chunk_iters);
    const size_t MT = d->m / 16, Bp = d->B > 0 ? d->B : 1;
    a.plogit = reinterpret_cast<float *>(workspace);
    a.partial = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) + ((MT * Bp * sizeof(float) + 255) & ~(size_t)255));
    a.set = ticket_set_of(workspace);

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (d->B > 0) {
        const dim3 grid(d->m / 16, a.nchunk, (d->B + 16 * kBT - 1) / (16 * kBT));
        launch_kernel(kKernScore, score_hidden, grid, dim3(kThreads), s, a);
    } else if (state && scores) {
        launch_kernel(kKernScore, score_hidden, dim3(1, 1, 1), dim3(kThreads), s, a);
    }
    return launch_status();
}
