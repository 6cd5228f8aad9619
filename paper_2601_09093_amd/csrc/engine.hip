// The pieces of Algorithm 1 around the three hot calls, so that a whole multi-step decode loop
// runs on the device without a host round trip:
//   step_reserve_pages  Section 4.2's trigger.  Before the next decode step a live trace whose
//                       length is a multiple of P needs a new page.  The trigger (memory full, the
//                       next step's KV cache does not fit) is read as: fewer free pages
//                       (refcount 0) than traces that need one; while that holds, the live trace
//                       with the lowest score is pruned and its pages released (Algorithm 1:
//                       argmin, ReleaseKVCache, T <- T \ {t*}), one trace at a time.  Then every
//                       trace that still needs a page, in ascending index, takes the smallest free
//                       page id.  The free pages are kept as a bitmap (and a count) in the workspace from
//                       call to call: releasing sets bits, allocating clears them, so a step costs a scan
//                       of NP / 32 words instead of NP reference counts.  step_freelist_rebuild makes the
//                       bitmap from the reference counts (the definition of "free"), step_freelist_add
//                       enters the pages a prune_free call has freed.
//   step_append_kv      the KV-cache write of NextToken(t): row L_i of every live trace, L_i += 1.
//   step_weighted_vote  WeightedVote of Algorithm 1 / Section 4.3: the answer whose traces' final
//                       scores sum highest.
// All integer results are bit-exact; the vote sums fp32 scores in trace index order.
#include "common.h"

namespace step {
namespace {

typedef unsigned long long u64;
constexpr int kThreads = 1024;
static_assert(kThreads == 1024, "block_excl_scan works on 1024-thread workgroups");
constexpr int kMaxN = 4096;

// sum of one int per thread over the workgroup, returned to every thread
__device__ int block_sum(int v, int *scratch /*[17]*/)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    int t = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) t += scratch[w];
    return t;
}

struct FreeListHeader {  // first 256 bytes of the reserve workspace
    int32_t stamp;        // freelist_stamp(NP) once the bitmap has been built for a pool of NP pages
    int32_t nfree;        // set bits of the bitmap
    int32_t pad[62];
};

__host__ __device__ inline int32_t freelist_stamp(int NP) { return (int32_t)((0x46524545u ^ ((u32)NP * 2654435761u)) | 1u); }

struct ReserveArgs {
    const float *scores;
    int32_t *refcounts, *block_tables, *seq_lens, *pruned, *n_pruned, *new_pages, *status;
    FreeListHeader *hdr;
    u32 *bitmap;  // ceil(NP / 64) * 2 words: bit p set <=> page p is free
    const int32_t *freed_pages, *n_freed;  // step_freelist_add only
    int N, MAXB, NP, P, words, cap;
};

// step_freelist_rebuild: bit p of the bitmap = (refcounts[p] == 0), count of set bits, stamp.  One workgroup;
// all loads of a thread are issued before the first is used (four pages per 16-byte load, 16 loads in flight),
// eight neighbouring lanes then assemble one 32-bit word of the bitmap.
__global__ __launch_bounds__(kThreads) void freelist_rebuild_kernel(const ReserveArgs a)
{
    __shared__ int scratch[32];
    const int tid = threadIdx.x, lane = tid & 63;
    int my_free = 0;
    constexpr int kBatch = 16;
    const int quads = a.words * 8;  // groups of four pages
    const bool vec_ok = (reinterpret_cast<uintptr_t>(a.refcounts) & 15) == 0;
    for (int base = 0; base < quads; base += kBatch * kThreads) {
        int4 v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int qd = base + u * kThreads + tid;
            const int p = qd * 4;
            v[u] = make_int4(1, 1, 1, 1);
            if (qd < quads) {
                if (vec_ok && p + 3 < a.NP) {
                    v[u] = *reinterpret_cast<const int4 *>(a.refcounts + p);
                } else {
                    if (p + 0 < a.NP) v[u].x = a.refcounts[p + 0];
                    if (p + 1 < a.NP) v[u].y = a.refcounts[p + 1];
                    if (p + 2 < a.NP) v[u].z = a.refcounts[p + 2];
                    if (p + 3 < a.NP) v[u].w = a.refcounts[p + 3];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int qd = base + u * kThreads + tid;
            u32 nib = (v[u].x == 0 ? 1u : 0u) | (v[u].y == 0 ? 2u : 0u) | (v[u].z == 0 ? 4u : 0u) |
                      (v[u].w == 0 ? 8u : 0u);
            u32 word = nib << (4 * (lane & 7));
            word |= __shfl_xor(word, 1);
            word |= __shfl_xor(word, 2);
            word |= __shfl_xor(word, 4);
            if ((lane & 7) == 0 && qd < quads) {
                a.bitmap[qd >> 3] = word;
                my_free += __popc(word);
            }
        }
    }
    const int nfree = block_sum(my_free, scratch);
    if (tid == 0) {
        a.hdr->nfree = nfree;
        a.hdr->stamp = freelist_stamp(a.NP);
    }
}

// step_freelist_add: the pages of a freed list (what prune_free reports) become free in the bitmap
__global__ __launch_bounds__(kThreads) void freelist_add_kernel(const ReserveArgs a)
{
    __shared__ int scratch[32];
    const int tid = threadIdx.x;
    if (a.hdr->stamp != freelist_stamp(a.NP)) {
        if (tid == 0) report(a.status, STEP_EFREELIST);
        return;
    }
    const int n = min(max(*a.n_freed, 0), a.cap);
    int added = 0;
    for (int i = tid; i < n; i += kThreads) {
        const int p = a.freed_pages[i];
        if ((u32)p >= (u32)a.NP) {
            report(a.status, STEP_EPAGE);
            continue;
        }
        const u32 bit = 1u << (p & 31);
        if (!(atomicOr(&a.bitmap[p >> 5], bit) & bit)) ++added;
    }
    added = block_sum(added, scratch);
    if (tid == 0) a.hdr->nfree += added;
}

__global__ __launch_bounds__(kThreads) void reserve_pages_kernel(const ReserveArgs a)
{
    __shared__ int lens[kMaxN];       // live length of trace t, 0 once pruned
    __shared__ int need_list[kMaxN];  // rank among the traces that need a page -> trace
    __shared__ int scratch[32];
    __shared__ u64 best_s[kThreads / 64];
    __shared__ int err_s;
    const int tid = threadIdx.x, lane = tid & 63;
    if (tid == 0) err_s = 0;
    __syncthreads();
    if (a.hdr->stamp != freelist_stamp(a.NP)) {  // no free list was built for this pool in this workspace
        if (tid == 0) {
            report(a.status, STEP_EFREELIST);
            *a.n_pruned = 0;
        }
        return;
    }

    // lengths, traces on a page boundary
    int my_need = 0;
    for (int i = tid; i < a.N; i += kThreads) {
        const int L = a.seq_lens[i];
        int keep = L;
        if (L < 0 || (long long)L > (long long)a.MAXB * a.P) {
            atomicCAS(&err_s, 0, (int)STEP_ELEN);
            keep = 0;
        } else if (L > 0 && L % a.P == 0) {
            if (L / a.P >= a.MAXB) atomicCAS(&err_s, 0, (int)STEP_ELEN);  // the row has no entry left
            ++my_need;
        }
        lens[i] = keep;
        a.new_pages[i] = -1;
    }
    int needed = block_sum(my_need, scratch);
    int nfree = a.hdr->nfree;
    __syncthreads();
    if (err_s == 0 && nfree < needed) {  // pruning will happen: every live score must be a number
        for (int i = tid; i < a.N; i += kThreads)
            if (lens[i] > 0) {
                const float s = a.scores[i];
                if (s != s) atomicCAS(&err_s, 0, (int)STEP_ENAN);
            }
    }
    __syncthreads();
    if (err_s != 0) {
        if (tid == 0) {
            report(a.status, err_s);
            *a.n_pruned = 0;
        }
        return;
    }

    int n_pruned = 0;
    while (nfree < needed) {  // uniform: both counts are workgroup-wide values
        // t* = argmin over live traces of (score, index)
        u64 key = ~0ull;
        for (int i = tid; i < a.N; i += kThreads)
            if (lens[i] > 0) {
                const u64 k2 = ((u64)order_key(a.scores[i]) << 32) | (u32)i;
                key = k2 < key ? k2 : key;
            }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const u32 lo = __shfl_xor((u32)key, off), hi = __shfl_xor((u32)(key >> 32), off);
            const u64 o = ((u64)hi << 32) | lo;
            key = o < key ? o : key;
        }
        __syncthreads();
        if (lane == 0) best_s[tid >> 6] = key;
        __syncthreads();
        key = best_s[0];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) key = best_s[w] < key ? best_s[w] : key;
        if (key == ~0ull) break;  // no live trace left (then needed == 0 as well)
        const int t = (int)(u32)key;
        const int L = lens[t];
        const int nb = (L + a.P - 1) / a.P;
        // ReleaseKVCache(t*)
        int my_freed = 0;
        for (int j = tid; j < a.MAXB; j += kThreads) {
            int32_t *entry = a.block_tables + (size_t)t * a.MAXB + j;
            if (j < nb) {
                const int p = *entry;
                if ((u32)p >= (u32)a.NP) {
                    report(a.status, STEP_EPAGE);
                } else {
                    const int old = atomicSub(&a.refcounts[p], 1);
                    if (old <= 0) {
                        atomicAdd(&a.refcounts[p], 1);
                        report(a.status, STEP_EREFCOUNT);
                    } else if (old == 1) {
                        const u32 bit = 1u << (p & 31);
                        if (!(atomicOr(&a.bitmap[p >> 5], bit) & bit)) ++my_freed;
                    }
                }
            }
            *entry = -1;
        }
        nfree += block_sum(my_freed, scratch);
        if (L % a.P == 0) --needed;
        __syncthreads();
        if (tid == 0) {
            lens[t] = 0;
            a.seq_lens[t] = 0;
            a.pruned[n_pruned] = t;
        }
        ++n_pruned;
        __syncthreads();
    }
    if (tid == 0) *a.n_pruned = n_pruned;

    // traces that still need a page, in ascending index
    int total_need = 0;
    for (int base = 0; base < a.N; base += kThreads) {
        const int i = base + tid;
        const int L = i < a.N ? lens[i] : 0;
        const int flag = (L > 0 && L % a.P == 0) ? 1 : 0;
        int tot;
        const int rk = total_need + block_excl_scan(flag, scratch, &tot);
        if (flag) need_list[rk] = i;
        total_need += tot;
    }
    __syncthreads();
    if (total_need == 0) {  // nothing to hand out: the bitmap is not even looked at
        if (tid == 0) a.hdr->nfree = nfree;
        return;
    }
    // free pages in ascending id: thread owns a contiguous range of bitmap words
    const int per = (a.words + kThreads - 1) / kThreads;
    const int w0 = min(tid * per, a.words), w1 = min(w0 + per, a.words);
    int cnt = 0;
    for (int wv = w0; wv < w1; ++wv) cnt += __popc(__atomic_load_n(&a.bitmap[wv], __ATOMIC_RELAXED));
    int total_free;
    int pos = block_excl_scan(cnt, scratch, &total_free);
    int taken = 0;
    if (cnt > 0 && pos < total_need)
        for (int wv = w0; wv < w1 && pos < total_need; ++wv) {
            u32 bits = __atomic_load_n(&a.bitmap[wv], __ATOMIC_RELAXED);
            u32 used = 0;
            while (bits && pos < total_need) {
                const int b = __ffs(bits) - 1;
                bits &= bits - 1;
                const int page = wv * 32 + b;
                const int i = need_list[pos++];
                used |= 1u << b;
                if (page >= a.NP || a.refcounts[page] != 0) {  // the bitmap does not match the reference counts
                    report(a.status, STEP_EFREELIST);
                    continue;
                }
                a.block_tables[(size_t)i * a.MAXB + lens[i] / a.P] = page;
                a.refcounts[page] = 1;
                a.new_pages[i] = page;
                ++taken;
            }
            if (used) a.bitmap[wv] &= ~used;  // this thread owns the word
        }
    taken = block_sum(taken, scratch);
    if (tid == 0) {
        if (total_free != nfree) report(a.status, STEP_EFREELIST);  // the count and the bitmap have come apart
        a.hdr->nfree = total_free - min(total_need, total_free);
    }
}

struct AppendArgs {
    const uint16_t *k_new, *v_new;
    uint16_t *k_pages, *v_pages;
    const int32_t *block_tables, *refcounts;
    int32_t *seq_lens, *status;
    int N, Hkv, D, MAXB, NP;
};

// one workgroup per trace: read L, write the Hkv rows of K and V, then L + 1
__global__ __launch_bounds__(256) void append_kv_kernel(const AppendArgs a)
{
    const int i = blockIdx.x;
    const int L = a.seq_lens[i];
    if (L == 0) return;
    if (L < 0 || (long long)L >= (long long)a.MAXB * kPageTokens) {
        if (threadIdx.x == 0) report(a.status, STEP_ELEN);
        return;
    }
    const int page = a.block_tables[(size_t)i * a.MAXB + L / kPageTokens];
    if ((u32)page >= (u32)a.NP) {
        if (threadIdx.x == 0) report(a.status, STEP_EPAGE);
        return;
    }
    if (a.refcounts && a.refcounts[page] != 1) {  // the row would land in a page another trace reads
        if (threadIdx.x == 0) report(a.status, STEP_EREFCOUNT);
        return;
    }
    const int slot = L % kPageTokens;
    const int chunks = a.D / 8;  // 16-byte pieces per row
    for (int idx = threadIdx.x; idx < a.Hkv * chunks; idx += blockDim.x) {
        const int g = idx / chunks, c = idx % chunks;
        const size_t src = ((size_t)i * a.Hkv + g) * a.D + c * 8;
        const size_t dst = (((size_t)page * a.Hkv + g) * kPageTokens + slot) * a.D + c * 8;
        *reinterpret_cast<uint4 *>(a.k_pages + dst) = *reinterpret_cast<const uint4 *>(a.k_new + src);
        *reinterpret_cast<uint4 *>(a.v_pages + dst) = *reinterpret_cast<const uint4 *>(a.v_new + src);
    }
    __syncthreads();
    if (threadIdx.x == 0) a.seq_lens[i] = L + 1;
}

__global__ __launch_bounds__(kThreads) void weighted_vote_kernel(int N, const int32_t *answer, const float *scores,
                                                                  int32_t *winner, float *weight, int32_t *status)
{
    __shared__ int ans_s[kMaxN];
    __shared__ float sc_s[kMaxN];
    __shared__ u64 best_s[kThreads / 64];
    __shared__ int err_s;
    const int tid = threadIdx.x, lane = tid & 63;
    if (tid == 0) err_s = 0;
    __syncthreads();
    for (int i = tid; i < N; i += kThreads) {
        ans_s[i] = answer[i];
        sc_s[i] = scores[i];
        if (ans_s[i] >= 0 && sc_s[i] != sc_s[i]) err_s = STEP_ENAN;
    }
    __syncthreads();
    if (err_s != 0) {
        if (tid == 0) {
            report(status, err_s);
            *winner = -1;
            *weight = 0.f;
        }
        return;
    }
    // best = max weight, ties to the smaller answer id: one 64-bit key (weight image, ~answer)
    u64 key = 0ull;  // below every real key
    for (int i = tid; i < N; i += kThreads) {
        const int ai = ans_s[i];
        if (ai < 0) continue;
        float w = 0.f;
        for (int j = 0; j < N; ++j)
            if (ans_s[j] == ai) w = w + sc_s[j];  // trace index order
        const u64 k2 = ((u64)order_key(w) << 32) | (u32)(0x7fffffff - ai);
        key = k2 > key ? k2 : key;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const u32 lo = __shfl_xor((u32)key, off), hi = __shfl_xor((u32)(key >> 32), off);
        const u64 o = ((u64)hi << 32) | lo;
        key = o > key ? o : key;
    }
    if (lane == 0) best_s[tid >> 6] = key;
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kThreads / 64; ++w) key = best_s[w] > key ? best_s[w] : key;
        if (key == 0ull) {
            *winner = -1;
            *weight = 0.f;
        } else {
            const u32 img = (u32)(key >> 32);
            const u32 bits = (img & 0x80000000u) ? (img & 0x7fffffffu) : ~img;  // inverse of order_key
            *winner = 0x7fffffff - (int)(u32)key;
            *weight = __uint_as_float(bits);
        }
    }
}

}  // namespace
}  // namespace step

using namespace step;

extern "C" size_t step_reserve_workspace_bytes(int32_t N, int32_t MAXB, int32_t NP)
{
    if (N < 0 || MAXB < 0 || NP < 0) return 0;
    const size_t words = (((size_t)NP + 63) / 64) * 2;
    return ((words * sizeof(u32) + 255) & ~(size_t)255) + 256;
}

namespace {
bool freelist_args(ReserveArgs &a, int32_t NP, void *workspace, size_t workspace_bytes)
{
    if (NP < 0) return false;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < step_reserve_workspace_bytes(0, 0, NP)) return false;
    a.hdr = reinterpret_cast<FreeListHeader *>(workspace);
    a.bitmap = reinterpret_cast<u32 *>(reinterpret_cast<char *>(workspace) + 256);
    a.NP = NP;
    a.words = (int)((((size_t)NP + 63) / 64) * 2);
    return true;
}
}  // namespace

extern "C" int step_freelist_rebuild(int32_t NP, const int32_t *refcounts, void *workspace, size_t workspace_bytes,
                                     void *stream)
{
    if (NP < 0 || (NP > 0 && !refcounts)) return STEP_EINVAL;
    ReserveArgs a = {};
    if (!freelist_args(a, NP, workspace, workspace_bytes)) return STEP_EWORKSPACE;
    a.refcounts = const_cast<int32_t *>(refcounts);
    launch_kernel(kKernFreelist, freelist_rebuild_kernel, dim3(1), dim3(kThreads), reinterpret_cast<hipStream_t>(stream), a);
    return launch_status();
}

extern "C" int step_freelist_add(int32_t NP, const int32_t *freed_pages, const int32_t *n_freed, int32_t capacity,
                                 void *workspace, size_t workspace_bytes, int32_t *status, void *stream)
{
    if (NP < 0 || capacity < 0 || !n_freed || (capacity > 0 && !freed_pages)) return STEP_EINVAL;
    ReserveArgs a = {};
    if (!freelist_args(a, NP, workspace, workspace_bytes)) return STEP_EWORKSPACE;
    a.freed_pages = freed_pages; a.n_freed = n_freed; a.cap = capacity; a.status = status;
    launch_kernel(kKernFreelist, freelist_add_kernel, dim3(1), dim3(kThreads), reinterpret_cast<hipStream_t>(stream), a);
    return launch_status();
}

extern "C" int step_reserve_pages(int32_t N, int32_t MAXB, int32_t NP, int32_t P, const float *scores,
                                  int32_t *refcounts, int32_t *block_tables, int32_t *seq_lens, int32_t *pruned,
                                  int32_t *n_pruned, int32_t *new_pages, void *workspace, size_t workspace_bytes,
                                  int32_t *status, void *stream)
{
    if (N < 0 || N > kMaxN || MAXB < 0 || NP < 0 || P <= 0) return STEP_EINVAL;
    if (!n_pruned) return STEP_EINVAL;
    if (N > 0 && (!scores || !seq_lens || !block_tables || !refcounts || !pruned || !new_pages)) return STEP_EINVAL;
    ReserveArgs a = {};
    if (!freelist_args(a, NP, workspace, workspace_bytes)) return STEP_EWORKSPACE;
    a.scores = scores; a.refcounts = refcounts; a.block_tables = block_tables; a.seq_lens = seq_lens;
    a.pruned = pruned; a.n_pruned = n_pruned; a.new_pages = new_pages; a.status = status;
    a.N = N; a.MAXB = MAXB; a.P = P;
    launch_kernel(kKernReserve, reserve_pages_kernel, dim3(1), dim3(kThreads), reinterpret_cast<hipStream_t>(stream), a);
    return launch_status();
}

extern "C" int step_append_kv(const step_attn_dims *d, const uint16_t *k_new, const uint16_t *v_new,
                              uint16_t *k_pages, uint16_t *v_pages, const int32_t *block_tables,
                              const int32_t *refcounts, int32_t *seq_lens, int32_t *status, void *stream)
{
    if (!d || d->N < 0 || d->Hkv <= 0 || d->MAXB < 0 || d->NP < 0 || d->P != kPageTokens) return STEP_EINVAL;
    if (d->D <= 0 || d->D % 8) return STEP_EINVAL;
    if (d->N == 0) return STEP_OK;
    if (!k_new || !v_new || !k_pages || !v_pages || !block_tables || !seq_lens) return STEP_EINVAL;
    if (!aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(k_pages, 16) || !aligned(v_pages, 16)) return STEP_EINVAL;
    AppendArgs a;
    a.k_new = k_new; a.v_new = v_new; a.k_pages = k_pages; a.v_pages = v_pages;
    a.block_tables = block_tables; a.refcounts = refcounts; a.seq_lens = seq_lens; a.status = status;
    a.N = d->N; a.Hkv = d->Hkv; a.D = d->D; a.MAXB = d->MAXB; a.NP = d->NP;
    launch_kernel(kKernAppend, append_kv_kernel, dim3(d->N), dim3(256), reinterpret_cast<hipStream_t>(stream), a);
    return launch_status();
}

extern "C" int step_weighted_vote(int32_t N, const int32_t *answer, const float *scores, int32_t *winner,
                                  float *weight, int32_t *status, void *stream)
{
    if (N < 0 || N > kMaxN || !winner || !weight) return STEP_EINVAL;
    if (N > 0 && (!answer || !scores)) return STEP_EINVAL;
    launch_kernel(kKernVote, weighted_vote_kernel, dim3(1), dim3(kThreads), reinterpret_cast<hipStream_t>(stream), N,
                  answer, scores, winner, weight, status);
    return launch_status();
}
