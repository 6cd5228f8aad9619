// prune_free: Algorithm 1's pruning branch applied k times -- t* = argmin score_t over the live
// traces, ReleaseKVCache(t*), T <- T \ {t*} (Section 4.2: prune the lowest average step score and
// release its KV cache).  Integer work only; every output is bit-exact.
//
// prune_select : one workgroup.  Builds 64-bit keys (order-preserving image of the fp32 score in
//                the high word, trace index in the low word; dead traces get the all-ones key),
//                sorts them with a bitonic network (exchanges closer than 64 keys are wavefront
//                shuffles, farther ones go through LDS) and writes the first k indices.  Also
//                validates lengths and scores and clears the freed-page bitmap.
// prune_release: one thread per (pruned trace, block-table entry): atomic decrement of the page's
//                refcount; the decrement that reaches zero sets the page's bit in the bitmap.
// prune_compact: the bitmap in ascending page order (popcount + prefix sum) gives the freed page ids, 1024
//                bitmap words per workgroup; then the pruned traces are marked dead.
// prune_fused  : all of the above in one workgroup, for small problems.
#include <mutex>

#include "common.h"

namespace step {
namespace {

typedef unsigned long long u64;
constexpr int kSelThreads = 1024;
static_assert(kSelThreads == 1024, "block_excl_scan works on 1024-thread workgroups");
constexpr int kMaxN = 4096;
constexpr int kRankN = 256;  // up to this many keys are ordered by counting, not by sorting

// Few keys: the place of a live key among the selected is the number of smaller keys (keys are distinct, the trace
// index is part of them; the keys of dead traces are all ~0 and are not placed).  Every thread reads all npad keys as
// LDS broadcasts -- no exchange stages, no barriers in between.  On return keys[0 .. live) is ascending.
__device__ __forceinline__ void order_by_counting(u64 *keys, int npad)
{
    const int tid = threadIdx.x;
    const u64 mine = tid < npad ? keys[tid] : ~0ull;
    int rank = 0;
    if (mine != ~0ull) {
        for (int j = 0; j < npad; j += 4) {  // (npad is a power of two, at least 4)
            rank += (keys[j] < mine) + (keys[j + 1] < mine) + (keys[j + 2] < mine) + (keys[j + 3] < mine);
        }
    }
    __syncthreads();
    if (mine != ~0ull) keys[rank] = mine;
    __syncthreads();
}

struct PruneHeader {  // first 256 bytes of the workspace
    int32_t k_eff;    // number of traces actually pruned (0 after a selection error)
};

struct PruneArgs {
    const float *scores;
    int32_t *refcounts, *block_tables, *seq_lens, *pruned, *freed_pages, *n_freed, *status;
    PruneHeader *hdr;
    u32 *bitmap;  // ceil(NP / 32) words
    int N, MAXB, NP, P, k, npad, words;
};

__global__ __launch_bounds__(kSelThreads) void prune_select(const PruneArgs a)
{
    __shared__ u64 keys[kMaxN];
    __shared__ int live_count, err;
    const int tid = threadIdx.x;
    if (tid == 0) {
        live_count = 0;
        err = 0;
    }
    for (int wv = tid; wv < a.words; wv += kSelThreads) a.bitmap[wv] = 0u;
    __syncthreads();
    int my_live = 0;
    for (int i = tid; i < a.npad; i += kSelThreads) {
        u64 key = ~0ull;
        if (i < a.N) {
            const int L = a.seq_lens[i];
            if (L < 0 || (long long)L > (long long)a.MAXB * a.P) {
                atomicCAS(&err, 0, (int)STEP_ELEN);
            } else if (L > 0) {
                const float s = a.scores[i];
                if (s != s) atomicCAS(&err, 0, (int)STEP_ENAN);
                key = ((u64)order_key(s) << 32) | (u32)i;
                ++my_live;
            }
        }
        keys[i] = key;
    }
    if (my_live) atomicAdd(&live_count, my_live);
    __syncthreads();
    if (err == 0 && a.k > live_count) {
        __syncthreads();
        if (tid == 0) err = STEP_EKLIVE;
    }
    __syncthreads();
    if (err != 0) {
        if (tid == 0) {
            report(a.status, err);
            a.hdr->k_eff = 0;
        }
        return;
    }
    // ascending order of the keys: by counting when they are few, else a bitonic sort
    if (a.npad <= kRankN) {
        order_by_counting(keys, a.npad);
    } else if (a.npad <= kSelThreads) {
        // one key per thread; exchanges at distance < 64 stay inside a wavefront (shuffles), larger
        // distances go through LDS
        u64 key = tid < a.npad ? keys[tid] : ~0ull;
        for (int size = 2; size <= a.npad; size <<= 1) {
            const bool asc = (tid & size) == 0;
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                u64 other;
                if (stride >= 64) {
                    __syncthreads();
                    keys[tid] = key;
                    __syncthreads();
                    other = keys[tid ^ stride];
                } else {
                    const u32 lo = __shfl_xor((u32)key, stride), hi = __shfl_xor((u32)(key >> 32), stride);
                    other = ((u64)hi << 32) | lo;
                }
                const bool lower = (tid & stride) == 0;       // this thread keeps the smaller key when ascending
                const bool take_min = lower == asc;
                key = take_min ? (key < other ? key : other) : (key > other ? key : other);
            }
        }
        __syncthreads();
        if (tid < a.npad) keys[tid] = key;
        __syncthreads();
    } else {
        for (int size = 2; size <= a.npad; size <<= 1) {
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                for (int t = tid; t < (a.npad >> 1); t += kSelThreads) {
                    const int lo = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
                    const int hi = lo + stride;
                    const bool asc = (lo & size) == 0;
                    const u64 x = keys[lo], y = keys[hi];
                    if ((x > y) == asc) {
                        keys[lo] = y;
                        keys[hi] = x;
                    }
                }
                __syncthreads();
            }
        }
    }
    for (int j = tid; j < a.k; j += kSelThreads) a.pruned[j] = (int32_t)(u32)keys[j];
    if (tid == 0) a.hdr->k_eff = a.k;
}

__global__ __launch_bounds__(256) void prune_release(const PruneArgs a)
{
    const int r = blockIdx.y;
    if (r >= a.hdr->k_eff) return;
    const int t = a.pruned[r];
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= a.MAXB) return;
    const int L = a.seq_lens[t];
    const int nb = (L + a.P - 1) / a.P;
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
                atomicOr(&a.bitmap[p >> 5], 1u << (p & 31));
            }
        }
    }
    *entry = -1;
}

// One workgroup per 1024 bitmap words, one word per thread.  A workgroup needs the number of freed pages
// in the words before its own: it counts them itself (the whole bitmap is a few kilobytes, read from the
// caches), so the workgroups need nothing from each other; the last one also reports the total.
__global__ __launch_bounds__(kSelThreads) void prune_compact(const PruneArgs a)
{
    __shared__ int scratch[32];
    const int tid = threadIdx.x;
    const int k_eff = a.hdr->k_eff;
    const int seg0 = blockIdx.x * kSelThreads;
    const int wv = seg0 + tid;
    u32 bits = 0;
    int before = 0;
    if (k_eff > 0) {
        if (wv < a.words) bits = a.bitmap[wv];
        for (int w = tid; w < seg0; w += kSelThreads) before += __popc(a.bitmap[w]);
    }
    int base = 0;
    if (blockIdx.x > 0) (void)block_excl_scan(before, scratch, &base);  // uniform branch; base = sum over the workgroup
    int total;
    int pos = base + block_excl_scan(__popc(bits), scratch, &total);
    while (bits) {
        const int b = __ffs(bits) - 1;
        bits &= bits - 1;
        a.freed_pages[pos++] = wv * 32 + b;
    }
    if (blockIdx.x == gridDim.x - 1 && tid == 0) *a.n_freed = base + total;
    if (blockIdx.x == 0)
        for (int r = tid; r < k_eff; r += kSelThreads) a.seq_lens[a.pruned[r]] = 0;
}

// Small problems (N <= 1024 traces, at most 8192 block-table entries to release, a bitmap that fits
// LDS): the three phases above in ONE workgroup, with the keys, the lengths and the freed-page
// bitmap in LDS, so a prune of a few traces costs one launch instead of three.
constexpr int kFusedN = 1024;
constexpr int kFusedWords = 8192;    // bitmap words in LDS: pools of up to 262144 pages
constexpr int kFusedEntries = 8192;  // k * MAXB

__global__ __launch_bounds__(kSelThreads) void prune_fused(const PruneArgs a)
{
    __shared__ u64 keys[kFusedN];
    __shared__ int lens[kFusedN];
    __shared__ u32 bitmap[kFusedWords];
    __shared__ int scratch[32];
    __shared__ int live_count, err;
    const int tid = threadIdx.x;
    if (tid == 0) {
        live_count = 0;
        err = 0;
    }
    for (int wv = tid; wv < a.words; wv += kSelThreads) bitmap[wv] = 0u;
    __syncthreads();
    {
        u64 key = ~0ull;
        int L = 0;
        if (tid < a.N) {
            L = a.seq_lens[tid];
            const float s = a.scores[tid];  // requested together with the length (a dead trace's score is not looked at)
            if (L < 0 || (long long)L > (long long)a.MAXB * a.P) {
                atomicCAS(&err, 0, (int)STEP_ELEN);
            } else if (L > 0) {
                if (s != s) atomicCAS(&err, 0, (int)STEP_ENAN);
                key = ((u64)order_key(s) << 32) | (u32)tid;
            }
        }
        keys[tid] = key;
        lens[tid] = L;
        const u64 live_mask = __ballot(key != ~0ull);
        if ((tid & 63) == 0 && live_mask) atomicAdd(&live_count, __popcll(live_mask));
    }
    __syncthreads();
    if (err == 0 && a.k > live_count) {
        __syncthreads();
        if (tid == 0) err = STEP_EKLIVE;
    }
    __syncthreads();
    if (err != 0) {
        if (tid == 0) {
            report(a.status, err);
            *a.n_freed = 0;
        }
        return;
    }
    // ascending order of the keys: by counting when they are few, else a bitonic sort with one key per thread
    if (a.npad <= kRankN) {
        order_by_counting(keys, a.npad);
    } else {
        u64 key = keys[tid];
        for (int size = 2; size <= a.npad; size <<= 1) {
            const bool asc = (tid & size) == 0;
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                u64 other;
                if (stride >= 64) {
                    __syncthreads();
                    keys[tid] = key;
                    __syncthreads();
                    other = keys[tid ^ stride];
                } else {
                    const u32 lo = __shfl_xor((u32)key, stride), hi = __shfl_xor((u32)(key >> 32), stride);
                    other = ((u64)hi << 32) | lo;
                }
                const bool take_min = ((tid & stride) == 0) == asc;
                key = take_min ? (key < other ? key : other) : (key > other ? key : other);
            }
        }
        __syncthreads();
        keys[tid] = key;
        __syncthreads();
    }
    if (tid < a.k) a.pruned[tid] = (int32_t)(u32)keys[tid];
    // release: (pruned trace, block-table entry) pairs, four per thread and trip: first the four entries are
    // requested, then the four decrements, then their results are looked at -- two memory round trips per trip
    // instead of two per entry
    const int entries = a.k * a.MAXB;
    constexpr int kRel = 4;
    for (int e0 = tid; e0 < entries; e0 += kRel * kSelThreads) {
        int32_t *entry[kRel];
        int page[kRel], old[kRel];
        bool used[kRel];
#pragma unroll
        for (int u = 0; u < kRel; ++u) {
            const int e = e0 + u * kSelThreads;
            used[u] = false;
            entry[u] = nullptr;
            page[u] = -1;
            if (e < entries) {
                const int r = e / a.MAXB, j = e - r * a.MAXB;
                const int t = (int)(u32)keys[r];
                entry[u] = a.block_tables + (size_t)t * a.MAXB + j;
                used[u] = j < (lens[t] + a.P - 1) / a.P;
                if (used[u]) page[u] = *entry[u];
            }
        }
#pragma unroll
        for (int u = 0; u < kRel; ++u) {
            old[u] = 1 << 30;
            if (used[u]) {
                if ((u32)page[u] >= (u32)a.NP) {
                    report(a.status, STEP_EPAGE);
                    used[u] = false;
                } else {
                    old[u] = atomicSub(&a.refcounts[page[u]], 1);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kRel; ++u) {
            if (used[u]) {
                if (old[u] <= 0) {
                    atomicAdd(&a.refcounts[page[u]], 1);
                    report(a.status, STEP_EREFCOUNT);
                } else if (old[u] == 1) {
                    atomicOr(&bitmap[page[u] >> 5], 1u << (page[u] & 31));
                }
            }
            if (entry[u]) *entry[u] = -1;
        }
    }
    __syncthreads();
    // compact the bitmap in ascending page order
    const int per = (a.words + kSelThreads - 1) / kSelThreads;
    const int w0 = min(tid * per, a.words), w1 = min(w0 + per, a.words);
    int cnt = 0;
    for (int wv = w0; wv < w1; ++wv) cnt += __popc(bitmap[wv]);
    int total;
    int pos = block_excl_scan(cnt, scratch, &total);
    if (cnt > 0)
        for (int wv = w0; wv < w1; ++wv) {
            u32 bits = bitmap[wv];
            while (bits) {
                const int b = __ffs(bits) - 1;
                bits &= bits - 1;
                a.freed_pages[pos++] = wv * 32 + b;
            }
        }
    if (tid == 0) *a.n_freed = total;
    if (tid < a.k) a.seq_lens[(int)(u32)keys[tid]] = 0;
}

}  // namespace
}  // namespace step

using namespace step;

extern "C" size_t step_prune_workspace_bytes(int32_t N, int32_t MAXB, int32_t NP)
{
    if (N < 0 || MAXB < 0 || NP < 0) return 0;
    const size_t words = ((size_t)NP + 31) / 32;
    return 256 + ((words * sizeof(u32) + 255) & ~(size_t)255);
}

namespace {

// Shared by prune_free (scratch = the caller's workspace) and prune_free_static (scratch = this
// library's own device array): argument checks, then the launches.  `scratch` is a device address.
int run_prune(int32_t N, int32_t MAXB, int32_t NP, int32_t P, const float *scores, int32_t k, int32_t *refcounts,
              int32_t *block_tables, int32_t *seq_lens, int32_t *pruned, int32_t *freed_pages, int32_t *n_freed,
              void *scratch, int32_t *status, void *stream)
{
    PruneArgs a;
    a.scores = scores; a.refcounts = refcounts; a.block_tables = block_tables; a.seq_lens = seq_lens;
    a.pruned = pruned; a.freed_pages = freed_pages; a.n_freed = n_freed; a.status = status;
    a.hdr = reinterpret_cast<PruneHeader *>(scratch);
    a.bitmap = reinterpret_cast<u32 *>(reinterpret_cast<char *>(scratch) + 256);
    a.N = N; a.MAXB = MAXB; a.NP = NP; a.P = P; a.k = k;
    a.npad = 4;
    while (a.npad < N) a.npad <<= 1;
    a.words = (int)(((size_t)NP + 31) / 32);

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    static const bool force_multi = getenv("STEP_PRUNE_MULTI") != nullptr;  // testing aid: always three kernels
    if (!force_multi && N <= kFusedN && a.words <= kFusedWords && (long long)k * MAXB <= kFusedEntries) {
        launch_kernel(kKernPruneFused, prune_fused, dim3(1), dim3(kSelThreads), s, a);
        return launch_status();
    }
    launch_kernel(kKernPruneSelect, prune_select, dim3(1), dim3(kSelThreads), s, a);
    if (k > 0 && MAXB > 0)
        launch_kernel(kKernPruneRelease, prune_release, dim3((MAXB + 255) / 256, k), dim3(256), s, a);
    launch_kernel(kKernPruneCompact, prune_compact, dim3((unsigned)((a.words + kSelThreads - 1) / kSelThreads > 0 ? (a.words + kSelThreads - 1) / kSelThreads : 1)), dim3(kSelThreads), s, a);
    return launch_status();
}

bool prune_args_ok(int32_t N, int32_t MAXB, int32_t NP, int32_t P, const float *scores, int32_t k,
                   const int32_t *refcounts, const int32_t *block_tables, const int32_t *seq_lens,
                   const int32_t *pruned, const int32_t *freed_pages, const int32_t *n_freed)
{
    if (N < 0 || N > kMaxN || MAXB < 0 || NP < 0 || P <= 0 || k < 0 || k > N) return false;
    if (!n_freed) return false;
    if (N > 0 && (!scores || !seq_lens || !block_tables || !refcounts)) return false;
    if (k > 0 && (!pruned || !freed_pages)) return false;
    return true;
}

// ---------------------------------------------------------------------------------------------
// prune_free_static: the scratch of the three-kernel path (header + freed-page bitmap) lives in a
// device array of this library instead of a caller's workspace, for callers that cannot allocate.
// Every GPU holds its own copy of the array at its own address; the address is looked up once per
// device and kept.  The array's name is never used as a pointer in host code.
// ---------------------------------------------------------------------------------------------
constexpr int kStaticMaxNP = 1 << 22;  // pages the static bitmap covers (512 KiB + the 256-byte header)
static __device__ __align__(256) unsigned char scratch[256 + kStaticMaxNP / 8];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, nullptr until looked up

int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return STEP_ELAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return STEP_ELAUNCH;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return STEP_OK;
}

}  // namespace

extern "C" int prune_free(int32_t N, int32_t MAXB, int32_t NP, int32_t P, const float *scores, int32_t k,
                          int32_t *refcounts, int32_t *block_tables, int32_t *seq_lens, int32_t *pruned,
                          int32_t *freed_pages, int32_t *n_freed, void *workspace, size_t workspace_bytes,
                          int32_t *status, void *stream)
{
    if (!prune_args_ok(N, MAXB, NP, P, scores, k, refcounts, block_tables, seq_lens, pruned, freed_pages, n_freed))
        return STEP_EINVAL;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < step_prune_workspace_bytes(N, MAXB, NP))
        return STEP_EWORKSPACE;
    return run_prune(N, MAXB, NP, P, scores, k, refcounts, block_tables, seq_lens, pruned, freed_pages, n_freed,
                     workspace, status, stream);
}

extern "C" int32_t step_prune_static_max_pages(void) { return kStaticMaxNP; }

extern "C" int prune_free_static(int32_t N, int32_t MAXB, int32_t NP, int32_t P, const float *scores, int32_t k,
                                 int32_t *refcounts, int32_t *block_tables, int32_t *seq_lens, int32_t *pruned,
                                 int32_t *freed_pages, int32_t *n_freed, int32_t *status, void *stream)
{
    if (!prune_args_ok(N, MAXB, NP, P, scores, k, refcounts, block_tables, seq_lens, pruned, freed_pages, n_freed))
        return STEP_EINVAL;
    if (NP > kStaticMaxNP) return STEP_EWORKSPACE;  // the pool is larger than the static bitmap covers
    void *ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc != STEP_OK) return rc;
    return run_prune(N, MAXB, NP, P, scores, k, refcounts, block_tables, seq_lens, pruned, freed_pages, n_freed, ptr,
                     status, stream);
}
