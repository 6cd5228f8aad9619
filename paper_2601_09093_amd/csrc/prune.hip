// prune_free: Algorithm 1's pruning branch applied k times -- t* = argmin score_t over the live
// traces, ReleaseKVCache(t*), T <- T \ {t*} (Section 4.2: prune the lowest average step score and
// release its KV cache).  Integer work only; every output is bit-exact.
//
// prune_select : one workgroup.  Builds 64-bit keys (order-preserving image of the fp32 score in
//                the high word, trace index in the low word; dead traces get the all-ones key),
//                sorts them with a bitonic network in LDS and writes the first k indices.  Also
//                validates lengths and scores and clears the freed-page bitmap.
// prune_release: one thread per (pruned trace, block-table entry): atomic decrement of the page's
//                refcount; the decrement that reaches zero sets the page's bit in the bitmap.
// prune_compact: one workgroup scans the bitmap in ascending page order (popcount + prefix sum)
//                and writes the freed page ids; then marks the pruned traces dead.
#include "common.h"

namespace step {
namespace {

typedef unsigned long long u64;
constexpr int kSelThreads = 1024;
constexpr int kMaxN = 4096;

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

__device__ __forceinline__ u32 order_key(float s)
{
    u32 u = __float_as_uint(s);
    if (u == 0x80000000u) u = 0u;  // -0 == +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

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
    // bitonic sort, ascending
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

__global__ __launch_bounds__(kSelThreads) void prune_compact(const PruneArgs a)
{
    __shared__ int scan[kSelThreads];
    const int tid = threadIdx.x;
    const int k_eff = a.hdr->k_eff;
    const int per = (a.words + kSelThreads - 1) / kSelThreads;
    const int w0 = min(tid * per, a.words), w1 = min(w0 + per, a.words);
    int cnt = 0;
    if (k_eff > 0)
        for (int wv = w0; wv < w1; ++wv) cnt += __popc(a.bitmap[wv]);
    scan[tid] = cnt;
    __syncthreads();
    for (int off = 1; off < kSelThreads; off <<= 1) {  // inclusive Hillis-Steele scan
        const int v = tid >= off ? scan[tid - off] : 0;
        __syncthreads();
        scan[tid] += v;
        __syncthreads();
    }
    int pos = scan[tid] - cnt;
    if (k_eff > 0)
        for (int wv = w0; wv < w1; ++wv) {
            u32 bits = a.bitmap[wv];
            while (bits) {
                const int b = __ffs(bits) - 1;
                bits &= bits - 1;
                a.freed_pages[pos++] = wv * 32 + b;
            }
        }
    if (tid == kSelThreads - 1) *a.n_freed = scan[tid];
    for (int r = tid; r < k_eff; r += kSelThreads) a.seq_lens[a.pruned[r]] = 0;
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

extern "C" int prune_free(int32_t N, int32_t MAXB, int32_t NP, int32_t P, const float *scores, int32_t k,
                          int32_t *refcounts, int32_t *block_tables, int32_t *seq_lens, int32_t *pruned,
                          int32_t *freed_pages, int32_t *n_freed, void *workspace, size_t workspace_bytes,
                          int32_t *status, void *stream)
{
    if (N < 0 || N > kMaxN || MAXB < 0 || NP < 0 || P <= 0 || k < 0 || k > N) return STEP_EINVAL;
    if (!n_freed) return STEP_EINVAL;
    if (N > 0 && (!scores || !seq_lens || !block_tables || !refcounts)) return STEP_EINVAL;
    if (k > 0 && (!pruned || !freed_pages)) return STEP_EINVAL;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < step_prune_workspace_bytes(N, MAXB, NP))
        return STEP_EWORKSPACE;

    PruneArgs a;
    a.scores = scores; a.refcounts = refcounts; a.block_tables = block_tables; a.seq_lens = seq_lens;
    a.pruned = pruned; a.freed_pages = freed_pages; a.n_freed = n_freed; a.status = status;
    a.hdr = reinterpret_cast<PruneHeader *>(workspace);
    a.bitmap = reinterpret_cast<u32 *>(reinterpret_cast<char *>(workspace) + 256);
    a.N = N; a.MAXB = MAXB; a.NP = NP; a.P = P; a.k = k;
    a.npad = 2;
    while (a.npad < N) a.npad <<= 1;
    a.words = (int)(((size_t)NP + 31) / 32);

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(prune_select, dim3(1), dim3(kSelThreads), 0, s, a);
    if (k > 0 && MAXB > 0)
        hipLaunchKernelGGL(prune_release, dim3((MAXB + 255) / 256, k), dim3(256), 0, s, a);
    hipLaunchKernelGGL(prune_compact, dim3(1), dim3(kSelThreads), 0, s, a);
    return launch_status();
}
