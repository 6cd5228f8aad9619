/*
 * libstep -- C ABI of the decode-step hot path of STEP (arxiv 2601.09093) on one MI355X (gfx950).
 *
 * One decode step over N parallel reasoning traces of one prompt is three hot calls, in this order
 * (step_reserve_pages / step_append_kv / step_weighted_vote further down complete Algorithm 1):
 *   paged_decode_attn   the attention inside NextToken(t) of Algorithm 1, for all live traces,
 *   step_score          y = f(h) for the traces at a step boundary, then "Update score_t"
 *                       (Section 4.1 equation; Section 4.3 running average),
 *   prune_free          argmin score_t / ReleaseKVCache / T <- T \ {t*} of Algorithm 1, k times.
 *
 * Conventions for every call
 *   - Every pointer is a DEVICE pointer owned by the caller unless it says "host".  The library
 *     allocates nothing; scratch memory comes in through `workspace` (256-byte aligned).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *     work on it and never synchronise; arrays may be reused once the stream reaches that point.
 *   - Return value: STEP_OK, or an error found on the host before anything was enqueued.
 *   - Errors only the device can see (a page id outside the pool, a length past the block-table
 *     row, a boundary row outside `hidden`, a NaN score, a refcount that would go negative) are
 *     reported in `*status` (device int32, caller-zeroed): the first non-zero code wins and stays.
 *     A call that reports such an error produces unspecified outputs but never reads or writes
 *     outside the arrays described here.  status may be NULL (errors are then dropped).
 *   - bf16 arrays are passed as uint16_t bit patterns.
 */
#ifndef STEP_H
#define STEP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum step_error {
    STEP_OK = 0,
    STEP_EINVAL = 1,     /* host: bad dimension, null or misaligned pointer, k > N              */
    STEP_EWORKSPACE = 2, /* host: workspace smaller than the matching *_workspace_bytes()       */
    STEP_ELAUNCH = 3,    /* host: the HIP runtime refused a launch (hipGetLastError was non-zero)*/
    STEP_EPAGE = 16,     /* device: block-table entry outside [0, NP) among a trace's used pages */
    STEP_ELEN = 17,      /* device: seq_lens[i] < 0 or > MAXB * P                                */
    STEP_EINDEX = 18,    /* device: boundary_idx outside [0, R) or trace_of outside [0, N)       */
    STEP_ENAN = 19,      /* device: NaN score on a live trace                                    */
    STEP_EREFCOUNT = 20, /* device: a released page had refcount <= 0                            */
    STEP_EKLIVE = 21,    /* device: k larger than the number of live traces                      */
    STEP_EPLAN = 22,     /* device: the workspace holds no shared-prefix lengths made for these dims */
    STEP_EFREELIST = 23  /* device: no free list in the workspace, or it disagrees with refcounts */
};

/* Human-readable name of an error code (host pointer to a static string). */
const char *step_strerror(int code);
/* Library version, "major.minor". */
const char *step_version(void);

/* ------------------------------------------------------------------------------------------ */
/* Paged grouped-query decode attention (the attention of NextToken in Algorithm 1).           */
/* ------------------------------------------------------------------------------------------ */

typedef struct {
    int32_t N;    /* traces, at most 2048                                                       */
    int32_t Hq;   /* query heads                                                                */
    int32_t Hkv;  /* KV heads; Hq % Hkv == 0, group size G = Hq / Hkv in {1, 2, 4, 8}           */
    int32_t D;    /* head dimension, 64 or 128                                                  */
    int32_t P;    /* tokens per page, must be 16                                                */
    int32_t MAXB; /* row width of block_tables                                                  */
    int32_t NP;   /* pages in the pool                                                          */
    float scale;  /* logit scale, normally 1/sqrt(D)                                            */
} step_attn_dims;

/* Bytes of workspace paged_decode_attn needs for these dims (host function, no device work). */
size_t step_attn_workspace_bytes(const step_attn_dims *dims);
/* Wavefronts per KV head that stage 1 keeps resident on the current device for these dims (host
 * function; 0 on bad dims): (compute units x resident waves per unit) / Hkv.  The work is cut so
 * that each of them streams the same number of pages.  The streaming kernels are built for one wave
 * per SIMD (four per compute unit).  The environment variable STEP_ATTN_WAVES_PER_CU, read once, overrides
 * the count (tuning aid; more than four per unit run as a second round). */
int32_t step_attn_waves_per_head(const step_attn_dims *dims);

/*
 * For every trace i with L = seq_lens[i] > 0 and every query head h (KV head g = h / G):
 *   x_t = scale * <q[i][h], K[page(t)][g][t % P]>,  t in [0, L),  page(t) = block_tables[i][t / P]
 *   out[i][h] = sum_t softmax(x)_t * V[page(t)][g][t % P]          rounded to bf16 (nearest even).
 * The query is the newest token, whose K/V row is already in the cache: L includes it, no mask.
 * A trace with L == 0 (pruned) gets a zero output row.  Pages may be shared between traces (the
 * prompt's); slots past a trace's last token and unreferenced pages are never read into a result.
 *
 *   q            [N][Hq][D]        bf16, 16-byte aligned
 *   k_pages      [NP][Hkv][P][D]   bf16, 16-byte aligned (one (page, head) tile is contiguous)
 *   v_pages      [NP][Hkv][P][D]   bf16, same layout, separate array
 *   block_tables [N][MAXB]         int32, -1 in unused entries
 *   seq_lens     [N]               int32
 *   out          [N][Hq][D]        bf16, written for every trace
 *   workspace    >= step_attn_workspace_bytes(dims), 256-byte aligned; holds split-K partials
 * Arithmetic: exact bf16 products, fp32 accumulation, fp32 running max and exponentials; the
 * softmax weights are rounded to bf16 before they multiply V (the normaliser is summed from the
 * same rounded weights).  Result within 2e-2
 * max-abs of the float64 definition for N(0,1) inputs.
 * Shared prompts: the traces are taken in blocks of 16 * QT / G consecutive indices (QT = 1 while the waves of a
 * KV head outnumber such blocks at least three to one, else 2); the leading block-table entries that every live trace of a block has in common (whole pages all
 * of them attend to completely, up to 1024) are found on the device and computed once per block on the
 * matrix cores.  The environment variable STEP_ATTN_PREFIX=0, read once, turns that off (testing aid: the
 * pages are then streamed per trace like private pages).  N * MAXB must stay below 2^30.
 */
int paged_decode_attn(const step_attn_dims *dims, const uint16_t *q, const uint16_t *k_pages,
                      const uint16_t *v_pages, const int32_t *block_tables, const int32_t *seq_lens,
                      uint16_t *out, void *workspace, size_t workspace_bytes, int32_t *status, void *stream);

/*
 * The same call in two halves, for a model with several layers: all layers of one decode step see the
 * same block_tables and seq_lens, so the per-block shared-prefix lengths are found once per step and every
 * layer's attention reuses them.  step_attn_plan finds them (and reports lengths outside the block-table
 * row) and leaves them, with a stamp of the dims, in `workspace`; paged_decode_attn_planned is
 * paged_decode_attn without that search and must be given the same dims, block_tables, seq_lens and
 * workspace, unchanged since (the layers run one after another on one stream and share the workspace).
 * On a workspace whose stamp is not the one of its dims it reports STEP_EPLAN (the output is then
 * unspecified; no access leaves the arrays).  Same arguments, layouts and errors as paged_decode_attn.
 */
int step_attn_plan(const step_attn_dims *dims, const int32_t *block_tables, const int32_t *seq_lens,
                   void *workspace, size_t workspace_bytes, int32_t *status, void *stream);
int paged_decode_attn_planned(const step_attn_dims *dims, const uint16_t *q, const uint16_t *k_pages,
                              const uint16_t *v_pages, const int32_t *block_tables, const int32_t *seq_lens,
                              uint16_t *out, void *workspace, size_t workspace_bytes, int32_t *status,
                              void *stream);

/* ------------------------------------------------------------------------------------------ */
/* Step scorer + running-mean trace score (Section 4.1 equation, Section 4.3 equation).        */
/* ------------------------------------------------------------------------------------------ */

enum step_activation { STEP_ACT_RELU = 0 /* the paper's (Table 5) */, STEP_ACT_GELU = 1 /* exact erf form */ };

typedef struct {
    int32_t R;   /* rows of hidden                                                              */
    int32_t d;   /* hidden size of the LLM, multiple of 128                                     */
    int32_t m;   /* width of the scorer's hidden layer, multiple of 16                          */
    int32_t B;   /* step boundaries in this call (may be 0)                                     */
    int32_t N;   /* traces (length of score_sum / score_cnt / scores); 0 if those are NULL      */
    int32_t act; /* enum step_activation                                                        */
} step_score_dims;

size_t step_score_workspace_bytes(const step_score_dims *dims);

/*
 * For b in [0, B): x = hidden[boundary_idx[b]];  z = W1 x + b1;  logits[b] = <W2, act(z)> + b2;
 * probs[b] = 1 / (1 + exp(-logits[b])).
 * Then, if the running-mean state is passed (score_sum and score_cnt not NULL; trace_of is then
 * required when B > 0), for b = 0 .. B-1 in this order: t = trace_of[b];
 * score_sum[t] += probs[b] (fp32); score_cnt[t] += 1; and finally, if scores is not NULL, for every
 * t in [0, N): scores[t] = score_cnt[t] > 0 ? score_sum[t] / score_cnt[t] (IEEE fp32 divide) : +inf
 * (a trace with no finished step yet is pruned after every scored one).
 *
 *   hidden [R][d] bf16 (16-byte aligned rows) | boundary_idx [B] int32 | W1 [m][d] bf16 row-major
 *   b1 [m] fp32 | W2 [m] bf16 | b2 [1] fp32 (device) | logits, probs [B] fp32
 *   trace_of [B] int32 | score_sum [N] fp32, score_cnt [N] int32 (in/out, or both NULL) | scores [N] fp32 or NULL
 * Arithmetic: bf16 products on the matrix cores with fp32 accumulation; the hidden activations
 * stay fp32.  logits within 1e-3 max-abs of the float64 definition.  m <= 16384.
 * One kernel launch: the workgroups that split W1 hand their sums over through `workspace` and through
 * arrival counters that belong to the library (device words that are zero between calls); every sum is
 * taken in a fixed order, so results are bit-identical from call to call.  Calls that may be in flight at
 * the same time (different streams, replays of different recorded graphs) must be given different
 * workspaces; the library keeps one counter set per workspace address, for the 64 most recently used
 * addresses, so such calls do not interfere as long as no more than 64 scorer workspaces are in use.
 */
int step_score(const step_score_dims *dims, const uint16_t *hidden, const int32_t *boundary_idx,
               const uint16_t *W1, const float *b1, const uint16_t *W2, const float *b2,
               float *logits, float *probs, const int32_t *trace_of, float *score_sum,
               int32_t *score_cnt, float *scores, void *workspace, size_t workspace_bytes,
               int32_t *status, void *stream);

/* ------------------------------------------------------------------------------------------ */
/* Prune the k lowest-scoring live traces and release their pages (Algorithm 1, k times).      */
/* ------------------------------------------------------------------------------------------ */

size_t step_prune_workspace_bytes(int32_t N, int32_t MAXB, int32_t NP);

/*
 * Live traces are those with seq_lens[i] > 0.  The k live traces with the smallest
 * (scores[i], i) are pruned (ties go to the lower index; -0 == +0), reported in that order.
 * For each pruned t and each j < ceil(seq_lens[t] / P): p = block_tables[t][j], refcounts[p] -= 1;
 * a page whose count reaches 0 is freed.  freed_pages receives the freed ids in ascending order,
 * *n_freed their number.  Then block_tables[t][*] = -1 and seq_lens[t] = 0.
 * k == 0 is a no-op (*n_freed = 0).  On a device-reported error the selection is abandoned
 * before any array is modified when the error is in the selection (STEP_ENAN, STEP_EKLIVE,
 * STEP_ELEN); a bad page id or refcount met during release is reported and that page skipped.
 *
 *   scores [N] fp32 | refcounts [NP] int32 in/out | block_tables [N][MAXB] int32 in/out
 *   seq_lens [N] int32 in/out | pruned [k] int32 out | freed_pages [min(NP, k*MAXB)] int32 out
 *   n_freed [1] int32 out | workspace >= step_prune_workspace_bytes(N, MAXB, NP)
 * Integer work only: every output is bit-exact with the definition.  N <= 4096.
 */
int prune_free(int32_t N, int32_t MAXB, int32_t NP, int32_t P, const float *scores, int32_t k,
               int32_t *refcounts, int32_t *block_tables, int32_t *seq_lens, int32_t *pruned,
               int32_t *freed_pages, int32_t *n_freed, void *workspace, size_t workspace_bytes,
               int32_t *status, void *stream);

/*
 * prune_free for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors
 * as prune_free, without `workspace`: the scratch of the kernels (a 256-byte header and the freed-page
 * bitmap, one bit per page) lives in a device array that is part of this library's code object,
 * 512 KiB + 256 bytes, held by every GPU the library runs on until the process ends.  It covers pools
 * of up to step_prune_static_max_pages() = 4194304 pages; a larger NP returns STEP_EWORKSPACE and
 * nothing is enqueued.  The call allocates and frees nothing.  Its first call on a device looks up the
 * array's address (not a stream operation; make that call outside graph capture).  All calls on one GPU
 * share the array: two calls that overlap in time on one GPU (different streams) race on it; calls
 * on one stream, or ordered by events, are safe, and every call clears what it needs cleared.
 */
int32_t step_prune_static_max_pages(void);
int prune_free_static(int32_t N, int32_t MAXB, int32_t NP, int32_t P, const float *scores, int32_t k,
                      int32_t *refcounts, int32_t *block_tables, int32_t *seq_lens, int32_t *pruned,
                      int32_t *freed_pages, int32_t *n_freed, int32_t *status, void *stream);

/* ------------------------------------------------------------------------------------------ */
/* Memory-triggered pruning + page allocation (Section 4.2; the GPUMemoryFull branch of         */
/* Algorithm 1), the KV-cache write of NextToken, and WeightedVote (Section 4.3).               */
/* With these a multi-step decode loop runs on the device with no host round trip:              */
/*   step_reserve_pages -> step_append_kv -> paged_decode_attn -> step_score                    */
/* ------------------------------------------------------------------------------------------ */

size_t step_reserve_workspace_bytes(int32_t N, int32_t MAXB, int32_t NP);

/*
 * The free pages of the pool are kept, from call to call, as a bitmap and a count in the workspace of
 * step_reserve_pages (a page is free when its reference count is 0; that remains the definition).
 *   step_freelist_rebuild  makes the free list from refcounts [NP]; call it once after the workspace has
 *                          been allocated and again whenever refcounts changed other than through
 *                          step_reserve_pages or step_freelist_add.
 *   step_freelist_add      enters the pages that a prune_free call reports as freed: freed_pages
 *                          [capacity], *n_freed (device) of them (STEP_EPAGE for an id outside the pool).
 * A call on a workspace that holds no free list for a pool of NP pages reports STEP_EFREELIST and changes
 * nothing.  Both calls need workspace >= step_reserve_workspace_bytes(0, 0, NP).
 */
int step_freelist_rebuild(int32_t NP, const int32_t *refcounts, void *workspace, size_t workspace_bytes, void *stream);
int step_freelist_add(int32_t NP, const int32_t *freed_pages, const int32_t *n_freed, int32_t capacity,
                      void *workspace, size_t workspace_bytes, int32_t *status, void *stream);

/*
 * Before the next decode step: a live trace with seq_lens[i] % P == 0 needs a new page for its next
 * token.  While fewer pages are free (refcount 0) than traces need one, the live trace with the
 * smallest (scores[i], i) is pruned exactly as prune_free prunes one trace (pages released, row set
 * to -1, seq_len 0): the memory trigger of Section 4.2 / the GPUMemoryFull branch of Algorithm 1,
 * read as "the pool cannot hold the pages the next decode step opens".  Then every trace that
 * still needs a page, in ascending index, takes the smallest free page id:
 * block_tables[i][seq_lens[i] / P] = page, refcounts[page] = 1, new_pages[i] = page.
 * The free pages are read from, and kept up to date in, the free list of the workspace (above): a step
 * that prunes nothing costs a scan of NP / 32 bitmap words, and none at all when no trace needs a page.
 *
 *   scores [N] fp32 | refcounts [NP], block_tables [N][MAXB], seq_lens [N] int32 in/out
 *   pruned [N] int32 out (first *n_pruned entries, pruning order) | n_pruned [1] int32 out
 *   new_pages [N] int32 out (-1 where no page was given) | workspace >= step_reserve_workspace_bytes
 * Device-reported errors: STEP_EFREELIST (no free list in the workspace: nothing is modified; or a page the
 * list calls free has a non-zero reference count: that page is skipped), STEP_ELEN (bad length, or a trace
 * on a page boundary whose row is full), STEP_ENAN (pruning needed and a live score is NaN) -- both before
 * anything is modified; STEP_EPAGE / STEP_EREFCOUNT while releasing (that entry is skipped).  N <= 4096.
 */
int step_reserve_pages(int32_t N, int32_t MAXB, int32_t NP, int32_t P, const float *scores,
                       int32_t *refcounts, int32_t *block_tables, int32_t *seq_lens, int32_t *pruned,
                       int32_t *n_pruned, int32_t *new_pages, void *workspace, size_t workspace_bytes,
                       int32_t *status, void *stream);

/*
 * For every live trace i (L = seq_lens[i] > 0): the K and V rows of its newest token,
 * k_new[i][g][:], v_new[i][g][:], are written to page block_tables[i][L / P], slot L % P, of every
 * KV head g, and seq_lens[i] becomes L + 1.  dims: N, Hkv, D (multiple of 8), P = 16, MAXB, NP are
 * used.  k_new, v_new [N][Hkv][D] bf16, 16-byte aligned.  refcounts may be NULL; when given, a
 * target page with refcount != 1 is refused (STEP_EREFCOUNT): a shared page is never written.
 * Device-reported errors skip that trace: STEP_ELEN (row full), STEP_EPAGE, STEP_EREFCOUNT.
 */
int step_append_kv(const step_attn_dims *dims, const uint16_t *k_new, const uint16_t *v_new,
                   uint16_t *k_pages, uint16_t *v_pages, const int32_t *block_tables,
                   const int32_t *refcounts, int32_t *seq_lens, int32_t *status, void *stream);

/*
 * answer[i] >= 0 is the final answer id of trace i, -1 means it has none (pruned, unfinished).  The
 * weight of an answer is the fp32 sum, in trace index order, of scores[j] over the traces that gave
 * it; *winner is the answer with the largest weight (ties: smallest id; -1 if nobody answered) and
 * *weight its weight.  STEP_ENAN if a voting trace's score is NaN.  N <= 4096.
 */
int step_weighted_vote(int32_t N, const int32_t *answer, const float *scores, int32_t *winner,
                       float *weight, int32_t *status, void *stream);

/* ------------------------------------------------------------------------------------------ */
/* Measurement aid: a plain copy kernel of known size (dst[i] = src[i], 16-byte units), used   */
/* to calibrate profiler byte counters against known traffic.  bytes % 16 == 0.               */
/* ------------------------------------------------------------------------------------------ */
int step_calib_copy(void *dst, const void *src, size_t bytes, void *stream);

/* ------------------------------------------------------------------------------------------ */
/* Measurement aid: a bare read of KV tiles, to see what the memory system delivers to the       */
/* access pattern of attention's streaming kernel with no arithmetic behind it.  k_pages and     */
/* v_pages are pools [NP][Hkv][16][128] bf16 (4096-byte tiles).  `waves` x Hkv single-wave        */
/* workgroups are launched; wave (w, g) reads the K and V tiles of KV head g of the pages          */
/* page_ids[w * pages_per_wave .. + pages_per_wave) (device int32; ids outside [0, NP) read page */
/* 0), two pages in flight.  pattern 0: 1 KB contiguous per load instruction; 1: the matrix-core */
/* operand pattern.  nontemporal != 0: streaming (non-temporal) loads.  sink: one device word.   */
/* ------------------------------------------------------------------------------------------ */
int step_read_probe(const void *k_pages, const void *v_pages, const int32_t *page_ids, int32_t waves,
                    int32_t pages_per_wave, int32_t Hkv, int32_t NP, int32_t pattern, int32_t nontemporal,
                    uint32_t *sink, void *stream);

/* ------------------------------------------------------------------------------------------ */
/* Measurement aid: the duration of every kernel the library launches.                          */
/* After step_profile_begin(cap), each of the next `cap` kernel launches of any entry point      */
/* carries two HIP events (from a pool of `cap` pairs created by that call) that take the         */
/* kernel's begin and end timestamps on the stream it runs on; later launches are not timed.     */
/* step_profile_end waits for the recorded events, writes for launch j < n, in launch order, the */
/* kernel's id to kernel_ids[j] and its duration in milliseconds to ms[j] (HOST arrays of         */
/* capacity cap), destroys the pool and returns n, or -STEP_EINVAL.                              */
/* step_profile_kernel_name maps an id to a name (host pointer to a static string).              */
/* Benchmark use only: not thread safe, creates and destroys events, not for graph capture.      */
/* ------------------------------------------------------------------------------------------ */
int step_profile_begin(int cap);
int step_profile_end(int32_t *kernel_ids, float *ms, int cap);
const char *step_profile_kernel_name(int id);

#ifdef __cplusplus
}
#endif
#endif /* STEP_H */
