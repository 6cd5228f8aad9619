// step_score: the step scorer y = sigma(W2 act(W1 h + b1) + b2) of Section 4.1 ("Model
// Architecture"; Table 5 fixes act = ReLU, hidden width 512) on the hidden states of the traces at a
// step boundary, followed by the running-average trace score of Section 4.3 ("Update score_t" in
// Algorithm 1).
//
// score_hidden: the dense projection W1 X^T on the matrix cores (v_mfma_f32_16x16x32_bf16).  One
//   workgroup owns 16 rows of W1 (one MFMA tile of hidden units) and up to 32 boundaries; its
//   sixteen waves split the contraction over d, 128 values per iteration, and are summed through LDS.  The
//   gather hidden[boundary_idx[b]] is fused into the B-operand loads.  Bias, activation and the
//   product with the 16 matching entries of W2 follow in registers; the workgroup writes one
//   partial logit per boundary.
// score_finish: adds the partial logits in a fixed order, applies the sigmoid, then one thread
//   replays the boundaries in index order to update (sum, count) per trace -- fp32 addition is
//   not associative and a trace may own several boundaries, so the order is part of the result.
#include "common.h"

namespace step {
namespace {

constexpr int kWaves = 16;  // the contraction over d is split over the waves of a workgroup
constexpr int kBT = 2;  // boundary tiles (of 16) per workgroup

struct ScoreArgs {
    const uint16_t *hidden, *W1, *W2;
    const int32_t *boundary_idx, *trace_of;
    const float *b1, *b2;
    float *logits, *probs, *score_sum, *scores, *partial;  // partial [m/16][B]
    int32_t *score_cnt, *status;
    int R, d, m, B, N, act;
};

__device__ __forceinline__ float activate(float z, int act)
{
    if (act == STEP_ACT_RELU) return fmaxf(z, 0.f);
    return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
}

__global__ __launch_bounds__(64 * kWaves) void score_hidden(const ScoreArgs a)
{
    __shared__ float red[kWaves][kBT][4][64];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int row16 = lane & 15, kg = lane >> 4;
    const int m0 = blockIdx.x * 16;
    const int b0 = blockIdx.y * (16 * kBT);

    // rows of `hidden` feeding the B operand of each boundary tile (column = lane % 16)
    const uint16_t *xrow[kBT];
#pragma unroll
    for (int t = 0; t < kBT; ++t) {
        const int b = b0 + t * 16 + row16;
        int rix = 0;
        if (b < a.B) {
            rix = a.boundary_idx[b];
            if ((u32)rix >= (u32)a.R) {
                if (blockIdx.x == 0 && kg == 0 && w == 0) report(a.status, STEP_EINDEX);
                rix = 0;
            }
        }
        xrow[t] = a.hidden + (size_t)rix * a.d;
    }
    const bool tile1 = (b0 + 16 < a.B);  // wave-uniform: second boundary tile in use
    const uint16_t *wrow = a.W1 + (size_t)(m0 + row16) * a.d;

    f32x4 c0 = {0.f, 0.f, 0.f, 0.f}, c1 = {0.f, 0.f, 0.f, 0.f};
    const int iters = a.d / 128;
    for (int it = w; it < iters; it += kWaves) {
        // the contraction index is permuted identically for both operands: lane group kg takes the
        // 32 consecutive values kbase + 32 kg .. +32, eight per MFMA, so a lane reads 64 contiguous
        // bytes per iteration and the four groups cover 256 contiguous bytes of the row
        const int kbase = it * 128 + kg * 32;
        const uint4 *wp = reinterpret_cast<const uint4 *>(wrow + kbase);
        const uint4 *x0 = reinterpret_cast<const uint4 *>(xrow[0] + kbase);
        const uint4 *x1 = reinterpret_cast<const uint4 *>(xrow[1] + kbase);
        uint4 av[4], bv0[4], bv1[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) av[s] = wp[s];
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
    if (w < kBT) {
        const int b = b0 + w * 16 + row16;
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = m0 + kg * 4 + i;
            float z = a.b1[row];
#pragma unroll
            for (int ww = 0; ww < kWaves; ++ww) z += red[ww][w][i][lane];
            s = fmaf(bf16_lo((u32)a.W2[row]), activate(z, a.act), s);
        }
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        if (kg == 0 && b < a.B) a.partial[(size_t)blockIdx.x * a.B + b] = s;
    }
}

constexpr int kFinishThreads = 256;
constexpr int kFinishChunk = 1024;  // boundaries whose (trace, prob) are staged in LDS at a time
constexpr int kStateMax = 2048;     // traces whose (sum, count) state is staged in LDS

__global__ __launch_bounds__(kFinishThreads) void score_finish(const ScoreArgs a)
{
    __shared__ float prob_s[kFinishChunk];
    __shared__ int trace_s[kFinishChunk];
    __shared__ float sum_s[kStateMax];
    __shared__ int cnt_s[kStateMax];
    const int tid = threadIdx.x;
    const int mt = a.m / 16;
    const float b2 = a.b2[0];
    const bool state = a.score_sum != nullptr;
    const bool staged = state && a.N <= kStateMax;  // keep the sequential replay off global memory
    if (staged)
        for (int t = tid; t < a.N; t += kFinishThreads) {
            sum_s[t] = a.score_sum[t];
            cnt_s[t] = a.score_cnt[t];
        }
    for (int base = 0; base < a.B; base += kFinishChunk) {
        const int nbd = min(kFinishChunk, a.B - base);
        for (int bb = tid; bb < nbd; bb += kFinishThreads) {
            const int b = base + bb;
            // partial logits are summed in a fixed order, four independent accumulators in flight
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
            int t = 0;
            for (; t + 3 < mt; t += 4) {
                s0 += a.partial[(size_t)(t + 0) * a.B + b];
                s1 += a.partial[(size_t)(t + 1) * a.B + b];
                s2 += a.partial[(size_t)(t + 2) * a.B + b];
                s3 += a.partial[(size_t)(t + 3) * a.B + b];
            }
            for (; t < mt; ++t) s0 += a.partial[(size_t)t * a.B + b];
            const float logit = b2 + ((s0 + s1) + (s2 + s3));
            const float prob = 1.0f / (1.0f + expf(-logit));
            a.logits[b] = logit;
            a.probs[b] = prob;
            prob_s[bb] = prob;
            trace_s[bb] = state ? a.trace_of[b] : 0;
        }
        if (!state) continue;  // uniform
        __syncthreads();
        if (tid == 0) {
            // boundaries in index order: fp32 addition is not associative and a trace may own several
            for (int bb = 0; bb < nbd; ++bb) {
                const int t = trace_s[bb];
                if ((u32)t >= (u32)a.N) {
                    report(a.status, STEP_EINDEX);
                    continue;
                }
                if (staged) {
                    sum_s[t] = sum_s[t] + prob_s[bb];
                    cnt_s[t] = cnt_s[t] + 1;
                } else {
                    a.score_sum[t] = a.score_sum[t] + prob_s[bb];
                    a.score_cnt[t] = a.score_cnt[t] + 1;
                }
            }
        }
        __syncthreads();
    }
    if (!state) return;
    __threadfence_block();
    __syncthreads();
    for (int t = tid; t < a.N; t += kFinishThreads) {
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

bool dims_ok(const step_score_dims *d)
{
    if (!d) return false;
    if (d->R < 0 || d->d <= 0 || d->m <= 0 || d->B < 0 || d->N < 0) return false;
    if (d->d % 128 || d->m % 16) return false;
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
    return (((size_t)(d->m / 16) * (size_t)(d->B > 0 ? d->B : 1) * sizeof(float)) + 255) & ~(size_t)255;
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
    a.partial = reinterpret_cast<float *>(workspace);
    a.score_cnt = score_cnt; a.status = status;
    a.R = d->R; a.d = d->d; a.m = d->m; a.B = d->B; a.N = d->N; a.act = d->act;

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (d->B > 0) {
        const dim3 grid(d->m / 16, (d->B + 16 * kBT - 1) / (16 * kBT));
        hipLaunchKernelGGL(score_hidden, grid, dim3(64 * kWaves), 0, s, a);
    }
    if (d->B > 0 || (state && scores)) hipLaunchKernelGGL(score_finish, dim3(1), dim3(kFinishThreads), 0, s, a);
    return launch_status();
}
