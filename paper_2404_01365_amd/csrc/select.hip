// Selectors other than the prompt statistic, and the similarity of selected sets.
//
//  * weight_norm_kernel: the static score of the paper's magnitude baseline (Section 5.1,
//    "Setup"): ||W1_j||_2, times ||Wg_j||_2 for GLU blocks.  One wavefront per neuron, 16-byte
//    non-temporal loads (the weights pass once), fp32 sums: a single pass over 2*F*d weights,
//    bandwidth-bound.
//  * sample_score_kernel / sample_mark_kernel: sampling-based selection (Appendix B).  Weighted
//    sampling without replacement is run as exponential clocks: neuron j rings at e_j / s_j with
//    e_j a unit exponential variate supplied by the caller; the earliest rings win.  The order
//    is decided on q_j = s_j / e_j (IEEE single-precision division, capped at 1e38), largest
//    first, so the exact top-k kernel does the draw; neurons already taken by the top-k half
//    are marked 3e38 and come first.
//  * jaccard_kernel: |A n B| / |A u B| for every pair of ascending index lists (Section 4.1).
#include "common.h"

namespace griffin {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_s;
typedef __attribute__((ext_vector_type(4))) float f32x4_s;

template <bool BF16>
__global__ __launch_bounds__(256) void weight_norm_kernel(const void *W1, const void *Wg, int64_t ld, int n, int d,
                                                          float *score)
{
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= n)
        return;
    float a = 0.0f, b = 0.0f;
    if (BF16) {
        const uint16_t *r1 = (const uint16_t *)W1 + (int64_t)j * ld;
        const uint16_t *rg = Wg ? (const uint16_t *)Wg + (int64_t)j * ld : nullptr;
        for (int c = lane * 8; c < d; c += 512) {       // d is a multiple of 8
            const u32x4_s v = __builtin_nontemporal_load((const u32x4_s *)(r1 + c));
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float lo = __uint_as_float(v[t] << 16), hi = __uint_as_float(v[t] & 0xFFFF0000u);
                a = fmaf(lo, lo, a);
                a = fmaf(hi, hi, a);
            }
            if (rg) {
                const u32x4_s g = __builtin_nontemporal_load((const u32x4_s *)(rg + c));
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float lo = __uint_as_float(g[t] << 16), hi = __uint_as_float(g[t] & 0xFFFF0000u);
                    b = fmaf(lo, lo, b);
                    b = fmaf(hi, hi, b);
                }
            }
        }
    } else {
        const float *r1 = (const float *)W1 + (int64_t)j * ld;
        const float *rg = Wg ? (const float *)Wg + (int64_t)j * ld : nullptr;
        for (int c = lane * 4; c < d; c += 256) {       // d is a multiple of 8
            const f32x4_s v = *(const f32x4_s *)(r1 + c);
            a = fmaf(v[0], v[0], a); a = fmaf(v[1], v[1], a); a = fmaf(v[2], v[2], a); a = fmaf(v[3], v[3], a);
            if (rg) {
                const f32x4_s g = *(const f32x4_s *)(rg + c);
                b = fmaf(g[0], g[0], b); b = fmaf(g[1], g[1], b); b = fmaf(g[2], g[2], b); b = fmaf(g[3], g[3], b);
            }
        }
    }
    a = wave_sum(a);
    b = wave_sum(b);
    if (lane == 0)
        score[j] = Wg ? sqrtf(a) * sqrtf(b) : sqrtf(a);
}

__global__ __launch_bounds__(256) void sample_score_kernel(const float *s, const float *e, int n, float *q)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j < n)
        q[j] = fminf(s[j] / e[j], 1.0e38f);
}

__global__ __launch_bounds__(256) void sample_mark_kernel(const int32_t *idx_top, int k_top, int n, float *q)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < k_top) {
        const int j = idx_top[t];
        if (j >= 0 && j < n)
            q[j] = 3.0e38f;
    }
}

// one workgroup per ordered pair (a, b); the matrix is symmetric and its diagonal is 1
__global__ __launch_bounds__(256) void jaccard_kernel(const int32_t *idx, int n_sets, int k, float *out)
{
    __shared__ int sh[4];
    const int a = blockIdx.x / n_sets, b = blockIdx.x % n_sets;
    const int32_t *A = idx + (int64_t)a * k, *B = idx + (int64_t)b * k;
    int cnt = 0;
    for (int i = threadIdx.x; i < k; i += 256) {
        const int32_t v = A[i];
        int lo = 0, hi = k;                    // first position of B not below v
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (B[mid] < v) lo = mid + 1; else hi = mid;
        }
        cnt += (lo < k && B[lo] == v) ? 1 : 0;
    }
    cnt = (int)wave_sum((float)cnt);           // k <= 2^20, exact in fp32
    if ((threadIdx.x & 63) == 0)
        sh[threadIdx.x >> 6] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int inter = sh[0] + sh[1] + sh[2] + sh[3];
        const int uni = 2 * k - inter;
        out[(int64_t)a * n_sets + b] = uni > 0 ? (float)inter / (float)uni : 1.0f;
    }
}

int launch_weight_norm(const griffin_layer &L, float *score, hipStream_t st)
{
    dim3 grid((L.n + 3) / 4), block(256);
    if (L.dtype == GRIFFIN_BF16)
        hipLaunchKernelGGL(weight_norm_kernel<true>, grid, block, 0, st, L.W1, L.Wg, L.ld, L.n, L.d, score);
    else
        hipLaunchKernelGGL(weight_norm_kernel<false>, grid, block, 0, st, L.W1, L.Wg, L.ld, L.n, L.d, score);
    return check_launch("weight_norm_kernel");
}

int launch_select_sampled(const float *s, const float *e, int32_t n, int32_t k, int32_t k_top, int32_t *idx_out,
                          float *q, int32_t *idx_top, hipStream_t st)
{
    int rc;
    hipLaunchKernelGGL(sample_score_kernel, dim3((n + 255) / 256), dim3(256), 0, st, s, e, n, q);
    if ((rc = check_launch("sample_score_kernel")) != GRIFFIN_OK)
        return rc;
    if (k_top > 0) {
        if ((rc = launch_topk(s, 1, n, k_top, idx_top, st)) != GRIFFIN_OK)
            return rc;
        hipLaunchKernelGGL(sample_mark_kernel, dim3((k_top + 255) / 256), dim3(256), 0, st, idx_top, k_top, n, q);
        if ((rc = check_launch("sample_mark_kernel")) != GRIFFIN_OK)
            return rc;
    }
    return launch_topk(q, 1, n, k, idx_out, st);
}

int launch_jaccard(const int32_t *idx, int32_t n_sets, int32_t k, float *out, hipStream_t st)
{
    hipLaunchKernelGGL(jaccard_kernel, dim3(n_sets * n_sets), dim3(256), 0, st, idx, n_sets, k, out);
    return check_launch("jaccard_kernel");
}

}  // namespace griffin
