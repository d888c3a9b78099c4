// Relative activations and the statistic s (Section 4.1 and Eq. 6), and the batch-shared
// statistic of Eq. 7.
//
//   r_i^2 = sum_j Z_ij^2            (row i of Z scaled by 1/r_i is the "relative activation")
//   s_j   = sqrt( sum_{i in sequence} Z_ij^2 / r_i^2 )
//
// r_i^2 needs the whole row, so the scaling cannot finish inside one tile of the GEMM that
// makes Z: the GEMM's epilogue leaves one sum-of-squares partial per (row, column tile), this
// file turns them into the weights w_i = 1/r_i^2 (0 for an all-zero row) and streams Z once
// more, coalesced along the neuron axis, to accumulate sum_i w_i Z_ij^2.  The token range of
// every sequence is cut into `rc` chunks handled by different workgroups; a last small kernel
// adds the chunk partials in a fixed order and takes the square root.  All of it is
// bandwidth-bound: S*F fp32 reads.
#include "common.h"

namespace griffin {

// w[i] = 1 / sum_t rowpart[i][t]; one wavefront per row
__global__ __launch_bounds__(256) void row_weight_kernel(const float *rowpart, int nt, int64_t M, float *w)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= M)
        return;
    float acc = 0.0f;
    for (int t = lane; t < nt; t += 64)
        acc += rowpart[i * nt + t];
    acc = wave_sum(acc);
    if (lane == 0)
        w[i] = acc > 0.0f ? 1.0f / acc : 0.0f;
}

// s2part[seq][chunk][j] = sum over the chunk's rows of w_i Z_ij^2
template <int VEC>
__global__ __launch_bounds__(256) void col_stat_kernel(const float *Z, int64_t ldz, const float *w, int F,
                                                       SeqTable seqs, int rc, float *s2part)
{
    const int seq = blockIdx.z, chunk = blockIdx.y;
    const int j = (blockIdx.x * 256 + threadIdx.x) * VEC;
    if (j >= F)
        return;
    const int64_t lo0 = seqs.cu[seq], len = seqs.cu[seq + 1] - lo0;
    const int64_t lo = lo0 + len * chunk / rc, hi = lo0 + len * (chunk + 1) / rc;
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v)
        acc[v] = 0.0f;
    const float *zp = Z + lo * ldz + j;
    int64_t i = lo;
    for (; i + 4 <= hi; i += 4) {
        float zz[4][VEC], ww[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            ww[r] = w[i + r];
            if (VEC == 4) {
                float4 t = *(const float4 *)(zp + r * ldz);
                zz[r][0] = t.x; zz[r][1 % VEC] = t.y; zz[r][2 % VEC] = t.z; zz[r][3 % VEC] = t.w;
            } else {
                zz[r][0] = zp[r * ldz];
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int v = 0; v < VEC; ++v)
                acc[v] = fmaf(zz[r][v] * zz[r][v], ww[r], acc[v]);
        zp += 4 * ldz;
    }
    for (; i < hi; ++i) {
        const float wi = w[i];
#pragma unroll
        for (int v = 0; v < VEC; ++v)
            acc[v] = fmaf(zp[v] * zp[v], wi, acc[v]);
        zp += ldz;
    }
    float *o = s2part + ((int64_t)seq * rc + chunk) * F + j;
#pragma unroll
    for (int v = 0; v < VEC; ++v)
        o[v] = acc[v];
}

// s[seq][j] = sqrt(sum_chunk s2part[seq][chunk][j]) in ascending chunk order
// (one wavefront per 64 columns so that the few columns still fill the chip; eight loads in flight
// per lane, added in chunk order)
__global__ __launch_bounds__(64) void stat_finalize_kernel(const float *s2part, int rc, int F, float *s,
                                                           float *s_out)
{
    const int seq = blockIdx.y;
    const int j = blockIdx.x * 64 + threadIdx.x;
    if (j >= F)
        return;
    const float *p = s2part + (int64_t)seq * rc * F + j;
    float acc = 0.0f;
    int c = 0;
    for (; c + 8 <= rc; c += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = p[(int64_t)(c + u) * F];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            acc += v[u];
    }
    for (; c < rc; ++c)
        acc += p[(int64_t)c * F];
    const float v = sqrtf(acc);
    s[(int64_t)seq * F + j] = v;
    if (s_out)
        s_out[(int64_t)seq * F + j] = v;
}

// Eq. 7: sbar_j = sum_b s[b][j] / sqrt(S_b), b ascending, empty sequences skipped
__global__ __launch_bounds__(256) void stat_shared_kernel(const float *s, SeqTable seqs, int F, float *sbar)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= F)
        return;
    float acc = 0.0f;
    for (int b = 0; b < seqs.n; ++b) {
        const int len = seqs.cu[b + 1] - seqs.cu[b];
        if (len > 0)
            acc += s[(int64_t)b * F + j] / sqrtf((float)len);
    }
    sbar[j] = acc;
}

// number of token chunks per sequence: enough workgroups to fill the chip, at least ~16 rows each
int stat_row_chunks(int64_t total_tokens, int32_t n_seqs, int32_t F)
{
    const int64_t col_blocks = (F + 1023) / 1024;
    int64_t want = 2048 / (col_blocks * (n_seqs > 0 ? n_seqs : 1));
    const int64_t avg = total_tokens / (n_seqs > 0 ? n_seqs : 1);
    if (want > avg / 16)
        want = avg / 16;
    if (want > 64)
        want = 64;
    return want < 1 ? 1 : (int)want;
}

int launch_stat(const float *Z, int64_t ldz, const float *rowpart, int nt, int64_t M, int32_t F,
                const SeqTable &seqs, int rc, float *w, float *s2part, float *s, float *s_out,
                hipStream_t st)
{
    int rcode;
    if (M > 0) {
        hipLaunchKernelGGL(row_weight_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, st, rowpart, nt, M, w);
        if ((rcode = check_launch("row_weight_kernel")) != GRIFFIN_OK)
            return rcode;
    }
    const bool vec4 = (F % 4 == 0) && (ldz % 4 == 0) && (((uintptr_t)Z & 15) == 0);
    if (vec4) {
        dim3 grid((F / 4 + 255) / 256, rc, seqs.n);
        hipLaunchKernelGGL(col_stat_kernel<4>, grid, dim3(256), 0, st, Z, ldz, w, F, seqs, rc, s2part);
    } else {
        dim3 grid((F + 255) / 256, rc, seqs.n);
        hipLaunchKernelGGL(col_stat_kernel<1>, grid, dim3(256), 0, st, Z, ldz, w, F, seqs, rc, s2part);
    }
    if ((rcode = check_launch("col_stat_kernel")) != GRIFFIN_OK)
        return rcode;
    hipLaunchKernelGGL(stat_finalize_kernel, dim3((F + 63) / 64, seqs.n), dim3(64), 0, st, s2part, rc, F, s, s_out);
    return check_launch("stat_finalize_kernel");
}

int launch_stat_shared(const float *s, const SeqTable &seqs, int32_t n, float *sbar, hipStream_t st)
{
    hipLaunchKernelGGL(stat_shared_kernel, dim3((n + 255) / 256), dim3(256), 0, st, s, seqs, n, sbar);
    return check_launch("stat_shared_kernel");
}

}  // namespace griffin
