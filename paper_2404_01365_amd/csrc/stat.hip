// Relative activations and the statistic s (Section 4.1 and Eq. 6), and the batch-shared
// statistic of Eq. 7.
//
//   r_i^2 = sum_j Z_ij^2            (row i of Z scaled by 1/r_i is the "relative activation")
//   s_j   = sqrt( sum_{i in sequence} Z_ij^2 / r_i^2 )
//
// r_i^2 needs the whole row, so the scaling cannot finish inside one tile of the GEMM that
// makes Z: the GEMM's epilogue leaves one sum-of-squares partial per (row, column tile), the
// kernel here turns them into the weights w_i = 1/r_i^2 (0 for an all-zero row) and streams Z once
// more, coalesced along the neuron axis, to accumulate sum_i w_i Z_ij^2.  The tokens of every
// sequence are cut into chunks of the same number of rows (so that prompts of different lengths
// give workgroups of the same size: with the same number of chunks per prompt the long prompts'
// workgroups ran on alone while most of the chip sat idle), handled by different workgroups; a last
// small kernel adds a sequence's chunk partials in a fixed order and takes the square root.  All of
// it is bandwidth-bound: S*F fp32 reads.
#include "common.h"

namespace griffin {

// first chunk of every sequence in the global list of chunks (sequence b owns chunks first[b] .. first[b+1]-1)
struct ChunkTable {
    int32_t first[GRIFFIN_MAX_SEQS + 1];
};

// s2part[chunk][j] = sum over the chunk's rows of w_i Z_ij^2, w_i = 1 / sum_t rowpart[i][t] (0 for an all-zero
// row).  A workgroup first turns the row partials of its own rows into weights (one wavefront per row: lanes
// over the column tiles, then a wave sum; every column block of a chunk repeats this for the same few rows,
// which is far cheaper than a kernel of its own in front of this one) and keeps them in LDS.
constexpr int STAT_ROWS_LDS = 256;

template <int VEC>
__global__ __launch_bounds__(256) void col_stat_kernel(const float *Z, int64_t ldz, const float *rowpart, int nt, int F,
                                                       SeqTable seqs, ChunkTable chunks, int rows_per_chunk, float *s2part)
{
    __shared__ float w_s[STAT_ROWS_LDS];
    const int g = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = (blockIdx.x * 256 + threadIdx.x) * VEC;
    const bool live = j < F;
    const int jc = live ? j : 0;              // columns past the end: loads stay in bounds, nothing is stored
    // the sequence this chunk belongs to: the last b with first[b] <= g (empty sequences own no chunk)
    int b0 = 0, b1 = seqs.n;
    while (b1 - b0 > 1) {
        const int mid = (b0 + b1) >> 1;
        if (chunks.first[mid] <= g) b0 = mid; else b1 = mid;
    }
    const int64_t lo = (int64_t)seqs.cu[b0] + (int64_t)(g - chunks.first[b0]) * rows_per_chunk;
    const int64_t end = seqs.cu[b0 + 1];
    const int64_t hi = lo + rows_per_chunk < end ? lo + rows_per_chunk : end;
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v)
        acc[v] = 0.0f;
    for (int64_t r0 = lo; r0 < hi; r0 += STAT_ROWS_LDS) {
        const int nr = (int)(hi - r0 < STAT_ROWS_LDS ? hi - r0 : STAT_ROWS_LDS);
        __syncthreads();                       // the weights of the block before have been used
        for (int r = wave; r < nr; r += 4) {
            const float *rp = rowpart + (r0 + r) * nt;
            float a = 0.0f;
            for (int t = lane; t < nt; t += 64)
                a += rp[t];
            a = wave_sum(a);
            if (lane == 0)
                w_s[r] = a > 0.0f ? 1.0f / a : 0.0f;
        }
        __syncthreads();
        const float *zp = Z + r0 * ldz + jc;
        int i = 0;
        for (; i + 4 <= nr; i += 4) {
            float zz[4][VEC], ww[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                ww[r] = w_s[i + r];
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
        for (; i < nr; ++i) {
            const float wi = w_s[i];
#pragma unroll
            for (int v = 0; v < VEC; ++v)
                acc[v] = fmaf(zp[v] * zp[v], wi, acc[v]);
            zp += ldz;
        }
    }
    if (live) {
        float *o = s2part + (int64_t)g * F + j;
#pragma unroll
        for (int v = 0; v < VEC; ++v)
            o[v] = acc[v];
    }
}

// s[seq][j] = sqrt(sum of the sequence's chunk partials s2part[chunk][j]) in ascending chunk order
// (one wavefront per 64 columns so that the few columns still fill the chip; eight loads in flight
// per lane, added in chunk order); a sequence without tokens has no chunk and gets s = 0
__global__ __launch_bounds__(64) void stat_finalize_kernel(const float *s2part, ChunkTable chunks, int F, float *s,
                                                           float *s_out)
{
    const int seq = blockIdx.y;
    const int j = blockIdx.x * 64 + threadIdx.x;
    if (j >= F)
        return;
    const int c0 = chunks.first[seq], rc = chunks.first[seq + 1] - c0;
    const float *p = s2part + (int64_t)c0 * F + j;
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

// Rows per chunk, the same for every sequence: enough chunks over all sequences to fill the chip
// (about eight workgroups per CU), at least 16 rows each.
int stat_rows_per_chunk(int64_t total_tokens, int32_t F)
{
    const int64_t col_blocks = (F + 1023) / 1024;
    const int64_t target = 2048 / col_blocks > 1 ? 2048 / col_blocks : 1;
    const int64_t rows = (total_tokens + target - 1) / target;
    return (int)(rows < 16 ? 16 : (rows > (1 << 20) ? (1 << 20) : rows));
}

// upper bound of the number of chunks of any split of total_tokens into n_seqs sequences
int64_t stat_max_chunks(int64_t total_tokens, int32_t n_seqs, int32_t F)
{
    return total_tokens / stat_rows_per_chunk(total_tokens, F) + n_seqs;
}

int launch_stat(const float *Z, int64_t ldz, const float *rowpart, int nt, int64_t M, int32_t F,
                const SeqTable &seqs, float *s2part, float *s, float *s_out, hipStream_t st)
{
    int rcode;
    const int R = stat_rows_per_chunk(M, F);
    ChunkTable chunks;
    int32_t n_chunks = 0;
    for (int b = 0; b < seqs.n; ++b) {
        chunks.first[b] = n_chunks;
        n_chunks += (int32_t)(((int64_t)seqs.cu[b + 1] - seqs.cu[b] + R - 1) / R);
    }
    for (int b = seqs.n; b <= GRIFFIN_MAX_SEQS; ++b)
        chunks.first[b] = n_chunks;
    if (n_chunks > 0) {
        const bool vec4 = (F % 4 == 0) && (ldz % 4 == 0) && (((uintptr_t)Z & 15) == 0);
        if (vec4) {
            dim3 grid((F / 4 + 255) / 256, n_chunks);
            hipLaunchKernelGGL(col_stat_kernel<4>, grid, dim3(256), 0, st, Z, ldz, rowpart, nt, F, seqs, chunks, R, s2part);
        } else {
            dim3 grid((F + 255) / 256, n_chunks);
            hipLaunchKernelGGL(col_stat_kernel<1>, grid, dim3(256), 0, st, Z, ldz, rowpart, nt, F, seqs, chunks, R, s2part);
        }
        if ((rcode = check_launch("col_stat_kernel")) != GRIFFIN_OK)
            return rcode;
    }
    hipLaunchKernelGGL(stat_finalize_kernel, dim3((F + 63) / 64, seqs.n), dim3(64), 0, st, s2part, chunks, F, s, s_out);
    return check_launch("stat_finalize_kernel");
}

int launch_stat_shared(const float *s, const SeqTable &seqs, int32_t n, float *sbar, hipStream_t st)
{
    hipLaunchKernelGGL(stat_shared_kernel, dim3((n + 255) / 256), dim3(256), 0, st, s, seqs, n, sbar);
    return check_launch("stat_shared_kernel");
}

}  // namespace griffin
