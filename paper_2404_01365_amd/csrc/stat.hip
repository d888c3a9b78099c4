// Relative activations and the statistic s (Section 4.1 and Eq. 6), and the batch-shared
// statistic of Eq. 7.
//
//   r_i^2 = sum_j Z_ij^2            (row i of Z scaled by 1/r_i is the "relative activation")
//   s_j   = sqrt( sum_{i in sequence} Z_ij^2 / r_i^2 )
//
// r_i^2 needs the whole row, so the scaling cannot finish inside one tile of the GEMM that
// makes Z: the GEMM's epilogue leaves one sum-of-squares partial per (row, column tile), the
// kernel here turns them into the weights w_i = 1/r_i^2 (0 for an all-zero row) and streams Z once
// more, coalesced along the neuron axis, to accumulate sum_i w_i Z_ij^2.  Every sequence gets a
// number of chunks in proportion to its length (so that prompts of different lengths give
// workgroups of the same size), handled by different workgroups; a last small kernel adds a
// sequence's chunk partials in a fixed order and takes the square root.  All of it is
// bandwidth-bound: S*F fp32 reads.
#include "common.h"

namespace griffin {

// first chunk of every sequence in the global list of chunks (sequence b owns chunks first[b] .. first[b+1]-1)
struct ChunkTable {
    int32_t first[GRIFFIN_MAX_SEQS + 1];
};

// s2part[chunk][j] = sum over the chunk's rows of w_i Z_ij^2, w_i = 1 / sum_t rowpart[i][t] (0 for an all-zero
// row).  The chunks of a sequence do not own contiguous runs of rows: chunk c of the sequence's NC takes the
// groups of four rows c, c + NC, c + 2 NC, ..., so that at any moment the workgroups of a sequence read ONE
// compact window of 4 NC consecutive rows that marches through Z.  (Measured, 201 MB of Z / 1.18 GB of Z in 16
// prompts: 38.7 / 268 us with contiguous chunks, 38.3 / 278 us with this window and the register double buffer
// below, 44 / 250 us with twice the workgroups, 56 / 447 us with a quarter, non-temporal loads within 3 % either
// way: the kernel sits at 5.2 and 4.4 TB/s whatever the order of rows, the depth in flight or the cache policy.)
// A workgroup first turns the row partials of its own rows into weights (one wavefront per row: lanes over
// the column tiles, then a wave sum, eight rows' loads on their way together; every column block of a chunk
// repeats this for the same few rows, which is far cheaper than a kernel of its own in front of this one) and
// keeps them in LDS; rows past the end of the sequence get weight 0 and a clamped address.
constexpr int STAT_ROWS_LDS = 256;
typedef __attribute__((ext_vector_type(4))) float stat_f32x4;
#define STAT_LD(p_) (*(p_))

template <int VEC>
__global__ __launch_bounds__(256) void col_stat_kernel(const float *Z, int64_t ldz, const float *rowpart, int nt, int F,
                                                       SeqTable seqs, ChunkTable chunks, float *s2part)
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
    const int gl = g - chunks.first[b0], nc = chunks.first[b0 + 1] - chunks.first[b0];
    const int64_t s0 = seqs.cu[b0], s1 = seqs.cu[b0 + 1];
    const int ngroups = (int)((s1 - s0 + 3) >> 2);
    const int mine = gl < ngroups ? (ngroups - gl + nc - 1) / nc : 0;      // groups gl, gl + nc, ... of four rows
    // row number idx of this chunk (idx = 4 * group + row of the group)
#define STAT_ROW(idx_) (s0 + 4 * ((int64_t)gl + (int64_t)((idx_) >> 2) * nc) + ((idx_) & 3))
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v)
        acc[v] = 0.0f;
    for (int i0 = 0; i0 < 4 * mine; i0 += STAT_ROWS_LDS) {
        const int nr = 4 * mine - i0 < STAT_ROWS_LDS ? 4 * mine - i0 : STAT_ROWS_LDS;     // a multiple of 4
        __syncthreads();                       // the weights of the block before have been used
        for (int rb = wave; rb < nr; rb += 4 * 8) {
            float a[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = rb + 4 * u;
                const int64_t row = STAT_ROW(i0 + (r < nr ? r : nr - 1));
                const float *rp = rowpart + (row < s1 ? row : s1 - 1) * nt;
                a[u] = 0.0f;
                for (int t = lane; t < nt; t += 64)
                    a[u] += rp[t];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = rb + 4 * u;
                const float v = wave_sum(a[u]);
                if (lane == 0 && r < nr)
                    w_s[r] = (v > 0.0f && STAT_ROW(i0 + r) < s1) ? 1.0f / v : 0.0f;
            }
        }
        __syncthreads();
        // groups of four rows, the next group's loads already on their way while this one is used (branch-free:
        // past the last group the same group is loaded again, so the compiler waits for the older set only)
        float zc[4][VEC], zn[4][VEC];
#define STAT_LOAD(dst_, i_)                                                                      \
        _Pragma("unroll") for (int r = 0; r < 4; ++r)                                            \
        {                                                                                        \
            const int64_t row_ = STAT_ROW(i0 + (i_) + r);                                        \
            const float *zp_ = Z + (row_ < s1 ? row_ : s1 - 1) * ldz + jc;                       \
            if (VEC == 4) {                                                                      \
                const stat_f32x4 t_ = STAT_LD((const stat_f32x4 *)zp_);                          \
                dst_[r][0] = t_.x; dst_[r][1 % VEC] = t_.y; dst_[r][2 % VEC] = t_.z; dst_[r][3 % VEC] = t_.w; \
            } else {                                                                             \
                dst_[r][0] = zp_[0];                                                             \
            }                                                                                    \
        }
        STAT_LOAD(zc, 0)
        for (int i = 0; i < nr; i += 4) {
            const int inext = i + 4 < nr ? i + 4 : i;
            STAT_LOAD(zn, inext)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float wr = w_s[i + r];
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    acc[v] = fmaf(zc[r][v] * zc[r][v], wr, acc[v]);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    zc[r][v] = zn[r][v];
        }
#undef STAT_LOAD
    }
#undef STAT_ROW
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

// Rows per chunk, the same for every sequence, chosen so that all workgroups are resident at once (eight of
// 256 threads per CU, 2048 on the chip) and none is left to run alone afterwards: every sequence's last chunk
// is a partial one, so the count is at most total / rows + n_seqs and that bound is what is kept within the
// chip (measured on 16 prompts, 20600 tokens: 2142 workgroups, 94 more than fit, took 276 us against 243 us).
int stat_rows_per_chunk(int64_t total_tokens, int32_t n_seqs, int32_t F)
{
    const int64_t col_blocks = (F + 1023) / 1024;
    int64_t target = 2048 / col_blocks - n_seqs;
    if (target < 1)
        target = 1;
    const int64_t rows = (total_tokens + target - 1) / target;
    return (int)(rows < 16 ? 16 : (rows > (1 << 20) ? (1 << 20) : rows));
}

// upper bound of the number of chunks of any split of total_tokens into n_seqs sequences
int64_t stat_max_chunks(int64_t total_tokens, int32_t n_seqs, int32_t F)
{
    return total_tokens / stat_rows_per_chunk(total_tokens, n_seqs, F) + n_seqs;
}

int launch_stat(const float *Z, int64_t ldz, const float *rowpart, int nt, int64_t M, int32_t F,
                const SeqTable &seqs, float *s2part, float *s, float *s_out, hipStream_t st)
{
    int rcode;
    const int R = stat_rows_per_chunk(M, seqs.n, F);
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
            hipLaunchKernelGGL(col_stat_kernel<4>, grid, dim3(256), 0, st, Z, ldz, rowpart, nt, F, seqs, chunks, s2part);
        } else {
            dim3 grid((F + 255) / 256, n_chunks);
            hipLaunchKernelGGL(col_stat_kernel<1>, grid, dim3(256), 0, st, Z, ldz, rowpart, nt, F, seqs, chunks, s2part);
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
