// Expert set E (Section 4.2): indices of the k largest entries of the statistic s.
// Exact selection, ties to the lowest index, indices returned ascending.
//
// One workgroup per score row.  fp32 scores are mapped to uint32 keys whose unsigned order is
// the floats' order; a 4-pass, 8-bit-per-pass radix select over LDS histograms finds the k-th
// largest key tau and how many entries equal to tau are still needed; an ordered compaction
// (block-wide exclusive scan of per-thread counts over contiguous chunks) then writes every
// index with key > tau plus the first `need` indices with key == tau, in ascending order.
// D_ff <= 2^20 keys are re-read from L2 on every pass (98 KB for Gemma's 24576).
#include "common.h"

namespace griffin {

constexpr int TOPK_THREADS = 1024;

__device__ __forceinline__ uint32_t order_key(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exclusive scan of one value per thread across the workgroup; `total` gets the sum.
// `sh` must hold TOPK_THREADS/64 + 1 entries.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *sh, uint32_t &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        uint32_t t = __shfl_up(inc, off, 64);
        if (lane >= off)
            inc += t;
    }
    __syncthreads();            // sh may still be read from a previous call
    if (lane == 63)
        sh[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int w = 0; w < TOPK_THREADS / 64; ++w) {
            uint32_t t = sh[w];
            sh[w] = run;
            run += t;
        }
        sh[TOPK_THREADS / 64] = run;
    }
    __syncthreads();
    total = sh[TOPK_THREADS / 64];
    return sh[wave] + inc - v;
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_select_kernel(const float *scores, int n, int k,
                                                                   int32_t *idx_out)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t suffix[2][257];
    __shared__ uint32_t sh_digit, sh_need;
    __shared__ uint32_t sh_scan[TOPK_THREADS / 64 + 1];

    const float *row = scores + (int64_t)blockIdx.x * n;
    int32_t *out = idx_out + (int64_t)blockIdx.x * k;
    const int tid = threadIdx.x;

    uint32_t prefix = 0, mask = 0, need = (uint32_t)k;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256)
            hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += TOPK_THREADS) {
            const uint32_t key = order_key(row[i]);
            if ((key & mask) == prefix)
                atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        // suffix sums S[b] = sum_{b' >= b} hist[b'] (Hillis-Steele over 256 bins), S[256] = 0
        if (tid < 256)
            suffix[0][tid] = hist[tid];
        if (tid == 0) {
            suffix[0][256] = 0;
            suffix[1][256] = 0;
        }
        __syncthreads();
        int cur = 0;
        for (int off = 1; off < 256; off <<= 1) {
            if (tid < 256) {
                uint32_t v = suffix[cur][tid];
                if (tid + off < 256)
                    v += suffix[cur][tid + off];
                suffix[cur ^ 1][tid] = v;
            }
            __syncthreads();
            cur ^= 1;
        }
        // the digit of the k-th largest: the one bin with S[b] >= need > S[b+1]
        if (tid < 256) {
            const uint32_t here = suffix[cur][tid], above = suffix[cur][tid + 1];
            if (here >= need && above < need) {
                sh_digit = (uint32_t)tid;
                sh_need = need - above;
            }
        }
        __syncthreads();
        prefix |= sh_digit << shift;
        mask |= 255u << shift;
        need = sh_need;
        __syncthreads();
    }
    const uint32_t tau = prefix;   // key of the k-th largest score; `need` entries equal to it are kept

    // ordered compaction over contiguous per-thread chunks
    const int chunk = (n + TOPK_THREADS - 1) / TOPK_THREADS;
    const int lo = min(tid * chunk, n), hi = min(lo + chunk, n);
    uint32_t c_gt = 0, c_eq = 0;
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = order_key(row[i]);
        c_gt += key > tau;
        c_eq += key == tau;
    }
    uint32_t tot_gt, tot_eq;
    uint32_t p_gt = block_exclusive_scan(c_gt, sh_scan, tot_gt);
    uint32_t p_eq = block_exclusive_scan(c_eq, sh_scan, tot_eq);
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = order_key(row[i]);
        if (key > tau) {
            out[p_gt + min(p_eq, need)] = i;
            ++p_gt;
        } else if (key == tau) {
            if (p_eq < need)
                out[p_gt + p_eq] = i;
            ++p_eq;
        }
    }
}

int launch_topk(const float *scores, int32_t n_rows, int32_t n, int32_t k, int32_t *idx, hipStream_t st)
{
    hipLaunchKernelGGL(topk_select_kernel, dim3(n_rows), dim3(TOPK_THREADS), 0, st, scores, n, k, idx);
    return check_launch("topk_select_kernel");
}

}  // namespace griffin
