// Expert set E (Section 4.2): indices of the k largest entries of the statistic s.
// Exact selection, ties to the lowest index, indices returned ascending.
//
// One workgroup per score row.  fp32 scores are mapped to uint32 keys whose unsigned order is
// the floats' order; a radix select over LDS histograms (eight bits per step) finds the k-th
// largest key tau and how many entries equal to tau are still needed; an ordered compaction
// (block-wide exclusive scan of per-thread counts over contiguous chunks) then writes every
// index with key > tau plus the first `need` indices with key == tau, in ascending order.
// Rows of up to 32768 scores (every model shape in use) keep their keys in registers, spread the
// first step over the actual range of the row and finish on a short list of candidates
// (topk_select_reg_kernel); longer rows take four passes with the keys in LDS (up to 36864) or
// re-read from L2 on every pass (up to 2^20).
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

// CACHED: the row's keys are read from global memory once (coalesced, eight loads in flight per
// thread) into LDS and every later pass works from there; without it each of the five passes
// pays the global-memory latency of its loads again, one after the other.
constexpr int TOPK_CACHE_KEYS = 36864;       // 144 KB of LDS

template <bool CACHED>
__global__ __launch_bounds__(TOPK_THREADS) void topk_select_kernel(const float *scores, int n, int k,
                                                                   int32_t *idx_out)
{
    __shared__ uint32_t keys[CACHED ? TOPK_CACHE_KEYS : 1];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh_digit, sh_need;
    __shared__ uint32_t sh_scan[TOPK_THREADS / 64 + 1];

    const float *row = scores + (int64_t)blockIdx.x * n;
    int32_t *out = idx_out + (int64_t)blockIdx.x * k;
    const int tid = threadIdx.x;

    if (CACHED) {
        int i = tid;
        for (; i + 7 * TOPK_THREADS < n; i += 8 * TOPK_THREADS) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                v[u] = row[i + u * TOPK_THREADS];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                keys[i + u * TOPK_THREADS] = order_key(v[u]);
        }
        for (; i < n; i += TOPK_THREADS)
            keys[i] = order_key(row[i]);
        __syncthreads();
    }
#define TOPK_KEY(i_) (CACHED ? keys[i_] : order_key(row[i_]))

    uint32_t prefix = 0, mask = 0, need = (uint32_t)k;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256)
            hist[tid] = 0;
        __syncthreads();
        // the statistic's values sit in a narrow range, so in the first passes most keys of a wave
        // share one digit: lanes that agree with the wave's first candidate send ONE atomic with
        // their count, the others go singly
        for (int i0 = 0; i0 < n; i0 += TOPK_THREADS) {
            const int i = i0 + tid;
            uint32_t key = 0;
            bool cand = false;
            if (i < n) {
                key = TOPK_KEY(i);
                cand = (key & mask) == prefix;
            }
            const uint32_t digit = (key >> shift) & 255u;
            const uint64_t cmask = __ballot(cand);
            if (cmask != 0) {
                const int leader = __builtin_ctzll(cmask);
                const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)digit, leader);
                const uint64_t same = __ballot(cand && digit == d0);
                if ((int)(tid & 63) == leader)
                    atomicAdd(&hist[d0], (uint32_t)__builtin_popcountll(same));
                else if (cand && digit != d0)
                    atomicAdd(&hist[digit], 1u);
            }
        }
        __syncthreads();
        // the digit of the k-th largest: the one bin b with S[b] >= need > S[b+1], S[b] = sum of the
        // bins b' >= b.  One wavefront: lane l owns bins 4l .. 4l+3, suffix sums across lanes by shuffles.
        if (tid < 64) {
            const uint32_t h0 = hist[4 * tid], h1 = hist[4 * tid + 1], h2 = hist[4 * tid + 2], h3 = hist[4 * tid + 3];
            const uint32_t loc = h0 + h1 + h2 + h3;
            uint32_t suf = loc;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t t = __shfl_down(suf, off, 64);
                if (tid + off < 64)
                    suf += t;
            }
            const uint32_t s4 = suf - loc, s3 = s4 + h3, s2 = s3 + h2, s1 = s2 + h1, s0 = s1 + h0;
            if (s0 >= need && s4 < need) {
                uint32_t dg, above;
                if (s3 >= need) { dg = 3; above = s4; }
                else if (s2 >= need) { dg = 2; above = s3; }
                else if (s1 >= need) { dg = 1; above = s2; }
                else { dg = 0; above = s1; }
                sh_digit = 4u * tid + dg;
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
        const uint32_t key = TOPK_KEY(i);
        c_gt += key > tau;
        c_eq += key == tau;
    }
    uint32_t tot_gt, tot_eq;
    uint32_t p_gt = block_exclusive_scan(c_gt, sh_scan, tot_gt);
    uint32_t p_eq = block_exclusive_scan(c_eq, sh_scan, tot_eq);
    for (int i = lo; i < hi; ++i) {
        const uint32_t key = TOPK_KEY(i);
        if (key > tau) {
            out[p_gt + min(p_eq, need)] = i;
            ++p_gt;
        } else if (key == tau) {
            if (p_eq < need)
                out[p_gt + p_eq] = i;
            ++p_eq;
        }
    }
#undef TOPK_KEY
}

// Rows of up to TOPK_REG_KEYS scores.  One CU does all the work of a row, so what counts is the number of
// instructions per key and the latency chains between them (with the keys in LDS and one shared histogram
// a pass over 11008 keys took 2-5 us: eleven dependent LDS reads per wave, and the sixteen waves' atomics
// meeting in the few bins that the narrow range of the statistic fills):
//   * the keys come in coalesced, pass through LDS once (padded by one word in 32 so that the chunk-strided
//     read-back is free of bank conflicts) and then live in registers, a contiguous chunk of at most KPT per
//     thread, so every pass is straight-line code;
//   * the select works on rel = key - min key, and its first pass takes the eight bits below the highest set
//     bit of (max - min): the row spreads over all 256 bins whatever exponent the scores share (with the key's
//     own top byte the statistic fills a handful of bins and whole waves' adds meet there), every wavefront
//     adds into a histogram of its own, and the sixteen are summed once;
//   * the bin of the k-th largest holds a few per cent of the row: those keys go into a short list in LDS and
//     the remaining digits (eight bits at a time) are found on the list, not in three more passes over the row;
//   * the two counts of the compaction ride in one packed scan, and the selected indices are put in order
//     in LDS (where the keys were) and leave as coalesced stores.
constexpr int TOPK_REG_KEYS = 32768;
constexpr int TOPK_WAVES = TOPK_THREADS / 64;

template <int KPT>
__global__ __launch_bounds__(TOPK_THREADS) void topk_select_reg_kernel(const float *scores, int n, int k,
                                                                       int32_t *idx_out)
{
    __shared__ uint32_t stage[TOPK_REG_KEYS + TOPK_REG_KEYS / 32];     // keys on the way in, indices on the way out
    __shared__ uint32_t whist[TOPK_WAVES][256];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sh_digit, sh_need, sh_ncand;
    __shared__ uint32_t sh_scan[TOPK_WAVES], sh_max[TOPK_WAVES];

    const float *row = scores + (int64_t)blockIdx.x * n;
    int32_t *out = idx_out + (int64_t)blockIdx.x * k;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    {
        int i = tid;
        for (; i + 7 * TOPK_THREADS < n; i += 8 * TOPK_THREADS) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                v[u] = row[i + u * TOPK_THREADS];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int a = i + u * TOPK_THREADS;
                stage[a + (a >> 5)] = order_key(v[u]);
            }
        }
        for (; i < n; i += TOPK_THREADS)
            stage[i + (i >> 5)] = order_key(row[i]);
    }
    __syncthreads();
    // this thread's contiguous chunk of the row, in registers from here on
    const int chunk = (n + TOPK_THREADS - 1) / TOPK_THREADS;       // <= KPT
    const int lo = min(tid * chunk, n);
    const int nv = min(chunk, n - lo);                             // keys this thread holds
    uint32_t key[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const int a = min(lo + j, n - 1);
        key[j] = stage[a + (a >> 5)];
    }

    // ---- the range of the keys: the select works on rel = key - kmin, whose top eight bits BELOW the highest
    // set bit of (kmax - kmin) spread the row over all 256 bins of the first pass, whatever exponent the
    // scores have in common (with the key's own top byte the statistic fills a handful of bins)
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
    for (int j = 0; j < KPT; ++j)
        if (j < nv) {
            kmin = min(kmin, key[j]);
            kmax = max(kmax, key[j]);
        }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, m, 64));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, m, 64));
    }
    if (lane == 0) {
        sh_scan[wave] = kmin;
        sh_max[wave] = kmax;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < TOPK_WAVES; ++w) {
        kmin = min(kmin, sh_scan[w]);
        kmax = max(kmax, sh_max[w]);
    }
    const uint32_t range = kmax - kmin;
    const int nbits = range ? 32 - __builtin_clz(range) : 0;
    const int shift0 = nbits > 8 ? nbits - 8 : 0;
#pragma unroll
    for (int j = 0; j < KPT; ++j)
        key[j] -= kmin;                         // rel; order and ties are those of the keys

    // ---- first pass over all keys: digit = rel >> shift0
    uint32_t need = (uint32_t)k;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        whist[wave][lane * 4 + q] = 0;          // a wave's LDS accesses are performed in order: no barrier needed
    // With the digits spread over the bins the lanes of a wave rarely meet, and a plain add per lane is the
    // cheapest pass (1200-2800 clocks less than aggregating).  A row with many equal scores would send whole
    // waves to one bin, one add after the other: each wave looks at its first slot once, and if more than eight
    // of its lanes share a digit there it takes the aggregating form (the lanes that share the digit of the
    // wave's first key send one add with their count, the others add singly) for all its slots.
    bool aggregate = false;
    {
        const bool cand = 0 < nv;
        const uint64_t cmask = __ballot(cand);
        if (cmask != 0) {
            const uint32_t digit = key[0] >> shift0;
            const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)digit, __builtin_ctzll(cmask));
            aggregate = __builtin_popcountll(__ballot(cand && digit == d0)) > 8;
        }
    }
    if (!aggregate) {
#pragma unroll
        for (int j = 0; j < KPT; ++j)
            if (j < nv)
                atomicAdd(&whist[wave][key[j] >> shift0], 1u);
    } else {
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const bool cand = j < nv;
            const uint64_t cmask = __ballot(cand);
            if (cmask != 0) {
                const uint32_t digit = key[j] >> shift0;
                const int leader = __builtin_ctzll(cmask);
                const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)digit, leader);
                const uint64_t same = __ballot(cand && digit == d0);
                if (lane == leader)
                    atomicAdd(&whist[wave][d0], (uint32_t)__builtin_popcountll(same));
                else if (cand && digit != d0)
                    atomicAdd(&whist[wave][digit], 1u);
            }
        }
    }
    if (tid == 0)
        sh_ncand = 0;
    __syncthreads();
// the bin of the need-th largest: sums the waves' histograms, then one wavefront finds the one bin b with
// S[b] >= need > S[b+1], S[b] = sum of the bins b' >= b (lane l owns bins 4l .. 4l+3, suffix sums by shuffles)
#define TOPK_FIND_BIN(SUM_WAVES_)                                                                              \
    {                                                                                                          \
        if (SUM_WAVES_) {                                                                                      \
            if (tid < 256) {                                                                                   \
                uint32_t t_ = 0;                                                                               \
                _Pragma("unroll") for (int w = 0; w < TOPK_WAVES; ++w) t_ += whist[w][tid];                    \
                hist[tid] = t_;                                                                                \
            }                                                                                                  \
            __syncthreads();                                                                                   \
        }                                                                                                      \
        if (tid < 64) {                                                                                        \
            const uint32_t h0 = hist[4 * tid], h1 = hist[4 * tid + 1], h2 = hist[4 * tid + 2], h3 = hist[4 * tid + 3]; \
            hist[4 * tid] = hist[4 * tid + 1] = hist[4 * tid + 2] = hist[4 * tid + 3] = 0;   /* left empty for the next search */ \
            const uint32_t loc = h0 + h1 + h2 + h3;                                                            \
            uint32_t suf = loc;                                                                                \
            _Pragma("unroll") for (int off = 1; off < 64; off <<= 1)                                           \
            {                                                                                                  \
                const uint32_t t_ = __shfl_down(suf, off, 64);                                                 \
                if (tid + off < 64)                                                                            \
                    suf += t_;                                                                                 \
            }                                                                                                  \
            const uint32_t s4 = suf - loc, s3 = s4 + h3, s2 = s3 + h2, s1 = s2 + h1, s0 = s1 + h0;             \
            if (s0 >= need && s4 < need) {                                                                     \
                uint32_t dg, above;                                                                            \
                if (s3 >= need) { dg = 3; above = s4; }                                                        \
                else if (s2 >= need) { dg = 2; above = s3; }                                                   \
                else if (s1 >= need) { dg = 1; above = s2; }                                                   \
                else { dg = 0; above = s1; }                                                                   \
                sh_digit = 4u * tid + dg;                                                                      \
                sh_need = need - above;                                                                        \
            }                                                                                                  \
        }                                                                                                      \
        __syncthreads();                                                                                       \
    }
    TOPK_FIND_BIN(true)
    uint32_t tau = sh_digit << shift0;          // rel of the k-th largest, low bits still to come
    need = sh_need;

    if (shift0 > 0) {
        // ---- the keys of that bin (a few per cent of the row) go into a list in LDS (the staging area is free:
        // all keys are in registers), low bits only; the remaining digits are found on the list
        const uint32_t bin = sh_digit, low_mask = (1u << shift0) - 1u;
#pragma unroll
        for (int j = 0; j < KPT; ++j)
            if (j < nv && (key[j] >> shift0) == bin)
                stage[atomicAdd(&sh_ncand, 1u)] = key[j] & low_mask;
        __syncthreads();
        const int ncand = (int)sh_ncand;
        uint32_t lprefix = 0;                   // the digits found so far, as the high bits of the low part
        for (int bits = shift0; bits > 0;) {
            const int w = bits < 8 ? bits : 8, sh = bits - w;
            // the list is short: its entries add straight into the one histogram, which every search leaves empty
            for (int i = tid; i < ncand; i += TOPK_THREADS) {
                const uint32_t v = stage[i];
                if ((v >> bits) == (lprefix >> bits))
                    atomicAdd(&hist[(v >> sh) & ((1u << w) - 1u)], 1u);
            }
            __syncthreads();
            TOPK_FIND_BIN(false)
            lprefix |= sh_digit << sh;
            need = sh_need;
            bits = sh;
        }
        tau |= lprefix;
        __syncthreads();                        // the list has been read for the last time: the area is written again below
    }
#undef TOPK_FIND_BIN
    // tau: rel of the k-th largest score; `need` entries equal to it are kept

    // ordered compaction: both counts in one packed scan (each total is at most 32768: 16 bits apiece)
    uint32_t cnt = 0;
#pragma unroll
    for (int j = 0; j < KPT; ++j)
        if (j < nv)
            cnt += (key[j] > tau ? 1u : 0u) + (key[j] == tau ? 0x10000u : 0u);
    uint32_t inc = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(inc, off, 64);
        if (lane >= off)
            inc += t;
    }
    if (lane == 63)
        sh_scan[wave] = inc;
    __syncthreads();
    uint32_t base = 0;
#pragma unroll
    for (int w = 0; w < TOPK_WAVES; ++w)
        base += w < wave ? sh_scan[w] : 0u;
    const uint32_t excl = base + inc - cnt;
    uint32_t p_gt = excl & 0xFFFFu, p_eq = excl >> 16;
    // the keys are all in registers: the staging area now collects the selected indices in order
    // (a key above tau and a kept key equal to tau land at the same formula: p_gt + min(p_eq, need))
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const bool gt = j < nv && key[j] > tau, eq = j < nv && key[j] == tau;
        if (gt || (eq && p_eq < need))
            stage[p_gt + min(p_eq, need)] = (uint32_t)(lo + j);
        p_gt += gt ? 1u : 0u;
        p_eq += eq ? 1u : 0u;
    }
    __syncthreads();
    for (int i = tid; i < k; i += TOPK_THREADS)
        out[i] = (int32_t)stage[i];
}

int launch_topk(const float *scores, int32_t n_rows, int32_t n, int32_t k, int32_t *idx, hipStream_t st)
{
    if (n <= TOPK_REG_KEYS) {
        const int chunk = (n + TOPK_THREADS - 1) / TOPK_THREADS;
        dim3 grid(n_rows), block(TOPK_THREADS);
        if (chunk <= 4) hipLaunchKernelGGL(topk_select_reg_kernel<4>, grid, block, 0, st, scores, n, k, idx);
        else if (chunk <= 8) hipLaunchKernelGGL(topk_select_reg_kernel<8>, grid, block, 0, st, scores, n, k, idx);
        else if (chunk <= 12) hipLaunchKernelGGL(topk_select_reg_kernel<12>, grid, block, 0, st, scores, n, k, idx);
        else if (chunk <= 16) hipLaunchKernelGGL(topk_select_reg_kernel<16>, grid, block, 0, st, scores, n, k, idx);
        else if (chunk <= 24) hipLaunchKernelGGL(topk_select_reg_kernel<24>, grid, block, 0, st, scores, n, k, idx);
        else hipLaunchKernelGGL(topk_select_reg_kernel<32>, grid, block, 0, st, scores, n, k, idx);
        return check_launch("topk_select_reg_kernel");
    }
    if (n <= TOPK_CACHE_KEYS)
        hipLaunchKernelGGL(topk_select_kernel<true>, dim3(n_rows), dim3(TOPK_THREADS), 0, st, scores, n, k, idx);
    else
        hipLaunchKernelGGL(topk_select_kernel<false>, dim3(n_rows), dim3(TOPK_THREADS), 0, st, scores, n, k, idx);
    return check_launch("topk_select_kernel");
}

}  // namespace griffin
