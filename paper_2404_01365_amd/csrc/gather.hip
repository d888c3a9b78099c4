// Compaction (Section 4.2; Eq. 4-5): the selected neurons' rows of Wg, W1 and W2 (and the
// selected entries of bg, b1) are copied into dense [k][d] arrays.  With the neuron-major
// layout every selected neuron is one contiguous row in each matrix, so the gather is a
// row copy: 16-byte loads and stores, one workgroup per selected neuron; HBM-bound.
#include "common.h"

namespace griffin {

struct GatherParams {
    const void *src[3];
    void *dst[3];
    const void *bsrc[2];
    void *bdst[2];
    const int32_t *idx;
    int64_t ld_src, ld_dst;   // bytes
    int32_t row_chunks;       // 16-byte chunks per row
    int32_t n_src, k, esize;
};

// One workgroup per selected neuron: its rows of the matrices that are there (three for a gated block)
// are one run of 16-byte chunks, taken GATHER_U x 256 at a time: all loads of a pass leave before the
// first store (a thread keeps up to GATHER_U x 16 bytes on their way: for rows up to 5120 bf16 elements the
// whole neuron is in flight at once; measured on 425 MB: 82 us with four loads per thread, 72 us with eight
// or sixteen, 84 us with the load-store-load-store loop of one workgroup per row).  Stores carry the
// non-temporal hint, and so do the loads when the block is larger than the Infinity Cache can have kept
// from the prompt GEMM that has just read two thirds of it (NT_LOAD; on a 270 MB block plain loads take
// 41 us, non-temporal ones 46 us; on 425 MB it is 77 us against 72 us).
// With the three rows of a neuron stored side by side in the target, a workgroup writes one contiguous piece.
constexpr int GATHER_U = 8;
typedef __attribute__((ext_vector_type(4))) uint32_t gather_u32x4;

template <bool NT_LOAD>
__global__ __launch_bounds__(256) void compact_rows_kernel(GatherParams p)
{
    const int t = blockIdx.x;
    int row = p.idx[t];
    row = row < 0 ? 0 : (row >= p.n_src ? p.n_src - 1 : row);
    // the matrices present, in order (Wg may be absent: Eq. 2; W2 may live only in its transposed copy)
    const char *s0, *s1, *s2;
    char *o0, *o1, *o2;
    int nm = 0;
    s0 = s1 = s2 = nullptr;
    o0 = o1 = o2 = nullptr;
#pragma unroll
    for (int m = 0; m < 3; ++m) {
        if (!p.src[m])
            continue;
        const char *sp = (const char *)p.src[m] + (int64_t)row * p.ld_src;
        char *op = (char *)p.dst[m] + (int64_t)t * p.ld_dst;
        if (nm == 0) { s0 = sp; o0 = op; }
        else if (nm == 1) { s1 = sp; o1 = op; }
        else { s2 = sp; o2 = op; }
        ++nm;
    }
    const int rc = p.row_chunks, total = nm * rc;
    for (int base = 0; base < total; base += 256 * GATHER_U) {
        gather_u32x4 v[GATHER_U];
        int64_t off[GATHER_U];
        int mi[GATHER_U];
#pragma unroll
        for (int u = 0; u < GATHER_U; ++u) {
            const int q = base + u * 256 + (int)threadIdx.x;
            const int qc = q < total ? q : total - 1;          // clamped: the load stays in bounds, nothing is stored
            mi[u] = (qc >= rc) + (qc >= 2 * rc);
            off[u] = (int64_t)(qc - mi[u] * rc) * 16;
            const char *sp = mi[u] == 0 ? s0 : (mi[u] == 1 ? s1 : s2);
            v[u] = NT_LOAD ? __builtin_nontemporal_load((const gather_u32x4 *)(sp + off[u])) : *(const gather_u32x4 *)(sp + off[u]);
        }
#pragma unroll
        for (int u = 0; u < GATHER_U; ++u) {
            const int q = base + u * 256 + (int)threadIdx.x;
            if (q < total) {
                char *op = mi[u] == 0 ? o0 : (mi[u] == 1 ? o1 : o2);
                __builtin_nontemporal_store(v[u], (gather_u32x4 *)(op + off[u]));
            }
        }
    }
}

// The second copy of the compact W2, output-feature-major (the paper's own orientation of W_2):
// W2t[c][t] = W2[idx[t]][c] for t < k, zero for k <= t < ldt.  A workgroup moves a 64-neuron x
// 64-feature tile through LDS: 128-byte pieces of 64 gathered rows in, 128-byte pieces of 64
// feature rows out (bf16 only, d a multiple of 64, ldt a multiple of 64).
__global__ __launch_bounds__(256) void compact_transpose_kernel(const uint16_t *W2, int64_t ld, int n_src,
                                                                const int32_t *idx, int k, uint16_t *W2t, int64_t ldt)
{
    __shared__ uint16_t tile[64][66];            // [neuron][feature], padded
    const int t0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int tid = threadIdx.x;
    // in: thread (row r = tid >> 2 (+0), quarter q = tid & 3) reads 16 features of one gathered row
    {
        const int r = tid >> 2, q = tid & 3;
        const int t = t0 + r;
        uint32_t v[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        if (t < k) {
            int row = idx[t];
            row = row < 0 ? 0 : (row >= n_src ? n_src - 1 : row);
            const uint4 *src = (const uint4 *)(W2 + (int64_t)row * ld + c0 + q * 16);
            const uint4 a = src[0], b = src[1];
            v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            tile[r][q * 16 + 2 * e] = (uint16_t)(v[e] & 0xFFFFu);
            tile[r][q * 16 + 2 * e + 1] = (uint16_t)(v[e] >> 16);
        }
    }
    __syncthreads();
    // out: thread (feature c = tid >> 2, quarter q) writes 16 neurons of one feature row
    {
        const int c = tid >> 2, q = tid & 3;
        uint32_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            v[e] = (uint32_t)tile[q * 16 + 2 * e][c] | ((uint32_t)tile[q * 16 + 2 * e + 1][c] << 16);
        uint4 *dst = (uint4 *)(W2t + (int64_t)(c0 + c) * ldt + t0 + q * 16);
        dst[0] = make_uint4(v[0], v[1], v[2], v[3]);
        dst[1] = make_uint4(v[4], v[5], v[6], v[7]);
    }
}

__global__ __launch_bounds__(256) void compact_bias_kernel(GatherParams p)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= p.k)
        return;
    int row = p.idx[t];
    row = row < 0 ? 0 : (row >= p.n_src ? p.n_src - 1 : row);
    for (int m = 0; m < 2; ++m) {
        if (!p.bsrc[m])
            continue;
        if (p.esize == 2)
            ((uint16_t *)p.bdst[m])[t] = ((const uint16_t *)p.bsrc[m])[row];
        else
            ((uint32_t *)p.bdst[m])[t] = ((const uint32_t *)p.bsrc[m])[row];
    }
}

int launch_compact(const griffin_layer &L, const int32_t *idx, int32_t k, const griffin_layer &C,
                   hipStream_t st)
{
    GatherParams p;
    const int es = L.dtype == GRIFFIN_BF16 ? 2 : 4;
    p.src[0] = L.Wg; p.src[1] = L.W1; p.src[2] = L.W2;
    p.dst[0] = (void *)C.Wg; p.dst[1] = (void *)C.W1; p.dst[2] = (void *)C.W2;
    if (!C.W2)
        p.src[2] = nullptr;        // the target keeps W2 only in its transposed copy
    p.bsrc[0] = L.bg; p.bsrc[1] = L.b1;
    p.bdst[0] = (void *)C.bg; p.bdst[1] = (void *)C.b1;
    p.idx = idx;
    p.ld_src = L.ld * es;
    p.ld_dst = C.ld * es;
    p.row_chunks = (int32_t)((int64_t)L.d * es / 16);
    p.n_src = L.n; p.k = k; p.esize = es;
    // blocks that the 256 MB Infinity Cache may still hold in good part are read with plain loads
    const int nmat = (L.Wg ? 1 : 0) + 1 + (C.W2 ? 1 : 0);
    if ((int64_t)nmat * L.n * L.ld * es > ((int64_t)384 << 20))
        hipLaunchKernelGGL(compact_rows_kernel<true>, dim3(k), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL(compact_rows_kernel<false>, dim3(k), dim3(256), 0, st, p);
    int rc = check_launch("compact_rows_kernel");
    if (rc != GRIFFIN_OK)
        return rc;
    if (C.W2t) {
        dim3 grid((unsigned)(C.ldt / 64), L.d / 64);
        hipLaunchKernelGGL(compact_transpose_kernel, grid, dim3(256), 0, st, (const uint16_t *)L.W2, L.ld, L.n, idx, k,
                           (uint16_t *)C.W2t, C.ldt);
        if ((rc = check_launch("compact_transpose_kernel")) != GRIFFIN_OK)
            return rc;
    }
    if (L.bg || L.b1) {
        hipLaunchKernelGGL(compact_bias_kernel, dim3((k + 255) / 256), dim3(256), 0, st, p);
        rc = check_launch("compact_bias_kernel");
    }
    return rc;
}

}  // namespace griffin
