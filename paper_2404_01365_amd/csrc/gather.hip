// Compaction (Section 4.2; Eq. 4-5): the selected neurons' rows of Wg, W1 and W2 (and the
// selected entries of bg, b1) are copied into dense [k][d] arrays.  With the neuron-major
// layout every selected neuron is one contiguous row in each matrix, so the gather is a
// row copy: 16-byte loads and stores, one workgroup per (row, matrix); HBM-bound.
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

__global__ __launch_bounds__(256) void compact_rows_kernel(GatherParams p)
{
    const int t = blockIdx.x;
    const int m = blockIdx.y;
    if (!p.src[m])
        return;
    int row = p.idx[t];
    row = row < 0 ? 0 : (row >= p.n_src ? p.n_src - 1 : row);
    const uint4 *s = (const uint4 *)((const char *)p.src[m] + (int64_t)row * p.ld_src);
    uint4 *o = (uint4 *)((char *)p.dst[m] + (int64_t)t * p.ld_dst);
    for (int c = threadIdx.x; c < p.row_chunks; c += 256)
        o[c] = s[c];
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
    p.bsrc[0] = L.bg; p.bsrc[1] = L.b1;
    p.bdst[0] = (void *)C.bg; p.bdst[1] = (void *)C.b1;
    p.idx = idx;
    p.ld_src = L.ld * es;
    p.ld_dst = C.ld * es;
    p.row_chunks = (int32_t)((int64_t)L.d * es / 16);
    p.n_src = L.n; p.k = k; p.esize = es;
    hipLaunchKernelGGL(compact_rows_kernel, dim3(k, 3), dim3(256), 0, st, p);
    int rc = check_launch("compact_rows_kernel");
    if (rc != GRIFFIN_OK)
        return rc;
    if (L.bg || L.b1) {
        hipLaunchKernelGGL(compact_bias_kernel, dim3((k + 255) / 256), dim3(256), 0, st, p);
        rc = check_launch("compact_bias_kernel");
    }
    return rc;
}

}  // namespace griffin
