// Generation phase: one token through a (compact or full) gated FF block
// (Section 4.2 "Generation with Expert Neurons"; Eq. 1 and Eq. 4-5):
//     z_j = sigma(wg_j . x + bg_j) * (w1_j . x + b1_j),   y = sum_j z_j W2[j][:] + b2.
//
// The work is a single pass over 3*n*d weights at one flop per byte, so the kernel is built to
// keep HBM busy: the three matrices are neuron-major, a wavefront owns a neuron, streams its
// three contiguous rows with 16-byte loads (all issued before the first use), reduces the two
// dot products with DPP (no LDS), and folds z_j * W2[j][:] into per-lane fp32 accumulators.
// A workgroup covers a contiguous slab of neurons; its waves are folded through LDS once at
// the end and the workgroup writes one fp32 partial row.  A second, tiny kernel sums the
// partial rows in a fixed order (deterministic), adds b2 and converts to the output type.
#include "common.h"

namespace griffin {

constexpr int DEC_WAVES = 8;
constexpr int DEC_THREADS = DEC_WAVES * 64;
constexpr int DEC_LDS_FLOATS = 16384;   // 64 KB fold buffer
constexpr int DEC_MAX_PARTS = 256;

struct DecodeParams {
    const void *Wg, *W1, *W2, *bg, *b1;
    const int32_t *idx;
    const void *x;
    float *part;
    int64_t ld;
    int32_t d, n, n_src, act, P;
};

struct MultiPtrs {
    const void *p[GRIFFIN_MAX_BATCH][5];   // Wg, W1, W2, bg, b1 of every row's own block
};

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// A 16-byte chunk of a row: 8 bf16 or 4 fp32 elements.  x stays in its storage form in
// registers (packed bf16 pairs feed v_dot2_f32_bf16 directly; fp32 feeds FMA).
template <bool BF16>
struct Chunk {
    static constexpr int E = BF16 ? 8 : 4;   // elements per chunk
    static __device__ __forceinline__ float dot(const uint4 &w, const uint4 &x, float acc)
    {
        if (BF16) {
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.x), __builtin_bit_cast(bf16x2, x.x), acc, false);
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.y), __builtin_bit_cast(bf16x2, x.y), acc, false);
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.z), __builtin_bit_cast(bf16x2, x.z), acc, false);
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.w), __builtin_bit_cast(bf16x2, x.w), acc, false);
        } else {
            acc = fmaf(__uint_as_float(w.x), __uint_as_float(x.x), acc);
            acc = fmaf(__uint_as_float(w.y), __uint_as_float(x.y), acc);
            acc = fmaf(__uint_as_float(w.z), __uint_as_float(x.z), acc);
            acc = fmaf(__uint_as_float(w.w), __uint_as_float(x.w), acc);
        }
        return acc;
    }
    static __device__ __forceinline__ void axpy(float z, const uint4 &w, float (&y)[BF16 ? 8 : 4])
    {
        if (BF16) {
            y[0] = fmaf(z, bf16_lo(w.x), y[0]); y[1] = fmaf(z, bf16_hi(w.x), y[1]);
            y[2] = fmaf(z, bf16_lo(w.y), y[2]); y[3] = fmaf(z, bf16_hi(w.y), y[3]);
            y[4 % E] = fmaf(z, bf16_lo(w.z), y[4 % E]); y[5 % E] = fmaf(z, bf16_hi(w.z), y[5 % E]);
            y[6 % E] = fmaf(z, bf16_lo(w.w), y[6 % E]); y[7 % E] = fmaf(z, bf16_hi(w.w), y[7 % E]);
        } else {
            y[0] = fmaf(z, __uint_as_float(w.x), y[0]); y[1] = fmaf(z, __uint_as_float(w.y), y[1]);
            y[2] = fmaf(z, __uint_as_float(w.z), y[2]); y[3] = fmaf(z, __uint_as_float(w.w), y[3]);
        }
    }
};

template <bool BF16, int NIT>
__device__ __forceinline__ void decode_body(const DecodeParams &p, const void *Wg, const void *W1,
                                            const void *W2, const void *bg, const void *b1,
                                            float *lds)
{
    constexpr int E = Chunk<BF16>::E;
    constexpr int ES = BF16 ? 2 : 4;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int b = blockIdx.y;
    const int part_id = blockIdx.x;
    const int d = p.d;
    const int nch = d / E;

    // x[b] into registers; lanes past the end hold zeros so clamped loads add nothing
    uint4 xr[NIT];
    const uint4 *xrow = (const uint4 *)((const char *)p.x + (int64_t)b * d * ES);
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int c = it * 64 + lane;
        xr[it] = c < nch ? xrow[c] : make_uint4(0, 0, 0, 0);
    }

    float ya[NIT][E];
#pragma unroll
    for (int it = 0; it < NIT; ++it)
#pragma unroll
        for (int e = 0; e < E; ++e)
            ya[it][e] = 0.0f;

    int cc[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it)
        cc[it] = min(it * 64 + lane, nch - 1);

    const int lo = (int)(((int64_t)p.n * part_id) / p.P);
    const int hi = (int)(((int64_t)p.n * (part_id + 1)) / p.P);
    const int32_t *idx = p.idx ? p.idx + (int64_t)b * p.n : nullptr;
    const int64_t row_bytes = p.ld * ES;

    for (int j = lo + wave; j < hi; j += DEC_WAVES) {
        int row = j;
        if (idx) {
            row = idx[j];
            row = row < 0 ? 0 : (row >= p.n_src ? p.n_src - 1 : row);
        }
        const uint4 *r1 = (const uint4 *)((const char *)W1 + row * row_bytes);
        const uint4 *r2 = (const uint4 *)((const char *)W2 + row * row_bytes);
        uint4 v1[NIT], v2[NIT];
        float g = 0.0f, u = 0.0f;
        if (Wg) {
            const uint4 *rg = (const uint4 *)((const char *)Wg + row * row_bytes);
            uint4 vg[NIT];
#pragma unroll
            for (int it = 0; it < NIT; ++it)
                vg[it] = rg[cc[it]];
#pragma unroll
            for (int it = 0; it < NIT; ++it)
                v1[it] = r1[cc[it]];
#pragma unroll
            for (int it = 0; it < NIT; ++it)
                v2[it] = r2[cc[it]];
#pragma unroll
            for (int it = 0; it < NIT; ++it)
                g = Chunk<BF16>::dot(vg[it], xr[it], g);
        } else {
#pragma unroll
            for (int it = 0; it < NIT; ++it)
                v1[it] = r1[cc[it]];
#pragma unroll
            for (int it = 0; it < NIT; ++it)
                v2[it] = r2[cc[it]];
        }
#pragma unroll
        for (int it = 0; it < NIT; ++it)
            u = Chunk<BF16>::dot(v1[it], xr[it], u);
        u = wave_sum(u);
        if (b1)
            u += load_scalar<BF16>(b1, row);
        float z;
        if (Wg) {
            g = wave_sum(g);
            if (bg)
                g += load_scalar<BF16>(bg, row);
            z = act_apply(p.act, g) * u;
        } else {
            z = act_apply(p.act, u);
        }
#pragma unroll
        for (int it = 0; it < NIT; ++it)
            Chunk<BF16>::axpy(z, v2[it], ya[it]);
    }

    // fold the workgroup's waves through LDS: each round the upper `h` active waves park their
    // accumulators in h slots and the lower h waves add them (fixed order, deterministic)
    const int slots = min(DEC_WAVES / 2, DEC_LDS_FLOATS / d);
    int active = DEC_WAVES;
    while (active > 1) {
        const int h = min(slots, active / 2);
        if (wave >= active - h && wave < active) {
            float *slot = lds + (int64_t)(wave - (active - h)) * d;
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int c = it * 64 + lane;
                if (c < nch) {
#pragma unroll
                    for (int e = 0; e < E; e += 4)
                        *(float4 *)(slot + c * E + e) =
                            make_float4(ya[it][e], ya[it][e + 1], ya[it][e + 2], ya[it][e + 3]);
                }
            }
        }
        __syncthreads();
        if (wave < h) {
            const float *slot = lds + (int64_t)wave * d;
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int c = it * 64 + lane;
                if (c < nch) {
#pragma unroll
                    for (int e = 0; e < E; e += 4) {
                        float4 t = *(const float4 *)(slot + c * E + e);
                        ya[it][e] += t.x; ya[it][e + 1] += t.y;
                        ya[it][e + 2] += t.z; ya[it][e + 3] += t.w;
                    }
                }
            }
        }
        __syncthreads();
        active -= h;
    }

    if (wave == 0) {
        float *out = p.part + ((int64_t)b * p.P + part_id) * d;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int c = it * 64 + lane;
            if (c < nch) {
#pragma unroll
                for (int e = 0; e < E; e += 4)
                    *(float4 *)(out + c * E + e) =
                        make_float4(ya[it][e], ya[it][e + 1], ya[it][e + 2], ya[it][e + 3]);
            }
        }
    }
}

template <bool BF16, int NIT>
__global__ __launch_bounds__(DEC_THREADS) void ff_decode_kernel(DecodeParams p)
{
    __shared__ __attribute__((aligned(16))) float lds[DEC_LDS_FLOATS];
    decode_body<BF16, NIT>(p, p.Wg, p.W1, p.W2, p.bg, p.b1, lds);
}

template <bool BF16, int NIT>
__global__ __launch_bounds__(DEC_THREADS) void ff_decode_multi_kernel(DecodeParams p, MultiPtrs m)
{
    __shared__ __attribute__((aligned(16))) float lds[DEC_LDS_FLOATS];
    const void *const *q = m.p[blockIdx.y];
    decode_body<BF16, NIT>(p, q[0], q[1], q[2], q[3], q[4], lds);
}

// y[b][c] = sum_p part[b][p][c] + b2[c], p ascending; one workgroup per 32 columns of one row.
struct B2Ptrs {
    const void *p[GRIFFIN_MAX_BATCH];    // b2 of every row's own block (multi path)
};

template <bool BF16, bool MULTI>
__global__ __launch_bounds__(256) void ff_decode_reduce_kernel(const float *part, int P, int d,
                                                               const void *b2_one, B2Ptrs b2_multi,
                                                               void *y)
{
    __shared__ float4 sm[32][8];
    const int q = threadIdx.x & 7;       // column quad inside the 32-column slab
    const int pg = threadIdx.x >> 3;     // partial-row group
    const int b = blockIdx.y;
    const void *b2 = MULTI ? b2_multi.p[b] : b2_one;
    const int c = blockIdx.x * 32 + q * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < d) {
        const float *base = part + (int64_t)b * P * d + c;
        for (int pp = pg; pp < P; pp += 32) {
            float4 t = *(const float4 *)(base + (int64_t)pp * d);
            acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
        }
    }
    sm[pg][q] = acc;
    __syncthreads();
    if (threadIdx.x < 8 && c < d) {
        float4 s = sm[0][q];
        for (int g = 1; g < 32; ++g) {
            float4 t = sm[g][q];
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
        if (b2) {
            s.x += load_scalar<BF16>(b2, c);
            s.y += load_scalar<BF16>(b2, c + 1);
            s.z += load_scalar<BF16>(b2, c + 2);
            s.w += load_scalar<BF16>(b2, c + 3);
        }
        const int64_t o = (int64_t)b * d + c;
        if (BF16) {
            uint2 w;
            w.x = f32_to_bf16_bits(s.x) | (f32_to_bf16_bits(s.y) << 16);
            w.y = f32_to_bf16_bits(s.z) | (f32_to_bf16_bits(s.w) << 16);
            *(uint2 *)((uint16_t *)y + o) = w;
        } else {
            *(float4 *)((float *)y + o) = s;
        }
    }
}

int decode_parts(int32_t n, int32_t batch)
{
    int P = (512 + batch - 1) / batch;
    if (P > DEC_MAX_PARTS) P = DEC_MAX_PARTS;
    if (P < 8) P = 8;
    const int by_work = (n + DEC_WAVES - 1) / DEC_WAVES;
    if (P > by_work) P = by_work;
    return P < 1 ? 1 : P;
}

template <bool BF16, int NIT>
static void launch_one(const DecodeParams &p, const MultiPtrs *m, int batch, hipStream_t st)
{
    dim3 grid(p.P, batch), block(DEC_THREADS);
    if (m)
        hipLaunchKernelGGL((ff_decode_multi_kernel<BF16, NIT>), grid, block, 0, st, p, *m);
    else
        hipLaunchKernelGGL((ff_decode_kernel<BF16, NIT>), grid, block, 0, st, p);
}

template <bool BF16>
static int launch_nit(int nit, const DecodeParams &p, const MultiPtrs *m, int batch, hipStream_t st)
{
    switch (nit) {
    case 1: launch_one<BF16, 1>(p, m, batch, st); break;
    case 2: launch_one<BF16, 2>(p, m, batch, st); break;
    case 4: launch_one<BF16, 4>(p, m, batch, st); break;
    case 6: launch_one<BF16, 6>(p, m, batch, st); break;
    case 8: launch_one<BF16, 8>(p, m, batch, st); break;
    case 10: launch_one<BF16, 10>(p, m, batch, st); break;
    case 12: launch_one<BF16, 12>(p, m, batch, st); break;
    case 16: launch_one<BF16, 16>(p, m, batch, st); break;
    default: return GRIFFIN_EUNSUPPORTED;
    }
    return GRIFFIN_OK;
}

// smallest supported per-lane chunk count that covers d; 0 if d is too wide for this build
int decode_nit(int32_t d, bool bf16)
{
    const int nch = d / (bf16 ? 8 : 4);
    const int need = (nch + 63) / 64;
    static const int sizes[] = {1, 2, 4, 6, 8, 10, 12, 16};
    for (int s : sizes)
        if (s >= need)
            return s;
    return 0;
}

// one-shot instrumentation: events recorded around the streaming kernel of the next decode
static thread_local hipEvent_t g_probe_begin = nullptr, g_probe_end = nullptr;

void set_decode_probe(hipEvent_t begin, hipEvent_t end)
{
    g_probe_begin = begin;
    g_probe_end = end;
}

int launch_decode(const DecodeJob &job, hipStream_t st)
{
    const int nit = decode_nit(job.d, job.bf16);
    if (nit == 0)
        return GRIFFIN_EUNSUPPORTED;
    const int P = decode_parts(job.n, job.batch);
    if (job.part_bytes < (size_t)P * job.batch * job.d * sizeof(float))
        return GRIFFIN_EWORKSPACE;

    DecodeParams p;
    p.Wg = job.Wg; p.W1 = job.W1; p.W2 = job.W2; p.bg = job.bg; p.b1 = job.b1;
    p.idx = job.idx; p.n_src = job.idx ? job.n_src : job.n;
    p.x = job.x; p.part = job.part; p.ld = job.ld;
    p.d = job.d; p.n = job.n; p.act = job.act; p.P = P;

    MultiPtrs m;
    B2Ptrs b2m;
    for (int b = 0; b < GRIFFIN_MAX_BATCH; ++b)
        b2m.p[b] = nullptr;
    const void *b2 = job.b2;
    if (job.multi) {
        for (int b = 0; b < job.batch; ++b) {
            const griffin_layer &c = job.multi[b];
            m.p[b][0] = c.Wg; m.p[b][1] = c.W1; m.p[b][2] = c.W2; m.p[b][3] = c.bg; m.p[b][4] = c.b1;
            b2m.p[b] = c.b2;
        }
        for (int b = job.batch; b < GRIFFIN_MAX_BATCH; ++b)
            for (int q = 0; q < 5; ++q)
                m.p[b][q] = nullptr;
    }
    const hipEvent_t ev_begin = g_probe_begin, ev_end = g_probe_end;
    g_probe_begin = g_probe_end = nullptr;
    if (ev_begin && hipEventRecord(ev_begin, st) != hipSuccess)
        return set_hip_error(hipGetLastError(), "hipEventRecord");
    int rc = job.bf16 ? launch_nit<true>(nit, p, job.multi ? &m : nullptr, job.batch, st)
                      : launch_nit<false>(nit, p, job.multi ? &m : nullptr, job.batch, st);
    if (rc != GRIFFIN_OK)
        return rc;
    rc = check_launch("ff_decode_kernel");
    if (rc != GRIFFIN_OK)
        return rc;
    if (ev_end && hipEventRecord(ev_end, st) != hipSuccess)
        return set_hip_error(hipGetLastError(), "hipEventRecord");

    dim3 rgrid((job.d + 31) / 32, job.batch), rblock(256);
    if (job.multi) {
        if (job.bf16)
            hipLaunchKernelGGL((ff_decode_reduce_kernel<true, true>), rgrid, rblock, 0, st, job.part, P, job.d, b2, b2m, job.y);
        else
            hipLaunchKernelGGL((ff_decode_reduce_kernel<false, true>), rgrid, rblock, 0, st, job.part, P, job.d, b2, b2m, job.y);
    } else {
        if (job.bf16)
            hipLaunchKernelGGL((ff_decode_reduce_kernel<true, false>), rgrid, rblock, 0, st, job.part, P, job.d, b2, b2m, job.y);
        else
            hipLaunchKernelGGL((ff_decode_reduce_kernel<false, false>), rgrid, rblock, 0, st, job.part, P, job.d, b2, b2m, job.y);
    }
    return check_launch("ff_decode_reduce_kernel");
}

}  // namespace griffin
