// Generation phase: one token through a (compact or full) gated FF block
// (Section 4.2 "Generation with Expert Neurons"; Eq. 1 and Eq. 4-5):
//     z_j = sigma(wg_j . x + bg_j) * (w1_j . x + b1_j),   y = sum_j z_j W2[j][:] + b2.
//
// One pass over 3*n*d weights at one flop per byte: the kernel is shaped by what HBM likes.
// Measured on MI355X, read bandwidth is highest when the requests in flight at any moment
// cover a compact window of addresses and each CU keeps only ~32-64 KB outstanding; many
// lightly loaded waves beat few waves with deep queues.  So:
//   * a TEAM of R wavefronts owns a neuron: wave r streams the r-th 1 KB piece of the
//     neuron's three rows (16 bytes per lane), so a wave holds only its slab of x (one chunk)
//     and of y (one chunk of fp32 accumulators) and registers do not limit occupancy;
//   * teams take neurons round-robin across the whole chip (team T, step s -> neurons
//     (s*NT + T)*G ... +G-1), so at any time the chip reads one contiguous window of rows
//     per matrix (one window in all when the three rows of a neuron are stored side by
//     side, i.e. Wg, W1, W2 interleaved with ld = 3d);
//   * the two dot products are reduced inside the wave with DPP, combined across the team's
//     waves through a few LDS words and one barrier per G neurons, and the loads of the next
//     two steps are already in flight while that happens (three register sets; the loads are
//     branch-free so the compiler waits for the oldest set only; with one step of lookahead a
//     wave streams only one step's bytes per memory latency, which is what bounds narrow rows);
//   * each workgroup folds its teams' y slabs in LDS (one team for rows of 4 KB and more) and
//     writes one fp32 partial row; a second tiny kernel adds the partial rows in a fixed
//     order (deterministic), adds b2 and converts to the output type.
#include "common.h"

namespace griffin {

constexpr int DEC_G = 1;                 // neurons per team step
constexpr int DEC_MAX_WAVES = 16;        // waves per workgroup
constexpr int DEC_MAX_PARTS = 256;       // partial rows per batch row
constexpr int DEC_NB_MAX = 4;            // rows of x sharing one pass over the weights
constexpr int DEC_FOLD_FLOATS = 8192;    // LDS floats for folding teams (d <= 8192)

struct DecodeParams {
    const void *Wg, *W1, *W2, *bg, *b1;
    const int32_t *idx;
    const void *x;
    float *part;
    int64_t ld;
    int32_t d, n, n_src, act, P, batch;
    int32_t R, teams;        // waves per team, teams per workgroup
};

struct MultiPtrs {
    const void *p[GRIFFIN_MAX_BATCH][5];   // Wg, W1, W2, bg, b1 of every row's own block
};

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
// cache-policy bits of a raw buffer store on gfx942/gfx950: sc0 (bit 0) and sc1 (bit 4) = write through to memory
[[maybe_unused]] constexpr int DEC_AUX_WRITE_THROUGH = 1 | 16;

// by value on purpose: bit-casting a vector element expression (v.y) in place picks element 0
__device__ __forceinline__ bf16x2 as_bf16x2(uint32_t v) { return __builtin_bit_cast(bf16x2, v); }

// A 16-byte chunk of a row: 8 bf16 or 4 fp32 elements.
template <bool BF16>
struct Chunk {
    static constexpr int E = BF16 ? 8 : 4;
    static __device__ __forceinline__ float dot(const u32x4 &w, const u32x4 &x)
    {
        float acc = 0.0f;
        if (BF16) {
            acc = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(w.x), as_bf16x2(x.x), acc, false);
            acc = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(w.y), as_bf16x2(x.y), acc, false);
            acc = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(w.z), as_bf16x2(x.z), acc, false);
            acc = __builtin_amdgcn_fdot2_f32_bf16(as_bf16x2(w.w), as_bf16x2(x.w), acc, false);
        } else {
            acc = fmaf(__uint_as_float(w.x), __uint_as_float(x.x), acc);
            acc = fmaf(__uint_as_float(w.y), __uint_as_float(x.y), acc);
            acc = fmaf(__uint_as_float(w.z), __uint_as_float(x.z), acc);
            acc = fmaf(__uint_as_float(w.w), __uint_as_float(x.w), acc);
        }
        return acc;
    }
    static __device__ __forceinline__ void axpy(float z, const u32x4 &w, float (&y)[8])
    {
        if (BF16) {
            y[0] = fmaf(z, bf16_lo(w.x), y[0]); y[1] = fmaf(z, bf16_hi(w.x), y[1]);
            y[2] = fmaf(z, bf16_lo(w.y), y[2]); y[3] = fmaf(z, bf16_hi(w.y), y[3]);
            y[4] = fmaf(z, bf16_lo(w.z), y[4]); y[5] = fmaf(z, bf16_hi(w.z), y[5]);
            y[6] = fmaf(z, bf16_lo(w.w), y[6]); y[7] = fmaf(z, bf16_hi(w.w), y[7]);
        } else {
            y[0] = fmaf(z, __uint_as_float(w.x), y[0]); y[1] = fmaf(z, __uint_as_float(w.y), y[1]);
            y[2] = fmaf(z, __uint_as_float(w.z), y[2]); y[3] = fmaf(z, __uint_as_float(w.w), y[3]);
        }
    }
};

// GATED and INDEXED are compile-time so that the three row loads of a neuron are issued
// back to back with no branch between them (a branch there makes the compiler wait for the
// first load before issuing the next).
// NB = rows of x that share the block's weights in one pass (the weights are streamed once for
// NB rows; 1 for the per-row variants).
template <bool BF16, bool GATED, bool INDEXED, bool BIAS, int NB>
__device__ __forceinline__ void decode_body(const DecodeParams &p, const void *Wg, const void *W1,
                                            const void *W2, const void *bg, const void *b1,
                                            float (*red)[2 * DEC_G * DEC_NB_MAX][16], float *fold)
{
    constexpr int E = Chunk<BF16>::E;
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int G = DEC_G;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, in an SGPR
    const int R = p.R;
    const int team = wave / R, wt = wave - team * R;
    const int b = blockIdx.y * NB;           // first of this block's NB rows
    const int d = p.d, nch = d / E;

    const int c = wt * 64 + lane;            // this lane's 16-byte chunk of every row
    const bool valid = c < nch;
    const int cc = valid ? c : nch - 1;      // clamped: loads stay in bounds, x = 0 kills the terms
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    u32x4 xr[NB];
    float ya[NB][8];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const bool live = valid && b + nb < p.batch;     // rows past the batch behave as x = 0
        xr[nb] = live ? ((const u32x4 *)((const char *)p.x + (int64_t)(b + nb) * d * ES))[cc] : zero4;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            ya[nb][e] = 0.0f;
    }

    const int NT = gridDim.x * p.teams;              // teams on the chip for this batch row
    const int T = blockIdx.x * p.teams + team;
    const int nsteps = (p.n + NT * G - 1) / (NT * G);
    const int32_t *idx = INDEXED ? p.idx + (int64_t)b * p.n : nullptr;
    const int64_t row_bytes = p.ld * ES;
    constexpr int NV = 2 * G * NB;                   // values to combine across the team per step
    float(*myred)[2 * G * DEC_NB_MAX][16] = red + team * 2;   // [parity][value][wave of the team]


    // Loads are branch-free (slots past the last neuron re-read the last row, which stays in
    // L2, and are masked when z is formed) so that the compiler can wait for exactly the
    // older buffer while the newer one is still in flight.
    u32x4 buf[3][G][3];
    int rows[3][G];
    float bias[3][G][2];

// the weights are read once per call: non-temporal loads (no allocation in the caches on the way)
// stream measurably faster than plain ones (135 MB: 20.4 us against 24.0 us in a bare read loop)
#define DEC_STREAM_LOAD(ptr_) __builtin_nontemporal_load(ptr_)
#define DEC_LOAD(B_, s_)                                                                     \
    {                                                                                        \
        _Pragma("unroll") for (int g = 0; g < G; ++g)                                        \
        {                                                                                    \
            const int j_ = min(((s_) * NT + T) * G + g, p.n - 1);                            \
            int row_ = j_;                                                                   \
            if (INDEXED) {                                                                   \
                row_ = idx[j_];                                                              \
                row_ = row_ < 0 ? 0 : (row_ >= p.n_src ? p.n_src - 1 : row_);                \
            }                                                                                \
            if (GATED)                                                                       \
                buf[B_][g][0] = DEC_STREAM_LOAD((const u32x4 *)((const char *)Wg + row_ * row_bytes) + cc); \
            buf[B_][g][1] = DEC_STREAM_LOAD((const u32x4 *)((const char *)W1 + row_ * row_bytes) + cc);     \
            buf[B_][g][2] = DEC_STREAM_LOAD((const u32x4 *)((const char *)W2 + row_ * row_bytes) + cc);     \
            if (BIAS) {                                                                      \
                bias[B_][g][0] = (GATED && bg) ? load_scalar<BF16>(bg, row_) : 0.0f;         \
                bias[B_][g][1] = b1 ? load_scalar<BF16>(b1, row_) : 0.0f;                    \
            }                                                                                \
            rows[B_][g] = row_;                                                              \
        }                                                                                    \
    }

#define DEC_CONSUME(B_, s_)                                                                  \
    {                                                                                        \
        float pv_[NV];                                                                       \
        _Pragma("unroll") for (int nb = 0; nb < NB; ++nb)                                    \
            _Pragma("unroll") for (int g = 0; g < G; ++g)                                    \
        {                                                                                    \
            pv_[(nb * G + g) * 2] = GATED ? wave_sum(Chunk<BF16>::dot(buf[B_][g][0], xr[nb])) : 0.0f; \
            pv_[(nb * G + g) * 2 + 1] = wave_sum(Chunk<BF16>::dot(buf[B_][g][1], xr[nb]));   \
        }                                                                                    \
        if (lane == 0) {                                                                     \
            _Pragma("unroll") for (int v = 0; v < NV; ++v) myred[(s_) & 1][v][wt] = pv_[v];  \
        }                                                                                    \
        __syncthreads();                                                                     \
        _Pragma("unroll") for (int q = 0; q < (NV + 3) / 4; ++q)                             \
        {                                                                                    \
            float q_ = q * 4 + (lane >> 4) < NV ? myred[(s_) & 1][q * 4 + (lane >> 4)][lane & 15] : 0.0f; \
            q_ = row16_sum(q_);                                                              \
            _Pragma("unroll") for (int h = 0; h < 2; ++h)                                    \
            {                                                                                \
                if (q * 4 + 2 * h < NV) {                                                    \
                    const int pair_ = q * 2 + h;         /* = nb * G + g */                  \
                    const int nb_ = pair_ / G, g_ = pair_ % G;                               \
                    const int j_ = ((s_) * NT + T) * G + g_;                                 \
                    float gg_ = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(q_), 32 * h));      \
                    float uu_ = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(q_), 32 * h + 16)); \
                    if (BIAS) {                                                              \
                        gg_ += bias[B_][g_][0];                                              \
                        uu_ += bias[B_][g_][1];                                              \
                    }                                                                        \
                    float z_ = GATED ? act_apply(p.act, gg_) * uu_ : act_apply(p.act, uu_);  \
                    z_ = j_ < p.n ? z_ : 0.0f;                                               \
                    Chunk<BF16>::axpy(z_, buf[B_][g_][2], ya[nb_]);                          \
                }                                                                            \
            }                                                                                \
        }                                                                                    \
    }

    if (nsteps > 0) {
        DEC_LOAD(0, 0)
        DEC_LOAD(1, 1)             // steps past the end re-read the last row and contribute nothing
    }
    // zero the padding entries of the cross-wave buffers once (the first rows are already on their way)
    for (int i = threadIdx.x; i < p.teams * 2 * 2 * G * DEC_NB_MAX * 16; i += blockDim.x)
        (&red[0][0][0])[i] = 0.0f;
    __syncthreads();
    for (int s = 0; s < nsteps; s += 3) {
        DEC_LOAD(2, s + 2)
        DEC_CONSUME(0, s)
        if (s + 1 >= nsteps)
            break;
        DEC_LOAD(0, s + 3)
        DEC_CONSUME(1, s + 1)
        if (s + 2 >= nsteps)
            break;
        DEC_LOAD(1, s + 4)
        DEC_CONSUME(2, s + 2)
    }
#undef DEC_LOAD
#undef DEC_STREAM_LOAD
#undef DEC_CONSUME
    (void)rows;

    // fold the workgroup's teams (fixed order), then one fp32 partial row per workgroup and x row
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        for (int t = 1; t < p.teams; ++t) {
            if (team == t && valid) {
#pragma unroll
                for (int e = 0; e < E; e += 4)
                    *(float4 *)(fold + c * E + e) = make_float4(ya[nb][e], ya[nb][e + 1], ya[nb][e + 2], ya[nb][e + 3]);
            }
            __syncthreads();
            if (team == 0 && valid) {
#pragma unroll
                for (int e = 0; e < E; e += 4) {
                    const float4 v = *(const float4 *)(fold + c * E + e);
                    ya[nb][e] += v.x; ya[nb][e + 1] += v.y; ya[nb][e + 2] += v.z; ya[nb][e + 3] += v.w;
                }
            }
            __syncthreads();
        }
        // The partial row is private to this kernel and the one that adds the rows up, so its columns are
        // stored in the order that makes every store instruction one contiguous kilobyte: quad e/4 of
        // chunk c goes to float4 slot (e/4) * nch + c (a lane's 8 columns would otherwise leave as two
        // instructions that each fill every other 16 bytes).  The stores are write-through (sc0 sc1): the rows
        // then sit in memory when the kernel ends instead of as dirty lines in eight L2s that the end of the
        // kernel has to write back before the adding kernel may start (0.4 us per layer-token less than with
        // plain or non-temporal stores, measured on three shapes).
        if (team == 0 && valid && b + nb < p.batch) {
#if defined(__HIP_DEVICE_COMPILE__)      // the host pass has no buffer builtins
            float *out = p.part + ((int64_t)(b + nb) * p.P + blockIdx.x) * d;
            const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc((void *)out, 0, 0x7FFFFFFE, 0x00020000);
#pragma unroll
            for (int e = 0; e < E; e += 4) {
                const f32x4 v = {ya[nb][e], ya[nb][e + 1], ya[nb][e + 2], ya[nb][e + 3]};
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), rp, ((e / 4) * nch + c) * 16, 0,
                                                       DEC_AUX_WRITE_THROUGH);
            }
#endif
        }
    }
}

template <bool BF16, bool GATED, bool INDEXED, bool BIAS, int NB>
__global__ __launch_bounds__(DEC_MAX_WAVES * 64) void ff_decode_kernel(DecodeParams p)
{
    __shared__ float red[DEC_MAX_WAVES * 2][2 * DEC_G * DEC_NB_MAX][16];
    __shared__ __attribute__((aligned(16))) float fold[DEC_FOLD_FLOATS];
    decode_body<BF16, GATED, INDEXED, BIAS, NB>(p, p.Wg, p.W1, p.W2, p.bg, p.b1, red, fold);
}

template <bool BF16, bool GATED, bool BIAS>
__global__ __launch_bounds__(DEC_MAX_WAVES * 64) void ff_decode_multi_kernel(DecodeParams p, MultiPtrs m)
{
    __shared__ float red[DEC_MAX_WAVES * 2][2 * DEC_G * DEC_NB_MAX][16];
    __shared__ __attribute__((aligned(16))) float fold[DEC_FOLD_FLOATS];
    const void *const *q = m.p[blockIdx.y];
    decode_body<BF16, GATED, false, BIAS, 1>(p, q[0], q[1], q[2], q[3], q[4], red, fold);
}

struct B2Ptrs {
    const void *p[GRIFFIN_MAX_BATCH];    // b2 of every row's own block (multi path)
};

// y[b] = sum_p part[b][p] + b2, the rows p taken in a fixed order.  A workgroup of eight wavefronts owns
// RED_Q float4 slots (one 128-byte line) of every partial row: lane (r, q) of wave w reads slot q of the
// rows p = 8 w + r, + 64, + 128, + 192 (all four loads on their way at once; a wave instruction covers
// eight whole lines), adds them in that order, the eight lanes of a slot are added with wave shuffles and
// the eight waves through LDS.  nch > 0 says that the rows come from the streaming kernel, which stores
// quad h of 16-byte chunk c at slot h * nch + c (bf16 blocks: 8 columns per chunk); 0 = columns in order.
constexpr int RED_Q = 8, RED_WAVES = 8;
template <bool BF16, bool MULTI>
__global__ __launch_bounds__(RED_WAVES * 64) void ff_decode_reduce_kernel(const float *part, int P, int d, int nch,
                                                                           const void *b2_one, B2Ptrs b2_multi,
                                                                           void *y)
{
    __shared__ float4 fold[RED_WAVES][RED_Q];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.y;
    const int r = lane >> 3, qi = lane & 7;
    const int nq = d >> 2;
    const int q = blockIdx.x * RED_Q + qi;
    const int qc = q < nq ? q : nq - 1;            // clamped: loads stay in bounds, the result is not stored
    const float *base = part + (int64_t)b * P * d + (int64_t)qc * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int p0 = wave * 8 + r; p0 < P; p0 += 256) {
        float4 t[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int pp = p0 + 64 * i;
            const f32x4 v = pp < P ? __builtin_nontemporal_load((const f32x4 *)(base + (int64_t)pp * d)) : (f32x4){0.f, 0.f, 0.f, 0.f};
            t[i] = make_float4(v.x, v.y, v.z, v.w);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc.x += t[i].x; acc.y += t[i].y; acc.z += t[i].z; acc.w += t[i].w;
        }
    }
    // the eight lanes (r = 0..7) that hold the same slot
#pragma unroll
    for (int m = 8; m < 64; m <<= 1) {
        acc.x += __shfl_xor(acc.x, m, 64); acc.y += __shfl_xor(acc.y, m, 64);
        acc.z += __shfl_xor(acc.z, m, 64); acc.w += __shfl_xor(acc.w, m, 64);
    }
    if (r == 0)
        fold[wave][qi] = acc;
    __syncthreads();
    if (threadIdx.x < RED_Q && q < nq) {
        float4 s = fold[0][qi];
#pragma unroll
        for (int w = 1; w < RED_WAVES; ++w) {
            const float4 v = fold[w][qi];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        const int c = nch > 0 ? (q % nch) * 8 + (q / nch) * 4 : q * 4;      // first of this slot's four columns
        const void *b2 = MULTI ? b2_multi.p[b] : b2_one;
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

// grid of the kernel above for rows of d floats
static dim3 reduce_grid(int d, int batch) { return dim3((d / 4 + RED_Q - 1) / RED_Q, batch); }

// waves per team for a row of d elements, 0 if this build cannot cover it
static int decode_team_waves(int32_t d, bool bf16)
{
    const int nch = d / (bf16 ? 8 : 4);
    const int R = (nch + 63) / 64;
    return (R <= DEC_MAX_WAVES && d <= DEC_FOLD_FLOATS) ? R : 0;
}

// workgroups (= partial rows) per batch row: enough to fill the chip when the rows of a batch
// are taken DEC_NB_MAX at a time
int decode_parts(int32_t n, int32_t batch)
{
    const int groups = batch <= 2 ? 1 : (batch + DEC_NB_MAX - 1) / DEC_NB_MAX;
    int P = (512 + groups - 1) / groups;
    if (P > DEC_MAX_PARTS) P = DEC_MAX_PARTS;
    if (P < 8) P = 8;
    const int by_work = (n + 2 * DEC_G - 1) / (2 * DEC_G);
    if (P > by_work) P = by_work;
    return P < 1 ? 1 : P;
}

// one-shot instrumentation: events recorded around the streaming kernel of the next decode
static thread_local hipEvent_t g_probe_begin = nullptr, g_probe_mid = nullptr, g_probe_end = nullptr;

void set_decode_probe(hipEvent_t begin, hipEvent_t mid, hipEvent_t end)
{
    g_probe_begin = begin;
    g_probe_mid = mid;
    g_probe_end = end;
}

int launch_decode(const DecodeJob &job, hipStream_t st)
{
    const int R = decode_team_waves(job.d, job.bf16);
    if (R == 0)
        return GRIFFIN_EUNSUPPORTED;
    int P = decode_parts(job.n, job.batch);
    // five rows and more through one shared block: the matrix-core path
    const bool batch_path = !job.multi && !job.idx && job.batch >= DEC_BATCH_MIN_ROWS &&
                            decode_batch_supported(job.d, job.n, job.bf16);
    // five rows and more with their own sets inside one block: one masked pass over the whole block, if
    // the caller's workspace was sized for the whole block (else row by row through the index lists)
    const bool masked_path = !job.multi && job.idx && job.batch >= DEC_BATCH_MIN_ROWS && job.W2 &&
                             decode_batch_supported(job.d, job.n_src, job.bf16) &&
                             job.part_bytes >= decode_masked_workspace_floats(job.d, job.n_src, job.batch) * sizeof(float);
    if (!masked_path &&
        job.part_bytes < (batch_path ? decode_batch_workspace_floats(job.d, job.n, job.batch)
                                     : (size_t)P * job.batch * job.d) * sizeof(float))
        return GRIFFIN_EWORKSPACE;

    DecodeParams p;
    p.Wg = job.Wg; p.W1 = job.W1; p.W2 = job.W2; p.bg = job.bg; p.b1 = job.b1;
    p.idx = job.idx; p.n_src = job.idx ? job.n_src : job.n;
    p.x = job.x; p.part = job.part; p.ld = job.ld;
    p.d = job.d; p.n = job.n; p.act = job.act; p.P = P; p.batch = job.batch;
    p.R = R;
    // about eight waves per workgroup, one workgroup per CU: measured best (more waves or
    // more loads in flight per CU lower the achieved bandwidth)
    p.teams = R >= 8 ? 1 : 8 / R;

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

    const hipEvent_t ev_begin = g_probe_begin, ev_mid = g_probe_mid, ev_end = g_probe_end;
    g_probe_begin = g_probe_mid = g_probe_end = nullptr;
    if (ev_begin && hipEventRecord(ev_begin, st) != hipSuccess)
        return set_hip_error(hipGetLastError(), "hipEventRecord");

    if (decode_split_supported(job)) {
        int rc = launch_decode_split(job, st, ev_mid);
        if (rc == GRIFFIN_OK && ev_end && hipEventRecord(ev_end, st) != hipSuccess)
            return set_hip_error(hipGetLastError(), "hipEventRecord");
        return rc;
    }
    if (!job.W2 && !job.multi)
        return GRIFFIN_EUNSUPPORTED;       // only the transposed copy is there and this call cannot use it
    if (batch_path || masked_path) {
        int rc = masked_path ? launch_decode_batch_front(job, job.n_src, job.idx, job.n, &P, st)
                             : launch_decode_batch_front(job, job.n, nullptr, 0, &P, st);
        if (rc != GRIFFIN_OK)
            return rc;
        if (ev_mid && hipEventRecord(ev_mid, st) != hipSuccess)
            return set_hip_error(hipGetLastError(), "hipEventRecord");
        dim3 rgrid = reduce_grid(job.d, job.batch), rblock(RED_WAVES * 64);
        hipLaunchKernelGGL((ff_decode_reduce_kernel<true, false>), rgrid, rblock, 0, st, job.part, P, job.d, 0, b2, b2m, job.y);
        rc = check_launch("ff_decode_reduce_kernel");
        if (rc == GRIFFIN_OK && ev_end && hipEventRecord(ev_end, st) != hipSuccess)
            return set_hip_error(hipGetLastError(), "hipEventRecord");
        return rc;
    }

    // rows through one shared block are taken NB at a time (weights streamed once per NB rows)
    const bool shared_block = !job.multi && !job.idx;
    const int NB = !shared_block || job.batch == 1 ? 1 : (job.batch == 2 ? 2 : DEC_NB_MAX);
    dim3 grid(P, (job.batch + NB - 1) / NB), block(p.teams * R * 64);
    const bool gated = job.multi ? job.multi[0].Wg != nullptr : job.Wg != nullptr;
    const bool indexed = job.idx != nullptr;
    const bool bias = job.multi ? (job.multi[0].bg || job.multi[0].b1) : (job.bg || job.b1);
#define DEC_GO1(BF, GA, IX, BI, NB_) hipLaunchKernelGGL((ff_decode_kernel<BF, GA, IX, BI, NB_>), grid, block, 0, st, p)
#define DEC_GO(BF, GA, IX, BI)                                         \
    {                                                                  \
        if (IX || NB == 1) DEC_GO1(BF, GA, IX, BI, 1);                 \
        else if (NB == 2) DEC_GO1(BF, GA, false, BI, 2);               \
        else DEC_GO1(BF, GA, false, BI, DEC_NB_MAX);                   \
    }
#define DEC_GO_MULTI(BF, GA, BI) hipLaunchKernelGGL((ff_decode_multi_kernel<BF, GA, BI>), grid, block, 0, st, p, m)
#define DEC_PICK3(BF, GA, IX) { if (bias) DEC_GO(BF, GA, IX, true) else DEC_GO(BF, GA, IX, false) }
#define DEC_PICK2(BF, GA) { if (indexed) DEC_PICK3(BF, GA, true) else DEC_PICK3(BF, GA, false) }
#define DEC_PICKM(BF, GA) { if (bias) DEC_GO_MULTI(BF, GA, true); else DEC_GO_MULTI(BF, GA, false); }
    if (job.multi) {
        if (job.bf16) { if (gated) DEC_PICKM(true, true) else DEC_PICKM(true, false) }
        else          { if (gated) DEC_PICKM(false, true) else DEC_PICKM(false, false) }
    } else if (job.bf16) {
        if (gated) DEC_PICK2(true, true) else DEC_PICK2(true, false)
    } else {
        if (gated) DEC_PICK2(false, true) else DEC_PICK2(false, false)
    }
#undef DEC_PICK3
#undef DEC_PICK2
#undef DEC_PICKM
#undef DEC_GO
#undef DEC_GO1
#undef DEC_GO_MULTI
    int rc = check_launch("ff_decode_kernel");
    if (rc != GRIFFIN_OK)
        return rc;
    if (ev_mid && hipEventRecord(ev_mid, st) != hipSuccess)
        return set_hip_error(hipGetLastError(), "hipEventRecord");

    dim3 rgrid = reduce_grid(job.d, job.batch), rblock(RED_WAVES * 64);
    const int nch = job.bf16 ? job.d / 8 : 0;       // the streaming kernel's order of columns (fp32 rows: in order)
    if (job.multi) {
        if (job.bf16)
            hipLaunchKernelGGL((ff_decode_reduce_kernel<true, true>), rgrid, rblock, 0, st, job.part, P, job.d, nch, b2, b2m, job.y);
        else
            hipLaunchKernelGGL((ff_decode_reduce_kernel<false, true>), rgrid, rblock, 0, st, job.part, P, job.d, nch, b2, b2m, job.y);
    } else {
        if (job.bf16)
            hipLaunchKernelGGL((ff_decode_reduce_kernel<true, false>), rgrid, rblock, 0, st, job.part, P, job.d, nch, b2, b2m, job.y);
        else
            hipLaunchKernelGGL((ff_decode_reduce_kernel<false, false>), rgrid, rblock, 0, st, job.part, P, job.d, nch, b2, b2m, job.y);
    }
    rc = check_launch("ff_decode_reduce_kernel");
    if (rc == GRIFFIN_OK && ev_end && hipEventRecord(ev_end, st) != hipSuccess)
        return set_hip_error(hipGetLastError(), "hipEventRecord");
    return rc;
}

}  // namespace griffin
