// Generation phase, one token, for blocks that carry W2 a second time in the paper's own
// orientation (W2t [d][ldt], row c = output feature c; Section 3: W_2 is D x D_FF):
//
//     z_j = sigma(wg_j . x + bg_j) * (w1_j . x + b1_j)        ff_decode_gu_kernel
//     y_c = sum_j W2t[c][j] z_j + b2_c                        ff_decode_down_kernel
//
// With W2 stored neuron-major a workgroup that owns some neurons can only produce a partial
// output row, and on this chip the 256 partial rows cost a 4 MB burst at the end of the stream
// plus a second kernel to add them.  With W2t the second line is a plain matrix-vector product
// whose rows are the output features, so both kernels are pure streams with a few KB of output:
//   * ff_decode_gu_kernel: a team of R = d/512 waves per neuron, wave r streams the r-th 1 KB
//     piece of the neuron's Wg and W1 rows (non-temporal, next neuron's pieces in flight),
//     dot products against its piece of x with v_dot2_f32_bf16, DPP sums, the team's waves
//     meet through a few LDS words, z_j goes out as one float; teams take neurons round-robin
//     over the chip.  z beyond n (up to ldt) is zeroed.
//   * ff_decode_down_kernel: a workgroup of R waves owns 2R output features, a wave two rows of
//     W2t (1 KB pieces, non-temporal, three pieces per row in flight); z comes from the caches with
//     the same lookahead; one DPP sum per
//     row at the end; y leaves in its final type.  No partial rows, no third kernel.
#include "common.h"

namespace griffin {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_s;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_sp;
typedef __attribute__((ext_vector_type(4))) float f32x4_sp;

__device__ __forceinline__ bf16x2_s sp_bf16x2(uint32_t v) { return __builtin_bit_cast(bf16x2_s, v); }

__device__ __forceinline__ float sp_dot(const u32x4_sp &w, const u32x4_sp &x)
{
    float acc = __builtin_amdgcn_fdot2_f32_bf16(sp_bf16x2(w.x), sp_bf16x2(x.x), 0.0f, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(sp_bf16x2(w.y), sp_bf16x2(x.y), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(sp_bf16x2(w.z), sp_bf16x2(x.z), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(sp_bf16x2(w.w), sp_bf16x2(x.w), acc, false);
    return acc;
}

struct SplitParams {
    const void *Wg, *W1, *bg, *b1, *b2, *W2t;
    const void *x;
    void *y;
    float *z;               // [ldt]
    int64_t ld, ldt;
    int32_t d, n, act, R, teams;
};

template <bool GATED, bool BIAS>
__global__ __launch_bounds__(1024) void ff_decode_gu_kernel(SplitParams p)
{
    __shared__ float red[16 * 2][2][16];      // [team * 2 + parity][g or u][wave of the team]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int R = p.R;
    const int team = wave / R, wt = wave - team * R;
    const int cc = wt * 64 + lane;            // this lane's 16-byte chunk of every row (d = 512 R: always inside)
    const u32x4_sp xr = ((const u32x4_sp *)p.x)[cc];

    const int NT = gridDim.x * p.teams;       // teams on the chip
    const int T = blockIdx.x * p.teams + team;
    const int nsteps = (p.n + NT - 1) / NT;
    const int64_t row_bytes = p.ld * 2;
    // three register sets: the pieces of the next two neurons are in flight while one is used (one
    // step of lookahead leaves 2 KB per wave in flight, and the stream then runs at 2 KB per memory
    // latency per wave, well under what HBM can deliver)
    u32x4_sp buf[4][2];
    float bias[4][2];
#define SP_LOAD(B_, s_)                                                                              \
    {                                                                                                \
        const int j_ = min((s_) * NT + T, p.n - 1);                                                  \
        if (GATED)                                                                                   \
            buf[B_][0] = __builtin_nontemporal_load((const u32x4_sp *)((const char *)p.Wg + j_ * row_bytes) + cc); \
        buf[B_][1] = __builtin_nontemporal_load((const u32x4_sp *)((const char *)p.W1 + j_ * row_bytes) + cc);     \
        if (BIAS) {                                                                                  \
            bias[B_][0] = (GATED && p.bg) ? bf16_bits_to_f32(((const uint16_t *)p.bg)[j_]) : 0.0f;   \
            bias[B_][1] = p.b1 ? bf16_bits_to_f32(((const uint16_t *)p.b1)[j_]) : 0.0f;              \
        }                                                                                            \
    }
#define SP_CONSUME(B_, s_)                                                                           \
    {                                                                                                \
        const float pg_ = GATED ? wave_sum(sp_dot(buf[B_][0], xr)) : 0.0f;                           \
        const float pu_ = wave_sum(sp_dot(buf[B_][1], xr));                                          \
        if (lane == 0) {                                                                             \
            red[team * 2 + ((s_) & 1)][0][wt] = pg_;                                                 \
            red[team * 2 + ((s_) & 1)][1][wt] = pu_;                                                 \
        }                                                                                            \
        __syncthreads();                                                                             \
        if (wt == 0) {                                                                               \
            float q_ = lane < 32 ? red[team * 2 + ((s_) & 1)][lane >> 4][lane & 15] : 0.0f;          \
            q_ = row16_sum(q_);                                                                      \
            float gg_ = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(q_), 0));            \
            float uu_ = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(q_), 16));           \
            if (BIAS) {                                                                              \
                gg_ += bias[B_][0];                                                                  \
                uu_ += bias[B_][1];                                                                  \
            }                                                                                        \
            const int j_ = (s_) * NT + T;                                                            \
            if (lane == 0 && j_ < p.n)                                                               \
                p.z[j_] = GATED ? act_apply(p.act, gg_) * uu_ : act_apply(p.act, uu_);               \
        }                                                                                            \
    }

    if (nsteps > 0) {
        SP_LOAD(0, 0)
        SP_LOAD(1, 1)                      // steps past the end re-read the last row and store nothing
        SP_LOAD(2, 2)
    }
    // entries of the cross-wave words beyond the team's R waves stay zero
    for (int i = threadIdx.x; i < 16 * 2 * 2 * 16; i += blockDim.x)
        (&red[0][0][0])[i] = 0.0f;
    // the tail of z that pads W2t's rows
    if (blockIdx.x == 0)
        for (int64_t i = p.n + threadIdx.x; i < p.ldt; i += blockDim.x)
            p.z[i] = 0.0f;
    __syncthreads();
    for (int s = 0; s < nsteps; s += 4) {
        SP_LOAD(3, s + 3)
        SP_CONSUME(0, s)
        if (s + 1 >= nsteps)
            break;
        SP_LOAD(0, s + 4)
        SP_CONSUME(1, s + 1)
        if (s + 2 >= nsteps)
            break;
        SP_LOAD(1, s + 5)
        SP_CONSUME(2, s + 2)
        if (s + 3 >= nsteps)
            break;
        SP_LOAD(2, s + 6)
        SP_CONSUME(3, s + 3)
    }
#undef SP_LOAD
#undef SP_CONSUME
}

__global__ __launch_bounds__(1024) void ff_decode_down_kernel(SplitParams p)
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int R = blockDim.x >> 6;
    const int c = (blockIdx.x * R + wave) * 2;                         // rows c and c + 1 of W2t
    const uint16_t *r0 = (const uint16_t *)p.W2t + (int64_t)c * p.ldt + lane * 8;
    const uint16_t *r1 = r0 + p.ldt;
    const int nchunks = (int)(p.ldt / 512);
    // the first pieces are on their way while z moves into LDS; three pieces per row in flight
    // (pieces past the end: the last one again, unused)
    const int last = (nchunks - 1) * 512;
    // three pieces per row in flight (pieces past the end: the last one again, unused); z is read
    // straight from global memory with the same lookahead (22 KB shared by every wave of the chip:
    // cache hits after the first touch), so nothing waits for a staging step
    const float *zl = p.z + lane * 8;
    u32x4_sp w0[3], w1[3];
    f32x4_sp za[3], zb[3];
#pragma unroll
    for (int u = 0; u < 3; ++u) {
        const int o = min(u * 512, last);
        w0[u] = __builtin_nontemporal_load((const u32x4_sp *)(r0 + o));
        w1[u] = __builtin_nontemporal_load((const u32x4_sp *)(r1 + o));
        za[u] = *(const f32x4_sp *)(zl + o);
        zb[u] = *(const f32x4_sp *)(zl + o + 4);
    }
    float acc0 = 0.0f, acc1 = 0.0f;
#define SP_FMA8(acc_, w_, za_, zb_)                                                                                   \
    acc_ = fmaf(__uint_as_float(w_.x << 16), za_.x, acc_); acc_ = fmaf(__uint_as_float(w_.x & 0xFFFF0000u), za_.y, acc_); \
    acc_ = fmaf(__uint_as_float(w_.y << 16), za_.z, acc_); acc_ = fmaf(__uint_as_float(w_.y & 0xFFFF0000u), za_.w, acc_); \
    acc_ = fmaf(__uint_as_float(w_.z << 16), zb_.x, acc_); acc_ = fmaf(__uint_as_float(w_.z & 0xFFFF0000u), zb_.y, acc_); \
    acc_ = fmaf(__uint_as_float(w_.w << 16), zb_.z, acc_); acc_ = fmaf(__uint_as_float(w_.w & 0xFFFF0000u), zb_.w, acc_);
    for (int i0 = 0; i0 < nchunks; i0 += 3) {
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int i = i0 + u;
            if (i < nchunks) {                                             // wave-uniform
                SP_FMA8(acc0, w0[u], za[u], zb[u])
                SP_FMA8(acc1, w1[u], za[u], zb[u])
                const int nx = min((i + 3) * 512, last);
                w0[u] = __builtin_nontemporal_load((const u32x4_sp *)(r0 + nx));
                w1[u] = __builtin_nontemporal_load((const u32x4_sp *)(r1 + nx));
                za[u] = *(const f32x4_sp *)(zl + nx);
                zb[u] = *(const f32x4_sp *)(zl + nx + 4);
            }
        }
    }
#undef SP_FMA8
    acc0 = wave_sum(acc0);
    acc1 = wave_sum(acc1);
    if (lane == 0) {
        if (p.b2) {
            acc0 += bf16_bits_to_f32(((const uint16_t *)p.b2)[c]);
            acc1 += bf16_bits_to_f32(((const uint16_t *)p.b2)[c + 1]);
        }
        ((uint32_t *)p.y)[c >> 1] = f32_to_bf16_bits(acc0) | (f32_to_bf16_bits(acc1) << 16);
    }
}

constexpr int64_t SPLIT_MAX_LDT = (int64_t)1 << 21;

// Can this job take the two-stream path?  One row through one bf16 block that has W2t.
bool decode_split_supported(const DecodeJob &job)
{
    return job.bf16 && job.W2t && !job.multi && !job.idx && job.batch == 1 && job.d % 512 == 0 &&
           job.d / 512 <= 16 && job.ldt % 512 == 0 && job.ldt >= job.n && job.ldt <= SPLIT_MAX_LDT;
}

int launch_decode_split(const DecodeJob &job, hipStream_t st, hipEvent_t ev_mid)
{
    if (job.part_bytes < (size_t)job.ldt * sizeof(float))
        return GRIFFIN_EWORKSPACE;
    SplitParams p;
    p.Wg = job.Wg; p.W1 = job.W1; p.bg = job.bg; p.b1 = job.b1; p.b2 = job.b2; p.W2t = job.W2t;
    p.x = job.x; p.y = job.y; p.z = job.part;
    p.ld = job.ld; p.ldt = job.ldt;
    p.d = job.d; p.n = job.n; p.act = job.act;
    const int R = job.d / 512;
    p.R = R;
    p.teams = R >= 8 ? 1 : 8 / R;
    int P = (job.n + p.teams - 1) / p.teams;       // workgroups: one neuron per team at least
    if (P > 256) P = 256;
    const bool gated = job.Wg != nullptr, bias = job.bg || job.b1;
    dim3 g1(P), b1(p.teams * R * 64);
    if (gated) {
        if (bias) hipLaunchKernelGGL((ff_decode_gu_kernel<true, true>), g1, b1, 0, st, p);
        else hipLaunchKernelGGL((ff_decode_gu_kernel<true, false>), g1, b1, 0, st, p);
    } else {
        if (bias) hipLaunchKernelGGL((ff_decode_gu_kernel<false, true>), g1, b1, 0, st, p);
        else hipLaunchKernelGGL((ff_decode_gu_kernel<false, false>), g1, b1, 0, st, p);
    }
    int rc = check_launch("ff_decode_gu_kernel");
    if (rc != GRIFFIN_OK)
        return rc;
    if (ev_mid && hipEventRecord(ev_mid, st) != hipSuccess)
        return set_hip_error(hipGetLastError(), "hipEventRecord");
    hipLaunchKernelGGL(ff_decode_down_kernel, dim3(job.d / (2 * R)), dim3(R * 64), 0, st, p);
    return check_launch("ff_decode_down_kernel");
}

}  // namespace griffin
