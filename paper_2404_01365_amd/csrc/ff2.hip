// The prompt's own output with the full block (Section 5.1: the prompt phase uses every
// neuron; Eq. 1):  Y = Z W_2^T + b_2 for every prompt token, from the activations Z that the
// selection pass already produced.
//
// A dense contraction (2*S*D_ff*d flop), so bf16 blocks run on the matrix cores.  W_2 is taken
// in the paper's own layout, W2p[d][D_ff] (row c = output feature c), which makes both operands
// K-contiguous ("NT"), exactly the shape of the first GEMM.  Three routes, chosen in launch_ff2:
//   * the usual one (D_ff in whole 64-element k-tiles): a bf16 copy of Z (made here by
//     ff2_z_to_bf16_kernel, or already left by the first GEMM's epilogue) goes through the
//     direct-to-LDS kernel of the first GEMM in its plain mode (256-token x 256-feature tiles,
//     launch_gemm_nt_partials), the long contraction over D_ff cut into ranges that each write
//     an fp32 slab, and ff2_split_sum_kernel adds the slabs in a fixed order, adds b_2 and
//     converts;
//   * D_ff not in whole k-tiles: the register-staged kernel of this file (fp32 Z converted to
//     bf16 on its way through registers into LDS, 16-byte loads, double-buffered, BK = 64, a
//     256-token x 128-feature tile, 4 waves of 128 x 64, v_mfma_f32_32x32x16_bf16, XOR-swizzled
//     LDS rows), with the same ranges and the same sum;
//   * shapes the tiles cannot take (D_ff not a multiple of 8, fp32 blocks): a plain fp32 kernel.
#include "common.h"

namespace griffin {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

struct Ff2Params {
    const float *Z;
    const void *W2p, *b2;
    void *Y;
    float *part;             // [splits][M][d] fp32 when the contraction is split, else unused
    int64_t ldz, ldw, ldy;
    int32_t M, F, d, mt, nt, splits, kt_per_split;
};

constexpr int P_BM = 256, P_BN = 128, P_BK = 64;

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

__global__ __launch_bounds__(256) void ff2_bf16_mfma_kernel(Ff2Params p)
{
    __shared__ u32x4 As[2][P_BM * 8];   // [buffer][row][8 chunks], chunk c of row r at c ^ (r & 7)
    __shared__ u32x4 Bs[2][P_BN * 8];

    const int ntile = p.mt * p.nt, nblk = ntile * p.splits;
    const int per_xcd = (nblk + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= nblk)
        return;
    // prompts are short and D_ff is long: the contraction is cut into `splits` ranges of
    // k-tiles so that every CU has a tile to work on
    const int split = logical / ntile, tile = logical % ntile;
    const int tile_n = tile / p.mt, tile_m = tile % p.mt;
    const int m0 = tile_m * P_BM, n0 = tile_n * P_BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    const int lr = tid >> 3, lc = tid & 7;
    int64_t zo[8], wo[4];
#pragma unroll
    for (int q = 0; q < 8; ++q)
        zo[q] = (int64_t)min(m0 + lr + 32 * q, p.M - 1) * p.ldz + lc * 8;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        wo[q] = (int64_t)min(n0 + lr + 32 * q, p.d - 1) * p.ldw + lc * 8;
    const uint16_t *Wp = (const uint16_t *)p.W2p;
    f32x4 za[8][2];
    u32x4 rb[4];
    const f32x4 zf = {0.f, 0.f, 0.f, 0.f};
    const u32x4 zu = {0u, 0u, 0u, 0u};

#define FF2_LOAD_TILE(k0)                                                                 \
    {                                                                                     \
        const bool ok_ = (k0) + lc * 8 < p.F;      /* D_ff is a multiple of 8 here */     \
        _Pragma("unroll") for (int q = 0; q < 8; ++q)                                     \
        {                                                                                 \
            za[q][0] = ok_ ? *(const f32x4 *)(p.Z + zo[q] + (k0)) : zf;                   \
            za[q][1] = ok_ ? *(const f32x4 *)(p.Z + zo[q] + (k0) + 4) : zf;               \
        }                                                                                 \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                     \
            rb[q] = ok_ ? *(const u32x4 *)(Wp + wo[q] + (k0)) : zu;                       \
    }
#define FF2_STORE_TILE(buf)                                                               \
    {                                                                                     \
        _Pragma("unroll") for (int q = 0; q < 8; ++q)                                     \
        {                                                                                 \
            const int row_ = lr + 32 * q;                                                 \
            u32x4 v_;                                                                     \
            v_.x = pack_bf16(za[q][0].x, za[q][0].y);                                     \
            v_.y = pack_bf16(za[q][0].z, za[q][0].w);                                     \
            v_.z = pack_bf16(za[q][1].x, za[q][1].y);                                     \
            v_.w = pack_bf16(za[q][1].z, za[q][1].w);                                     \
            As[buf][row_ * 8 + (lc ^ (row_ & 7))] = v_;                                   \
        }                                                                                 \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                     \
        {                                                                                 \
            const int row_ = lr + 32 * q;                                                 \
            Bs[buf][row_ * 8 + (lc ^ (row_ & 7))] = rb[q];                                \
        }                                                                                 \
    }
#define FF2_READ_FRAGS(F_, buf, kk)                                                       \
    {                                                                                     \
        const int ch_ = (2 * (kk) + lh) ^ sw;                                             \
        _Pragma("unroll") for (int mi = 0; mi < 4; ++mi)                                  \
            fa[F_][mi] = As[buf][(wm * 128 + mi * 32 + l31) * 8 + ch_];                   \
        _Pragma("unroll") for (int ni = 0; ni < 2; ++ni)                                  \
            fb[F_][ni] = Bs[buf][(wn * 64 + ni * 32 + l31) * 8 + ch_];                    \
    }
#define FF2_MFMA(F_)                                                                      \
    {                                                                                     \
        _Pragma("unroll") for (int mi = 0; mi < 4; ++mi)                                  \
            _Pragma("unroll") for (int ni = 0; ni < 2; ++ni)                              \
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                    \
                    __builtin_bit_cast(bf16x8, fa[F_][mi]), __builtin_bit_cast(bf16x8, fb[F_][ni]), acc[mi][ni], 0, 0, 0); \
    }

    f32x16 acc[4][2];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                acc[mi][ni][i] = 0.0f;

    const int KT_ALL = (p.F + P_BK - 1) / P_BK;
    const int kt0 = split * p.kt_per_split;
    const int KT = min(p.kt_per_split, KT_ALL - kt0);      // >= 1 by construction
    const int l31 = lane & 31, lh = lane >> 5, sw = lane & 7;
    u32x4 fa[2][4], fb[2][2];

    FF2_LOAD_TILE(kt0 * P_BK)
    FF2_STORE_TILE(0)
    __syncthreads();
    FF2_READ_FRAGS(0, 0, 0)
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        const bool more = kt + 1 < KT;
        if (more)
            FF2_LOAD_TILE((kt0 + kt + 1) * P_BK)
        FF2_READ_FRAGS(1, buf, 1)
        FF2_MFMA(0)
        FF2_READ_FRAGS(0, buf, 2)
        FF2_MFMA(1)
        FF2_READ_FRAGS(1, buf, 3)
        FF2_MFMA(0)
        if (more)
            FF2_STORE_TILE(buf ^ 1)
        FF2_MFMA(1)
        __syncthreads();
        if (more)
            FF2_READ_FRAGS(0, buf ^ 1, 0)
    }
#undef FF2_LOAD_TILE
#undef FF2_STORE_TILE
#undef FF2_READ_FRAGS
#undef FF2_MFMA

    // lane holds column (feature) l31 of each 32x32 tile and rows (i>>2)*8 + lh*4 + (i&3)
    if (p.splits > 1) {
        float *part = p.part + (int64_t)split * p.M * p.d;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int col = n0 + wn * 64 + ni * 32 + l31;
            if (col < p.d) {
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int row = m0 + wm * 128 + mi * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
                        if (row < p.M)
                            part[(int64_t)row * p.d + col] = acc[mi][ni][i];
                    }
            }
        }
        return;
    }
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
        const int col = n0 + wn * 64 + ni * 32 + l31;
        if (col < p.d) {
            const float bias = p.b2 ? bf16_bits_to_f32(((const uint16_t *)p.b2)[col]) : 0.0f;
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int row = m0 + wm * 128 + mi * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
                    if (row < p.M)
                        ((uint16_t *)p.Y)[(int64_t)row * p.ldy + col] = (uint16_t)f32_to_bf16_bits(acc[mi][ni][i] + bias);
                }
        }
    }
}

// Y = sum over the splits (ascending, deterministic) + b2, converted to bf16
__global__ __launch_bounds__(256) void ff2_split_sum_kernel(Ff2Params p)
{
    const int64_t total = (int64_t)p.M * p.d;
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= total)
        return;
    float4 a = *(const float4 *)(p.part + i);
    for (int s = 1; s < p.splits; ++s) {
        const float4 t = *(const float4 *)(p.part + (int64_t)s * total + i);
        a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
    }
    const int row = (int)(i / p.d), col = (int)(i % p.d);      // d is a multiple of 4 on this path
    if (p.b2) {
        const uint16_t *b = (const uint16_t *)p.b2 + col;
        a.x += bf16_bits_to_f32(b[0]); a.y += bf16_bits_to_f32(b[1]);
        a.z += bf16_bits_to_f32(b[2]); a.w += bf16_bits_to_f32(b[3]);
    }
    uint16_t *y = (uint16_t *)p.Y + (int64_t)row * p.ldy + col;
    y[0] = (uint16_t)f32_to_bf16_bits(a.x); y[1] = (uint16_t)f32_to_bf16_bits(a.y);
    y[2] = (uint16_t)f32_to_bf16_bits(a.z); y[3] = (uint16_t)f32_to_bf16_bits(a.w);
}

// plain fp32 path: one output per thread, 64 x 4 outputs per workgroup share the Z rows via L1
template <bool BF16>
__global__ __launch_bounds__(256) void ff2_plain_kernel(Ff2Params p)
{
    const int col = blockIdx.x * 64 + (threadIdx.x & 63);
    const int row = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (col >= p.d || row >= p.M)
        return;
    const float *z = p.Z + (int64_t)row * p.ldz;
    float acc = 0.0f;
    for (int j = 0; j < p.F; ++j)
        acc = fmaf(z[j], load_scalar<BF16>(p.W2p, (int64_t)col * p.ldw + j), acc);
    if (p.b2)
        acc += load_scalar<BF16>(p.b2, col);
    store_scalar<BF16>(p.Y, (int64_t)row * p.ldy + col, acc);
}

// Z fp32 -> bf16 copy [M][F] (rounded to nearest even), 8 elements per thread
__global__ __launch_bounds__(256) void ff2_z_to_bf16_kernel(const float *Z, int64_t ldz, int64_t M, int32_t F, uint16_t *Zb)
{
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;       // F is a multiple of 64 on this path
    if (i >= M * F)
        return;
    const int64_t row = i / F;
    const int col = (int)(i % F);
    const f32x4 a = *(const f32x4 *)(Z + row * ldz + col), b = *(const f32x4 *)(Z + row * ldz + col + 4);
    u32x4 o;
    o.x = pack_bf16(a.x, a.y); o.y = pack_bf16(a.z, a.w); o.z = pack_bf16(b.x, b.y); o.w = pack_bf16(b.z, b.w);
    *(u32x4 *)(Zb + i) = o;
}

static inline size_t ff2_align256(size_t v) { return (v + 255) & ~(size_t)255; }

// the direct-to-LDS GEMM takes the shape when D_ff comes in whole 64-wide k-tiles
static bool ff2_dma_ok(const float *Z, int64_t ldz, int64_t M, int32_t F, int32_t d, bool bf16, const void *W2p, int64_t ldw)
{
    return bf16 && ldz % 4 == 0 && (((uintptr_t)Z | (uintptr_t)W2p) & 15) == 0 && gemm_nt_partials_ok(M, d, F, F, ldw);
}

static bool ff2_tiles_ok(const float *Z, int64_t ldz, int32_t F, int32_t d, bool bf16, const void *W2p, int64_t ldw)
{
    return bf16 && F % 8 == 0 && d % 4 == 0 && ldz % 4 == 0 && ldw % 8 == 0 &&
           (((uintptr_t)Z | (uintptr_t)W2p) & 15) == 0;
}

// how many ranges the contraction is cut into, and k-tiles per range
static void ff2_split_plan(int64_t M, int32_t F, int32_t d, int *splits, int *kt_per_split)
{
    const int ntile = (int)((M + P_BM - 1) / P_BM) * ((d + P_BN - 1) / P_BN);
    const int KT = (F + P_BK - 1) / P_BK;
    int s = (512 + ntile - 1) / ntile;
    if (s > 16) s = 16;
    if (s > KT / 8) s = KT / 8;          // at least 8 k-tiles per range
    if (s < 1) s = 1;
    const int per = (KT + s - 1) / s;
    *splits = (KT + per - 1) / per;      // no empty range
    *kt_per_split = per;
}

size_t ff2_workspace_bytes(int64_t M, int32_t F, int32_t d)
{
    int splits, per;
    ff2_split_plan(M, F, d, &splits, &per);
    size_t need = splits > 1 ? (size_t)splits * M * d * sizeof(float) : 0;
    if (M >= 1 && F % 64 == 0 && d % 4 == 0) {
        // direct-to-LDS path: a bf16 copy of Z, then one fp32 slab per range of the contraction
        gemm_nt_split_plan(M, d, F, &splits, &per);
        const size_t dma = ff2_align256((size_t)M * F * 2) + (size_t)splits * M * d * sizeof(float);
        if (dma > need)
            need = dma;
    }
    return need;
}

// Does the prompt-output product of this shape run from a bf16 copy of Z [M][F] at the head of its workspace?
bool ff2_takes_zb(const float *Z, int64_t ldz, int64_t M, int32_t F, int32_t d, bool bf16, const void *W2p, int64_t ldw)
{
    return M >= 1 && ff2_dma_ok(Z, ldz, M, F, d, bf16, W2p, ldw);
}

int launch_ff2(const float *Z, int64_t ldz, int64_t M, int32_t F, int32_t d, bool bf16, const void *W2p,
               int64_t ldw, const void *b2, void *Y, int64_t ldy, float *ws, size_t ws_bytes, hipStream_t st,
               bool zb_ready)
{
    if (M == 0)
        return GRIFFIN_OK;
    Ff2Params p;
    p.Z = Z; p.W2p = W2p; p.b2 = b2; p.Y = Y; p.part = ws;
    p.ldz = ldz; p.ldw = ldw; p.ldy = ldy;
    p.M = (int32_t)M; p.F = F; p.d = d;
    p.splits = 1; p.kt_per_split = (F + P_BK - 1) / P_BK;
    if (ff2_dma_ok(Z, ldz, M, F, d, bf16, W2p, ldw)) {
        int per;
        gemm_nt_split_plan(M, d, F, &p.splits, &per);
        const size_t zb_bytes = ff2_align256((size_t)M * F * 2);
        if (!ws || ((uintptr_t)ws & 15) || ws_bytes < zb_bytes + (size_t)p.splits * M * d * sizeof(float))
            return GRIFFIN_EWORKSPACE;
        uint16_t *Zb = (uint16_t *)ws;
        p.part = (float *)((char *)ws + zb_bytes);
        int rc = GRIFFIN_OK;
        if (!zb_ready) {
            const int64_t oct = M * F / 8;
            hipLaunchKernelGGL(ff2_z_to_bf16_kernel, dim3((unsigned)((oct + 255) / 256)), dim3(256), 0, st, Z, ldz, M, F, Zb);
            if ((rc = check_launch("ff2_z_to_bf16_kernel")) != GRIFFIN_OK)
                return rc;
        }
        if ((rc = launch_gemm_nt_partials(Zb, F, W2p, ldw, M, d, F, p.splits, per, p.part, st)) != GRIFFIN_OK)
            return rc;
        const int64_t quads = (int64_t)M * d / 4;
        hipLaunchKernelGGL(ff2_split_sum_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, p);
        return check_launch("ff2_split_sum_kernel");
    }
    if (ff2_tiles_ok(Z, ldz, F, d, bf16, W2p, ldw)) {
        ff2_split_plan(M, F, d, &p.splits, &p.kt_per_split);
        if (p.splits > 1 && (!ws || ws_bytes < ff2_workspace_bytes(M, F, d) || ((uintptr_t)ws & 15)))
            return GRIFFIN_EWORKSPACE;
        p.mt = (int32_t)((M + P_BM - 1) / P_BM);
        p.nt = (d + P_BN - 1) / P_BN;
        const int nblk = p.mt * p.nt * p.splits;
        hipLaunchKernelGGL(ff2_bf16_mfma_kernel, dim3(((nblk + 7) / 8) * 8), dim3(256), 0, st, p);
        int rc = check_launch("ff2_bf16_mfma_kernel");
        if (rc != GRIFFIN_OK || p.splits == 1)
            return rc;
        const int64_t quads = (int64_t)M * d / 4;
        hipLaunchKernelGGL(ff2_split_sum_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, p);
        return check_launch("ff2_split_sum_kernel");
    }
    p.mt = p.nt = 0;
    dim3 grid((d + 63) / 64, (unsigned)((M + 3) / 4));
    if (bf16)
        hipLaunchKernelGGL(ff2_plain_kernel<true>, grid, dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL(ff2_plain_kernel<false>, grid, dim3(256), 0, st, p);
    return check_launch("ff2_plain_kernel");
}

}  // namespace griffin
