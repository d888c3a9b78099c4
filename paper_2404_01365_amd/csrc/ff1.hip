// Prompt phase, first half: the FF activations of every prompt token (Section 3, Eq. 3 applied
// row-wise; Eq. 2 when there is no gate),
//     Z = sigma(X Wg^T + bg) * (X W1^T + b1),
// together with one sum-of-squares partial per (token row, column tile) from which the row
// norms of Section 4.1 are finished elsewhere.
//
// bf16: a dense contraction, so it runs on the matrix cores.  One workgroup (4 wavefronts, 2x2)
// owns a 128-token x 128-neuron tile of BOTH products: the X tile is staged once in LDS and
// feeds two sets of v_mfma_f32_32x32x16_bf16 accumulators (gate and up), so the epilogue finds
// g_ij and u_ij in the same lane and applies sigma, the gating product, the store of Z and the
// row sum-of-squares without another pass.  Global->LDS copies are 16-byte, double-buffered
// through registers; LDS rows are XOR-swizzled in 16-byte chunks so the ds_read_b128 operand
// fetches are conflict-free.  Workgroup ids are remapped so that each XCD (ids congruent mod 8
// land on the same XCD) walks a contiguous range of tiles and reuses W tiles in its own L2.
//
// fp32: a plain LDS-tiled FMA kernel (64x64 tile); exists for exactness tests and small cases.
#include "common.h"

namespace griffin {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;   // one 16-byte chunk (8 bf16)

constexpr int G_BN = 128, G_BK = 64;
constexpr int G_THREADS = 256;
constexpr int F_BM = 64, F_BN = 64, F_BK = 16;

struct Ff1Params {
    const void *X, *Wg, *W1, *bg, *b1;
    float *Z, *rowpart;
    int64_t ldx, ldw, ldz;
    int32_t M, F, d, nt, mt;
};

// Epilogue shared by the MFMA kernels: sigma, gating, store of Z, row sums of z^2.
// Lane holds column (neuron) l31 of each 32x32 tile and rows (i>>2)*8 + lh*4 + (i&3), i = 0..15.
template <int ACT, bool GATED, int MI>
__device__ __forceinline__ void ff1_mfma_epilogue(const Ff1Params &p, f32x16 (&accU)[MI][2], f32x16 (&accG)[MI][2],
                                                  float (*rs)[64 * MI], int m0, int n0, int tile_n)
{
    constexpr int BM = 64 * MI;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, l31 = lane & 31, lh = lane >> 5;
    float b1j[2], bgj[2];
    int col[2];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
        col[ni] = n0 + wn * 64 + ni * 32 + l31;
        const int cj = min(col[ni], p.F - 1);
        b1j[ni] = p.b1 ? bf16_bits_to_f32(((const uint16_t *)p.b1)[cj]) : 0.0f;
        bgj[ni] = (GATED && p.bg) ? bf16_bits_to_f32(((const uint16_t *)p.bg)[cj]) : 0.0f;
    }
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int lrow = wm * (32 * MI) + mi * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
            const int grow = m0 + lrow;
            float sq = 0.0f;
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                const float u = accU[mi][ni][i] + b1j[ni];
                float z;
                if (GATED)
                    z = act_apply_t<ACT>(accG[mi][ni][i] + bgj[ni]) * u;
                else
                    z = act_apply_t<ACT>(u);
                if (col[ni] < p.F) {
                    sq = fmaf(z, z, sq);
                    if (grow < p.M)
                        __builtin_nontemporal_store(z, &p.Z[(int64_t)grow * p.ldz + col[ni]]);
                }
            }
            // sum over the 32 lanes that share this row
            sq = row16_sum(sq);
            sq += __shfl_xor(sq, 16, 64);
            if (l31 == 0)
                rs[wn][lrow] = sq;
        }
    }
    __syncthreads();
    for (int r = tid; r < BM; r += G_THREADS)
        if (m0 + r < p.M)
            p.rowpart[(int64_t)(m0 + r) * p.nt + tile_n] = rs[0][r] + rs[1][r];
}

// ------------------------------------------------------------------------------------ bf16 / MFMA, direct-to-LDS
// Main path (d a multiple of 32).  Operand tiles go from global memory straight into LDS
// (global_load_lds_dwordx4: lane l of a wave instruction fills 16-byte slot l of a 1 KB region,
// no VGPR staging, no ds_write), BK = 32, four LDS stages, so three k-tiles (~3000 MFMA
// cycles) of loads are in flight.  A row of a stage is 64 B = 4 slots; logical chunk c of row r
// sits in slot c ^ ((r >> 2) & 3), which keeps the ds_read_b128 operand fetches conflict-free;
// the swizzle is applied by choosing which global chunk each lane loads.  The loop body is
// branch-free (loads past the last k-tile re-read the last one into a dead stage) so that the
// scheduler can interleave LDS reads and loads between MFMAs: k-step 1's fragments are read
// under k-step 0's MFMAs, the next tile's first fragments and the tile three ahead under k-step
// 1's.  One bare s_barrier per k-tile, preceded by the vmcnt wait that says tile kt+1 landed.
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void gbl_cvoid_t;

template <int ACT, bool GATED, int MI>
__global__ __launch_bounds__(G_THREADS) void ff1_bf16_mfma_kernel(Ff1Params p)
{
    constexpr int BM = 64 * MI;
    constexpr int NS = 4, BK = 32;
    constexpr int A_SLOTS = BM * 4, B_SLOTS = G_BN * 4;
    constexpr int STAGE = A_SLOTS + (GATED ? 2 : 1) * B_SLOTS;
    constexpr int AQ = MI;                       // 16-row regions of X per wave per k-tile
    constexpr int NLOADS = AQ + (GATED ? 4 : 2);  // LDS-DMA instructions per wave per k-tile
    // s_waitcnt immediates: vmcnt in bits [3:0] and [15:14], expcnt/lgkmcnt fields left at "no wait"
    constexpr int WAIT_ONE_TILE = 0x0F70 | (NLOADS & 15) | ((NLOADS >> 4) << 14);
    constexpr int WAIT_TWO_TILES = 0x0F70 | ((2 * NLOADS) & 15) | (((2 * NLOADS) >> 4) << 14);
    __shared__ u32x4 lds[NS * STAGE];
    __shared__ float rs[2][BM];

    // XCD-aware tile order
    const int nblk = p.mt * p.nt;
    const int per_xcd = (nblk + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= nblk)
        return;
    const int tile_n = logical / p.mt, tile_m = logical % p.mt;
    const int m0 = tile_m * BM, n0 = tile_n * G_BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // loader: lane -> (row of the region, slot in the row) -> global chunk (un-swizzled)
    const int lrow = lane >> 2, lp = lane & 3;
    int64_t xoff[AQ], woff[2];
#pragma unroll
    for (int q = 0; q < AQ; ++q) {
        const int row = (wave * AQ + q) * 16 + lrow;
        xoff[q] = (int64_t)min(m0 + row, p.M - 1) * p.ldx + (lp ^ ((row >> 2) & 3)) * 8;
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int row = (wave * 2 + q) * 16 + lrow;
        woff[q] = (int64_t)min(n0 + row, p.F - 1) * p.ldw + (lp ^ ((row >> 2) & 3)) * 8;
    }
    const uint16_t *Xp = (const uint16_t *)p.X, *W1p = (const uint16_t *)p.W1, *Wgp = (const uint16_t *)p.Wg;
    const int KT = p.d / BK;

#define FF1_ISSUE(kt_)                                                                                   \
    {                                                                                                    \
        u32x4 *st_ = lds + ((kt_) % NS) * STAGE;                                                         \
        const int k0_ = min((kt_), KT - 1) * BK;                                                         \
        _Pragma("unroll") for (int q = 0; q < AQ; ++q)                                                   \
            __builtin_amdgcn_global_load_lds((gbl_cvoid_t *)(Xp + xoff[q] + k0_),                        \
                                             (lds_void_t *)(st_ + (wave * AQ + q) * 64), 16, 0, 0);      \
        _Pragma("unroll") for (int q = 0; q < 2; ++q)                                                    \
            __builtin_amdgcn_global_load_lds((gbl_cvoid_t *)(W1p + woff[q] + k0_),                       \
                                             (lds_void_t *)(st_ + A_SLOTS + (wave * 2 + q) * 64), 16, 0, 0); \
        if (GATED) {                                                                                     \
            _Pragma("unroll") for (int q = 0; q < 2; ++q)                                                \
                __builtin_amdgcn_global_load_lds((gbl_cvoid_t *)(Wgp + woff[q] + k0_),                   \
                                                 (lds_void_t *)(st_ + A_SLOTS + B_SLOTS + (wave * 2 + q) * 64), 16, 0, 0); \
        }                                                                                                \
    }
// Operand fragments are fetched with ds_read_b128 written as inline asm: the compiler makes every
// LDS load it knows about wait for ALL LDS-DMA in flight (it cannot tell the stages apart), which
// would serialise the pipeline.  The asm reads are invisible to that logic; their completion is
// awaited explicitly (FF1_WAIT_FRAGS names the registers, so the MFMAs that use them stay behind
// it), and sched_barrier keeps the hand-made interleaving of reads, DMA issues and MFMAs.
#define FF1_DS_READ(dst, addr, off) asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"((addr) + (uint32_t)(off)))
#define FF1_BARRIER()                                                                                    \
    {                                                                                                    \
        asm volatile("" ::: "memory");                                                                   \
        __builtin_amdgcn_s_barrier();                                                                    \
        asm volatile("" ::: "memory");                                                                   \
    }
#define FF1_PIN() __builtin_amdgcn_sched_barrier(0)

    f32x16 accU[MI][2], accG[MI][2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                accU[mi][ni][i] = 0.0f;
                accG[mi][ni][i] = 0.0f;
            }

    const int l31 = lane & 31, lh = lane >> 5, sw = (l31 >> 2) & 3;
    // byte addresses (inside a stage) of this lane's fragment rows, per k-step
    uint32_t abase[2], bbase[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int ch = (2 * kk + lh) ^ sw;
        abase[kk] = (uint32_t)(((wm * (32 * MI) + l31) * 4 + ch) * 16);
        bbase[kk] = (uint32_t)((A_SLOTS + (wn * 64 + l31) * 4 + ch) * 16);
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void_t *)lds;   // LDS byte address of stage 0
    u32x4 fa[2][MI], f1[2][2], fg[2][2];
    constexpr int NREADS = MI + (GATED ? 4 : 2);
    constexpr int NMFMA = MI * 2;                  // MFMA pairs (up, gate) or singles per k-step
    constexpr int NSLOTS = NMFMA > NREADS ? NMFMA : NREADS;   // interleaving slots per k-step (NLOADS == NREADS)

// read number r (0 .. NREADS-1) of fragment set F_ from stage address sa_/sb_
#define FF1_READ_ONE(F_, r, sa_, sb_)                                                          \
    {                                                                                          \
        if ((r) < MI) FF1_DS_READ(fa[F_][(r) % MI], sa_, ((r) % MI) * 2048);                   \
        else if ((r) < MI + 2) FF1_DS_READ(f1[F_][((r) - MI) % 2], sb_, (((r) - MI) % 2) * 2048); \
        else FF1_DS_READ(fg[F_][((r) - MI) % 2], sb_, B_SLOTS * 16 + (((r) - MI) % 2) * 2048); \
    }
// MFMA(s) number m (0 .. NMFMA-1) of fragment set F_: tile (mi, ni) of the up product and, gated, of the gate product
#define FF1_MFMA_ONE(F_, m)                                                                    \
    {                                                                                          \
        const int mi_ = (m) / 2, ni_ = (m) % 2;                                                \
        accU[mi_][ni_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                              \
            __builtin_bit_cast(bf16x8, fa[F_][mi_]), __builtin_bit_cast(bf16x8, f1[F_][ni_]), accU[mi_][ni_], 0, 0, 0); \
        if (GATED)                                                                             \
            accG[mi_][ni_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                          \
                __builtin_bit_cast(bf16x8, fa[F_][mi_]), __builtin_bit_cast(bf16x8, fg[F_][ni_]), accG[mi_][ni_], 0, 0, 0); \
    }
#define FF1_WAIT_FRAGS(F_)                                                                     \
    {                                                                                          \
        if (MI == 4)                                                                           \
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(fa[F_][0]), "+v"(fa[F_][1]), "+v"(fa[F_][MI - 2]), "+v"(fa[F_][MI - 1]), \
                         "+v"(f1[F_][0]), "+v"(f1[F_][1]), "+v"(fg[F_][0]), "+v"(fg[F_][1]));  \
        else                                                                                   \
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(fa[F_][0]), "+v"(fa[F_][1]),            \
                         "+v"(f1[F_][0]), "+v"(f1[F_][1]), "+v"(fg[F_][0]), "+v"(fg[F_][1]));  \
    }

    FF1_ISSUE(0)
    FF1_ISSUE(1)
    FF1_ISSUE(2)
    __builtin_amdgcn_s_waitcnt(WAIT_TWO_TILES);      // tile 0 landed
    FF1_BARRIER()
    if (!GATED) {
        fg[0][0] = fg[0][1] = fg[1][0] = fg[1][1] = (u32x4){0u, 0u, 0u, 0u};
    }
    {
        const uint32_t sa = lds0 + abase[0], sb = lds0 + bbase[0];
#pragma unroll
        for (int r = 0; r < NREADS; ++r)
            FF1_READ_ONE(0, r, sa, sb)
    }
    for (int kt = 0; kt < KT; ++kt) {
        const uint32_t st_cur = lds0 + (uint32_t)((kt % NS) * STAGE * 16);
        const uint32_t st_nxt = lds0 + (uint32_t)(((kt + 1) % NS) * STAGE * 16);
        // ---- k-step 0 of tile kt; k-step 1's fragments are fetched underneath
        FF1_WAIT_FRAGS(0)
        {
            const uint32_t sa = st_cur + abase[1], sb = st_cur + bbase[1];
            FF1_PIN();
#pragma unroll
            for (int m = 0; m < NSLOTS; ++m) {
                if (m < NREADS)
                    FF1_READ_ONE(1, m, sa, sb)
                if (m < NMFMA)
                    FF1_MFMA_ONE(0, m)
                FF1_PIN();
            }
        }
        // tile kt+1 has landed for this wave when only tile kt+2's loads are outstanding; past the
        // barrier it has landed for every wave, and every wave is done reading tile kt-1, whose
        // stage the loads of tile kt+3 overwrite
        FF1_WAIT_FRAGS(1)
        __builtin_amdgcn_s_waitcnt(WAIT_ONE_TILE);
        FF1_BARRIER()
        // ---- k-step 1; the first fragments of tile kt+1 and the loads of tile kt+3 go underneath
        {
            const uint32_t sa = st_nxt + abase[0], sb = st_nxt + bbase[0];
            u32x4 *st_ = lds + ((kt + 3) % NS) * STAGE;
            const int k0_ = min(kt + 3, KT - 1) * BK;
            FF1_PIN();
#pragma unroll
            for (int m = 0; m < NSLOTS; ++m) {
                if (m < NREADS)
                    FF1_READ_ONE(0, m, sa, sb)
                if (m < AQ)
                    __builtin_amdgcn_global_load_lds((gbl_cvoid_t *)(Xp + xoff[m % AQ] + k0_),
                                                     (lds_void_t *)(st_ + (wave * AQ + (m % AQ)) * 64), 16, 0, 0);
                else if (m < AQ + 2)
                    __builtin_amdgcn_global_load_lds((gbl_cvoid_t *)(W1p + woff[(m - AQ) % 2] + k0_),
                                                     (lds_void_t *)(st_ + A_SLOTS + (wave * 2 + (m - AQ) % 2) * 64), 16, 0, 0);
                else if (GATED && m < AQ + 4)
                    __builtin_amdgcn_global_load_lds((gbl_cvoid_t *)(Wgp + woff[(m - AQ) % 2] + k0_),
                                                     (lds_void_t *)(st_ + A_SLOTS + B_SLOTS + (wave * 2 + (m - AQ) % 2) * 64), 16, 0, 0);
                if (m < NMFMA)
                    FF1_MFMA_ONE(1, m)
                FF1_PIN();
            }
        }
    }
    FF1_WAIT_FRAGS(0)                                 // the reads issued for the tile past the end
    __builtin_amdgcn_s_waitcnt(0x0F70);               // no LDS-DMA may outlive the loop
    FF1_BARRIER()
#undef FF1_ISSUE
#undef FF1_BARRIER
#undef FF1_DS_READ
#undef FF1_PIN
#undef FF1_READ_ONE
#undef FF1_MFMA_ONE
#undef FF1_WAIT_FRAGS

    ff1_mfma_epilogue<ACT, GATED, MI>(p, accU, accG, rs, m0, n0, tile_n);
}

// ------------------------------------------------------------------------------------ bf16 / MFMA, register-staged
// Fallback for d not a multiple of 32 (the k tail is zero-filled in registers, which the
// direct-to-LDS loads cannot do): 16-byte global loads staged through VGPRs into two LDS
// buffers of BK = 64.
template <int ACT, bool GATED, int MI, bool KTAIL>
__global__ __launch_bounds__(G_THREADS) void ff1_bf16_mfma_staged_kernel(Ff1Params p)
{
    constexpr int BM = 64 * MI;
    constexpr int AQ = BM / 32;      // 16-byte chunks of X a thread stages per k-tile
    // [buffer][row][8 chunks of 16 B], chunk c of row r stored at c ^ (r & 7)
    __shared__ u32x4 As[2][BM * 8];
    __shared__ u32x4 B1s[2][G_BN * 8];
    __shared__ u32x4 Bgs[GATED ? 2 : 1][GATED ? G_BN * 8 : 1];
    __shared__ float rs[2][BM];

    // XCD-aware tile order
    const int nblk = p.mt * p.nt;
    const int per_xcd = (nblk + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= nblk)
        return;
    const int tile_n = logical / p.mt, tile_m = logical % p.mt;
    const int m0 = tile_m * BM, n0 = tile_n * G_BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // global -> register staging: thread covers chunk `lc` of rows lr + 32 q.  Row offsets are
    // clamped once (rows past the end re-read the last row; their results are never stored).
    const int lr = tid >> 3, lc = tid & 7;
    const uint16_t *xb = (const uint16_t *)p.X + lc * 8;
    const uint16_t *w1b = (const uint16_t *)p.W1 + lc * 8;
    const uint16_t *wgb = GATED ? (const uint16_t *)p.Wg + lc * 8 : nullptr;
    int64_t xo[AQ], wo[4];
#pragma unroll
    for (int q = 0; q < AQ; ++q)
        xo[q] = (int64_t)min(m0 + lr + 32 * q, p.M - 1) * p.ldx;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        wo[q] = (int64_t)min(n0 + lr + 32 * q, p.F - 1) * p.ldw;
    u32x4 ra[AQ], r1[4], rg[4];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

// global -> registers for the k-tile starting at k0 (with KTAIL, chunks past d read as zero)
#define FF1_LOAD_TILE(k0)                                                     \
    {                                                                         \
        const bool ok_ = !KTAIL || (k0) + lc * 8 < p.d;                       \
        _Pragma("unroll") for (int q = 0; q < AQ; ++q)                        \
            ra[q] = ok_ ? *(const u32x4 *)(xb + xo[q] + (k0)) : zero4;        \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                         \
        {                                                                     \
            r1[q] = ok_ ? *(const u32x4 *)(w1b + wo[q] + (k0)) : zero4;       \
            if (GATED)                                                        \
                rg[q] = ok_ ? *(const u32x4 *)(wgb + wo[q] + (k0)) : zero4;   \
        }                                                                     \
    }
// registers -> LDS buffer `buf`
#define FF1_STORE_TILE(buf)                                                   \
    {                                                                         \
        _Pragma("unroll") for (int q = 0; q < AQ; ++q)                        \
        {                                                                     \
            const int row_ = lr + 32 * q;                                     \
            As[buf][row_ * 8 + (lc ^ (row_ & 7))] = ra[q];                    \
        }                                                                     \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                         \
        {                                                                     \
            const int row_ = lr + 32 * q;                                     \
            const int slot_ = row_ * 8 + (lc ^ (row_ & 7));                   \
            B1s[buf][slot_] = r1[q];                                          \
            if (GATED)                                                        \
                Bgs[buf][slot_] = rg[q];                                      \
        }                                                                     \
    }
// LDS -> MFMA operand fragments of k-step kk of buffer `buf`
#define FF1_READ_FRAGS(F_, buf, kk)                                           \
    {                                                                         \
        const int ch_ = (2 * (kk) + lh) ^ sw;                                 \
        _Pragma("unroll") for (int mi = 0; mi < MI; ++mi)                     \
            fa[F_][mi] = As[buf][(wm * (32 * MI) + mi * 32 + l31) * 8 + ch_]; \
        _Pragma("unroll") for (int ni = 0; ni < 2; ++ni)                      \
        {                                                                     \
            f1[F_][ni] = B1s[buf][(wn * 64 + ni * 32 + l31) * 8 + ch_];       \
            if (GATED)                                                        \
                fg[F_][ni] = Bgs[buf][(wn * 64 + ni * 32 + l31) * 8 + ch_];   \
        }                                                                     \
    }
#define FF1_MFMA(F_)                                                          \
    {                                                                         \
        _Pragma("unroll") for (int mi = 0; mi < MI; ++mi)                     \
            _Pragma("unroll") for (int ni = 0; ni < 2; ++ni)                  \
        {                                                                     \
            accU[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(           \
                __builtin_bit_cast(bf16x8, fa[F_][mi]), __builtin_bit_cast(bf16x8, f1[F_][ni]), accU[mi][ni], 0, 0, 0); \
            if (GATED)                                                        \
                accG[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(       \
                    __builtin_bit_cast(bf16x8, fa[F_][mi]), __builtin_bit_cast(bf16x8, fg[F_][ni]), accG[mi][ni], 0, 0, 0); \
        }                                                                     \
    }

    f32x16 accU[MI][2], accG[MI][2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                accU[mi][ni][i] = 0.0f;
                accG[mi][ni][i] = 0.0f;
            }

    const int KT = (p.d + G_BK - 1) / G_BK;
    const int l31 = lane & 31, lh = lane >> 5, sw = lane & 7;
    u32x4 fa[2][MI], f1[2][2], fg[2][2];      // operand fragments, double-buffered over k-steps

    FF1_LOAD_TILE(0)
    FF1_STORE_TILE(0)
    __syncthreads();
    FF1_READ_FRAGS(0, 0, 0)

    // Per k-tile: the next tile's global loads are issued first; each k-step's MFMAs run on
    // fragments read during the previous k-step; the staged registers go to the other LDS
    // buffer during the last two k-steps; one barrier, then the first fragments of the next
    // tile.
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        const bool more = kt + 1 < KT;
        if (more)
            FF1_LOAD_TILE((kt + 1) * G_BK)
        FF1_READ_FRAGS(1, buf, 1)
        FF1_MFMA(0)
        FF1_READ_FRAGS(0, buf, 2)
        FF1_MFMA(1)
        FF1_READ_FRAGS(1, buf, 3)
        FF1_MFMA(0)
        if (more)
            FF1_STORE_TILE(buf ^ 1)
        FF1_MFMA(1)
        __syncthreads();
        if (more)
            FF1_READ_FRAGS(0, buf ^ 1, 0)
    }

#undef FF1_LOAD_TILE
#undef FF1_STORE_TILE
#undef FF1_READ_FRAGS
#undef FF1_MFMA

    ff1_mfma_epilogue<ACT, GATED, MI>(p, accU, accG, rs, m0, n0, tile_n);
}

// ------------------------------------------------------------------------------------ fp32 / FMA
template <bool GATED>
__global__ __launch_bounds__(256) void ff1_f32_kernel(Ff1Params p, int act)
{
    __shared__ float Xs[F_BK][F_BM + 4];
    __shared__ float W1s[F_BK][F_BN + 4];
    __shared__ float Wgs[F_BK][F_BN + 4];

    const int tile_n = blockIdx.x, tile_m = blockIdx.y;
    const int m0 = tile_m * F_BM, n0 = tile_n * F_BN;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int lrow = tid >> 2, lq = tid & 3;   // staging: row, float4 along k

    const float *xp = (const float *)p.X + (int64_t)min(m0 + lrow, p.M - 1) * p.ldx + lq * 4;
    const float *w1p = (const float *)p.W1 + (int64_t)min(n0 + lrow, p.F - 1) * p.ldw + lq * 4;
    const float *wgp = GATED ? (const float *)p.Wg + (int64_t)min(n0 + lrow, p.F - 1) * p.ldw + lq * 4 : nullptr;

    float g[4][4], u[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            g[i][j] = u[i][j] = 0.0f;

    for (int k0 = 0; k0 < p.d; k0 += F_BK) {
        const bool ok = k0 + lq * 4 < p.d;   // d is a multiple of 4
        float4 vx = ok ? *(const float4 *)(xp + k0) : make_float4(0, 0, 0, 0);
        float4 v1 = ok ? *(const float4 *)(w1p + k0) : make_float4(0, 0, 0, 0);
        float4 vg = (GATED && ok) ? *(const float4 *)(wgp + k0) : make_float4(0, 0, 0, 0);
        __syncthreads();
        Xs[lq * 4 + 0][lrow] = vx.x; Xs[lq * 4 + 1][lrow] = vx.y; Xs[lq * 4 + 2][lrow] = vx.z; Xs[lq * 4 + 3][lrow] = vx.w;
        W1s[lq * 4 + 0][lrow] = v1.x; W1s[lq * 4 + 1][lrow] = v1.y; W1s[lq * 4 + 2][lrow] = v1.z; W1s[lq * 4 + 3][lrow] = v1.w;
        if (GATED) {
            Wgs[lq * 4 + 0][lrow] = vg.x; Wgs[lq * 4 + 1][lrow] = vg.y; Wgs[lq * 4 + 2][lrow] = vg.z; Wgs[lq * 4 + 3][lrow] = vg.w;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < F_BK; ++kk) {
            float a[4], b1v[4], bgv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = Xs[kk][ty * 4 + i];
                b1v[i] = W1s[kk][tx * 4 + i];
                bgv[i] = GATED ? Wgs[kk][tx * 4 + i] : 0.0f;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    u[i][j] = fmaf(a[i], b1v[j], u[i][j]);
                    if (GATED)
                        g[i][j] = fmaf(a[i], bgv[j], g[i][j]);
                }
        }
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int grow = m0 + ty * 4 + i;
        float sq = 0.0f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int colj = n0 + tx * 4 + j;
            if (colj < p.F) {
                float uu = u[i][j] + (p.b1 ? ((const float *)p.b1)[colj] : 0.0f);
                float z;
                if (GATED)
                    z = act_apply(act, g[i][j] + (p.bg ? ((const float *)p.bg)[colj] : 0.0f)) * uu;
                else
                    z = act_apply(act, uu);
                sq = fmaf(z, z, sq);
                if (grow < p.M)
                    p.Z[(int64_t)grow * p.ldz + colj] = z;
            }
        }
        // the 16 threads that share a row are one DPP row of the wavefront
        sq = row16_sum(sq);
        if (tx == 0 && grow < p.M)
            p.rowpart[(int64_t)grow * p.nt + tile_n] = sq;
    }
}

int ff1_ntiles(const griffin_layer &L)
{
    const int bn = L.dtype == GRIFFIN_BF16 ? G_BN : F_BN;
    return (L.n + bn - 1) / bn;
}

template <int ACT, int MI>
static void launch_mfma(const Ff1Params &p, bool gated, hipStream_t st)
{
    const int nblk = p.mt * p.nt;
    dim3 grid(((nblk + 7) / 8) * 8), block(G_THREADS);
    const bool ktail = p.d % 32 != 0;
    if (gated) {
        if (ktail) hipLaunchKernelGGL((ff1_bf16_mfma_staged_kernel<ACT, true, MI, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((ff1_bf16_mfma_kernel<ACT, true, MI>), grid, block, 0, st, p);
    } else {
        if (ktail) hipLaunchKernelGGL((ff1_bf16_mfma_staged_kernel<ACT, false, MI, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((ff1_bf16_mfma_kernel<ACT, false, MI>), grid, block, 0, st, p);
    }
}

template <int MI>
static void launch_mfma_act(const Ff1Params &p, int act, bool gated, hipStream_t st)
{
    switch (act) {
    case GRIFFIN_ACT_SILU: launch_mfma<GRIFFIN_ACT_SILU, MI>(p, gated, st); break;
    case GRIFFIN_ACT_GELU_TANH: launch_mfma<GRIFFIN_ACT_GELU_TANH, MI>(p, gated, st); break;
    default: launch_mfma<GRIFFIN_ACT_RELU, MI>(p, gated, st); break;
    }
}

int launch_ff1(const griffin_layer &L, const void *X, int64_t ldx, int64_t M, float *Z, int64_t ldz,
               float *rowpart, int32_t *nt_out, hipStream_t st)
{
    Ff1Params p;
    p.X = X; p.Wg = L.Wg; p.W1 = L.W1; p.bg = L.bg; p.b1 = L.b1;
    p.Z = Z; p.rowpart = rowpart;
    p.ldx = ldx; p.ldw = L.ld; p.ldz = ldz;
    p.M = (int32_t)M; p.F = L.n; p.d = L.d;
    p.nt = ff1_ntiles(L);
    *nt_out = p.nt;
    if (M == 0)
        return GRIFFIN_OK;
    const bool gated = L.Wg != nullptr;
    if (L.dtype == GRIFFIN_BF16) {
        // 256-token tiles halve the LDS traffic per flop; short prompts keep 128
        if (M > 128) {
            p.mt = (int32_t)((M + 255) / 256);
            launch_mfma_act<4>(p, L.act, gated, st);
        } else {
            p.mt = (int32_t)((M + 127) / 128);
            launch_mfma_act<2>(p, L.act, gated, st);
        }
        return check_launch("ff1_bf16_mfma_kernel");
    }
    p.mt = (int32_t)((M + F_BM - 1) / F_BM);
    dim3 grid(p.nt, p.mt), block(256);
    if (gated)
        hipLaunchKernelGGL(ff1_f32_kernel<true>, grid, block, 0, st, p, L.act);
    else
        hipLaunchKernelGGL(ff1_f32_kernel<false>, grid, block, 0, st, p, L.act);
    return check_launch("ff1_f32_kernel");
}

}  // namespace griffin
