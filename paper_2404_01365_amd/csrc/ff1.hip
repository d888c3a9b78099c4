// Prompt phase, first half: the FF activations of every prompt token (Section 3, Eq. 3 applied
// row-wise; Eq. 2 when there is no gate),
//     Z = sigma(X Wg^T + bg) * (X W1^T + b1),
// together with one sum-of-squares partial per (token row, column tile) from which the row
// norms of Section 4.1 are finished elsewhere.
//
// bf16: a dense contraction, so it runs on the matrix cores.  One workgroup (4 wavefronts, 2x2)
// owns a 256-token (128 for short prompts) x 128-neuron tile of BOTH products: the X tile is
// staged once in LDS and feeds two sets of v_mfma_f32_32x32x16_bf16 accumulators (gate and up),
// so the epilogue finds g_ij and u_ij in the same lane and applies sigma, the gating product,
// the store of Z and the row sum-of-squares without another pass.  Workgroup ids are remapped so
// that each XCD (ids congruent mod 8 land on the same XCD) walks a contiguous range of tiles and
// reuses W tiles in its own L2.  The main kernel loads tiles straight into LDS; a register-staged
// variant takes the shapes it cannot (d not a multiple of 64).
//
// fp32: a plain LDS-tiled FMA kernel (64x64 tile); exists for exactness tests and small cases.
#include "common.h"

#include <atomic>

namespace griffin {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;   // one 16-byte chunk (8 bf16)

constexpr int G_BN = 128, G_BK = 64;
constexpr int G_THREADS = 256;
constexpr int F_BM = 64, F_BN = 64, F_BK = 16;
// s_waitcnt immediate that waits for vmcnt <= n only (expcnt / lgkmcnt fields left at "no wait")
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

struct Ff1Params {
    const void *X, *Wg, *W1, *bg, *b1;
    float *Z, *rowpart;
    uint16_t *Zb;                    // optional bf16 copy of Z [M][ldzb] for the prompt-output product, or NULL
    int64_t ldx, ldw, ldz, ldzb;
    int32_t M, F, d, nt, mt;
    int32_t splits, kt_per_split;    // ranges of the contraction (1 for the activations) and 64-wide k-tiles per range
    int32_t z_stream;                // Z leaves with the non-temporal hint (see launch_ff1)
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
// Epilogue of the main kernel.  Its MFMAs take the weight fragment as the first operand, so the
// accumulator tiles are transposed: a lane holds ONE token (column l31 of the 32x32 tile) and the
// neurons (i>>2)*8 + lh*4 + (i&3): four consecutive neurons per group of four registers.  Z is
// then written 16 bytes at a time and a token's sum of squares needs no cross-lane step (the
// four partials per token, one per (wn, lh), meet in LDS).
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// PLAIN: the kernel serves as a plain C = A B^T with fp32 output (one range of a split contraction):
// no activation, no biases, no row sums; Z points at that range's [M][F] slab.
// One accumulator value out of its AGPR, at the point of use.  Left to itself the compiler copies all
// 256 accumulator registers into VGPRs at the end of the k loop and spills a hundred of them around
// the epilogue; the asm operand keeps each value in the accumulation file until it is wanted.
__device__ __forceinline__ float ff1_acc_read(float a)
{
    float v;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}

// EXTRA: the instantiation that also knows biases and the bf16 copy of Z; the lean one (most models: no FF
// biases, selection alone) is 2 % faster for not carrying those branches and registers through the epilogue.
template <int ACT, bool GATED, int MI, bool PLAIN, bool EQ2W = false, bool EXTRA = true>
__device__ __forceinline__ bool ff1_mfma_epilogue_t(const Ff1Params &p, f32x16 (&accU)[MI][2], f32x16 (&accG)[MI][2],
                                                    float (*rs)[64 * MI], uint32_t rs_lds, uint32_t patch_lds, int m0, int n0,
                                                    int tile_n)
{
    constexpr int BM = 64 * MI;
    // one B matrix (the plain product, or an Eq. 2 block) over a 256-column tile: accG = columns n0 + 128 ..
    constexpr bool WIDE = (PLAIN && GATED) || EQ2W;
    constexpr bool GLU = GATED && !PLAIN && !EQ2W;          // accG is the gate (Eq. 3)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, l31 = lane & 31, lh = lane >> 5;
    const bool vec = ((p.F | (int32_t)p.ldz) & 3) == 0 && ((uintptr_t)p.Z & 15) == 0;
    const bool hb = EXTRA && !PLAIN && (p.b1 != nullptr || (GLU && p.bg != nullptr));
    const uint16_t *b1p = (const uint16_t *)p.b1, *bgp = (const uint16_t *)p.bg;
    const bool bias8 = (((uintptr_t)p.b1 | (uintptr_t)p.bg) & 7) == 0;       // four biases per 8-byte load
    if (vec && (!hb || bias8)) {
        // The usual case (16-byte aligned rows of Z, F a multiple of 4).  A wave's
        // 32-token x 64-neuron block goes through a private LDS patch (32 rows of 256 B, 16-byte
        // chunk c of row r at c ^ (r & 15): writes and reads both spread evenly over the banks) and
        // leaves as 16-byte stores that cover four whole 256-byte row pieces per instruction;
        // storing straight from the accumulator layout would touch 32 different rows with 32 bytes
        // each.  Every LDS access here is inline asm: the next tile's first LDS-DMA loads are in
        // flight, and an access the compiler knows about would wait for them (and for the Z stores).
        const uint32_t patch = patch_lds + (uint32_t)(wave * 32 * 256);
#if defined(__HIP_DEVICE_COMPILE__)
        // the tile's rows of Z as a raw buffer (byte offsets inside a tile stay below 2^31: 256 rows of at most 2^20 floats;
        // cache-policy bit 1 = non-temporal)
        const __amdgpu_buffer_rsrc_t zrsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(p.Z + (int64_t)m0 * p.ldz), 0, 0x7FFFFFFE, 0x00020000);
#endif
        const uint32_t wr = patch + (uint32_t)(l31 * 256);
        const int rrow = lane >> 4, rch = lane & 15;
        // biases of this lane's 32 columns (four consecutive ones per register pair), fetched before any store
        // of Z leaves: a load behind the stores would wait for them all
        uint2 b1w[2][4], bgw[2][4];
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int c = min(n0 + wn * 64 + ni * 32 + g * 8 + lh * 4, p.F - 4);
                b1w[ni][g] = (hb && b1p) ? *(const uint2 *)(b1p + c) : make_uint2(0u, 0u);
                if (EQ2W)       // the second half's b1, 128 columns further on
                    bgw[ni][g] = (hb && b1p) ? *(const uint2 *)(b1p + min(c + G_BN, p.F - 4)) : make_uint2(0u, 0u);
                else
                    bgw[ni][g] = (hb && GLU && bgp) ? *(const uint2 *)(bgp + c) : make_uint2(0u, 0u);
            }
        // (the plain product's wide tile: the second set of accumulators holds the columns 128 further on)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int lrow = wm * (32 * MI) + mi * 32 + l31;
            float sq = 0.0f;
#pragma unroll
        for (int half = 0; half < (WIDE ? 2 : 1); ++half) {
        const int nh = n0 + half * G_BN;
        const int ncol = nh + wn * 64 + rch * 4;
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float u = ff1_acc_read(half == 0 ? accU[mi][ni][g * 4 + e] : accG[mi][ni][g * 4 + e]);
                        float gt = GLU ? ff1_acc_read(accG[mi][ni][g * 4 + e]) : 0.0f;
                        if (hb) {
                            const uint2 &bu = (EQ2W && half == 1) ? bgw[ni][g] : b1w[ni][g];
                            const uint32_t wu = e < 2 ? bu.x : bu.y, wg2 = e < 2 ? bgw[ni][g].x : bgw[ni][g].y;
                            u += __uint_as_float((e & 1) ? (wu & 0xFFFF0000u) : (wu << 16));
                            if (GLU)
                                gt += __uint_as_float((e & 1) ? (wg2 & 0xFFFF0000u) : (wg2 << 16));
                        }
                        v[e] = PLAIN ? u : (GLU ? act_apply_t<ACT>(gt) * u : act_apply_t<ACT>(u));
                    }
                    if (nh + wn * 64 + ni * 32 + g * 8 + lh * 4 >= p.F)
                        v = (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f};
                    sq = fmaf(v[0], v[0], sq); sq = fmaf(v[1], v[1], sq);
                    sq = fmaf(v[2], v[2], sq); sq = fmaf(v[3], v[3], sq);
                    const int cw = (ni * 8 + g * 2 + lh) ^ (l31 & 15);
                    asm volatile("ds_write_b128 %0, %1" :: "v"(wr + (uint32_t)(cw * 16)), "v"(v) : "memory");
                    // keep the groups apart: left alone, the scheduler pulls the accumulator reads of all
                    // 32 groups to the front and spills a hundred registers
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            // rows 4j + rrow of the patch, 16 bytes per lane
            const int tok0 = m0 + wm * (32 * MI) + mi * 32 + rrow;
            // all eight reads leave together; each store waits for its own row only (LDS returns in order)
            f32x4_t pv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int row = 4 * j + rrow;
                asm volatile("ds_read_b128 %0, %1" : "=v"(pv[j]) : "v"(patch + (uint32_t)(row * 256 + ((rch ^ (row & 15)) * 16))) : "memory");
            }
#if defined(__HIP_DEVICE_COMPILE__)      /* the host pass has no buffer builtins */
#define FF1_Z_STREAM_STORE(v_, elem_) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v_), zrsrc, (elem_) * 4, 0, 2)
#else
#define FF1_Z_STREAM_STORE(v_, elem_) (void)0
#endif
#define FF1_PATCH_STORE(j_)                                                                          \
            {                                                                                        \
                asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(pv[j_]) : "n"(7 - (j_)) : "memory");     \
                const int tok = tok0 + 4 * (j_);                                                     \
                if (tok < p.M && ncol < p.F) {                                                       \
                    if (p.z_stream)      /* a buffer store: the two flavours must stay two instructions */ \
                        FF1_Z_STREAM_STORE(pv[j_], (tok - m0) * (int)p.ldz + ncol);                  \
                    else                                                                             \
                        *(f32x4_t *)(p.Z + (int64_t)tok * p.ldz + ncol) = pv[j_];                    \
                    if (EXTRA && !PLAIN && p.Zb) {                                                   \
                        uint2 h_;                                                                    \
                        h_.x = f32_to_bf16_bits(pv[j_][0]) | (f32_to_bf16_bits(pv[j_][1]) << 16);    \
                        h_.y = f32_to_bf16_bits(pv[j_][2]) | (f32_to_bf16_bits(pv[j_][3]) << 16);    \
                        *(uint2 *)(p.Zb + (int64_t)tok * p.ldzb + ncol) = h_;                        \
                    }                                                                                \
                }                                                                                    \
                __builtin_amdgcn_sched_barrier(0);                                                   \
            }
            FF1_PATCH_STORE(0) FF1_PATCH_STORE(1) FF1_PATCH_STORE(2) FF1_PATCH_STORE(3)
            FF1_PATCH_STORE(4) FF1_PATCH_STORE(5) FF1_PATCH_STORE(6) FF1_PATCH_STORE(7)
#undef FF1_PATCH_STORE
#undef FF1_Z_STREAM_STORE
        }
            if (!PLAIN)     // the row's sum of squares over all the columns of the tile (both halves)
                asm volatile("ds_write_b32 %0, %1" :: "v"(rs_lds + (uint32_t)(((wn * 2 + lh) * BM + lrow) * 4)), "v"(sq) : "memory");
        }
        if (PLAIN)
            return true;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        for (int r = tid; r < BM; r += G_THREADS) {
            float q0, q1, q2, q3;
            const uint32_t ra = rs_lds + (uint32_t)(r * 4);
            asm volatile("ds_read_b32 %0, %1" : "=v"(q0) : "v"(ra));
            asm volatile("ds_read_b32 %0, %1" : "=v"(q1) : "v"(ra + (uint32_t)(BM * 4)));
            asm volatile("ds_read_b32 %0, %1" : "=v"(q2) : "v"(ra + (uint32_t)(2 * BM * 4)));
            asm volatile("ds_read_b32 %0, %1" : "=v"(q3) : "v"(ra + (uint32_t)(3 * BM * 4)));
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(q0), "+v"(q1), "+v"(q2), "+v"(q3));
            if (m0 + r < p.M)
                p.rowpart[(int64_t)(m0 + r) * p.nt + tile_n] = (q0 + q1) + (q2 + q3);
        }
        return true;
    }
    // biases, or rows of Z that 16-byte stores cannot take: element by element, no LDS patch
    // (LDS accesses the compiler knows about: they wait for whatever LDS-DMA is in flight)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int lrow = wm * (32 * MI) + mi * 32 + l31;
        const bool rowok = m0 + lrow < p.M;
        float *zrow = p.Z + (int64_t)min(m0 + lrow, p.M - 1) * p.ldz;
        float sq = 0.0f;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int col = n0 + wn * 64 + ni * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
                const int cj = min(col, p.F - 1);
                float u = ff1_acc_read(accU[mi][ni][i]);
                float gt = GATED ? ff1_acc_read(accG[mi][ni][i]) : 0.0f;
                if (!PLAIN && b1p) u += bf16_bits_to_f32(b1p[cj]);
                if (GLU && bgp) gt += bf16_bits_to_f32(bgp[cj]);
                if (EQ2W && b1p) gt += bf16_bits_to_f32(b1p[min(col + G_BN, p.F - 1)]);
                const float z = PLAIN ? u : (GLU ? act_apply_t<ACT>(gt) * u : act_apply_t<ACT>(u));
                if (col < p.F) {
                    sq = fmaf(z, z, sq);
                    if (rowok)
                        zrow[col] = z;
                }
                if (WIDE && col + G_BN < p.F) {
                    const float z2 = EQ2W ? act_apply_t<ACT>(gt) : gt;
                    sq = fmaf(z2, z2, sq);
                    if (rowok)
                        zrow[col + G_BN] = z2;
                }
            }
        }
        rs[wn * 2 + lh][lrow] = sq;
    }
    if (PLAIN)
        return false;
    __syncthreads();
    for (int r = tid; r < BM; r += G_THREADS)
        if (m0 + r < p.M)
            p.rowpart[(int64_t)(m0 + r) * p.nt + tile_n] = (rs[0][r] + rs[1][r]) + (rs[2][r] + rs[3][r]);
    return false;
}

// Main path (d a multiple of 64).  Operand tiles go from global memory straight into LDS
// (buffer_load_dwordx4 ... lds: lane l of a wave instruction fills 16-byte slot l of a 1 KB
// region; no VGPR staging, no ds_write).  A k-tile is BK = 64 elements = one whole 128-byte
// cache line per row: with half lines the other half is evicted from the 32 KB vector L1
// before the next k-tile asks for it, every line crosses the L2->L1 path twice and that path
// (64 B/clk) becomes the bound.  An instruction covers 8 rows x 128 B.  Two LDS stages; a row
// of a stage is 8 slots (128 B, half of the 256 bytes the LDS banks span), logical chunk c of
// row r in slot c ^ ((r >> 1) & 7): sixteen consecutive rows then land on sixteen different
// 16-byte bank groups, which keeps the ds_read_b128 operand fetches conflict-free (with
// c ^ (r & 7) rows two apart collide and the bank-conflict counter showed the LDS stalled for
// half of its active cycles); the swizzle is applied by choosing which global chunk each lane
// loads.  Per k-tile: four k-steps of MFMAs on fragments read one k-step ahead;
// after the third, vmcnt(0) + one bare s_barrier say that the next tile has landed for every
// wave and that every wave has read its last fragment of this tile, so the loads of the tile
// after next go into this tile's stage under the fourth k-step (first half) and under the next
// tile's first k-step (second half).  Loads past the last k-tile re-read the last one into a
// dead stage, which keeps the loop body branch-free.
typedef __attribute__((address_space(3))) void lds_void_t;
// slot swizzle of row r (rows of every stage section start at a multiple of 16)
#define FF1_SWZ(r) (((r) >> 1) & 7)

template <int ACT, bool GATED, int MI, bool PLAIN, bool EQ2W = false, bool EXTRA = true>
__global__ __launch_bounds__(G_THREADS) void ff1_bf16_mfma_kernel(Ff1Params p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass has no buffer-descriptor builtins; it only needs the launch stub
    constexpr int BM = 64 * MI, BK = 64;
    constexpr int STAGE = (BM + (GATED ? 2 : 1) * G_BN) * 8;   // 16-byte slots per stage
    constexpr int W1_SLOT = BM * 8, WG_SLOT = (BM + G_BN) * 8;
    constexpr int XQ = BM / 32, WQ = G_BN / 32;                // 8-row regions per wave per k-tile
    constexpr int NLOADS = XQ + (GATED ? 2 : 1) * WQ;          // LDS-DMA instructions per wave per k-tile
    constexpr int H1 = NLOADS / 2;
    // The plain product has one B matrix: its tile is 256 columns wide and the "gate" half of the
    // machinery (LDS section, fragments, accumulators) takes columns n0 + 128 .. n0 + 255, which
    // halves the X traffic per flop exactly as the dual product does.
    constexpr bool WIDE = (PLAIN && GATED) || EQ2W;        // EQ2W: an Eq. 2 block (no gate) through the same machinery
    static_assert(!EQ2W || (GATED && !PLAIN), "the Eq. 2 wide tile uses both LDS sections and both accumulator sets");
    constexpr int TILE_N = WIDE ? 2 * G_BN : G_BN;
    __shared__ u32x4 lds[2 * STAGE];
    __shared__ float rs[4][BM];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // XCD-aware tile order (workgroup ids congruent mod 8 share an XCD: each XCD walks its own
    // contiguous range of tiles, its workgroups side by side); with a split contraction the ranges
    // of one tile are `ntile` ids apart.  The grid holds one workgroup per CU and every workgroup
    // walks through its tiles itself, so that the first loads of the next tile can go out before
    // the epilogue of this one (a workgroup per tile leaves the CU idle while the next one starts).
    const int ntile = p.mt * p.nt, nblk = ntile * p.splits;
    // Order of the tiles: panels of PANEL_M token tiles; inside a panel the token tile runs fastest, then the
    // neuron tile.  The 32 workgroups of an XCD then work on 8 token tiles x 4 neuron tiles at any time (12
    // operand slices stream through its L2 per k-tile) instead of 32 token tiles x 1 neuron tile (33 slices)
    // when the prompt batch is long; a last panel of fewer token tiles is walked the same way.  With at most
    // PANEL_M token tiles this is the plain order "token tile fastest".
    constexpr int PANEL_M = 8;
    const int full_m = (p.mt / PANEL_M) * PANEL_M, full_tiles = full_m * p.nt;
    const int per_xcd = (nblk + 7) / 8;
    const int wg_per_xcd = gridDim.x >> 3;
    int slot = blockIdx.x >> 3;
    if (slot >= per_xcd || (int)(blockIdx.x & 7) * per_xcd + slot >= nblk)
        return;

    // per-tile addressing: the loader maps lane -> (row of the 8-row region, slot in the row) ->
    // global chunk (un-swizzled); byte offsets are relative to the tile's first row and fit 32 bits
    // (checked at launch).  Raw buffer descriptors (32-bit data format word of gfx9-family raw
    // buffers); every access is in range by construction, the record count is not relied upon.
    constexpr int RSRC_FLAGS = 0x00020000, RSRC_RECORDS = 0x7FFFFFFE;
    const int lrow = lane >> 3;
    int m0, n0, tile_n, kt0, KT;
    float *Zt;
    uint32_t xvo[XQ], wvo[WQ], wgvo[WQ];
    __amdgpu_buffer_rsrc_t rX, rW1, rWg;
#define FF1_TILE_ADDR(logical_)                                                                          \
    {                                                                                                    \
        const int split_ = (logical_) / ntile, tile_ = (logical_) % ntile;                               \
        {                                                                                                \
            const int in_full_ = tile_ < full_tiles ? 1 : 0;                                             \
            const int w_ = in_full_ ? tile_ % (PANEL_M * p.nt) : tile_ - full_tiles;                     \
            const int pm_ = in_full_ ? PANEL_M : p.mt - full_m;                                          \
            tile_n = w_ / pm_;                                                                           \
            m0 = ((in_full_ ? (tile_ / (PANEL_M * p.nt)) * PANEL_M : full_m) + w_ % pm_) * BM;           \
        }                                                                                                \
        n0 = tile_n * TILE_N;                                                                            \
        Zt = PLAIN ? p.Z + (int64_t)split_ * p.M * p.ldz : p.Z;                                          \
        _Pragma("unroll") for (int q = 0; q < XQ; ++q)                                                   \
            xvo[q] = (uint32_t)min((wave * XQ + q) * 8 + lrow, p.M - 1 - m0) * (uint32_t)(p.ldx * 2) +   \
                     (uint32_t)(((lane & 7) ^ FF1_SWZ((wave * XQ + q) * 8 + lrow)) * 16);                \
        _Pragma("unroll") for (int q = 0; q < WQ; ++q)                                                   \
        {                                                                                                \
            wvo[q] = (uint32_t)min((wave * WQ + q) * 8 + lrow, p.F - 1 - n0) * (uint32_t)(p.ldw * 2) +   \
                     (uint32_t)(((lane & 7) ^ FF1_SWZ((wave * WQ + q) * 8 + lrow)) * 16);                \
            wgvo[q] = WIDE ? (uint32_t)min(G_BN + (wave * WQ + q) * 8 + lrow, p.F - 1 - n0) * (uint32_t)(p.ldw * 2) + \
                             (uint32_t)(((lane & 7) ^ FF1_SWZ((wave * WQ + q) * 8 + lrow)) * 16)         \
                           : wvo[q];                                                                     \
        }                                                                                                \
        rX = __builtin_amdgcn_make_buffer_rsrc((void *)((const uint16_t *)p.X + (int64_t)m0 * p.ldx), 0, \
                                               RSRC_RECORDS, RSRC_FLAGS);                                \
        rW1 = __builtin_amdgcn_make_buffer_rsrc((void *)((const uint16_t *)p.W1 + (int64_t)n0 * p.ldw), 0, \
                                                RSRC_RECORDS, RSRC_FLAGS);                               \
        rWg = __builtin_amdgcn_make_buffer_rsrc((void *)((const uint16_t *)((GATED && !PLAIN && !EQ2W) ? p.Wg : p.W1) + (int64_t)n0 * p.ldw), 0, \
                                                RSRC_RECORDS, RSRC_FLAGS);                               \
        kt0 = split_ * p.kt_per_split;                                                                   \
        KT = min(p.kt_per_split, p.d / BK - kt0);      /* k-tiles of this range (>= 1 by construction) */ \
    }
    FF1_TILE_ADDR((int)(blockIdx.x & 7) * per_xcd + slot)

// LDS-DMA instruction number q (0 .. NLOADS-1: the X regions, then W1, then Wg) of k-tile kt_.
// The weight tiles carry the non-temporal hint (each is used by one wave of tiles and then never
// again; measured 3 % faster), the X tiles, which every column of tiles re-reads, do not.
#define FF1_LOAD_ONE(kt_, q)                                                                             \
    {                                                                                                    \
        u32x4 *st_ = lds + ((kt_) & 1) * STAGE;                                                          \
        const int so_ = (kt0 + min((kt_), KT - 1)) * (BK * 2);                                           \
        if ((q) < XQ)                                                                                    \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rX, (lds_void_t *)(st_ + (wave * XQ + (q) % XQ) * 64), 16, \
                                                     xvo[(q) % XQ], so_, 0, 0);                          \
        else if ((q) < XQ + WQ)                                                                          \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rW1, (lds_void_t *)(st_ + W1_SLOT + (wave * WQ + ((q) - XQ) % WQ) * 64), 16, \
                                                     wvo[((q) - XQ) % WQ], so_, 0, 2);                   \
        else if (GATED)                                                                                  \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rWg, (lds_void_t *)(st_ + WG_SLOT + (wave * WQ + ((q) - XQ) % WQ) * 64), 16, \
                                                     wgvo[((q) - XQ) % WQ], so_, 0, 2);                  \
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

    const int l31 = lane & 31, lh = lane >> 5, sw = FF1_SWZ(l31);
    // byte addresses (inside a stage) of this lane's fragment rows, per k-step
    uint32_t abase[4], bbase[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int ch = (2 * kk + lh) ^ sw;
        abase[kk] = (uint32_t)(((wm * (32 * MI) + l31) * 8 + ch) * 16);
        bbase[kk] = (uint32_t)(((BM + wn * 64 + l31) * 8 + ch) * 16);
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void_t *)lds;   // LDS byte address of stage 0
    u32x4 fa[2][MI], f1[2][2], fg[2][2];
    constexpr int NREADS = MI + (GATED ? 4 : 2);
    constexpr int NMFMA = MI * 2;                  // MFMA pairs (up, gate) or singles per k-step
    constexpr int NSLOTS = NMFMA > NREADS ? NMFMA : NREADS;   // interleaving slots per k-step
    static_assert(H1 <= NSLOTS && NLOADS - H1 <= NSLOTS, "the loads of a k-tile must fit two k-steps");

// read number r (0 .. NREADS-1) of fragment set F_ from stage addresses sa_/sb_ (32 rows = 4096 B apart)
#define FF1_READ_ONE(F_, r, sa_, sb_)                                                          \
    {                                                                                          \
        if ((r) < MI) FF1_DS_READ(fa[F_][(r) % MI], sa_, ((r) % MI) * 4096);                   \
        else if ((r) < MI + 2) FF1_DS_READ(f1[F_][((r) - MI) % 2], sb_, (((r) - MI) % 2) * 4096); \
        else FF1_DS_READ(fg[F_][((r) - MI) % 2], sb_, G_BN * 128 + (((r) - MI) % 2) * 4096);   \
    }
// MFMA(s) number m (0 .. NMFMA-1) of fragment set F_: tile (mi, ni) of the up product and, gated,
// of the gate product; weights first, so the result tile is neurons x tokens
#define FF1_MFMA_ONE(F_, m)                                                                    \
    {                                                                                          \
        const int mi_ = (m) / 2, ni_ = (m) % 2;                                                \
        accU[mi_][ni_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                              \
            __builtin_bit_cast(bf16x8, f1[F_][ni_]), __builtin_bit_cast(bf16x8, fa[F_][mi_]), accU[mi_][ni_], 0, 0, 0); \
        if (GATED)                                                                             \
            accG[mi_][ni_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                          \
                __builtin_bit_cast(bf16x8, fg[F_][ni_]), __builtin_bit_cast(bf16x8, fa[F_][mi_]), accG[mi_][ni_], 0, 0, 0); \
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
// one k-step: MFMAs on fragment set FM_, the reads of set FR_ (k-step KR_ of the stage at sr_)
// and up to NSLOTS loads (numbers L0_ .. L1_-1 of k-tile LT_) interleaved underneath
#define FF1_KSTEP(FM_, FR_, sr_, KR_, LT_, L0_, L1_)                                           \
    {                                                                                          \
        const uint32_t sa = (sr_) + abase[KR_], sb = (sr_) + bbase[KR_];                       \
        FF1_PIN();                                                                             \
        _Pragma("unroll") for (int m = 0; m < NSLOTS; ++m)                                     \
        {                                                                                      \
            if (m < NREADS)                                                                    \
                FF1_READ_ONE(FR_, m, sa, sb)                                                   \
            if ((L0_) + m < (L1_))                                                             \
                FF1_LOAD_ONE(LT_, (L0_) + m)                                                   \
            if (m < NMFMA)                                                                     \
                FF1_MFMA_ONE(FM_, m)                                                           \
            FF1_PIN();                                                                         \
        }                                                                                      \
    }

    // k-tile 0 of a tile goes to stage 0 in full.  Of k-tile 1 only loads that fill the X section of
    // stage 1 may go out with it: the weights' part of stage 1 (32 KB from its W1 section on) holds the
    // epilogue's patches of the tile before, so a load into it has to follow the epilogue.  With 256-token
    // tiles the first half of the loads is exactly the X regions; with 128-token tiles it would reach two
    // W1 regions, which therefore wait.  Blocks with one weight section keep the patches at the head of
    // stage 1 and send nothing early.
    constexpr int EARLY1 = GATED ? (H1 < XQ ? H1 : XQ) : 0;
    static_assert(EARLY1 <= XQ, "early loads of k-tile 1 must stay inside the X section of stage 1");
    // Global store instructions that EVERY wave issues in the epilogue's usual path on a tile that lies
    // wholly inside the matrix (8 per 32-token block, plus the row sums when all four waves write them).
    // The wait for k-tile 0 of the next tile may leave that many operations outstanding, no more: a
    // wave that issued fewer stores than the wait allows would sail through before its loads landed.
    constexpr int EPI_STORES = MI * 8 * (WIDE ? 2 : 1) + ((!PLAIN && MI == 4) ? 1 : 0);
    const uint32_t rs_lds = (uint32_t)(uintptr_t)(lds_void_t *)rs;
    const uint32_t patch_lds = lds0 + (uint32_t)(STAGE * 16) + (GATED ? (uint32_t)(BM * 128) : 0u);
#define FF1_FIRST_LOADS()                                                                      \
    {                                                                                          \
        _Pragma("unroll") for (int q = 0; q < NLOADS; ++q) FF1_LOAD_ONE(0, q)                  \
        _Pragma("unroll") for (int q = 0; q < EARLY1; ++q) FF1_LOAD_ONE(1, q)                  \
    }
    FF1_FIRST_LOADS()
    bool stores_known = false;         // the tile before was whole and took the epilogue's usual path
    if (!GATED) {
        fg[0][0] = fg[0][1] = fg[1][0] = fg[1][1] = (u32x4){0u, 0u, 0u, 0u};
    }
    for (;;) {
#pragma unroll
        for (int q = EARLY1; q < H1; ++q)
            FF1_LOAD_ONE(1, q)
        // k-tile 0 has landed when only the first half of k-tile 1 and (from the second tile on) the
        // epilogue's stores, all issued after it, are still outstanding
        if (stores_known && EXTRA && !PLAIN && p.Zb)      // twice the Z stores: more than the counter holds, 63 is as good
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(H1 + EPI_STORES + MI * 8 > 63 ? 63 : H1 + EPI_STORES + MI * 8));
        else if (stores_known)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(H1 + EPI_STORES > 63 ? 63 : H1 + EPI_STORES));
        else
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(H1));
        FF1_BARRIER()
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    accU[mi][ni][i] = 0.0f;
                    accG[mi][ni][i] = 0.0f;
                }
        {
            const uint32_t sa = lds0 + abase[0], sb = lds0 + bbase[0];
#pragma unroll
            for (int r = 0; r < NREADS; ++r)
                FF1_READ_ONE(0, r, sa, sb)
        }
        for (int kt = 0; kt < KT; ++kt) {
            const uint32_t st_cur = lds0 + (uint32_t)((kt & 1) * STAGE * 16);
            const uint32_t st_nxt = lds0 + (uint32_t)(((kt + 1) & 1) * STAGE * 16);
            FF1_WAIT_FRAGS(0)
            FF1_KSTEP(0, 1, st_cur, 1, kt + 1, H1, NLOADS)     // second half of the next tile's loads
            FF1_WAIT_FRAGS(1)
            FF1_KSTEP(1, 0, st_cur, 2, 0, 0, 0)
            FF1_WAIT_FRAGS(0)
            FF1_KSTEP(0, 1, st_cur, 3, 0, 0, 0)
            FF1_WAIT_FRAGS(1)
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));          // tile kt+1 has landed (this wave's part)
            FF1_BARRIER()                                      // ... every wave's part; tile kt is read out
            FF1_KSTEP(1, 0, st_nxt, 0, kt + 2, 0, H1)          // first half of the loads of the tile after next
        }
        FF1_WAIT_FRAGS(0)                                 // the reads issued for the tile past the end
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));         // no LDS-DMA of this tile is left in flight
        FF1_BARRIER()

        // this tile's coordinates for the epilogue; then the next tile's first loads go out
        Ff1Params pt = p;
        pt.Z = Zt;
        const int m0c = m0, n0c = n0, tile_nc = tile_n;
        const bool whole = m0 + BM <= p.M && n0 + TILE_N <= p.F;
        slot += wg_per_xcd;
        const int logical_n = (int)(blockIdx.x & 7) * per_xcd + slot;
        const bool more = slot < per_xcd && logical_n < nblk;
        if (more) {
            FF1_TILE_ADDR(logical_n)
            FF1_FIRST_LOADS()
        }
        const bool usual = ff1_mfma_epilogue_t<ACT, GATED, MI, PLAIN, EQ2W, EXTRA>(pt, accU, accG, rs, rs_lds, patch_lds, m0c, n0c, tile_nc);
        if (!more)
            break;
        FF1_BARRIER()              // every wave is done with its patch and the row sums
        stores_known = usual && whole;
    }
#undef FF1_TILE_ADDR
#undef FF1_FIRST_LOADS
#undef FF1_LOAD_ONE
#undef FF1_BARRIER
#undef FF1_DS_READ
#undef FF1_PIN
#undef FF1_READ_ONE
#undef FF1_MFMA_ONE
#undef FF1_WAIT_FRAGS
#undef FF1_KSTEP
#endif
}

// ------------------------------------------------------------------------------------ bf16 / MFMA, register-staged
// Fallback for d not a multiple of 64 or row strides too long for 32-bit byte offsets (the k tail is zero-filled in registers, which the
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

// one workgroup per CU (a multiple of 8, so that every XCD gets the same number), fewer if there are fewer tiles.
// The CU count is asked of the current device at every launch's first use on that device and kept per device.
static int ff1_grid(int nblk)
{
    constexpr int MAX_DEV = 64;
    static std::atomic<int> cus_of[MAX_DEV];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV)
        dev = -1;
    int cus = dev >= 0 ? cus_of[dev].load(std::memory_order_relaxed) : 0;
    if (cus == 0) {
        int n = 0;
        if (dev < 0 || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8)
            n = 256;
        cus = n & ~7;
        if (dev >= 0)
            cus_of[dev].store(cus, std::memory_order_relaxed);
    }
    const int want = ((nblk + 7) / 8) * 8;
    return want < cus ? want : cus;
}

template <int ACT, int MI>
static void launch_mfma(const Ff1Params &p, bool gated, bool wide, hipStream_t st)
{
    const int nblk = p.mt * p.nt;
    dim3 grid(ff1_grid(nblk)), block(G_THREADS);
    dim3 grid_all(((nblk + 7) / 8) * 8);           // the register-staged kernel takes one tile per workgroup
    // the direct-to-LDS kernel wants whole 64-element k-tiles and 32-bit byte offsets inside a tile
    const bool ktail = p.d % 64 != 0 || p.ldx > (1 << 21) || p.ldw > (1 << 21);
    if (gated) {
        if (ktail) hipLaunchKernelGGL((ff1_bf16_mfma_staged_kernel<ACT, true, MI, true>), grid_all, block, 0, st, p);
        else if (p.Zb || p.b1 || p.bg) hipLaunchKernelGGL((ff1_bf16_mfma_kernel<ACT, true, MI, false>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((ff1_bf16_mfma_kernel<ACT, true, MI, false, false, false>), grid, block, 0, st, p);
    } else {
        if (ktail) hipLaunchKernelGGL((ff1_bf16_mfma_staged_kernel<ACT, false, MI, true>), grid_all, block, 0, st, p);
        else if (wide) hipLaunchKernelGGL((ff1_bf16_mfma_kernel<ACT, true, MI, false, true>), grid, block, 0, st, p);   // 256-column tiles
        else hipLaunchKernelGGL((ff1_bf16_mfma_kernel<ACT, false, MI, false>), grid, block, 0, st, p);
    }
}

template <int MI>
static void launch_mfma_act(const Ff1Params &p, int act, bool gated, bool wide, hipStream_t st)
{
    switch (act) {
    case GRIFFIN_ACT_SILU: launch_mfma<GRIFFIN_ACT_SILU, MI>(p, gated, wide, st); break;
    case GRIFFIN_ACT_GELU_TANH: launch_mfma<GRIFFIN_ACT_GELU_TANH, MI>(p, gated, wide, st); break;
    default: launch_mfma<GRIFFIN_ACT_RELU, MI>(p, gated, wide, st); break;
    }
}

// Will the first GEMM's own epilogue leave a bf16 copy of Z beside the fp32 one?  Only the direct-to-LDS
// kernel's usual store path does (bf16 block, d in whole k-tiles, 16-byte aligned rows of Z, biases 8-byte aligned).
bool ff1_can_write_zb(const griffin_layer &L, int64_t ldx, const float *Z, int64_t ldz)
{
    const bool ktail = L.d % 64 != 0 || ldx > (1 << 21) || L.ld > (1 << 21);
    const bool vec = ((L.n | (int32_t)ldz) & 3) == 0 && ((uintptr_t)Z & 15) == 0;
    const bool bias8 = (((uintptr_t)L.b1 | (uintptr_t)L.bg) & 7) == 0;
    return L.dtype == GRIFFIN_BF16 && !ktail && vec && bias8;
}

int launch_ff1(const griffin_layer &L, const void *X, int64_t ldx, int64_t M, float *Z, int64_t ldz,
               float *rowpart, int32_t *nt_out, hipStream_t st, uint16_t *Zb, int64_t ldzb)
{
    Ff1Params p;
    p.X = X; p.Wg = L.Wg; p.W1 = L.W1; p.bg = L.bg; p.b1 = L.b1;
    p.Z = Z; p.rowpart = rowpart;
    p.Zb = (Zb && ff1_can_write_zb(L, ldx, Z, ldz)) ? Zb : nullptr;
    p.ldzb = ldzb;
    p.ldx = ldx; p.ldw = L.ld; p.ldz = ldz;
    p.M = (int32_t)M; p.F = L.n; p.d = L.d;
    p.splits = 1; p.kt_per_split = L.d / 64;
    // Z is read again at once by the statistic kernel.  While it fits the 256 MB Infinity Cache, plain stores leave it
    // there for that kernel; a Z several times that size is better sent past the caches (measured, statistic kernel
    // after plain / non-temporal stores: 201 MB of Z 38.3 / 44.6 us, 57 MB 14.5 / 16.4 us, 1.18 GB 284 / 243 us; the
    // product itself takes the same time either way).
    p.z_stream = ((int64_t)M * L.n * 4 > ((int64_t)384 << 20) && ldz <= (1 << 20)) ? 1 : 0;   // (32-bit byte offsets inside a tile)
    p.nt = ff1_ntiles(L);
    const bool gated = L.Wg != nullptr;
    // An Eq. 2 block on the direct-to-LDS kernel takes 256-column tiles (one row-sum partial per tile) when that
    // is the faster way to fill the chip: a 128-column tile of one product is bound by the L2->L1 path (~1400
    // clocks per k-tile), a 256-column tile by the matrix cores (~2550), and either comes in rounds of one tile per CU.
    bool wide = false;
    if (L.dtype == GRIFFIN_BF16 && !gated && !(L.d % 64 != 0 || ldx > (1 << 21) || L.ld > (1 << 21))) {
        const int64_t mt = M > 128 ? (M + 255) / 256 : (M + 127) / 128;
        const int64_t tn = mt * p.nt, tw = mt * ((L.n + 2 * G_BN - 1) / (2 * G_BN));
        wide = ((tw + 255) / 256) * 2550 < ((tn + 255) / 256) * 1400;
        if (wide)
            p.nt = (L.n + 2 * G_BN - 1) / (2 * G_BN);
    }
    *nt_out = p.nt;
    if (M == 0)
        return GRIFFIN_OK;
    if (L.dtype == GRIFFIN_BF16) {
        // 256-token tiles halve the LDS traffic per flop; short prompts keep 128
        if (M > 128) {
            p.mt = (int32_t)((M + 255) / 256);
            launch_mfma_act<4>(p, L.act, gated, wide, st);
        } else {
            p.mt = (int32_t)((M + 127) / 128);
            launch_mfma_act<2>(p, L.act, gated, wide, st);
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

// C[s] = A B^T over the s-th range of the contraction, fp32, for s = 0 .. splits-1, on the
// direct-to-LDS kernel: A [M][K] and B [N][K] bf16 with K a multiple of 64, C [splits][M][N].
// Used by the prompt-output GEMM (Section 5.1) on a bf16 copy of Z.
bool gemm_nt_partials_ok(int64_t M, int32_t N, int32_t K, int64_t lda, int64_t ldb)
{
    return M >= 1 && M <= (1 << 30) && K % 64 == 0 && N % 4 == 0 && lda % 8 == 0 && ldb % 8 == 0 &&
           lda <= (1 << 21) && ldb <= (1 << 21);
}

void gemm_nt_split_plan(int64_t M, int32_t N, int32_t K, int *splits, int *kt_per_split)
{
    const int bm = M > 128 ? 256 : 128;
    const int64_t ntile = ((M + bm - 1) / bm) * ((N + 2 * G_BN - 1) / (2 * G_BN));
    const int KT = K / 64;
    int best = 1;
    int64_t best_cost = -1;
    for (int s = 1; s <= 16 && s <= KT; ++s) {
        const int per = (KT + s - 1) / s;
        if (s > 1 && per < 16)
            break;
        const int used = (KT + per - 1) / per;
        const int64_t rounds = (ntile * used + 255) / 256;
        // in units of one k-tile on every CU (~1.1 us): 8 k-tiles' worth of prologue and epilogue per item, and
        // every range writes an fp32 slab that the sum reads again (8 bytes per element at ~5 TB/s: 5.4 MB per unit)
        const int64_t slab = (int64_t)used * ((M * N * 8) / 5400000);
        const int64_t cost = rounds * (per + 8) + slab;
        if (best_cost < 0 || cost < best_cost) {
            best_cost = cost;
            best = s;
        }
    }
    const int per = (KT + best - 1) / best;
    *splits = (KT + per - 1) / per;
    *kt_per_split = per;
}

int launch_gemm_nt_partials(const void *A, int64_t lda, const void *B, int64_t ldb, int64_t M, int32_t N, int32_t K,
                            int splits, int kt_per_split, float *C, hipStream_t st)
{
    Ff1Params p;
    p.X = A; p.Wg = nullptr; p.W1 = B; p.bg = nullptr; p.b1 = nullptr;
    p.Z = C; p.rowpart = nullptr;
    p.Zb = nullptr; p.ldzb = 0;
    p.ldx = lda; p.ldw = ldb; p.ldz = N;
    p.M = (int32_t)M; p.F = N; p.d = K;
    p.splits = splits; p.kt_per_split = kt_per_split;
    p.z_stream = 0;
    p.nt = (N + 2 * G_BN - 1) / (2 * G_BN);        // 256-column tiles: both sets of accumulators hold columns of B
    if (M > 128) {
        p.mt = (int32_t)((M + 255) / 256);
        const int nblk = p.mt * p.nt * splits;
        hipLaunchKernelGGL((ff1_bf16_mfma_kernel<GRIFFIN_ACT_RELU, true, 4, true>), dim3(ff1_grid(nblk)), dim3(G_THREADS), 0, st, p);
    } else {
        p.mt = (int32_t)((M + 127) / 128);
        const int nblk = p.mt * p.nt * splits;
        hipLaunchKernelGGL((ff1_bf16_mfma_kernel<GRIFFIN_ACT_RELU, true, 2, true>), dim3(ff1_grid(nblk)), dim3(G_THREADS), 0, st, p);
    }
    return check_launch("ff1_bf16_mfma_kernel");
}

}  // namespace griffin
