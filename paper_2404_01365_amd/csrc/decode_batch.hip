// Generation phase for a batch of rows that share ONE selected set (Section 5.3, Eq. 7: one
// expert set for the whole batch; Eq. 4-5 through it): 5 to 16 rows per pass over the weights.
//
//     Z[b][j] = sigma(wg_j . x_b + bg_j) * (w1_j . x_b + b1_j),   Y[b][:] = sum_j Z[b][j] W2[j][:]
//
// With 16 rows the two products of the first line are a skinny dense contraction
// (16 x d x n), so they run on the matrix cores; the weights are still read exactly once, so
// the pass stays bound by HBM.  Two kernels, because the two lines want different ownership:
//
//  * ff_batch_gu_kernel: a workgroup of R = d/512 wavefronts takes neurons two at a time,
//    round-robin over the chip (a compact window of rows is in flight at any time).  Wave r owns
//    the r-th 512-element slice of every row: its slice of the 16 x-rows lives in registers as
//    MFMA operand fragments (v_mfma_f32_16x16x32_bf16, x as the 16-row operand, the two neurons
//    in two of the 16 columns), its 1 KB pieces of the Wg and W1 rows go from global memory
//    straight into a private LDS ring (LDS-DMA, no VGPRs) and come back as operand fragments
//    with ds_read_b128.  A wave keeps its partial 16 x 2 tiles in LDS; there is no barrier per
//    group of neurons (one would tie the independent load streams to the slowest of them): the
//    waves meet once (more often only if the tiles outgrow LDS), add the tiles in wave order,
//    apply sigma and the gating product, and Z goes to a small LDS table that is written out at
//    the end ([n][16] fp32).
//  * ff_batch_down_kernel: the second line, also on the matrix cores.  Giving every workgroup all
//    d columns would cost one [16][d] partial per workgroup (64 MB for 256 of them), so the work
//    is cut in two directions: a workgroup owns 512 columns and one of NR ranges of neurons, and
//    writes one [16][512] partial into the partial-row buffer that the single-row path uses
//    (NR rows per batch row).  Details at the kernel.
// The partial rows are then added in a fixed order by the reduce kernel of the single-row path.
#include "common.h"
#include <atomic>

namespace griffin {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_b;
typedef __attribute__((ext_vector_type(4))) float f32x4_b;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_b;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_b;
typedef __attribute__((address_space(3))) void lds_void_b;
typedef __attribute__((address_space(1))) const void gbl_cvoid_b;

constexpr int BT_ROWS = 16;              // rows of x per pass
constexpr int BT_ZBLOCKS = 64;           // neuron groups per workgroup whose Z fits the LDS table
constexpr int BT_G = 2;                  // neurons per group (MFMA columns in use)
constexpr int BT_MAX_WG = 256;           // workgroups of the first kernel
constexpr int BT_COLS = 512;             // columns per workgroup of the second kernel
constexpr int BT_WAVES2 = 8;             // waves per workgroup of the second kernel (64 columns each)

struct BatchParams {
    const void *Wg, *W1, *W2, *bg, *b1;
    const void *x;           // [rows][d] bf16
    float *z;                // [n][16] fp32
    float *part;             // [rows][NR][d] fp32
    int64_t ld;
    int32_t d, n, act, rows; // rows <= 16
    int32_t P;               // workgroups of the first kernel
    int32_t NR, CS;          // neuron ranges x column slices of the second kernel
    int32_t TB;              // groups between two meetings of the first kernel's waves
    const uint32_t *mask;    // per neuron, bit b set if row b of this pass uses the neuron; NULL: every row uses all
};

// cache policy of the weight stream: read once, so non-temporal (135 MB in a bare LDS-DMA read
// loop: 20.4 us against 23.3 us with the default policy)
constexpr int BT_NT = 2;

constexpr int bt_vmcnt(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

template <bool GATED, int NSTG, int G, int MAXT>
__global__ __launch_bounds__(MAXT) void ff_batch_gu_kernel(BatchParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char bt_smem[];
    constexpr int NMAT = GATED ? 2 : 1;
    constexpr int LPB = G * NMAT;            // LDS-DMA instructions per wave per group of G neurons
    constexpr int UNIT = LPB * 1024;         // bytes of a wave's ring slot
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int R = blockDim.x >> 6;
    const int bq = lane & 15, q = lane >> 4;
    unsigned char *ring = bt_smem + wave * (NSTG * UNIT);
    unsigned char *red = bt_smem + R * (NSTG * UNIT);            // [R][TB][NMAT][G][16] floats
    unsigned char *ztab = red + R * p.TB * NMAT * G * 16 * 4;    // [BT_ZBLOCKS][G][16] floats
    const uint32_t ring_a = (uint32_t)(uintptr_t)(lds_void_b *)ring;
    const uint32_t red_a = (uint32_t)(uintptr_t)(lds_void_b *)red;
    const uint32_t ztab_a = (uint32_t)(uintptr_t)(lds_void_b *)ztab;

    // neuron pairs of this workgroup: wg, wg + P, ...
    const int npairs = (p.n + G - 1) / G;
    const int T = (int)blockIdx.x < npairs ? (npairs - (int)blockIdx.x + p.P - 1) / p.P : 0;
    if (T == 0)
        return;

    // this wave's slice of x as the 16-row MFMA operand: lane (row bq, k-group q), step s holds
    // x[bq][wave*512 + (4 s + q)*8 .. +8]
    u32x4_b xa[16];
    {
        const uint16_t *xr = (const uint16_t *)p.x + (int64_t)min(bq, p.rows - 1) * p.d + wave * 512 + q * 8;
        const u32x4_b zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int s = 0; s < 16; ++s)
            xa[s] = bq < p.rows ? *(const u32x4_b *)(xr + s * 32) : zero;
    }
    const uint16_t *w1p = (const uint16_t *)p.W1 + wave * 512 + lane * 8;
    const uint16_t *wgp = (const uint16_t *)(GATED ? p.Wg : p.W1) + wave * 512 + lane * 8;

// the four (two) 1 KB pieces of pair number t_ (clamped to the last pair: loads past the end land
// in a slot nobody reads, which keeps the loop free of branches around loads)
#define BT_ISSUE(t_)                                                                                      \
    {                                                                                                     \
        const int pr_ = (int)blockIdx.x + min((t_), T - 1) * p.P;                                         \
        unsigned char *sl_ = ring + ((t_) % NSTG) * UNIT;                                                 \
        _Pragma("unroll") for (int g_ = 0; g_ < G; ++g_)                                                  \
        {                                                                                                 \
            const int64_t r_ = (int64_t)min(G * pr_ + g_, p.n - 1) * p.ld;                                \
            __builtin_amdgcn_global_load_lds((gbl_cvoid_b *)(w1p + r_), (lds_void_b *)(sl_ + g_ * 1024), 16, 0, BT_NT); \
            if (GATED)                                                                                    \
                __builtin_amdgcn_global_load_lds((gbl_cvoid_b *)(wgp + r_), (lds_void_b *)(sl_ + (G + g_) * 1024), 16, 0, BT_NT); \
        }                                                                                                 \
    }
#define BT_BARRIER()                                                                                      \
    {                                                                                                     \
        asm volatile("" ::: "memory");                                                                    \
        __builtin_amdgcn_s_barrier();                                                                     \
        asm volatile("" ::: "memory");                                                                    \
    }

#pragma unroll
    for (int t = 0; t < NSTG - 1; ++t)
        BT_ISSUE(t)

    // LDS reads and writes below are inline asm: the compiler would make each one it knows about
    // wait for every LDS-DMA in flight, i.e. for the whole prefetch
    const uint32_t frag_off = (uint32_t)((bq & (G - 1)) * 1024 + q * 16);
    // operand fragments of the weights, two sets: the reads of one 4-step chunk run under the MFMAs
    // of the chunk before.  Only the lanes of MFMA columns 0 .. G-1 carry a neuron; the others never
    // read (their columns of the product are never looked at) and keep zeros.
    u32x4_b f1[2][4], fg[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            f1[i][s] = (u32x4_b){0u, 0u, 0u, 0u};
            fg[i][s] = (u32x4_b){0u, 0u, 0u, 0u};
        }
#define BT_READ(F_, unit_, c_)                                                                            \
    if (bq < G) {                                                                                         \
        _Pragma("unroll") for (int s = 0; s < 4; ++s)                                                     \
        {                                                                                                 \
            asm volatile("ds_read_b128 %0, %1" : "+v"(f1[F_][s]) : "v"((unit_) + (uint32_t)(((c_) * 4 + s) * 64))); \
            if (GATED)                                                                                    \
                asm volatile("ds_read_b128 %0, %1" : "+v"(fg[F_][s]) : "v"((unit_) + (uint32_t)(G * 1024 + ((c_) * 4 + s) * 64))); \
        }                                                                                                 \
    }
#define BT_WAITF(F_)                                                                                      \
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f1[F_][0]), "+v"(f1[F_][1]), "+v"(f1[F_][2]), "+v"(f1[F_][3]), \
                 "+v"(fg[F_][0]), "+v"(fg[F_][1]), "+v"(fg[F_][2]), "+v"(fg[F_][3]));
#define BT_MFMA(F_, c_)                                                                                   \
    _Pragma("unroll") for (int s = 0; s < 4; ++s)                                                         \
    {                                                                                                     \
        accU = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_b, xa[(c_) * 4 + s]),    \
                                                       __builtin_bit_cast(bf16x8_b, f1[F_][s]), accU, 0, 0, 0); \
        if (GATED)                                                                                        \
            accG = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_b, xa[(c_) * 4 + s]), \
                                                           __builtin_bit_cast(bf16x8_b, fg[F_][s]), accG, 0, 0, 0); \
    }
    __builtin_amdgcn_s_waitcnt(bt_vmcnt((NSTG - 2) * LPB));          // group 0 has landed
    BT_READ(0, ring_a + frag_off, 0)
    for (int t = 0; t < T; ++t) {
        BT_ISSUE(t + NSTG - 1)
        const uint32_t unit = ring_a + (uint32_t)((t % NSTG) * UNIT) + frag_off;
        const uint32_t unit_next = ring_a + (uint32_t)(((t + 1) % NSTG) * UNIT) + frag_off;
        f32x4_b accU = {0.f, 0.f, 0.f, 0.f}, accG = {0.f, 0.f, 0.f, 0.f};
        BT_WAITF(0)
        BT_READ(1, unit, 1)
        BT_MFMA(0, 0)
        BT_WAITF(1)
        BT_READ(0, unit, 2)
        BT_MFMA(1, 1)
        BT_WAITF(0)
        BT_READ(1, unit, 3)
        BT_MFMA(0, 2)
        BT_WAITF(1)
        // the first chunk of the next group goes underneath the last MFMAs: that group has landed when
        // only the NSTG-2 groups after it are still in flight
        __builtin_amdgcn_s_waitcnt(bt_vmcnt((NSTG - 2) * LPB));
        BT_READ(0, unit_next, 0)
        BT_MFMA(1, 3)
        // lane (column bq, row group q) holds rows 4q .. 4q+3 of column bq; columns 0 .. G-1 are the group.
        // Every wave keeps its partial tiles of up to TB groups in a region of its own: no barrier per group
        // (one would tie the eight independent load streams to the slowest of them).
        const int te = t % p.TB;
        if (bq < G) {
            const uint32_t ra = red_a + (uint32_t)(((((wave * p.TB + te) * NMAT) * G + bq) * 16 + q * 4) * 4);
            asm volatile("ds_write_b128 %0, %1" :: "v"(ra), "v"(accU) : "memory");
            if (GATED)
                asm volatile("ds_write_b128 %0, %1" :: "v"(ra + G * 16 * 4), "v"(accG) : "memory");
        }
        if (te == p.TB - 1 || t == T - 1) {
            // the waves meet: partial tiles are added in wave order, sigma and the gating product follow
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            BT_BARRIER()
            const int t_first = t - te;
            for (int i = tid; i < (te + 1) * (16 * G); i += blockDim.x) {
                const int ti = i / (16 * G), jj = (i >> 4) & (G - 1), b = i & 15;
                float pu[16], pg[16];
#pragma unroll
                for (int w = 0; w < 16; ++w) {
                    const uint32_t ra = red_a + (uint32_t)(((((min(w, R - 1) * p.TB + ti) * NMAT) * G + jj) * 16 + b) * 4);
                    asm volatile("ds_read_b32 %0, %1" : "=v"(pu[w]) : "v"(ra));
                    if (GATED)
                        asm volatile("ds_read_b32 %0, %1" : "=v"(pg[w]) : "v"(ra + G * 16 * 4));
                }
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(pu[0]), "+v"(pu[1]), "+v"(pu[2]), "+v"(pu[3]), "+v"(pu[4]), "+v"(pu[5]),
                             "+v"(pu[6]), "+v"(pu[7]), "+v"(pu[8]), "+v"(pu[9]), "+v"(pu[10]), "+v"(pu[11]), "+v"(pu[12]),
                             "+v"(pu[13]), "+v"(pu[14]), "+v"(pu[15]));
                if (GATED)
                    asm volatile("" : "+v"(pg[0]), "+v"(pg[1]), "+v"(pg[2]), "+v"(pg[3]), "+v"(pg[4]), "+v"(pg[5]),
                                 "+v"(pg[6]), "+v"(pg[7]), "+v"(pg[8]), "+v"(pg[9]), "+v"(pg[10]), "+v"(pg[11]), "+v"(pg[12]),
                                 "+v"(pg[13]), "+v"(pg[14]), "+v"(pg[15]));
                float u = 0.0f, g = 0.0f;
#pragma unroll
                for (int w = 0; w < 16; ++w) {
                    u += w < R ? pu[w] : 0.0f;
                    if (GATED)
                        g += w < R ? pg[w] : 0.0f;
                }
                const int j = min(G * ((int)blockIdx.x + (t_first + ti) * p.P) + jj, p.n - 1);
                if (p.b1) u += bf16_bits_to_f32(((const uint16_t *)p.b1)[j]);
                if (GATED && p.bg) g += bf16_bits_to_f32(((const uint16_t *)p.bg)[j]);
                float zv = GATED ? act_apply(p.act, g) * u : act_apply(p.act, u);
                if (p.mask && !((p.mask[j] >> b) & 1u))
                    zv = 0.0f;                 // this row's own expert set does not hold the neuron
                asm volatile("ds_write_b32 %0, %1" :: "v"(ztab_a + (uint32_t)((((t_first + ti) * G + jj) * 16 + b) * 4)), "v"(zv) : "memory");
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            BT_BARRIER()                         // the partial-tile regions may be written again
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_waitcnt(bt_vmcnt(0));          // no LDS-DMA may outlive the loop
    BT_BARRIER()
#undef BT_ISSUE
#undef BT_BARRIER
#undef BT_READ
#undef BT_WAITF
#undef BT_MFMA
    // Z of this workgroup's pairs -> global [n][16]
    const float *zt = (const float *)ztab;
    for (int i = tid; i < T * (16 * G); i += blockDim.x) {
        const int t = i / (16 * G), jj = (i >> 4) & (G - 1), b = i & 15;
        const int j = G * ((int)blockIdx.x + t * p.P) + jj;
        if (j < p.n)
            p.z[(int64_t)j * 16 + b] = zt[i];
    }
}

// Y partials on the matrix cores: workgroup (nr, cs) owns neurons [j_lo, j_hi) (bounds on
// multiples of 8, at most 488 of them) and columns cs*512 .. +511; wave w owns 64 of the columns
// (four 16-column MFMA tiles).
//   D[16 rows of the batch][16 columns] += A[16][32 neurons] * B[32 neurons][16 columns]
// A is Z: the workgroup first turns its range of Z into bf16 pairs hi + lo (fp32 accuracy is kept
// by feeding both) laid out [16][range] in LDS.  B is W2, whose memory order (columns
// contiguous) is the transpose of what an MFMA operand wants (neurons contiguous per lane):
// every wave brings its own 32-neuron x 64-column pieces (whole 128-byte lines, 8 rows per
// LDS-DMA instruction) into a private LDS ring and gathers the operands with 16-bit LDS reads.
// No wave waits for another after the first barrier.
constexpr int BD_ZLD = 520;              // elements per row of the Z tables in LDS
constexpr int BD_RANGE = 480;            // neurons per workgroup before rounding to multiples of 8
constexpr int BD_DEPTH = 3;              // ring slots per wave (a fourth, fitted into the LDS by trimming the tables, changed nothing)
constexpr int BD_REGION = 66;            // 16-byte units per 8-row region: 1 KB of rows + 32 B, so that the four
                                         // regions a gather touches (rows 8q + i) start on different LDS banks
constexpr int BD_SLOT = 4 * BD_REGION;   // a slot: 32 rows x 128 B in four regions

__global__ __launch_bounds__(BT_WAVES2 * 64) void ff_batch_down_kernel(BatchParams p, const float *__restrict__ z)
{
    __shared__ u32x4_b ring_s[BT_WAVES2 * BD_DEPTH * BD_SLOT];      // 99 KB
    __shared__ uint16_t zhi[16 * BD_ZLD], zlo[16 * BD_ZLD];         // 2 x 16.25 KB
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nr = blockIdx.x / p.CS, cs = blockIdx.x % p.CS;
    const int j_lo = (int)((int64_t)p.n * nr / p.NR) & ~7;
    const int j_hi = nr == p.NR - 1 ? p.n : ((int)((int64_t)p.n * (nr + 1) / p.NR) & ~7);
    const int range = j_hi - j_lo;                 // <= 488 by the choice of NR
    const int S = (range + 31) >> 5;

    // Z[j][b] fp32 -> hi/lo bf16 tables [b][j - j_lo], zero beyond the range.  The range holds at most
    // 16 x 32 neurons = 2048 groups of four batch rows: four 16-byte loads per thread, all issued before
    // the first is used (one load per trip of a loop would put sixteen memory latencies in a row in front
    // of the stream), and the first pieces of W2 leave right behind them.
    static_assert(BD_RANGE + 8 <= 16 * 32 && 16 * 32 + 8 <= BD_ZLD && BT_WAVES2 * 64 * 4 >= 16 * 32 * 4, "four groups per thread cover the range");
    f32x4_b zv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int u = tid + r * (BT_WAVES2 * 64), jr = u >> 2, qd = u & 3;
        zv[r] = jr < range ? *(const f32x4_b *)(z + (int64_t)(j_lo + jr) * 16 + qd * 4) : (f32x4_b){0.f, 0.f, 0.f, 0.f};
    }

    const int bq = lane & 15, q = lane >> 4;
    const int c0 = cs * BT_COLS + wave * 64;
    u32x4_b *ring = ring_s + wave * (BD_DEPTH * BD_SLOT);
    const uint32_t ring_a = (uint32_t)(uintptr_t)(lds_void_b *)ring;
    const uint32_t za = (uint32_t)(uintptr_t)(lds_void_b *)zhi + (uint32_t)((bq * BD_ZLD + q * 8) * 2);
    const uint32_t zb = (uint32_t)(uintptr_t)(lds_void_b *)zlo + (uint32_t)((bq * BD_ZLD + q * 8) * 2);
    const uint16_t *w2 = (const uint16_t *)p.W2 + c0 + (lane & 7) * 8;
    const int lrow = lane >> 3;
// the four LDS-DMA instructions of step s_: rows 8u .. 8u+7 of its 32 neurons, 128 bytes per row
#define BD_ISSUE(s_)                                                                                         \
    _Pragma("unroll") for (int u = 0; u < 4; ++u)                                                            \
    {                                                                                                        \
        const int row_ = min(j_lo + min((s_), S - 1) * 32 + u * 8 + lrow, p.n - 1);                          \
        __builtin_amdgcn_global_load_lds((gbl_cvoid_b *)(w2 + (int64_t)row_ * p.ld),                         \
                                         (lds_void_b *)(ring + ((s_) % BD_DEPTH) * BD_SLOT + u * BD_REGION), 16, 0, BT_NT); \
    }
    f32x4_b acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
        acc[t] = (f32x4_b){0.f, 0.f, 0.f, 0.f};
    if (S > 0) {
#pragma unroll
        for (int s = 0; s < BD_DEPTH - 1; ++s)
            BD_ISSUE(s)
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int u = tid + r * (BT_WAVES2 * 64), jr = u >> 2, qd = u & 3;
        if (jr < S * 32) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float v = zv[r][e];
                const uint32_t h = f32_to_bf16_bits(v);
                const float rest = v - bf16_bits_to_f32(h);
                zhi[(qd * 4 + e) * BD_ZLD + jr] = (uint16_t)h;
                zlo[(qd * 4 + e) * BD_ZLD + jr] = (uint16_t)f32_to_bf16_bits(rest);
            }
        }
    }
    __syncthreads();
    if (S > 0) {                 // an empty range (very few neurons) still writes its zero partial
    // LDS reads by inline asm: reads the compiler knows about would wait for every LDS-DMA in flight
    const uint32_t gat = (uint32_t)(q * BD_REGION * 16 + bq * 2);   // row 8q of the slot (region q), column bq of tile 0
    for (int s = 0; s < S; ++s) {
        BD_ISSUE(s + BD_DEPTH - 1)
        __builtin_amdgcn_s_waitcnt(bt_vmcnt((BD_DEPTH - 1) * 4));   // the pieces of step s have landed
        const uint32_t slot = ring_a + (uint32_t)((s % BD_DEPTH) * BD_SLOT * 16) + gat;
        u32x4_b ah, al;
        asm volatile("ds_read_b128 %0, %1" : "=v"(ah) : "v"(za + (uint32_t)(s * 64)));
        asm volatile("ds_read_b128 %0, %1" : "=v"(al) : "v"(zb + (uint32_t)(s * 64)));
        // eight 16-bit reads per 16-column tile into eight registers (two reads in flight into the
        // halves of one register do not merge), packed in pairs afterwards; all four tiles' reads are
        // issued before the one wait
        uint32_t e[4][8];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < 8; ++i)
                asm volatile("ds_read_u16 %0, %1" : "=v"(e[t][i]) : "v"(slot + (uint32_t)(t * 32 + i * 128)));
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(ah), "+v"(al),
                     "+v"(e[0][0]), "+v"(e[0][1]), "+v"(e[0][2]), "+v"(e[0][3]), "+v"(e[0][4]), "+v"(e[0][5]), "+v"(e[0][6]), "+v"(e[0][7]),
                     "+v"(e[1][0]), "+v"(e[1][1]), "+v"(e[1][2]), "+v"(e[1][3]), "+v"(e[1][4]), "+v"(e[1][5]), "+v"(e[1][6]), "+v"(e[1][7]));
        asm volatile("" : "+v"(e[2][0]), "+v"(e[2][1]), "+v"(e[2][2]), "+v"(e[2][3]), "+v"(e[2][4]), "+v"(e[2][5]), "+v"(e[2][6]), "+v"(e[2][7]),
                     "+v"(e[3][0]), "+v"(e[3][1]), "+v"(e[3][2]), "+v"(e[3][3]), "+v"(e[3][4]), "+v"(e[3][5]), "+v"(e[3][6]), "+v"(e[3][7]));
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const u32x4_b bw = {e[t][0] | (e[t][1] << 16), e[t][2] | (e[t][3] << 16), e[t][4] | (e[t][5] << 16), e[t][6] | (e[t][7] << 16)};
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_b, ah), __builtin_bit_cast(bf16x8_b, bw), acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_b, al), __builtin_bit_cast(bf16x8_b, bw), acc[t], 0, 0, 0);
        }
    }
    __builtin_amdgcn_s_waitcnt(bt_vmcnt(0));                   // no LDS-DMA may outlive the loop
    }
#undef BD_ISSUE
    // lane (column bq, row group q) holds rows 4q .. 4q+3 of the batch
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int b = 4 * q + i;
            if (b < p.rows)
                p.part[((int64_t)b * p.NR + nr) * p.d + c0 + t * 16 + bq] = acc[t][i];
        }
}

// Rows with their own expert sets through the FULL block in one pass (Section 4.2: every sample picks
// its own neurons): the sets of a batch cover nearly every neuron between them (16 half-sets of a
// 14336-neuron block: all of it), so streaming the block once and dropping, per row, the neurons its
// set does not hold moves 8 times fewer bytes than streaming 16 compact blocks.  mask[j] collects,
// for 16 rows, which of them selected neuron j.
__global__ __launch_bounds__(256) void batch_mask_zero_kernel(uint32_t *mask, int n)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j < n)
        mask[j] = 0u;
}

__global__ __launch_bounds__(256) void batch_mask_build_kernel(const int32_t *idx, int rows, int k, int n_src, uint32_t *mask)
{
    const int t = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
    if (t >= k || b >= rows)
        return;
    int j = idx[(int64_t)b * k + t];
    j = j < 0 ? 0 : (j >= n_src ? n_src - 1 : j);
    atomicOr(&mask[j], 1u << b);
}

// Can the batch path take this shape?  d in whole 512-element slices, at most 10 of them (one
// wave each, 168 registers per lane), and few enough neuron groups per workgroup for the LDS
// table of Z.
bool decode_batch_supported(int32_t d, int32_t n, bool bf16)
{
    if (!bf16 || d % 512 != 0 || d / 512 > 10 || n < 64)
        return false;
    const int npairs = (n + BT_G - 1) / BT_G;
    const int P = npairs < BT_MAX_WG ? npairs : BT_MAX_WG;
    return (npairs + P - 1) / P <= BT_ZBLOCKS;
}

int decode_batch_ranges(int32_t d, int32_t n)
{
    const int CS = d / BT_COLS;
    int NR = 256 / CS;                         // as many workgroups as fit the chip at once: one more than the CUs
                                               // (d = 3072: 43 x 6 = 258) and the stragglers double the kernel's time
    if (NR > 64) NR = 64;
    const int by_range = (n + BD_RANGE - 1) / BD_RANGE;
    if (NR < by_range) NR = by_range;          // a workgroup's range of Z must fit its LDS tables
    return NR < 1 ? 1 : NR;
}

// floats of workspace: partial rows [batch][NR][d], then Z [n][16]
size_t decode_batch_workspace_floats(int32_t d, int32_t n, int32_t batch)
{
    return (size_t)batch * decode_batch_ranges(d, n) * d + (size_t)n * 16 + 64;
}

// floats of workspace of the masked pass: the batch pass over the full block plus one mask word per neuron
size_t decode_masked_workspace_floats(int32_t d, int32_t n_src, int32_t batch)
{
    return decode_batch_workspace_floats(d, n_src, batch) + (size_t)n_src + 64;
}

// The membership words of every group of 16 rows, [groups][n_block], for callers that build them once
// per prompt (the sets do not change during generation, Section 4.2).
int launch_index_sets_build(const int32_t *idx, int32_t k, int32_t batch, int32_t n_block, uint32_t *sets, hipStream_t st)
{
    for (int r0 = 0; r0 < batch; r0 += BT_ROWS) {
        const int rows = batch - r0 < BT_ROWS ? batch - r0 : BT_ROWS;
        uint32_t *mask = sets + (size_t)(r0 / BT_ROWS) * n_block;
        hipLaunchKernelGGL(batch_mask_zero_kernel, dim3((n_block + 255) / 256), dim3(256), 0, st, mask, n_block);
        hipLaunchKernelGGL(batch_mask_build_kernel, dim3((k + 255) / 256, rows), dim3(256), 0, st,
                           idx + (int64_t)r0 * k, rows, k, n_block, mask);
    }
    return check_launch("batch_mask_build_kernel");
}

size_t index_sets_words(int32_t n_block, int32_t batch)
{
    return (size_t)((batch + BT_ROWS - 1) / BT_ROWS) * n_block;
}

// Runs both kernels for every group of up to 16 rows; leaves part[b][NR][d] for the reduce kernel.
// n_block neurons in the block; idx (or NULL) [batch][k]: the rows' own sets inside that block.
int launch_decode_batch_front(const DecodeJob &job, int32_t n_block, const int32_t *idx, int32_t k, int *NR_out,
                              hipStream_t st)
{
    const int R = job.d / 512;
    const int NR = decode_batch_ranges(job.d, n_block), CS = job.d / BT_COLS;
    *NR_out = NR;
    const bool gated = job.Wg != nullptr;
    const int NMAT = gated ? 2 : 1, UNIT = BT_G * NMAT * 1024;
    int NSTG = (128 * 1024) / (R * UNIT);
    if (NSTG > 4) NSTG = 4;
    if (NSTG < 2)
        return GRIFFIN_EUNSUPPORTED;
    const int npairs = (n_block + BT_G - 1) / BT_G;
    const int P1 = npairs < BT_MAX_WG ? npairs : BT_MAX_WG;
    const int Tmax = (npairs + P1 - 1) / P1;
    // room for the waves' partial tiles: all of a workgroup's groups if a ring of two slots or more
    // leaves that much, so that the waves meet only once
    const size_t tile = (size_t)R * NMAT * BT_G * 16 * 4, ztab_bytes = (size_t)BT_ZBLOCKS * BT_G * 16 * 4;
    const size_t budget = 150 * 1024;
    while (NSTG > 2 && (size_t)R * NSTG * UNIT + ztab_bytes + tile * Tmax > budget)
        --NSTG;
    if ((size_t)R * NSTG * UNIT + ztab_bytes + tile > budget)
        return GRIFFIN_EUNSUPPORTED;
    int TB = (int)((budget - (size_t)R * NSTG * UNIT - ztab_bytes) / tile);
    if (TB > Tmax) TB = Tmax;
    if (TB < 1)
        return GRIFFIN_EUNSUPPORTED;
    const size_t lds = (size_t)R * NSTG * UNIT + tile * TB + ztab_bytes;

    BatchParams p;
    p.Wg = job.Wg; p.W1 = job.W1; p.W2 = job.W2; p.bg = job.bg; p.b1 = job.b1;
    p.ld = job.ld; p.d = job.d; p.n = n_block; p.act = job.act;
    p.P = P1;
    p.NR = NR; p.CS = CS; p.TB = TB;
    size_t zoff = ((size_t)job.batch * NR * job.d + 63) & ~(size_t)63;
    p.z = job.part + zoff;
    uint32_t *mask = idx ? (uint32_t *)(p.z + (((size_t)n_block * 16 + 63) & ~(size_t)63)) : nullptr;
    p.mask = mask;

    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess)
        return set_hip_error(hipGetLastError(), "hipGetDevice");
    const uint64_t dev_bit = 1ull << (dev & 63);
    for (int r0 = 0; r0 < job.batch; r0 += BT_ROWS) {
        p.rows = job.batch - r0 < BT_ROWS ? job.batch - r0 : BT_ROWS;
        p.x = (const uint16_t *)job.x + (int64_t)r0 * job.d;
        p.part = job.part + (size_t)r0 * NR * job.d;
        if (job.sets) {
            p.mask = job.sets + (size_t)(r0 / BT_ROWS) * n_block;      // built once per prompt by the caller
        } else if (idx) {
            hipLaunchKernelGGL(batch_mask_zero_kernel, dim3((n_block + 255) / 256), dim3(256), 0, st, mask, n_block);
            hipLaunchKernelGGL(batch_mask_build_kernel, dim3((k + 255) / 256, p.rows), dim3(256), 0, st,
                               idx + (int64_t)r0 * k, p.rows, k, n_block, mask);
            int rcm = check_launch("batch_mask_build_kernel");
            if (rcm != GRIFFIN_OK)
                return rcm;
        }
        dim3 g1(p.P), b1(R * 64);
#define BT_GO2(GA, NS, MT)                                                                                     \
        {                                                                                                      \
            /* raising the dynamic LDS limit is needed once per kernel and device */                           \
            static std::atomic<uint64_t> attr_set_{0};                                                         \
            if (!(attr_set_.load(std::memory_order_acquire) & dev_bit)) {                                      \
                if (hipFuncSetAttribute((const void *)ff_batch_gu_kernel<GA, NS, BT_G, MT>,                    \
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) \
                    return set_hip_error(hipGetLastError(), "hipFuncSetAttribute");                            \
                attr_set_.fetch_or(dev_bit, std::memory_order_release);                                        \
            }                                                                                                  \
            hipLaunchKernelGGL((ff_batch_gu_kernel<GA, NS, BT_G, MT>), g1, b1, lds, st, p);                    \
        }
#define BT_GO(GA, NS) { if (R <= 8) BT_GO2(GA, NS, 512) else BT_GO2(GA, NS, 640) }
        if (gated) { if (NSTG == 4) BT_GO(true, 4) else if (NSTG == 3) BT_GO(true, 3) else BT_GO(true, 2) }
        else       { if (NSTG == 4) BT_GO(false, 4) else if (NSTG == 3) BT_GO(false, 3) else BT_GO(false, 2) }
#undef BT_GO
#undef BT_GO2
        int rc = check_launch("ff_batch_gu_kernel");
        if (rc != GRIFFIN_OK)
            return rc;
        dim3 g2(NR * CS), b2(BT_WAVES2 * 64);
        hipLaunchKernelGGL(ff_batch_down_kernel, g2, b2, 0, st, p, (const float *)p.z);
        rc = check_launch("ff_batch_down_kernel");
        if (rc != GRIFFIN_OK)
            return rc;
    }
    return GRIFFIN_OK;
}

}  // namespace griffin
