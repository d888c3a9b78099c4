// Internal helpers shared by the gfx950 kernels of the GRIFFIN feed-forward library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "griffin.h"

namespace griffin {

// ------------------------------------------------------------------ storage types
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
// the two bf16 values packed in one 32-bit word
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)
        return (u >> 16) | 0x40u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

template <bool BF16>
__device__ __forceinline__ float load_scalar(const void *p, int64_t i)
{
    if (BF16)
        return bf16_bits_to_f32(((const uint16_t *)p)[i]);
    return ((const float *)p)[i];
}

template <bool BF16>
__device__ __forceinline__ void store_scalar(void *p, int64_t i, float v)
{
    if (BF16)
        ((uint16_t *)p)[i] = (uint16_t)f32_to_bf16_bits(v);
    else
        ((float *)p)[i] = v;
}

// ------------------------------------------------------------------ sigma of Eq. 2 / Eq. 3
// silu(a) = a * sigmoid(a); tanh-GELU(a) = 0.5 a (1 + tanh(u)) = a * sigmoid(2u) with
// u = sqrt(2/pi) (a + 0.044715 a^3).  One v_exp_f32 and one v_rcp_f32 (1 ulp) each.
__device__ __forceinline__ float fast_sigmoid(float v) { return __builtin_amdgcn_rcpf(1.0f + __expf(-v)); }

__device__ __forceinline__ float act_silu(float a) { return a * fast_sigmoid(a); }

__device__ __forceinline__ float act_gelu_tanh(float a)
{
    const float u2 = 1.5957691216057308f * (a + 0.044715f * a * a * a);
    return a * fast_sigmoid(u2);
}

__device__ __forceinline__ float act_apply(int act, float a)
{
    if (act == GRIFFIN_ACT_SILU)
        return act_silu(a);
    if (act == GRIFFIN_ACT_GELU_TANH)
        return act_gelu_tanh(a);
    return fmaxf(a, 0.0f);
}

template <int ACT>
__device__ __forceinline__ float act_apply_t(float a)
{
    if (ACT == GRIFFIN_ACT_SILU)
        return act_silu(a);
    if (ACT == GRIFFIN_ACT_GELU_TANH)
        return act_gelu_tanh(a);
    return fmaxf(a, 0.0f);
}

// ------------------------------------------------------------------ wavefront (64 lanes) sums
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Sum over each row of 16 lanes; every lane of the row ends with the row's sum.
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_f32<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_f32<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_f32<0x141>(v);   // row_half_mirror
    v += dpp_f32<0x140>(v);   // row_mirror
    return v;
}

// Sum over the whole wavefront, returned uniformly (no LDS).
__device__ __forceinline__ float wave_sum(float v)
{
    v = row16_sum(v);
    float a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    float b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    float c = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (a + b) + (c + d);
}

// ------------------------------------------------------------------ host side
struct SeqTable {            // passed to kernels by value
    int32_t n;
    int32_t cu[GRIFFIN_MAX_SEQS + 1];
};

int set_hip_error(hipError_t e, const char *what);   // records text, returns GRIFFIN_EHIP
int check_launch(const char *what);                  // hipGetLastError -> status

// launchers (one per source file); all return a griffin_status
// Zb (optional): a bf16 copy of Z [M][ldzb] written by the same epilogue when ff1_can_write_zb() says so
int launch_ff1(const griffin_layer &L, const void *X, int64_t ldx, int64_t M, float *Z, int64_t ldz,
               float *rowpart, int32_t *nt_out, hipStream_t st, uint16_t *Zb = nullptr, int64_t ldzb = 0);
bool ff1_can_write_zb(const griffin_layer &L, int64_t ldx, const float *Z, int64_t ldz);
int ff1_ntiles(const griffin_layer &L);
int launch_stat(const float *Z, int64_t ldz, const float *rowpart, int nt, int64_t M, int32_t F,
                const SeqTable &seqs, float *s2part, float *s, float *s_out, hipStream_t st);
int64_t stat_max_chunks(int64_t total_tokens, int32_t n_seqs, int32_t F);
int launch_topk(const float *scores, int32_t n_rows, int32_t n, int32_t k, int32_t *idx, hipStream_t st);
int launch_stat_shared(const float *s, const SeqTable &seqs, int32_t n, float *sbar, hipStream_t st);
int launch_weight_norm(const griffin_layer &L, float *score, hipStream_t st);
int launch_select_sampled(const float *s, const float *e, int32_t n, int32_t k, int32_t k_top, int32_t *idx_out,
                          float *q, int32_t *idx_top, hipStream_t st);
int launch_jaccard(const int32_t *idx, int32_t n_sets, int32_t k, float *out, hipStream_t st);
int launch_compact(const griffin_layer &L, const int32_t *idx, int32_t k, const griffin_layer &C,
                   hipStream_t st);

bool gemm_nt_partials_ok(int64_t M, int32_t N, int32_t K, int64_t lda, int64_t ldb);
void gemm_nt_split_plan(int64_t M, int32_t N, int32_t K, int *splits, int *kt_per_split);
int launch_gemm_nt_partials(const void *A, int64_t lda, const void *B, int64_t ldb, int64_t M, int32_t N, int32_t K,
                            int splits, int kt_per_split, float *C, hipStream_t st);
// zb_ready: the bf16 copy of Z already sits at the head of ws (written by the first GEMM's epilogue)
int launch_ff2(const float *Z, int64_t ldz, int64_t M, int32_t F, int32_t d, bool bf16, const void *W2p,
               int64_t ldw, const void *b2, void *Y, int64_t ldy, float *ws, size_t ws_bytes, hipStream_t st,
               bool zb_ready = false);
bool ff2_takes_zb(const float *Z, int64_t ldz, int64_t M, int32_t F, int32_t d, bool bf16, const void *W2p, int64_t ldw);
size_t ff2_workspace_bytes(int64_t M, int32_t F, int32_t d);

struct DecodeJob {
    int32_t d, n, act, batch;
    bool bf16;
    int64_t ld;
    // single block (all rows) ...
    const void *Wg, *W1, *W2, *bg, *b1, *b2;
    const void *W2t;         // optional output-feature-major copy of W2, [d][ldt]
    int64_t ldt;
    // ... or one block per row (host array of `batch` layers), or an index list into one block
    const griffin_layer *multi;
    const int32_t *idx;      // [batch][n] rows of the full block, or NULL
    int32_t n_src;           // rows in the block idx points into
    const uint32_t *sets;    // optional membership words of idx, [groups of 16 rows][n_src], built beforehand
    const void *x;
    void *y;
    float *part;
    size_t part_bytes;
};
int launch_decode(const DecodeJob &job, hipStream_t st);
// one row through a block that carries W2t: two pure streams, no partial rows (decode_split.hip)
bool decode_split_supported(const DecodeJob &job);
int launch_decode_split(const DecodeJob &job, hipStream_t st, hipEvent_t ev_mid);
// rows 5.. of a batch through one shared block: matrix-core path (decode_batch.hip)
bool decode_batch_supported(int32_t d, int32_t n, bool bf16);
size_t decode_batch_workspace_floats(int32_t d, int32_t n, int32_t batch);
size_t decode_masked_workspace_floats(int32_t d, int32_t n_src, int32_t batch);
int launch_decode_batch_front(const DecodeJob &job, int32_t n_block, const int32_t *idx, int32_t k, int *NR_out,
                              hipStream_t st);
int launch_index_sets_build(const int32_t *idx, int32_t k, int32_t batch, int32_t n_block, uint32_t *sets, hipStream_t st);
size_t index_sets_words(int32_t n_block, int32_t batch);
constexpr int DEC_BATCH_MIN_ROWS = 5;
int decode_parts(int32_t n, int32_t batch);
void set_decode_probe(hipEvent_t begin, hipEvent_t mid, hipEvent_t end);

}  // namespace griffin
