// C ABI of the library: argument validation (before any HIP call), workspace carving and the
// order of kernel launches.  No allocation, no synchronisation, no host<->device copies.
#include <stdio.h>
#include <string.h>

#include <atomic>

#include "common.h"

namespace griffin {

static thread_local char g_hip_error[256] = "";

int set_hip_error(hipError_t e, const char *what)
{
    snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
    return GRIFFIN_EHIP;
}

int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? GRIFFIN_OK : set_hip_error(e, what);
}

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

constexpr int32_t MAX_DIM = 1 << 20;

// shape/pointer checks common to every entry point that takes a block description
static int check_layer(const griffin_layer *L)
{
    if (!L || !L->W1 || (!L->W2 && !L->W2t))
        return GRIFFIN_EINVAL;
    if (L->dtype != GRIFFIN_F32 && L->dtype != GRIFFIN_BF16)
        return GRIFFIN_EINVAL;
    if (L->act < GRIFFIN_ACT_SILU || L->act > GRIFFIN_ACT_RELU)
        return GRIFFIN_EINVAL;
    if (L->d <= 0 || L->n <= 0)
        return GRIFFIN_EINVAL;
    if (L->d > MAX_DIM || L->n > MAX_DIM || L->d % 8 != 0 || L->ld < L->d || L->ld % 8 != 0)
        return GRIFFIN_ESHAPE;
    if (!aligned16(L->W1) || !aligned16(L->W2) || !aligned16(L->Wg))
        return GRIFFIN_ESHAPE;
    if (!L->Wg && L->bg)
        return GRIFFIN_EINVAL;
    if (L->W2t) {       // the second, output-feature-major copy of W2: bf16, whole 512-element slices
        if (L->dtype != GRIFFIN_BF16)
            return GRIFFIN_EUNSUPPORTED;
        if (L->d % 512 != 0 || L->ldt < L->n || L->ldt % 512 != 0 || L->ldt > 2 * (int64_t)MAX_DIM || !aligned16(L->W2t))
            return GRIFFIN_ESHAPE;
    }
    return GRIFFIN_OK;
}

static int fill_seq_table(const int32_t *cu, int32_t n_seqs, SeqTable &t, int64_t *total)
{
    if (!cu || n_seqs < 1)
        return GRIFFIN_EINVAL;
    if (n_seqs > GRIFFIN_MAX_SEQS)
        return GRIFFIN_EUNSUPPORTED;
    if (cu[0] != 0)
        return GRIFFIN_ESHAPE;
    for (int b = 0; b < n_seqs; ++b)
        if (cu[b + 1] < cu[b])
            return GRIFFIN_ESHAPE;
    t.n = n_seqs;
    for (int b = 0; b <= n_seqs; ++b)
        t.cu[b] = cu[b];
    for (int b = n_seqs + 1; b <= GRIFFIN_MAX_SEQS; ++b)
        t.cu[b] = cu[n_seqs];
    *total = cu[n_seqs];
    return GRIFFIN_OK;
}

struct PrefillPlan {
    size_t off_z, off_rowpart, off_s2part, off_s, total;
    int nt;
};

static PrefillPlan plan_prefill(const griffin_layer &L, int64_t total_tokens, int32_t n_seqs, bool have_z)
{
    PrefillPlan pl;
    pl.nt = ff1_ntiles(L);
    size_t off = 0;
    pl.off_z = off;
    if (!have_z)
        off += align256((size_t)total_tokens * L.n * sizeof(float));
    pl.off_rowpart = off;
    off += align256((size_t)total_tokens * pl.nt * sizeof(float));
    pl.off_s2part = off;
    off += align256((size_t)stat_max_chunks(total_tokens, n_seqs, L.n) * L.n * sizeof(float));
    pl.off_s = off;
    off += align256((size_t)n_seqs * L.n * sizeof(float));
    pl.total = off;
    return pl;
}

}  // namespace griffin

using namespace griffin;

extern "C" {

const char *griffin_status_string(int status)
{
    switch (status) {
    case GRIFFIN_OK: return "ok";
    case GRIFFIN_EINVAL: return "invalid argument";
    case GRIFFIN_ESHAPE: return "inconsistent shape or alignment";
    case GRIFFIN_EWORKSPACE: return "workspace missing or too small";
    case GRIFFIN_EUNSUPPORTED: return "unsupported configuration";
    case GRIFFIN_EHIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

const char *griffin_last_hip_error(void) { return g_hip_error; }

const char *griffin_version(void) { return "griffin-gfx950 0.1"; }

int32_t griffin_k_from_fraction(int32_t d_ff, double keep)
{
    if (d_ff < 1)
        return 0;
    double v = keep * (double)d_ff + 0.5;
    int64_t k = v <= 1.0 ? 1 : (int64_t)v;
    if (k < 1) k = 1;
    if (k > d_ff) k = d_ff;
    return (int32_t)k;
}

size_t griffin_prefill_workspace_bytes(const griffin_layer *L, int64_t total_tokens, int32_t n_seqs,
                                       int32_t have_z_out)
{
    if (check_layer(L) != GRIFFIN_OK || total_tokens < 0 || n_seqs < 1 || n_seqs > GRIFFIN_MAX_SEQS)
        return 0;
    return plan_prefill(*L, total_tokens, n_seqs, have_z_out != 0).total;
}

int griffin_prefill_select(const griffin_layer *L, const void *X, int64_t ldx,
                           const int32_t *cu_seqlens_host, int32_t n_seqs, int32_t k,
                           int32_t *idx_out, float *s_out, float *Z_out, int64_t ldz,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_layer(L);
    if (rc != GRIFFIN_OK)
        return rc;
    SeqTable seqs;
    int64_t total = 0;
    if ((rc = fill_seq_table(cu_seqlens_host, n_seqs, seqs, &total)) != GRIFFIN_OK)
        return rc;
    if (!idx_out || (total > 0 && !X))
        return GRIFFIN_EINVAL;
    if (k < 1 || k > L->n)
        return GRIFFIN_ESHAPE;
    if (ldx < L->d || ldx % 8 != 0 || !aligned16(X) || total > (int64_t)1 << 30)
        return GRIFFIN_ESHAPE;
    if (Z_out && ldz < L->n)
        return GRIFFIN_ESHAPE;
    const PrefillPlan pl = plan_prefill(*L, total, n_seqs, Z_out != nullptr);
    if (!workspace || workspace_bytes < pl.total || ((uintptr_t)workspace & 255))
        return GRIFFIN_EWORKSPACE;

    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    float *Z = Z_out ? Z_out : (float *)(ws + pl.off_z);
    const int64_t zld = Z_out ? ldz : L->n;
    float *rowpart = (float *)(ws + pl.off_rowpart);
    float *s2part = (float *)(ws + pl.off_s2part);
    float *s = (float *)(ws + pl.off_s);

    int32_t nt = 0;
    if ((rc = launch_ff1(*L, X, ldx, total, Z, zld, rowpart, &nt, st)) != GRIFFIN_OK)
        return rc;
    if ((rc = launch_stat(Z, zld, rowpart, nt, total, L->n, seqs, s2part, s, s_out, st)) != GRIFFIN_OK)
        return rc;
    return launch_topk(s, n_seqs, L->n, k, idx_out, st);
}

int griffin_topk(const float *scores, int32_t n_rows, int32_t n, int32_t k, int32_t *idx_out, void *stream)
{
    if (!scores || !idx_out || n_rows < 0)
        return GRIFFIN_EINVAL;
    if (n < 1 || n > MAX_DIM || k < 1 || k > n)
        return GRIFFIN_ESHAPE;
    if (n_rows == 0)
        return GRIFFIN_OK;
    return launch_topk(scores, n_rows, n, k, idx_out, (hipStream_t)stream);
}

int griffin_stat_shared(const float *s, const int32_t *cu_seqlens_host, int32_t n_seqs, int32_t n,
                        float *sbar_out, void *stream)
{
    if (!s || !sbar_out)
        return GRIFFIN_EINVAL;
    if (n < 1 || n > MAX_DIM)
        return GRIFFIN_ESHAPE;
    SeqTable seqs;
    int64_t total = 0;
    int rc = fill_seq_table(cu_seqlens_host, n_seqs, seqs, &total);
    if (rc != GRIFFIN_OK)
        return rc;
    return launch_stat_shared(s, seqs, n, sbar_out, (hipStream_t)stream);
}

int griffin_weight_norm_score(const griffin_layer *L, float *score_out, void *stream)
{
    int rc = check_layer(L);
    if (rc != GRIFFIN_OK)
        return rc;
    if (!score_out)
        return GRIFFIN_EINVAL;
    return launch_weight_norm(*L, score_out, (hipStream_t)stream);
}

size_t griffin_select_sampled_workspace_bytes(int32_t n, int32_t k_top)
{
    if (n < 1 || k_top < 0 || k_top > n)
        return 0;
    return align256((size_t)n * sizeof(float)) + align256((size_t)(k_top > 0 ? k_top : 1) * sizeof(int32_t));
}

int griffin_select_sampled(const float *s, const float *e, int32_t n, int32_t k, int32_t k_top, int32_t *idx_out,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    if (!s || !e || !idx_out)
        return GRIFFIN_EINVAL;
    if (n < 1 || n > MAX_DIM || k < 1 || k > n || k_top < 0 || k_top > k)
        return GRIFFIN_ESHAPE;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < griffin_select_sampled_workspace_bytes(n, k_top))
        return GRIFFIN_EWORKSPACE;
    float *q = (float *)workspace;
    int32_t *idx_top = (int32_t *)((char *)workspace + align256((size_t)n * sizeof(float)));
    return launch_select_sampled(s, e, n, k, k_top, idx_out, q, idx_top, (hipStream_t)stream);
}

int griffin_jaccard(const int32_t *idx, int32_t n_sets, int32_t k, float *out, void *stream)
{
    if (!idx || !out)
        return GRIFFIN_EINVAL;
    if (n_sets < 1 || n_sets > GRIFFIN_MAX_SEQS || k < 1 || k > MAX_DIM)
        return GRIFFIN_ESHAPE;
    return launch_jaccard(idx, n_sets, k, out, (hipStream_t)stream);
}

int griffin_compact(const griffin_layer *L, const int32_t *idx, int32_t k, const griffin_layer *C, void *stream)
{
    int rc = check_layer(L);
    if (rc != GRIFFIN_OK)
        return rc;
    if ((rc = check_layer(C)) != GRIFFIN_OK)
        return rc;
    if (!idx || !L->W2)            // the neuron-major W2 of the full block is the source
        return GRIFFIN_EINVAL;
    if (k < 1 || k > L->n || C->n != k || C->d != L->d || C->dtype != L->dtype || C->act != L->act)
        return GRIFFIN_ESHAPE;
    if ((L->Wg == nullptr) != (C->Wg == nullptr) || (L->bg == nullptr) != (C->bg == nullptr) ||
        (L->b1 == nullptr) != (C->b1 == nullptr))
        return GRIFFIN_EINVAL;
    return launch_compact(*L, idx, k, *C, (hipStream_t)stream);
}

size_t griffin_prompt_out_workspace_bytes(int64_t total_tokens, int32_t d_ff, int32_t d)
{
    if (total_tokens < 1 || d_ff < 1 || d < 1 || total_tokens > ((int64_t)1 << 30))
        return 0;
    return ff2_workspace_bytes(total_tokens, d_ff, d);
}

int griffin_ff_prompt_out(const float *Z, int64_t ldz, int64_t total_tokens, int32_t d_ff, int32_t d,
                          int32_t dtype, const void *W2p, int64_t ldw, const void *b2, void *Y, int64_t ldy,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    if (!Z || !W2p || !Y || total_tokens < 0)
        return GRIFFIN_EINVAL;
    if (dtype != GRIFFIN_F32 && dtype != GRIFFIN_BF16)
        return GRIFFIN_EINVAL;
    if (d_ff < 1 || d < 1 || d_ff > MAX_DIM || d > MAX_DIM || ldz < d_ff || ldw < d_ff || ldy < d)
        return GRIFFIN_ESHAPE;
    const bool tiles = dtype == GRIFFIN_BF16 && d_ff % 8 == 0 && d % 4 == 0 && ldz % 4 == 0 && ldw % 8 == 0 &&
                       aligned16(Z) && aligned16(W2p);
    if (total_tokens > ((int64_t)1 << 30) || (!tiles && total_tokens > ((int64_t)1 << 18)))
        return GRIFFIN_EUNSUPPORTED;
    return launch_ff2(Z, ldz, total_tokens, d_ff, d, dtype == GRIFFIN_BF16, W2p, ldw, b2, Y, ldy,
                      (float *)workspace, workspace_bytes, (hipStream_t)stream);
}

size_t griffin_prompt_phase_workspace_bytes(const griffin_layer *L, int64_t total_tokens, int32_t n_seqs)
{
    if (check_layer(L) != GRIFFIN_OK || total_tokens < 0 || total_tokens > ((int64_t)1 << 30) || n_seqs < 1 ||
        n_seqs > GRIFFIN_MAX_SEQS)
        return 0;
    const size_t first = plan_prefill(*L, total_tokens, n_seqs, false).total;
    return first + align256(total_tokens > 0 ? ff2_workspace_bytes(total_tokens, L->n, L->d) : 0);
}

int griffin_prompt_phase(const griffin_layer *L, const void *W2p, int64_t ldw, const void *X, int64_t ldx,
                         const int32_t *cu_seqlens_host, int32_t n_seqs, int32_t k,
                         int32_t *idx_out, float *s_out, void *Y, int64_t ldy,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_layer(L);
    if (rc != GRIFFIN_OK)
        return rc;
    SeqTable seqs;
    int64_t total = 0;
    if ((rc = fill_seq_table(cu_seqlens_host, n_seqs, seqs, &total)) != GRIFFIN_OK)
        return rc;
    if (!idx_out || !W2p || !Y || (total > 0 && !X))
        return GRIFFIN_EINVAL;
    if (k < 1 || k > L->n)
        return GRIFFIN_ESHAPE;
    if (ldx < L->d || ldx % 8 != 0 || !aligned16(X) || total > (int64_t)1 << 30 || ldw < L->n || ldy < L->d)
        return GRIFFIN_ESHAPE;
    const bool bf16 = L->dtype == GRIFFIN_BF16;
    const bool tiles = bf16 && L->n % 8 == 0 && L->d % 4 == 0 && ldw % 8 == 0 && aligned16(W2p);
    if (!tiles && total > ((int64_t)1 << 18))
        return GRIFFIN_EUNSUPPORTED;
    const PrefillPlan pl = plan_prefill(*L, total, n_seqs, false);
    const size_t second = total > 0 ? ff2_workspace_bytes(total, L->n, L->d) : 0;
    if (!workspace || workspace_bytes < pl.total + align256(second) || ((uintptr_t)workspace & 255))
        return GRIFFIN_EWORKSPACE;

    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    float *Z = (float *)(ws + pl.off_z);
    float *rowpart = (float *)(ws + pl.off_rowpart);
    float *s2part = (float *)(ws + pl.off_s2part);
    float *s = (float *)(ws + pl.off_s);
    float *ws2 = (float *)(ws + pl.total);

    // the second product reads a bf16 copy of Z from the head of its workspace: let the first
    // product's epilogue write it there when both kernels agree on the shape
    const bool fuse = total > 0 && ff2_takes_zb(Z, L->n, total, L->n, L->d, bf16, W2p, ldw) &&
                      ff1_can_write_zb(*L, ldx, Z, L->n);
    int32_t nt = 0;
    if ((rc = launch_ff1(*L, X, ldx, total, Z, L->n, rowpart, &nt, st, fuse ? (uint16_t *)ws2 : nullptr, L->n)) != GRIFFIN_OK)
        return rc;
    if ((rc = launch_stat(Z, L->n, rowpart, nt, total, L->n, seqs, s2part, s, s_out, st)) != GRIFFIN_OK)
        return rc;
    if ((rc = launch_topk(s, n_seqs, L->n, k, idx_out, st)) != GRIFFIN_OK)
        return rc;
    return launch_ff2(Z, L->n, total, L->n, L->d, bf16, W2p, ldw, L->b2, Y, ldy, ws2, second, st, fuse);
}

int griffin_trace_next_decode(void *event_begin, void *event_mid, void *event_end)
{
    set_decode_probe((hipEvent_t)event_begin, (hipEvent_t)event_mid, (hipEvent_t)event_end);
    return GRIFFIN_OK;
}

size_t griffin_decode_workspace_bytes(int32_t d, int32_t n, int32_t batch)
{
    if (d < 1 || n < 1 || batch < 1 || batch > GRIFFIN_MAX_BATCH)
        return 0;
    size_t floats = (size_t)decode_parts(n, batch) * batch * d;
    if (batch >= DEC_BATCH_MIN_ROWS && decode_batch_supported(d, n, true)) {
        // also enough for the masked pass of griffin_ff_decode_indexed over a block of n neurons
        const size_t fb = decode_masked_workspace_floats(d, n, batch);
        if (fb > floats)
            floats = fb;
    }
    return floats * sizeof(float);
}

static int decode_common(const griffin_layer *L0, const griffin_layer *multi, const int32_t *idx, int32_t k,
                         int32_t batch, const void *x, void *y, void *ws, size_t ws_bytes, void *stream,
                         const uint32_t *sets = nullptr)
{
    if (batch < 0 || !x || !y)
        return GRIFFIN_EINVAL;
    if (batch > GRIFFIN_MAX_BATCH)
        return GRIFFIN_EUNSUPPORTED;
    if (!aligned16(x) || !aligned16(y))
        return GRIFFIN_ESHAPE;
    const int32_t n = idx ? k : L0->n;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < griffin_decode_workspace_bytes(L0->d, n, batch ? batch : 1))
        return GRIFFIN_EWORKSPACE;
    if (batch == 0)
        return GRIFFIN_OK;
    DecodeJob job;
    job.d = L0->d; job.n = n; job.act = L0->act; job.batch = batch;
    job.bf16 = L0->dtype == GRIFFIN_BF16;
    job.ld = L0->ld;
    job.Wg = L0->Wg; job.W1 = L0->W1; job.W2 = L0->W2; job.bg = L0->bg; job.b1 = L0->b1; job.b2 = L0->b2;
    job.W2t = L0->W2t; job.ldt = L0->ldt;
    job.multi = multi;
    job.idx = idx; job.n_src = L0->n;
    job.sets = sets;
    job.x = x; job.y = y;
    job.part = (float *)ws; job.part_bytes = ws_bytes;
    return launch_decode(job, (hipStream_t)stream);
}

int griffin_ff_decode(const griffin_layer *C, const void *x, void *y, int32_t batch, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    int rc = check_layer(C);
    if (rc != GRIFFIN_OK)
        return rc;
    return decode_common(C, nullptr, nullptr, 0, batch, x, y, workspace, workspace_bytes, stream);
}

int griffin_ff_decode_multi(const griffin_layer *Cs, int32_t batch, const void *x, void *y, void *workspace,
                            size_t workspace_bytes, void *stream)
{
    if (!Cs || batch < 1)
        return GRIFFIN_EINVAL;
    if (batch > GRIFFIN_MAX_BATCH)
        return GRIFFIN_EUNSUPPORTED;
    for (int b = 0; b < batch; ++b) {
        int rc = check_layer(&Cs[b]);
        if (rc != GRIFFIN_OK)
            return rc;
        const griffin_layer &a = Cs[0], &c = Cs[b];
        if (!c.W2)          // per-row blocks are streamed neuron-major; a block that carries W2t alone has no kernel here
            return GRIFFIN_EUNSUPPORTED;
        if (c.d != a.d || c.n != a.n || c.dtype != a.dtype || c.act != a.act || c.ld != a.ld ||
            (c.Wg == nullptr) != (a.Wg == nullptr) || (c.bg == nullptr) != (a.bg == nullptr) ||
            (c.b1 == nullptr) != (a.b1 == nullptr) || (c.b2 == nullptr) != (a.b2 == nullptr))
            return GRIFFIN_ESHAPE;
    }
    return decode_common(&Cs[0], Cs, nullptr, 0, batch, x, y, workspace, workspace_bytes, stream);
}

int griffin_ff_decode_indexed(const griffin_layer *L, const int32_t *idx, int32_t k, int32_t batch,
                              const void *x, void *y, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_layer(L);
    if (rc != GRIFFIN_OK)
        return rc;
    if (!idx)
        return GRIFFIN_EINVAL;
    if (k < 1 || k > L->n)
        return GRIFFIN_ESHAPE;
    return decode_common(L, nullptr, idx, k, batch, x, y, workspace, workspace_bytes, stream);
}

// ---------------------------------------------------------------- decode without a caller workspace
// The partial rows of griffin_ff_decode live in a file-scope device array instead of a workspace the
// caller allocated.  In host code the array's name is only a handle: its device address is asked for
// once per device (with that device current) and that address is what the kernels are given.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)8 << 20;
constexpr int STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
static std::atomic<void *> g_scratch_ptr[STATIC_MAX_DEVICES];

// device address of this device's copy of the array; GRIFFIN_EHIP if the runtime cannot give it
static int static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return set_hip_error(e, "hipGetDevice");
    if (dev < 0 || dev >= STATIC_MAX_DEVICES)
        return GRIFFIN_EUNSUPPORTED;
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        // two threads may both ask; they get the same address
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return set_hip_error(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return GRIFFIN_OK;
}

size_t griffin_ff_decode_static_max_bytes(void) { return STATIC_SCRATCH_BYTES; }

int griffin_ff_decode_static(const griffin_layer *C, const void *x, void *y, int32_t batch, void *stream)
{
    int rc = check_layer(C);
    if (rc != GRIFFIN_OK)
        return rc;
    if (batch < 0 || !x || !y)
        return GRIFFIN_EINVAL;
    if (batch > GRIFFIN_MAX_BATCH)
        return GRIFFIN_EUNSUPPORTED;
    // sizes are judged before the runtime is touched: what griffin_ff_decode would ask of a workspace
    // must fit the array
    const size_t need = griffin_decode_workspace_bytes(C->d, C->n, batch ? batch : 1);
    if (need == 0 || need > STATIC_SCRATCH_BYTES)
        return GRIFFIN_EWORKSPACE;
    if (batch == 0)
        return GRIFFIN_OK;
    void *ptr = nullptr;
    if ((rc = static_scratch(&ptr)) != GRIFFIN_OK)
        return rc;
    return decode_common(C, nullptr, nullptr, 0, batch, x, y, ptr, need, stream);
}

size_t griffin_index_sets_bytes(int32_t n, int32_t batch)
{
    if (n < 1 || n > MAX_DIM || batch < 1 || batch > GRIFFIN_MAX_BATCH)
        return 0;
    return index_sets_words(n, batch) * sizeof(uint32_t);
}

int griffin_index_sets_build(const int32_t *idx, int32_t k, int32_t batch, int32_t n, void *sets, size_t sets_bytes,
                             void *stream)
{
    if (!idx || !sets || batch < 0)
        return GRIFFIN_EINVAL;
    if (batch > GRIFFIN_MAX_BATCH)
        return GRIFFIN_EUNSUPPORTED;
    if (n < 1 || n > MAX_DIM || k < 1 || k > n || ((uintptr_t)sets & 3))
        return GRIFFIN_ESHAPE;
    if (batch == 0)
        return GRIFFIN_OK;
    if (sets_bytes < griffin_index_sets_bytes(n, batch))
        return GRIFFIN_EWORKSPACE;
    return launch_index_sets_build(idx, k, batch, n, (uint32_t *)sets, (hipStream_t)stream);
}

int griffin_ff_decode_indexed_sets(const griffin_layer *L, const int32_t *idx, int32_t k, const void *sets,
                                   int32_t batch, const void *x, void *y, void *workspace, size_t workspace_bytes,
                                   void *stream)
{
    int rc = check_layer(L);
    if (rc != GRIFFIN_OK)
        return rc;
    if (!idx || !sets)
        return GRIFFIN_EINVAL;
    if (k < 1 || k > L->n || ((uintptr_t)sets & 3))
        return GRIFFIN_ESHAPE;
    return decode_common(L, nullptr, idx, k, batch, x, y, workspace, workspace_bytes, stream, (const uint32_t *)sets);
}

}  // extern "C"
