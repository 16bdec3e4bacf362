// C-ABI of libsfb (see include/sfb.h for the contract): argument checks,
// workspace carving and the sequence of kernel launches of each call.  No device
// memory is allocated or freed here and nothing synchronises with the host.
#include "../../include/sfb.h"

#include <hip/hip_runtime.h>

#include <new>

#include "kernels.h"

// Kernel groups reported by the optional per-kernel timing.
enum KernelId : int {
    KID_FORWARD_BF16 = 0,
    KID_APPLY_BF16,
    KID_APPLY_TRANSPOSE,
    KID_SOFTMAX,
    KID_GEMM_F32_STORE,
    KID_GEMM_F32_RMW,
    KID_GEMM_F32_RESID,
    KID_GEMM_F32_SHRINK,
    KID_DIFF,
    KID_DML_SCALE,
    KID_FILL,
    KID_PROX,
    KID_POWER_ITERATION,
    KID_COPY,
    KID_SHADOW,
    KID_SCALE_ROWS,
    KID_CSR,
    KID_CSR_GATHER,
    KID_SDCA,
    KID_DUAL_TO_PRIMAL,
    KID_COUNT
};
static const char* const kKernelNames[KID_COUNT] = {
    "mlr_forward_bf16", "apply_bf16", "apply_bf16_transpose", "mlr_softmax", "gemm_f32_store", "gemm_f32_rmw(apply)", "gemm_f32_resid",
    "gemm_f32_shrink", "diff", "dml_scale", "fill", "prox_rows", "power_iteration", "copy", "shadow_convert", "scale_rows",
    "csr_to_operand", "csr_forward_gather", "sdca_mlr", "dual_to_primal"};

struct ProfSpan {
    hipEvent_t t0, t1;
    int kid;
};

struct sfb_ctx {
    int device;
    hipStream_t stream;
    char* ws;
    int64_t ws_bytes;
    int last_hip_error;
    // per-kernel timing (off by default): a fixed pool of event pairs
    bool prof_on;
    ProfSpan* spans;
    int span_cap;
    int span_used;
    int span_dropped;
    // bf16 working copy of one parameter matrix (sfb_shadow_attach)
    const float* shadow_W;
    uint16_t* shadow_buf;
    int64_t shadow_J, shadow_D;
    // low plane when that matrix is kept as two 16-bit planes (sfb_split_attach); shadow_buf is then the high plane
    uint16_t* split_lo;
    // CU / XCD counts of the device, per-device launch state, wait bound of the one-read softmax
    sfb::DeviceInfo dev;
    // route of sfb_mlr_sf_csr: 0 chosen from the number of stored entries, 1 dense contraction, 2 over the non-zeros
    int csr_route;
    // this device's copy of the library's static scratch array (sfb_apply_static), resolved by sfb_create
    char* static_scratch;
    int static_scratch_err;
};

// Scratch of sfb_apply_static: one array per GPU the library runs on, held until the process ends.  In host
// code the name is only a handle for hipGetSymbolAddress; kernels and copies get the address it returns.
static __device__ __align__(256) unsigned char scratch[SFB_STATIC_SCRATCH_BYTES];

namespace {

constexpr int64_t ALIGN = 256;
int64_t round_up(int64_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool valid_dtype(int32_t d) { return d == SFB_F32 || d == SFB_BF16; }

int hip_fail(sfb_ctx* ctx, hipError_t e)
{
    ctx->last_hip_error = (int)e;
    return SFB_EHIP;
}
#define SFB_TRY(expr)                                         \
    do {                                                      \
        hipError_t e_ = (expr);                               \
        if (e_ != hipSuccess) return hip_fail(ctx, e_);       \
    } while (0)

// Brackets a launch with two events when timing is on (and the pool has room).
struct ProfScope {
    sfb_ctx* c;
    ProfSpan* s;
    ProfScope(sfb_ctx* ctx, int kid) : c(ctx), s(nullptr)
    {
        if (!c->prof_on) return;
        if (c->span_used >= c->span_cap) {
            c->span_dropped++;
            return;
        }
        s = &c->spans[c->span_used++];
        s->kid = kid;
        (void)hipEventRecord(s->t0, c->stream);
    }
    ~ProfScope()
    {
        if (s) (void)hipEventRecord(s->t1, c->stream);
    }
};
#define SFB_RUN(kid, expr)                                    \
    do {                                                      \
        hipError_t e_;                                        \
        {                                                     \
            ProfScope scope_(ctx, (kid));                     \
            e_ = (expr);                                      \
        }                                                     \
        if (e_ != hipSuccess) return hip_fail(ctx, e_);       \
    } while (0)

struct ScLayout {
    int64_t power_floats;  // b[D] c[J] part[chunks*D] g[D]
    int64_t off_L;         // byte offset of the device scalar L
    int64_t total;
};
ScLayout sc_layout(int64_t J, int64_t D)
{
    ScLayout l;
    l.power_floats = D + J + sfb::power_chunks(J) * D + D;
    l.off_L = round_up(l.power_floats * 4);
    l.total = l.off_L + ALIGN;
    return l;
}

// k-split scratch shared by the two contractions of an ISTA iteration.
int64_t sc_partial_bytes(int64_t B, int64_t J, int64_t D)
{
    const int64_t a = sfb::gemm_f32_partial_bytes(B, D, J), b = sfb::gemm_f32_partial_bytes(B, J, D);
    return round_up(a > b ? a : b);
}

// Front of the workspace on the bf16 multiclass-logistic path: the tile-blocked logits, then the words the
// workgroups of the one-read softmax exchange.
int64_t bf16_logits_bytes(int64_t B, int64_t J)
{
    return round_up(sfb::mlr_logits_floats(B, J) * 4) + round_up(sfb::mlr_softmax_scratch_bytes(B, J));
}
void* bf16_softmax_scratch(sfb_ctx* ctx, int64_t B, int64_t J)
{
    return sfb::mlr_softmax_scratch_bytes(B, J) ? ctx->ws + round_up(sfb::mlr_logits_floats(B, J) * 4) : nullptr;
}

// True if W is currently kept as two planes by this context: its fp32 array is stale.
bool is_split(const sfb_ctx* ctx, const float* W) { return ctx->split_lo && ctx->shadow_W == W; }

int check_batch(int32_t model, int64_t J, int64_t D, const sfb_batch* b)
{
    if (!b || J <= 0 || D <= 0 || b->B < 0) return SFB_EINVAL;
    if (model != SFB_MLR && model != SFB_DML && model != SFB_SC) return SFB_EINVAL;
    if (!valid_dtype(b->in_dtype) || !valid_dtype(b->sf_dtype)) return SFB_EINVAL;
    if (b->in_dtype != b->sf_dtype) return SFB_EINVAL;
    if (model != SFB_MLR && b->in_dtype != SFB_F32) return SFB_EINVAL;
    if (b->in_dtype == SFB_BF16 && (J % 8 != 0 || D % 8 != 0)) return SFB_EINVAL;
    if (model == SFB_SC && (b->ista_iters < 0 || b->power_iters < 1 || !(b->lambda >= 0.f))) return SFB_EINVAL;
    return SFB_OK;
}

}  // namespace

extern "C" {

int sfb_create(sfb_ctx** out, int device_id, void* hip_stream)
{
    if (!out) return SFB_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device_id < 0 || device_id >= count) return SFB_EINVAL;
    sfb_ctx* c = new (std::nothrow) sfb_ctx;
    if (!c) return SFB_EINVAL;
    (void)hipGetLastError();
    c->device = device_id;
    c->stream = reinterpret_cast<hipStream_t>(hip_stream);
    c->ws = nullptr;
    c->ws_bytes = 0;
    c->last_hip_error = 0;
    c->prof_on = false;
    c->spans = nullptr;
    c->span_cap = 0;
    c->span_used = 0;
    c->span_dropped = 0;
    c->shadow_W = nullptr;
    c->shadow_buf = nullptr;
    c->shadow_J = c->shadow_D = 0;
    c->split_lo = nullptr;
    c->csr_route = 0;
    int cus = 0, xcds = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device_id) != hipSuccess || cus <= 0) {
        delete c;
        return SFB_EHIP;
    }
    if (hipDeviceGetAttribute(&xcds, hipDeviceAttributeNumberOfXccs, device_id) != hipSuccess || xcds <= 0 || xcds > cus)
        xcds = 1;   // unknown: one raster over all CUs (correct on any device, only the L2 locality is lost)
    c->dev.cus = cus;
    c->dev.xcds = xcds;
    // the address of this device's copy of the static scratch array (each GPU has its own)
    int prev = -1;
    (void)hipGetDevice(&prev);
    void* sp = nullptr;
    hipError_t e = hipSetDevice(device_id);
    if (e == hipSuccess) e = hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch));
    c->static_scratch = e == hipSuccess ? static_cast<char*>(sp) : nullptr;
    c->static_scratch_err = (int)e;
    if (e != hipSuccess) (void)hipGetLastError();
    if (prev >= 0 && prev != device_id) (void)hipSetDevice(prev);
    *out = c;
    return SFB_OK;
}

int sfb_destroy(sfb_ctx* ctx)
{
    if (!ctx) return SFB_EINVAL;
    if (ctx->spans) {
        for (int i = 0; i < ctx->span_cap; ++i) {
            (void)hipEventDestroy(ctx->spans[i].t0);
            (void)hipEventDestroy(ctx->spans[i].t1);
        }
        delete[] ctx->spans;
    }
    delete ctx;
    return SFB_OK;
}

int sfb_profile_enable(sfb_ctx* ctx, int on)
{
    if (!ctx) return SFB_EINVAL;
    if (on && !ctx->spans) {
        SFB_TRY(hipSetDevice(ctx->device));
        const int cap = 4096;
        ProfSpan* sp = new (std::nothrow) ProfSpan[cap];
        if (!sp) return SFB_EINVAL;
        for (int i = 0; i < cap; ++i) {
            hipError_t e = hipEventCreate(&sp[i].t0);
            if (e == hipSuccess) {
                e = hipEventCreate(&sp[i].t1);
                if (e != hipSuccess) (void)hipEventDestroy(sp[i].t0);
            }
            if (e != hipSuccess) {   // give back the pairs made so far
                for (int k = 0; k < i; ++k) {
                    (void)hipEventDestroy(sp[k].t0);
                    (void)hipEventDestroy(sp[k].t1);
                }
                delete[] sp;
                return hip_fail(ctx, e);
            }
        }
        ctx->spans = sp;
        ctx->span_cap = cap;
    }
    ctx->prof_on = on != 0;
    return SFB_OK;
}

int sfb_profile_collect(sfb_ctx* ctx, sfb_kernel_time* out, int max_entries, int* count)
{
    if (!ctx || !count || (max_entries > 0 && !out)) return SFB_EINVAL;
    *count = 0;
    SFB_TRY(hipSetDevice(ctx->device));
    SFB_TRY(hipStreamSynchronize(ctx->stream));
    float total[KID_COUNT] = {0};
    int launches[KID_COUNT] = {0};
    for (int i = 0; i < ctx->span_used; ++i) {
        float ms = 0.f;
        SFB_TRY(hipEventElapsedTime(&ms, ctx->spans[i].t0, ctx->spans[i].t1));
        total[ctx->spans[i].kid] += ms;
        launches[ctx->spans[i].kid] += 1;
    }
    ctx->span_used = 0;
    const int dropped = ctx->span_dropped;
    ctx->span_dropped = 0;
    int n = 0;
    for (int k = 0; k < KID_COUNT && n < max_entries; ++k) {
        if (!launches[k]) continue;
        out[n].name = kKernelNames[k];
        out[n].launches = launches[k];
        out[n].total_ms = total[k];
        ++n;
    }
    *count = n;
    return dropped ? SFB_ENOWS : SFB_OK;
}

int64_t sfb_workspace_bytes(int32_t model, int64_t J, int64_t D, const sfb_batch* batch)
{
    const int rc = check_batch(model, J, D, batch);
    if (rc != SFB_OK) return rc;
    const int64_t B = batch->B;
    switch (model) {
        case SFB_MLR:
            if (batch->in_dtype == SFB_BF16)   // logits (tile-blocked), aligned copy of X, bf16 copy of W
                return bf16_logits_bytes(B, J) + round_up(sfb::bf16_operand_bytes(B, D)) + sfb_shadow_bytes(J, D);
            return round_up(B * J * 4) + round_up(sfb::gemm_f32_partial_bytes(B, J, D));   // logits, k-split scratch
        case SFB_DML:
            return round_up(B * J * 4) + round_up(sfb::gemm_f32_partial_bytes(B, J, D));   // projections Q[B][K], k-split scratch
        default:
            return sc_layout(J, D).total + sc_partial_bytes(B, J, D);
    }
}

int64_t sfb_shadow_bytes(int64_t J, int64_t D)
{
    if (J <= 0 || D <= 0 || D % 8 != 0) return SFB_EINVAL;
    return round_up(sfb::bf16_operand_bytes(J, D));
}

int sfb_shadow_attach(sfb_ctx* ctx, const float* W, int64_t J, int64_t D, void* dev_ptr, int64_t bytes)
{
    if (!ctx || !W || !dev_ptr || !aligned16(W)) return SFB_EINVAL;
    if (ctx->split_lo) return SFB_EINVAL;   // a matrix is attached in split form: detach it first
    const int64_t need = sfb_shadow_bytes(J, D);
    if (need < 0) return SFB_EINVAL;
    if (bytes < need) return SFB_ENOWS;
    if (reinterpret_cast<uintptr_t>(dev_ptr) % ALIGN != 0) return SFB_EINVAL;
    SFB_TRY(hipSetDevice(ctx->device));
    SFB_RUN(KID_SHADOW, sfb::launch_shadow_from_w(W, static_cast<uint16_t*>(dev_ptr), J, D, ctx->stream));
    ctx->shadow_W = W;
    ctx->shadow_buf = static_cast<uint16_t*>(dev_ptr);
    ctx->shadow_J = J;
    ctx->shadow_D = D;
    return SFB_OK;
}

int sfb_shadow_detach(sfb_ctx* ctx)
{
    if (!ctx || ctx->split_lo) return SFB_EINVAL;
    ctx->shadow_W = nullptr;
    ctx->shadow_buf = nullptr;
    ctx->shadow_J = ctx->shadow_D = 0;
    return SFB_OK;
}

int64_t sfb_split_bytes(int64_t J, int64_t D)
{
    const int64_t plane = sfb_shadow_bytes(J, D);
    return plane < 0 ? plane : round_up(sfb::bf16_operand_bytes(J, D)) + round_up(sfb::split_lo_bytes(J, D));
}

int sfb_split_attach(sfb_ctx* ctx, const float* W, int64_t J, int64_t D, void* dev_ptr, int64_t bytes)
{
    if (!ctx || !W || !dev_ptr || !aligned16(W)) return SFB_EINVAL;
    if (ctx->shadow_buf && !(ctx->split_lo && ctx->shadow_W == W && ctx->shadow_J == J && ctx->shadow_D == D))
        return SFB_EINVAL;   // something else is attached (the same matrix in split form may be refreshed)
    const int64_t plane = sfb_shadow_bytes(J, D);
    if (plane < 0) return SFB_EINVAL;
    if (bytes < sfb_split_bytes(J, D)) return SFB_ENOWS;
    if (reinterpret_cast<uintptr_t>(dev_ptr) % ALIGN != 0) return SFB_EINVAL;
    SFB_TRY(hipSetDevice(ctx->device));
    uint16_t* hi = static_cast<uint16_t*>(dev_ptr);
    uint16_t* lo = hi + round_up(sfb::bf16_operand_bytes(J, D)) / 2;
    SFB_RUN(KID_SHADOW, sfb::launch_split_from_w(W, hi, lo, J, D, ctx->stream));
    ctx->shadow_W = W;
    ctx->shadow_buf = hi;
    ctx->shadow_J = J;
    ctx->shadow_D = D;
    ctx->split_lo = lo;
    return SFB_OK;
}

int sfb_split_export(sfb_ctx* ctx, float* W)
{
    if (!ctx || !W || !ctx->split_lo || ctx->shadow_W != W) return SFB_EINVAL;
    SFB_TRY(hipSetDevice(ctx->device));
    SFB_RUN(KID_SHADOW, sfb::launch_w_from_split(ctx->shadow_buf, ctx->split_lo, W, ctx->shadow_J, ctx->shadow_D, ctx->stream));
    return SFB_OK;
}

int sfb_split_detach(sfb_ctx* ctx)
{
    if (!ctx || !ctx->split_lo) return SFB_EINVAL;
    ctx->shadow_W = nullptr;
    ctx->shadow_buf = nullptr;
    ctx->shadow_J = ctx->shadow_D = 0;
    ctx->split_lo = nullptr;
    return SFB_OK;
}

int64_t sfb_apply_workspace_bytes(int64_t J, int64_t D, int64_t N, int32_t sf_dtype)
{
    if (J <= 0 || D <= 0 || N < 0 || !valid_dtype(sf_dtype)) return SFB_EINVAL;
    if (N == 0) return 0;
    if (sf_dtype == SFB_F32) return round_up(sfb::gemm_f32_partial_bytes(J, D, N));   // k-split scratch
    if (J % 8 != 0 || D % 8 != 0) return SFB_EINVAL;
    return round_up(sfb::apply_bf16_workspace_bytes(N, J, D));
}

int sfb_set_workspace(sfb_ctx* ctx, void* dev_ptr, int64_t bytes)
{
    if (!ctx || bytes < 0 || (bytes > 0 && !dev_ptr)) return SFB_EINVAL;
    if (reinterpret_cast<uintptr_t>(dev_ptr) % ALIGN != 0) return SFB_EINVAL;
    ctx->ws = static_cast<char*>(dev_ptr);
    ctx->ws_bytes = bytes;
    return SFB_OK;
}

int sfb_compute_sf(sfb_ctx* ctx, int32_t model, const float* W, int64_t J, int64_t D, const sfb_batch* batch,
                   void* U, void* V, int32_t* n_active)
{
    if (!ctx) return SFB_EINVAL;
    int rc = check_batch(model, J, D, batch);
    if (rc != SFB_OK) return rc;
    const int64_t B = batch->B;
    if (!W || !aligned16(W)) return SFB_EINVAL;
    if (is_split(ctx, W) && !(model == SFB_MLR && batch->in_dtype == SFB_BF16)) return SFB_EINVAL;   // fp32 array is stale
    if (B == 0) return SFB_OK;
    if (!batch->X || !U || !aligned16(batch->X) || !aligned16(U) || (V && !aligned16(V))) return SFB_EINVAL;
    const bool has_shadow = ctx->shadow_buf && ctx->shadow_W == W && ctx->shadow_J == J && ctx->shadow_D == D;
    if (is_split(ctx, W) && !has_shadow) return SFB_EINVAL;   // attached as planes of another shape: the fp32 array is stale
    int64_t need = sfb_workspace_bytes(model, J, D, batch);
    if (model == SFB_MLR && batch->in_dtype == SFB_BF16 && has_shadow) need -= sfb_shadow_bytes(J, D);
    if (need > 0 && (!ctx->ws || ctx->ws_bytes < need)) return SFB_ENOWS;
    SFB_TRY(hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;

    if (model == SFB_MLR) {
        if (!batch->Y) return SFB_EINVAL;
        const int32_t* y = static_cast<const int32_t*>(batch->Y);
        float* Z = reinterpret_cast<float*>(ctx->ws);
        const int64_t esz = batch->in_dtype == SFB_BF16 ? 2 : 4;
        if (batch->in_dtype == SFB_F32) {
            sfb::GemmF32Args g = {};
            g.dev = &ctx->dev;
            g.A = static_cast<const float*>(batch->X); g.lda = D; g.a_kstrided = false;
            g.B = W; g.ldb = D; g.b_kstrided = false;
            g.C = Z; g.ldc = J;
            g.M = B; g.N = J; g.K = D;
            g.epilogue = sfb::EPI_STORE;
            if (sfb::gemm_f32_partial_bytes(B, J, D) > 0) g.partial = reinterpret_cast<float*>(ctx->ws + round_up(B * J * 4));
            SFB_RUN(KID_GEMM_F32_STORE, sfb::launch_gemm_f32(g, st));
            SFB_RUN(KID_SOFTMAX, sfb::launch_mlr_softmax(Z, y, U, false, B, J, st));
        } else {
            uint16_t* Xa = reinterpret_cast<uint16_t*>(ctx->ws + bf16_logits_bytes(B, J));
            const uint16_t* Wb = ctx->shadow_buf;
            if (!has_shadow) {   // no working copy attached: make one for this call
                uint16_t* tmp = Xa + round_up(sfb::bf16_operand_bytes(B, D)) / 2;
                SFB_RUN(KID_SHADOW, sfb::launch_shadow_from_w(W, tmp, J, D, st));
                Wb = tmp;
            }
            SFB_RUN(KID_FORWARD_BF16,
                    sfb::launch_mlr_forward_bf16(static_cast<const uint16_t*>(batch->X), Wb, Z, Xa, B, J, D, ctx->dev, st));
            SFB_RUN(KID_SOFTMAX, sfb::launch_mlr_softmax(Z, y, U, true, B, J, st, true, bf16_softmax_scratch(ctx, B, J), &ctx->dev));
        }
        if (V && V != batch->X)
            SFB_RUN(KID_COPY, hipMemcpyAsync(V, batch->X, (size_t)(B * D * esz), hipMemcpyDeviceToDevice, st));
        return SFB_OK;
    }

    if (model == SFB_DML) {
        if (!batch->Y || !batch->sim || !V || !aligned16(batch->Y)) return SFB_EINVAL;
        float* Q = reinterpret_cast<float*>(ctx->ws);
        float* Vd = static_cast<float*>(V);
        // (the same launch clears the count of active pairs that the scaling kernel below adds to)
        SFB_RUN(KID_DIFF, sfb::launch_diff(static_cast<const float*>(batch->X), static_cast<const float*>(batch->Y), Vd,
                                           B * D, n_active, st));
        sfb::GemmF32Args g = {};
        g.dev = &ctx->dev;
        g.A = Vd; g.lda = D; g.a_kstrided = false;
        g.B = W; g.ldb = D; g.b_kstrided = false;
        g.C = Q; g.ldc = J;
        g.M = B; g.N = J; g.K = D;
        g.epilogue = sfb::EPI_STORE;
        if (sfb::gemm_f32_partial_bytes(B, J, D) > 0) g.partial = reinterpret_cast<float*>(ctx->ws + round_up(B * J * 4));
        SFB_RUN(KID_GEMM_F32_STORE, sfb::launch_gemm_f32(g, st));
        SFB_RUN(KID_DML_SCALE, sfb::launch_dml_scale(Q, batch->sim, static_cast<float*>(U), n_active, batch->margin, B, J, st));
        return SFB_OK;
    }

    // Sparse coding: codes by ISTA, residuals as the second factor.
    if (!V) return SFB_EINVAL;
    const ScLayout lay = sc_layout(J, D);
    float* scratch = reinterpret_cast<float*>(ctx->ws);
    float* Lp = reinterpret_cast<float*>(ctx->ws + lay.off_L);
    float* ksplit = sc_partial_bytes(B, J, D) > 0 ? reinterpret_cast<float*>(ctx->ws + lay.total) : nullptr;
    float* A = static_cast<float*>(U);
    float* R = static_cast<float*>(V);
    const float* X = static_cast<const float*>(batch->X);
    SFB_RUN(KID_POWER_ITERATION, sfb::launch_power_iteration(W, J, D, batch->power_iters, scratch, Lp, st));
    SFB_RUN(KID_FILL, sfb::launch_fill_u32(A, 0u, B * J, st));
    for (int it = 0; it <= batch->ista_iters; ++it) {
        if (it == 0) {
            // a = 0  =>  r = x
            SFB_RUN(KID_COPY, hipMemcpyAsync(R, X, (size_t)(B * D * 4), hipMemcpyDeviceToDevice, st));
        } else {
            sfb::GemmF32Args g = {};  // R = X - A W   (contraction over the basis index j)
            g.dev = &ctx->dev;
            g.A = A; g.lda = J; g.a_kstrided = false;
            g.B = W; g.ldb = D; g.b_kstrided = true;
            g.C = R; g.ldc = D;
            g.M = B; g.N = D; g.K = J;
            g.epilogue = sfb::EPI_RESID;
            g.aux = X;
            g.partial = ksplit;
            SFB_RUN(KID_GEMM_F32_RESID, sfb::launch_gemm_f32(g, st));
        }
        if (it == batch->ista_iters) break;
        sfb::GemmF32Args g = {};  // A = soft(A + (R W^T)/L, lambda/L)
        g.dev = &ctx->dev;
        g.A = R; g.lda = D; g.a_kstrided = false;
        g.B = W; g.ldb = D; g.b_kstrided = false;
        g.C = A; g.ldc = J;
        g.M = B; g.N = J; g.K = D;
        g.epilogue = sfb::EPI_SHRINK;
        g.aux = A;
        g.L_ptr = Lp;
        g.lambda = batch->lambda;
        g.partial = ksplit;
        SFB_RUN(KID_GEMM_F32_SHRINK, sfb::launch_gemm_f32(g, st));
    }
    return SFB_OK;
}

// Shared by sfb_apply (coef == nullptr) and sfb_apply_signed.
static int apply_impl(sfb_ctx* ctx, float* W, int64_t J, int64_t D, const void* U, const void* V, const float* coef,
                      int64_t N, int32_t sf_dtype, float eta)
{
    const int64_t need = coef ? sfb_apply_signed_workspace_bytes(J, D, N, sf_dtype)
                              : sfb_apply_workspace_bytes(J, D, N, sf_dtype);
    if (need < 0) return (int)need;
    if (need > 0 && (!ctx->ws || ctx->ws_bytes < need)) return SFB_ENOWS;
    if (is_split(ctx, W) && (sf_dtype != SFB_BF16 || ctx->shadow_J != J || ctx->shadow_D != D)) return SFB_EINVAL;
    SFB_TRY(hipSetDevice(ctx->device));
    if (sf_dtype == SFB_F32) {
        const int64_t part = round_up(sfb::gemm_f32_partial_bytes(J, D, N));
        const float* Vf = static_cast<const float*>(V);
        if (coef) {   // scaled copy of V behind the k-split scratch
            float* Vs = reinterpret_cast<float*>(ctx->ws + part);
            SFB_RUN(KID_SCALE_ROWS, sfb::launch_scale_rows(Vf, coef, Vs, N, D, ctx->stream));
            Vf = Vs;
        }
        sfb::GemmF32Args g = {};  // both factors are strided along the SF index
        g.dev = &ctx->dev;
        g.A = static_cast<const float*>(U); g.lda = J; g.a_kstrided = true;
        g.B = Vf; g.ldb = D; g.b_kstrided = true;
        g.C = W; g.ldc = D;
        g.M = J; g.N = D; g.K = N;
        g.epilogue = sfb::EPI_RMW;
        g.eta = eta;
        if (part > 0) g.partial = reinterpret_cast<float*>(ctx->ws);
        SFB_RUN(KID_GEMM_F32_RMW, sfb::launch_gemm_f32(g, ctx->stream));
        if (ctx->shadow_buf && ctx->shadow_W == W && ctx->shadow_J == J && ctx->shadow_D == D)
            SFB_RUN(KID_SHADOW, sfb::launch_shadow_from_w(W, ctx->shadow_buf, J, D, ctx->stream));
    } else {
        uint16_t* Wb = (ctx->shadow_buf && ctx->shadow_W == W && ctx->shadow_J == J && ctx->shadow_D == D)
                           ? ctx->shadow_buf
                           : nullptr;
        SFB_RUN(KID_APPLY_TRANSPOSE,
                sfb::launch_apply_bf16_transpose(static_cast<const uint16_t*>(U), static_cast<const uint16_t*>(V), coef,
                                                 N, J, D, ctx->ws, ctx->stream));
        SFB_RUN(KID_APPLY_BF16, sfb::launch_apply_bf16(W, Wb, is_split(ctx, W) ? ctx->split_lo : nullptr, N, J, D, eta,
                                                       ctx->ws, ctx->dev, ctx->stream));
    }
    return SFB_OK;
}

static int check_apply_args(sfb_ctx* ctx, const float* W, int64_t J, int64_t D, const void* U, const void* V, int64_t N,
                            int32_t sf_dtype)
{
    if (!ctx || J <= 0 || D <= 0 || N < 0 || !valid_dtype(sf_dtype)) return SFB_EINVAL;
    if (!W || !aligned16(W)) return SFB_EINVAL;
    if (N == 0) return SFB_OK;
    if (!U || !V || !aligned16(U) || !aligned16(V)) return SFB_EINVAL;
    if (sf_dtype == SFB_BF16 && (J % 8 != 0 || D % 8 != 0)) return SFB_EINVAL;
    return SFB_OK;
}

int sfb_apply(sfb_ctx* ctx, float* W, int64_t J, int64_t D, const void* U, const void* V, int64_t N,
              int32_t sf_dtype, float eta)
{
    const int rc = check_apply_args(ctx, W, J, D, U, V, N, sf_dtype);
    if (rc != SFB_OK || N == 0) return rc;
    return apply_impl(ctx, W, J, D, U, V, nullptr, N, sf_dtype, eta);
}

int sfb_apply_static(sfb_ctx* ctx, float* W, int64_t J, int64_t D, const void* U, const void* V, int64_t N,
                     int32_t sf_dtype, float eta)
{
    const int rc = check_apply_args(ctx, W, J, D, U, V, N, sf_dtype);
    if (rc != SFB_OK || N == 0) return rc;
    const int64_t need = sfb_apply_workspace_bytes(J, D, N, sf_dtype);
    if (need < 0) return (int)need;
    if (need > (int64_t)SFB_STATIC_SCRATCH_BYTES) return SFB_ETOOBIG;
    if (!ctx->static_scratch) return hip_fail(ctx, (hipError_t)ctx->static_scratch_err);
    // the same launches as sfb_apply, with the static array in the place of the caller's workspace
    char* const ws = ctx->ws;
    const int64_t ws_bytes = ctx->ws_bytes;
    ctx->ws = ctx->static_scratch;
    ctx->ws_bytes = (int64_t)SFB_STATIC_SCRATCH_BYTES;
    const int out = apply_impl(ctx, W, J, D, U, V, nullptr, N, sf_dtype, eta);
    ctx->ws = ws;
    ctx->ws_bytes = ws_bytes;
    return out;
}

int64_t sfb_apply_signed_workspace_bytes(int64_t J, int64_t D, int64_t N, int32_t sf_dtype)
{
    const int64_t base = sfb_apply_workspace_bytes(J, D, N, sf_dtype);
    if (base < 0 || sf_dtype != SFB_F32) return base;       // bf16: the coefficient goes into the V^T copy
    return base + round_up(N * D * 4);                       // fp32: scaled copy of V
}

int sfb_apply_signed(sfb_ctx* ctx, float* W, int64_t J, int64_t D, const void* U, const void* V, const float* coef,
                     int64_t N, int32_t sf_dtype, float eta)
{
    const int rc = check_apply_args(ctx, W, J, D, U, V, N, sf_dtype);
    if (rc != SFB_OK || N == 0) return rc;
    if (!coef || !aligned16(coef)) return SFB_EINVAL;
    return apply_impl(ctx, W, J, D, U, V, coef, N, sf_dtype, eta);
}

static int check_csr(const sfb_csr* m, int64_t cols)
{
    if (!m || m->rows < 0 || m->cols != cols || m->nnz < 0 || !valid_dtype(m->dtype)) return SFB_EINVAL;
    if (m->rows > 0 && (!m->indptr || !aligned16(m->indptr))) return SFB_EINVAL;
    if (m->nnz > 0 && (!m->indices || !m->values || !aligned16(m->indices) || !aligned16(m->values))) return SFB_EINVAL;
    return SFB_OK;
}

int sfb_csr_check(sfb_ctx* ctx, const sfb_csr* m, int64_t* violations)
{
    if (!ctx || !violations || !m) return SFB_EINVAL;
    const int rc = check_csr(m, m->cols);
    if (rc != SFB_OK || m->cols <= 0) return SFB_EINVAL;
    *violations = 0;
    if (m->rows == 0) return m->nnz == 0 ? SFB_OK : SFB_EINVAL;
    if (!ctx->ws || ctx->ws_bytes < ALIGN) return SFB_ENOWS;
    SFB_TRY(hipSetDevice(ctx->device));
    unsigned int* bad = reinterpret_cast<unsigned int*>(ctx->ws);
    SFB_RUN(KID_FILL, sfb::launch_fill_u32(bad, 0u, 1, ctx->stream));
    SFB_RUN(KID_CSR, sfb::launch_csr_check(m->indptr, m->indices, m->rows, m->cols, m->nnz, bad, ctx->stream));
    unsigned int host = 0;
    SFB_TRY(hipMemcpyAsync(&host, bad, sizeof(host), hipMemcpyDeviceToHost, ctx->stream));
    SFB_TRY(hipStreamSynchronize(ctx->stream));
    *violations = host;
    return SFB_OK;
}

// Bytes of the operand region of sfb_mlr_sf_csr behind the logits: the aligned dense copy of X (dense route) or
// the re-laid CSR rows (route over the non-zeros), whichever is larger.
static int64_t csr_operand_bytes(int64_t J, int64_t D, int64_t B, bool bf16)
{
    const int64_t dense = bf16 ? round_up(sfb::bf16_operand_bytes(B, D)) : round_up(B * D * 4);
    const int64_t gather = sfb::csr_gather_supported(B, J, D) ? round_up(sfb::csr_gather_workspace_bytes(B, D, bf16)) : 0;
    return dense > gather ? dense : gather;
}

int64_t sfb_mlr_sf_csr_workspace_bytes(int64_t J, int64_t D, int64_t B, int32_t dtype)
{
    if (!valid_dtype(dtype)) return SFB_EINVAL;
    sfb_batch b = {};
    b.B = B;
    b.in_dtype = b.sf_dtype = dtype;
    const int64_t base = sfb_workspace_bytes(SFB_MLR, J, D, &b);
    if (base < 0) return base;
    if (dtype == SFB_BF16)      // logits, exchange words, operand region, room for a bf16 copy of W
        return base - round_up(sfb::bf16_operand_bytes(B, D)) + csr_operand_bytes(J, D, B, true);
    return base + csr_operand_bytes(J, D, B, false);     // fp32: logits, k-split scratch, operand region
}

// Whether the logits of these CSR samples are computed over the stored entries only.  Measured on MI355X
// (J = 325000, D = 10000, bf16): the gather kernel takes, per group of up to 1024 samples, one pass over W
// (1.6 ms: 5e-13 s per element) plus 8.4e-11 s per class and stored entry of an average sample (a lane walks one
// sample, so the time follows the entries per sample, not their total); the dense MFMA product runs at about
// 1.45 PFLOP/s on ceil(B / 256) * 256 rows.  That puts the crossover near 1 % of non-zeros at B = 1024 and leaves
// batches of 256 and fewer to the dense product at any density.  fp32: both routes are slower (twice the bytes of W,
// twice the LDS reads per entry; the fp32 MFMA product runs at about 60 TFLOP/s), the gather route wins up to some 10 %.
static bool csr_use_gather(const sfb_ctx* ctx, int64_t B, int64_t J, int64_t D, int64_t nnz, bool bf16)
{
    if (!sfb::csr_gather_supported(B, J, D) || ctx->csr_route == 1) return false;
    if (ctx->csr_route == 2) return true;
    const double groups = (double)((B + 1023) / 1024), per_sample = (double)nnz / (double)B;
    const double gather = groups * ((bf16 ? 5e-13 : 1e-12) * (double)J * (double)D + (bf16 ? 8.4e-11 : 1.7e-10) * (double)J * per_sample);
    const double rows = (double)((B + 255) / 256 * 256);
    const double dense = 2.0 * rows * (double)J * (double)D / (bf16 ? 1.45e15 : 6e13);
    return gather < dense;
}

int sfb_set_csr_route(sfb_ctx* ctx, int route)
{
    if (!ctx || route < 0 || route > 2) return SFB_EINVAL;
    ctx->csr_route = route;
    return SFB_OK;
}

int sfb_mlr_sf_csr(sfb_ctx* ctx, const float* W, int64_t J, int64_t D, const sfb_csr* X, const int32_t* y, void* U)
{
    if (!ctx || J <= 0 || D <= 0) return SFB_EINVAL;
    int rc = check_csr(X, D);
    if (rc != SFB_OK) return rc;
    const int64_t B = X->rows;
    const bool bf16 = X->dtype == SFB_BF16;
    if (bf16 && (J % 8 != 0 || D % 8 != 0)) return SFB_EINVAL;
    if (!W || !aligned16(W)) return SFB_EINVAL;
    if (B == 0) return SFB_OK;
    if (!y || !U || !aligned16(U)) return SFB_EINVAL;
    const bool has_shadow = ctx->shadow_buf && ctx->shadow_W == W && ctx->shadow_J == J && ctx->shadow_D == D;
    if (is_split(ctx, W) && (!bf16 || !has_shadow)) return SFB_EINVAL;
    int64_t need = sfb_mlr_sf_csr_workspace_bytes(J, D, B, X->dtype);
    if (need < 0) return (int)need;
    if (bf16 && has_shadow) need -= sfb_shadow_bytes(J, D);
    if (!ctx->ws || ctx->ws_bytes < need) return SFB_ENOWS;
    SFB_TRY(hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;
    float* Z = reinterpret_cast<float*>(ctx->ws);
    const bool gather = csr_use_gather(ctx, B, J, D, X->nnz, bf16);
    if (!bf16) {
        const int64_t part = round_up(sfb::gemm_f32_partial_bytes(B, J, D));
        char* region = ctx->ws + round_up(B * J * 4) + part;
        if (gather) {
            SFB_RUN(KID_CSR_GATHER, sfb::launch_csr_forward_gather(X->indptr, X->indices, X->values, false, W, Z, B, J, D,
                                                                   X->nnz, region, st));
        } else {
            float* Xd = reinterpret_cast<float*>(region);
            SFB_RUN(KID_FILL, sfb::launch_fill_u32(Xd, 0u, B * D, st));
            SFB_RUN(KID_CSR, sfb::launch_csr_scatter(X->indptr, X->indices, X->values, false, nullptr, Xd, B, D, X->nnz, D, 1, st));
            sfb::GemmF32Args g = {};
            g.dev = &ctx->dev;
            g.A = Xd; g.lda = D; g.a_kstrided = false;
            g.B = W; g.ldb = D; g.b_kstrided = false;
            g.C = Z; g.ldc = J;
            g.M = B; g.N = J; g.K = D;
            g.epilogue = sfb::EPI_STORE;
            if (part > 0) g.partial = reinterpret_cast<float*>(ctx->ws + round_up(B * J * 4));
            SFB_RUN(KID_GEMM_F32_STORE, sfb::launch_gemm_f32(g, st));
        }
        SFB_RUN(KID_SOFTMAX, sfb::launch_mlr_softmax(Z, y, U, false, B, J, st));
        return SFB_OK;
    }
    const int64_t pitch = sfb::bf16_pitch(D);
    char* region = ctx->ws + bf16_logits_bytes(B, J);
    const uint16_t* Wb = ctx->shadow_buf;
    if (!has_shadow) {
        uint16_t* tmp = reinterpret_cast<uint16_t*>(region + csr_operand_bytes(J, D, B, true));
        SFB_RUN(KID_SHADOW, sfb::launch_shadow_from_w(W, tmp, J, D, st));
        Wb = tmp;
    }
    if (gather) {
        SFB_RUN(KID_CSR_GATHER, sfb::launch_csr_forward_gather(X->indptr, X->indices, X->values, true, Wb, Z, B, J, D, X->nnz,
                                                               region, st));
    } else {
        uint16_t* Xa = reinterpret_cast<uint16_t*>(region);
        SFB_RUN(KID_FILL, sfb::launch_fill_u32(Xa, 0u, sfb::bf16_operand_bytes(B, D) / 4, st));
        SFB_RUN(KID_CSR, sfb::launch_csr_scatter(X->indptr, X->indices, X->values, true, nullptr, Xa, B, D, X->nnz, -pitch, 1, st));
        SFB_RUN(KID_FORWARD_BF16, sfb::launch_mlr_forward_bf16(nullptr, Wb, Z, Xa, B, J, D, ctx->dev, st));
    }
    SFB_RUN(KID_SOFTMAX, sfb::launch_mlr_softmax(Z, y, U, true, B, J, st, true, bf16_softmax_scratch(ctx, B, J), &ctx->dev));
    return SFB_OK;
}

int64_t sfb_apply_csr_workspace_bytes(int64_t J, int64_t D, int64_t N, int32_t sf_dtype)
{
    const int64_t base = sfb_apply_workspace_bytes(J, D, N, sf_dtype);
    if (base < 0 || sf_dtype != SFB_F32) return base;   // bf16: V^T is written from the CSR rows
    return base + round_up(N * D * 4);                   // fp32: dense V
}

int sfb_apply_csr(sfb_ctx* ctx, float* W, int64_t J, int64_t D, const void* U, const sfb_csr* V, const float* coef,
                  float eta)
{
    if (!ctx || J <= 0 || D <= 0) return SFB_EINVAL;
    const int rc = check_csr(V, D);
    if (rc != SFB_OK) return rc;
    const int64_t N = V->rows;
    if (!W || !aligned16(W)) return SFB_EINVAL;
    if (N == 0) return SFB_OK;
    if (!U || !aligned16(U) || (coef && !aligned16(coef))) return SFB_EINVAL;
    if (V->dtype == SFB_BF16 && (J % 8 != 0 || D % 8 != 0)) return SFB_EINVAL;
    const int64_t need = sfb_apply_csr_workspace_bytes(J, D, N, V->dtype);
    if (need < 0) return (int)need;
    if (need > 0 && (!ctx->ws || ctx->ws_bytes < need)) return SFB_ENOWS;
    SFB_TRY(hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;
    const bool has_shadow = ctx->shadow_buf && ctx->shadow_W == W && ctx->shadow_J == J && ctx->shadow_D == D;
    if (is_split(ctx, W) && (V->dtype != SFB_BF16 || !has_shadow)) return SFB_EINVAL;
    if (V->dtype == SFB_F32) {
        const int64_t part = round_up(sfb::gemm_f32_partial_bytes(J, D, N));
        float* Vd = reinterpret_cast<float*>(ctx->ws + part);
        SFB_RUN(KID_FILL, sfb::launch_fill_u32(Vd, 0u, N * D, st));
        SFB_RUN(KID_CSR, sfb::launch_csr_scatter(V->indptr, V->indices, V->values, false, coef, Vd, N, D, V->nnz, D, 1, st));
        sfb::GemmF32Args g = {};
        g.dev = &ctx->dev;
        g.A = static_cast<const float*>(U); g.lda = J; g.a_kstrided = true;
        g.B = Vd; g.ldb = D; g.b_kstrided = true;
        g.C = W; g.ldc = D;
        g.M = J; g.N = D; g.K = N;
        g.epilogue = sfb::EPI_RMW;
        g.eta = eta;
        if (part > 0) g.partial = reinterpret_cast<float*>(ctx->ws);
        SFB_RUN(KID_GEMM_F32_RMW, sfb::launch_gemm_f32(g, st));
        if (has_shadow) SFB_RUN(KID_SHADOW, sfb::launch_shadow_from_w(W, ctx->shadow_buf, J, D, st));
        return SFB_OK;
    }
    const int64_t Np = sfb::bf16_pitch(N);
    uint16_t* Vt = sfb::apply_bf16_vt(ctx->ws, N, J);
    SFB_RUN(KID_FILL, sfb::launch_fill_u32(Vt, 0u, sfb::bf16_operand_bytes(D, N) / 4, st));
    SFB_RUN(KID_CSR, sfb::launch_csr_scatter(V->indptr, V->indices, V->values, true, coef, Vt, N, D, V->nnz, 1, -Np, st));
    SFB_RUN(KID_APPLY_TRANSPOSE, sfb::launch_apply_bf16_transpose(static_cast<const uint16_t*>(U), nullptr, nullptr, N, J,
                                                                  D, ctx->ws, st));
    SFB_RUN(KID_APPLY_BF16, sfb::launch_apply_bf16(W, has_shadow ? ctx->shadow_buf : nullptr,
                                                   is_split(ctx, W) ? ctx->split_lo : nullptr, N, J, D, eta, ctx->ws, ctx->dev, st));
    return SFB_OK;
}

int64_t sfb_sdca_workspace_bytes(int64_t J, int64_t D, int64_t B)
{
    if (J <= 0 || D <= 0 || B < 0) return SFB_EINVAL;
    return round_up(B * J * 4) + round_up(sfb::gemm_f32_partial_bytes(B, J, D));   // logits, k-split scratch
}

int sfb_sdca_mlr_sf(sfb_ctx* ctx, const float* W, int64_t J, int64_t D, const float* X, int64_t B, float* P,
                    float lambda, int64_t N, float beta, float* dU)
{
    if (!ctx || J <= 0 || D <= 0 || B < 0 || N <= 0) return SFB_EINVAL;
    if (!(lambda > 0.f) || !(beta > 0.f) || !(beta <= 1.f)) return SFB_EINVAL;
    if (!W || !aligned16(W) || is_split(ctx, W)) return SFB_EINVAL;
    if (B == 0) return SFB_OK;
    if (!X || !P || !dU || !aligned16(X) || !aligned16(P) || !aligned16(dU)) return SFB_EINVAL;
    const int64_t need = sfb_sdca_workspace_bytes(J, D, B);
    if (!ctx->ws || ctx->ws_bytes < need) return SFB_ENOWS;
    SFB_TRY(hipSetDevice(ctx->device));
    float* Zl = reinterpret_cast<float*>(ctx->ws);
    sfb::GemmF32Args g = {};
    g.dev = &ctx->dev;
    g.A = X; g.lda = D; g.a_kstrided = false;
    g.B = W; g.ldb = D; g.b_kstrided = false;
    g.C = Zl; g.ldc = J;
    g.M = B; g.N = J; g.K = D;
    g.epilogue = sfb::EPI_STORE;
    if (sfb::gemm_f32_partial_bytes(B, J, D) > 0) g.partial = reinterpret_cast<float*>(ctx->ws + round_up(B * J * 4));
    SFB_RUN(KID_GEMM_F32_STORE, sfb::launch_gemm_f32(g, ctx->stream));
    SFB_RUN(KID_SDCA, sfb::launch_sdca_mlr(Zl, X, P, dU, B, J, D, lambda, N, beta, ctx->stream));
    return SFB_OK;
}

int sfb_dual_to_primal_l2(sfb_ctx* ctx, const float* Z, float* W, int64_t J, int64_t D, float lambda)
{
    if (!ctx || !Z || !W || J <= 0 || D <= 0 || !(lambda > 0.f) || is_split(ctx, W) || is_split(ctx, Z)) return SFB_EINVAL;
    SFB_TRY(hipSetDevice(ctx->device));
    SFB_RUN(KID_DUAL_TO_PRIMAL, sfb::launch_div_scalar(Z, W, lambda, J * D, ctx->stream));
    if (ctx->shadow_buf && ctx->shadow_W == W && ctx->shadow_J == J && ctx->shadow_D == D)
        SFB_RUN(KID_SHADOW, sfb::launch_shadow_from_w(W, ctx->shadow_buf, J, D, ctx->stream));
    return SFB_OK;
}

int sfb_prox_rows(sfb_ctx* ctx, float* W, int64_t J, int64_t D, int32_t mode)
{
    if (!ctx || !W || J <= 0 || D <= 0 || is_split(ctx, W)) return SFB_EINVAL;
    if (mode != SFB_PROX_PROJECT && mode != SFB_PROX_NORMALIZE) return SFB_EINVAL;
    SFB_TRY(hipSetDevice(ctx->device));
    SFB_RUN(KID_PROX, sfb::launch_prox_rows(W, J, D, mode, ctx->stream));
    if (ctx->shadow_buf && ctx->shadow_W == W && ctx->shadow_J == J && ctx->shadow_D == D)
        SFB_RUN(KID_SHADOW, sfb::launch_shadow_from_w(W, ctx->shadow_buf, J, D, ctx->stream));
    return SFB_OK;
}

const char* sfb_strerror(int code)
{
    switch (code) {
        case SFB_OK: return "success";
        case SFB_EINVAL: return "invalid argument (null/misaligned pointer, shape, enum or dtype combination)";
        case SFB_ENOWS: return "workspace missing or smaller than sfb_workspace_bytes()";
        case SFB_EHIP: return "a HIP call failed (see sfb_last_hip_error)";
        case SFB_ETOOBIG: return "problem too large for the library's static scratch (SFB_STATIC_SCRATCH_BYTES)";
        default: return "unknown sfb status";
    }
}

int sfb_last_hip_error(const sfb_ctx* ctx) { return ctx ? ctx->last_hip_error : 0; }

const char* sfb_version(void) { return "0.1"; }

int sfb_set_wait_limit(sfb_ctx* ctx, int polls)
{
    if (!ctx) return SFB_EINVAL;
    ctx->dev.softmax_wait_polls = polls < 0 ? 1000 : polls;
    return SFB_OK;
}

int sfb_wait_fallbacks(sfb_ctx* ctx, int64_t* count)
{
    if (!ctx || !count) return SFB_EINVAL;
    SFB_TRY(hipSetDevice(ctx->device));
    SFB_TRY(hipStreamSynchronize(ctx->stream));
    unsigned long long n = 0;
    SFB_TRY(sfb::softmax_fallbacks(&n));
    *count = (int64_t)n;
    return SFB_OK;
}

}  // extern "C"
