// C-ABI of libsfb (see include/sfb.h for the contract): argument checks,
// workspace carving and the sequence of kernel launches of each call.  No device
// memory is allocated or freed here and nothing synchronises with the host.
#include "../../include/sfb.h"

#include <hip/hip_runtime.h>

#include <new>

#include "kernels.h"

struct sfb_ctx {
    int device;
    hipStream_t stream;
    char* ws;
    int64_t ws_bytes;
    int last_hip_error;
};

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
    c->device = device_id;
    c->stream = reinterpret_cast<hipStream_t>(hip_stream);
    c->ws = nullptr;
    c->ws_bytes = 0;
    c->last_hip_error = 0;
    *out = c;
    return SFB_OK;
}

int sfb_destroy(sfb_ctx* ctx)
{
    if (!ctx) return SFB_EINVAL;
    delete ctx;
    return SFB_OK;
}

int64_t sfb_workspace_bytes(int32_t model, int64_t J, int64_t D, const sfb_batch* batch)
{
    const int rc = check_batch(model, J, D, batch);
    if (rc != SFB_OK) return rc;
    const int64_t B = batch->B;
    switch (model) {
        case SFB_MLR:
        case SFB_DML:
            return round_up(B * J * 4);  // logits Z[B][J] / projections Q[B][K], fp32
        default:
            return sc_layout(J, D).total;
    }
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
    if (B == 0) return SFB_OK;
    if (!batch->X || !U || !aligned16(batch->X) || !aligned16(U) || (V && !aligned16(V))) return SFB_EINVAL;
    const int64_t need = sfb_workspace_bytes(model, J, D, batch);
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
            g.A = static_cast<const float*>(batch->X); g.lda = D; g.a_kstrided = false;
            g.B = W; g.ldb = D; g.b_kstrided = false;
            g.C = Z; g.ldc = J;
            g.M = B; g.N = J; g.K = D;
            g.epilogue = sfb::EPI_STORE;
            SFB_TRY(sfb::launch_gemm_f32(g, st));
            SFB_TRY(sfb::launch_mlr_softmax(Z, y, U, false, B, J, st));
        } else {
            SFB_TRY(sfb::launch_mlr_forward_bf16(static_cast<const uint16_t*>(batch->X), W, Z, B, J, D, st));
            SFB_TRY(sfb::launch_mlr_softmax(Z, y, U, true, B, J, st));
        }
        if (V && V != batch->X)
            SFB_TRY(hipMemcpyAsync(V, batch->X, (size_t)(B * D * esz), hipMemcpyDeviceToDevice, st));
        return SFB_OK;
    }

    if (model == SFB_DML) {
        if (!batch->Y || !batch->sim || !V || !aligned16(batch->Y)) return SFB_EINVAL;
        float* Q = reinterpret_cast<float*>(ctx->ws);
        float* Vd = static_cast<float*>(V);
        SFB_TRY(sfb::launch_diff(static_cast<const float*>(batch->X), static_cast<const float*>(batch->Y), Vd, B * D,
                                 st));
        sfb::GemmF32Args g = {};
        g.A = Vd; g.lda = D; g.a_kstrided = false;
        g.B = W; g.ldb = D; g.b_kstrided = false;
        g.C = Q; g.ldc = J;
        g.M = B; g.N = J; g.K = D;
        g.epilogue = sfb::EPI_STORE;
        SFB_TRY(sfb::launch_gemm_f32(g, st));
        if (n_active) SFB_TRY(sfb::launch_fill_u32(n_active, 0u, 1, st));
        SFB_TRY(sfb::launch_dml_scale(Q, batch->sim, static_cast<float*>(U), n_active, batch->margin, B, J, st));
        return SFB_OK;
    }

    // Sparse coding: codes by ISTA, residuals as the second factor.
    if (!V) return SFB_EINVAL;
    const ScLayout lay = sc_layout(J, D);
    float* scratch = reinterpret_cast<float*>(ctx->ws);
    float* Lp = reinterpret_cast<float*>(ctx->ws + lay.off_L);
    float* A = static_cast<float*>(U);
    float* R = static_cast<float*>(V);
    const float* X = static_cast<const float*>(batch->X);
    SFB_TRY(sfb::launch_power_iteration(W, J, D, batch->power_iters, scratch, Lp, st));
    SFB_TRY(sfb::launch_fill_u32(A, 0u, B * J, st));
    for (int it = 0; it <= batch->ista_iters; ++it) {
        if (it == 0) {
            // a = 0  =>  r = x
            SFB_TRY(hipMemcpyAsync(R, X, (size_t)(B * D * 4), hipMemcpyDeviceToDevice, st));
        } else {
            sfb::GemmF32Args g = {};  // R = X - A W   (contraction over the basis index j)
            g.A = A; g.lda = J; g.a_kstrided = false;
            g.B = W; g.ldb = D; g.b_kstrided = true;
            g.C = R; g.ldc = D;
            g.M = B; g.N = D; g.K = J;
            g.epilogue = sfb::EPI_RESID;
            g.aux = X;
            SFB_TRY(sfb::launch_gemm_f32(g, st));
        }
        if (it == batch->ista_iters) break;
        sfb::GemmF32Args g = {};  // A = soft(A + (R W^T)/L, lambda/L)
        g.A = R; g.lda = D; g.a_kstrided = false;
        g.B = W; g.ldb = D; g.b_kstrided = false;
        g.C = A; g.ldc = J;
        g.M = B; g.N = J; g.K = D;
        g.epilogue = sfb::EPI_SHRINK;
        g.aux = A;
        g.L_ptr = Lp;
        g.lambda = batch->lambda;
        SFB_TRY(sfb::launch_gemm_f32(g, st));
    }
    return SFB_OK;
}

int sfb_apply(sfb_ctx* ctx, float* W, int64_t J, int64_t D, const void* U, const void* V, int64_t N,
              int32_t sf_dtype, float eta)
{
    if (!ctx || J <= 0 || D <= 0 || N < 0 || !valid_dtype(sf_dtype)) return SFB_EINVAL;
    if (!W || !aligned16(W)) return SFB_EINVAL;
    if (N == 0) return SFB_OK;
    if (!U || !V || !aligned16(U) || !aligned16(V)) return SFB_EINVAL;
    if (sf_dtype == SFB_BF16 && (J % 8 != 0 || D % 8 != 0)) return SFB_EINVAL;
    SFB_TRY(hipSetDevice(ctx->device));
    if (sf_dtype == SFB_F32) {
        sfb::GemmF32Args g = {};  // both factors are strided along the SF index
        g.A = static_cast<const float*>(U); g.lda = J; g.a_kstrided = true;
        g.B = static_cast<const float*>(V); g.ldb = D; g.b_kstrided = true;
        g.C = W; g.ldc = D;
        g.M = J; g.N = D; g.K = N;
        g.epilogue = sfb::EPI_RMW;
        g.eta = eta;
        SFB_TRY(sfb::launch_gemm_f32(g, ctx->stream));
    } else {
        SFB_TRY(sfb::launch_apply_bf16(W, static_cast<const uint16_t*>(U), static_cast<const uint16_t*>(V), N, J, D,
                                       eta, ctx->stream));
    }
    return SFB_OK;
}

int sfb_prox_rows(sfb_ctx* ctx, float* W, int64_t J, int64_t D, int32_t mode)
{
    if (!ctx || !W || J <= 0 || D <= 0) return SFB_EINVAL;
    if (mode != SFB_PROX_PROJECT && mode != SFB_PROX_NORMALIZE) return SFB_EINVAL;
    SFB_TRY(hipSetDevice(ctx->device));
    SFB_TRY(sfb::launch_prox_rows(W, J, D, mode, ctx->stream));
    return SFB_OK;
}

const char* sfb_strerror(int code)
{
    switch (code) {
        case SFB_OK: return "success";
        case SFB_EINVAL: return "invalid argument (null/misaligned pointer, shape, enum or dtype combination)";
        case SFB_ENOWS: return "workspace missing or smaller than sfb_workspace_bytes()";
        case SFB_EHIP: return "a HIP call failed (see sfb_last_hip_error)";
        default: return "unknown sfb status";
    }
}

int sfb_last_hip_error(const sfb_ctx* ctx) { return ctx ? ctx->last_hip_error : 0; }

const char* sfb_version(void) { return "0.1"; }

void sfb_tune_bf16_variant(int forward_variant, int apply_variant)
{
    sfb::set_bf16_variant(forward_variant, apply_variant);
}

}  // extern "C"
