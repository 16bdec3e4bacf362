// Internal (C++) launch interface between the C-ABI layer and the HIP kernels.
// Every function only enqueues work on `stream` and returns the launch status.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sfb {

// What the launchers need to know of the device a context is bound to; read once when the context is created.
struct DeviceInfo {
    int cus = 0;                                   // compute units
    int xcds = 0;                                  // accelerator dies, one L2 each (workgroup ids go round-robin over them)
    bool gemm_bf16_lds_set[3] = {false, false, false};   // dynamic-LDS attribute of sf_gemm_kernel<mode> set on this device
    bool gemm_f32_lds_set[12] = {};                      // the same for the pipelined fp32 kernels (operand combination x tile shape)
    int softmax_wait_polls = 1000;                 // bound of the one-read softmax's wait for a partner's word
};

// ---------------------------------------------------------------------------
// fp32 MFMA GEMM family:  acc[m][n] = sum_k A(m,k) * B(n,k), followed by an
// epilogue that writes C[m*ldc + n].
//   operand layout "k-contiguous": A(m,k) = A[m*lda + k]
//   operand layout "k-strided":    A(m,k) = A[k*lda + m]
// ---------------------------------------------------------------------------
enum GemmEpilogue : int {
    EPI_STORE = 0,   // C = acc
    EPI_RMW = 1,     // C = C - eta * acc                      (rank-1 update sum applied to W)
    EPI_RESID = 2,   // C = aux - acc                          (sparse-coding residual x - W^T a)
    EPI_SHRINK = 3,  // C = soft(aux + acc / L, lambda / L)    (one ISTA step), L read from *L_ptr
};

struct GemmF32Args {
    const float* A;
    int64_t lda;
    bool a_kstrided;
    const float* B;
    int64_t ldb;
    bool b_kstrided;
    float* C;
    int64_t ldc;
    int64_t M, N, K;
    int epilogue;
    float eta;           // EPI_RMW
    const float* aux;    // EPI_RESID / EPI_SHRINK, same leading dimension as C; may alias C
    const float* L_ptr;  // EPI_SHRINK: device scalar
    float lambda;        // EPI_SHRINK
    float* partial;      // scratch of gemm_f32_partial_bytes(M, N, K) for the k-split, or null (no split)
    DeviceInfo* dev;     // the context's device facts; null: the plain kernel only
};
hipError_t launch_gemm_f32(const GemmF32Args& a, hipStream_t stream);
// Scratch a contraction of this shape can use to split its k range over several
// workgroups (0: it would not be split).  16-byte aligned.
int64_t gemm_f32_partial_bytes(int64_t M, int64_t N, int64_t K);

// ---------------------------------------------------------------------------
// bf16 MFMA kernel of the large MLR path (fp32 accumulate) and its layout helpers.
// ---------------------------------------------------------------------------
// Every bf16 operand of the kernel (the aligned copy of X, the working copy / high plane of W, U^T, V^T) is
// stored in blocks of 256 rows x 64 columns, columns zero-padded to bf16_pitch(cols): element (r, c) of a
// rows x cols operand sits at ((r / 256) * (pitch / 64) + c / 64) * 16384 + (r % 256) * 64 + c % 64, so that a
// k-slice of a 256-row tile is one 32 KB piece.  bf16_operand_bytes: size of such an array (whole row blocks).
int64_t bf16_pitch(int64_t cols);
int64_t bf16_operand_bytes(int64_t rows, int64_t cols);
// shadow = bf16(W) (round to nearest even), J x D, in that layout.
hipError_t launch_shadow_from_w(const float* W, uint16_t* shadow, int64_t J, int64_t D, hipStream_t stream);
// z(b, j) = sum_d X[b][d] * shadow(j, d);  X bf16 [B][D] row-major, or null if X_aligned (B x D in the operand
// layout, bf16_operand_bytes(B, D)) has already been filled.  The logits are stored tile by tile:
// Z is an array of 256 x 256 tiles (mlr_logits_floats(B, J) floats), tile (b / 256, j / 256) at index
// (j / 256) * ceil(B / 256) + b / 256, rows of 256 floats inside a tile; launch_mlr_softmax(..., blocked = true)
// reads that layout.
hipError_t launch_mlr_forward_bf16(const uint16_t* X, const uint16_t* W_shadow, float* Z, uint16_t* X_aligned,
                                   int64_t B, int64_t J, int64_t D, DeviceInfo& dev, hipStream_t stream);
// W[j][d] -= eta * sum_i U[i][j] * V[i][d];  U bf16 [N][J], V bf16 [N][D], W fp32 [J][D].
// Two steps: launch_apply_bf16_transpose writes U^T and V^T into `workspace`
// (apply_bf16_workspace_bytes, 256-byte aligned), launch_apply_bf16 consumes them.
// W_shadow (nullable): bf16 copy of W, refreshed with the new values.
int64_t mlr_logits_floats(int64_t B, int64_t J);
int64_t apply_bf16_workspace_bytes(int64_t N, int64_t J, int64_t D);
// coef (nullable, device, N floats): V^T is written as bf16(coef[i] * V[i][d]).
// U^T (J x N) and V^T (D x N) are written into the workspace in the operand layout.  V == nullptr: only U^T is
// written; the caller fills V^T at apply_bf16_vt(workspace, N, J) (bf16_operand_bytes(D, N), columns N.. zero).
uint16_t* apply_bf16_vt(void* workspace, int64_t N, int64_t J);
hipError_t launch_apply_bf16_transpose(const uint16_t* U, const uint16_t* V, const float* coef, int64_t N, int64_t J,
                                       int64_t D, void* workspace, hipStream_t stream);
// W_lo (nullable): W is kept as two 16-bit planes, W_shadow the high one (the value rounded
// to bf16) and W_lo the low one; both are updated and the fp32 array W is not touched.
hipError_t launch_apply_bf16(float* W, uint16_t* W_shadow, uint16_t* W_lo, int64_t N, int64_t J, int64_t D, float eta,
                             const void* workspace, DeviceInfo& dev, hipStream_t stream);
// fp32 W[J][D] <-> planes hi (a J x D bf16 operand, bf16_operand_bytes(J, D)) and lo (split_lo_bytes(J, D)
// bytes: 256 x 256 tiles in row-major tile order, one piece per workgroup of the apply):
// the halves of bits + 0x8000; bits = ((hi << 16) | lo) - 0x8000.
int64_t split_lo_bytes(int64_t J, int64_t D);
hipError_t launch_split_from_w(const float* W, uint16_t* hi, uint16_t* lo, int64_t J, int64_t D, hipStream_t stream);
hipError_t launch_w_from_split(const uint16_t* hi, const uint16_t* lo, float* W, int64_t J, int64_t D, hipStream_t stream);

// ---------------------------------------------------------------------------
// CSR rows (indptr int64 [rows + 1], indices int32, values fp32 or bf16).
// ---------------------------------------------------------------------------
// dst[r * row_stride + c * col_stride] = value (* coef[r] if coef) for every stored
// entry (r, c); dst must have been zero-filled.  In the operand layout of the bf16 contractions instead:
// row_stride = -P writes the rows x cols matrix itself (pitch P), col_stride = -P its transpose (cols x rows, pitch P).  Entries outside [0, cols) and row
// ranges outside [0, nnz] are skipped.
hipError_t launch_csr_scatter(const int64_t* indptr, const int32_t* indices, const void* values, bool bf16,
                              const float* coef, void* dst, int64_t rows, int64_t cols, int64_t nnz,
                              int64_t row_stride, int64_t col_stride, hipStream_t stream);
// Logits z(b, j) = sum over the stored entries (d, x) of CSR row b of W(j, d) x, computed over the non-zeros only
// (work proportional to nnz * J; W is read once).  bf16: W is a J x D bf16 operand (blocked layout above), Z the
// tile-blocked logits array of launch_mlr_forward_bf16, values bf16; fp32: W row-major fp32 [J][D], Z row-major
// [B][J], values fp32.  workspace: csr_gather_workspace_bytes(B, D, bf16) bytes, 256-byte aligned (the CSR rows
// re-laid per 64-sample slice and column chunk).  csr_gather_supported: whether this shape can take that route.
bool csr_gather_supported(int64_t B, int64_t J, int64_t D);
int64_t csr_gather_workspace_bytes(int64_t B, int64_t D, bool bf16);
hipError_t launch_csr_forward_gather(const int64_t* indptr, const int32_t* indices, const void* values, bool bf16,
                                     const void* W, float* Z, int64_t B, int64_t J, int64_t D, int64_t nnz,
                                     void* workspace, hipStream_t stream);
// Adds the number of format violations to *bad (device, zeroed by the caller).
hipError_t launch_csr_check(const int64_t* indptr, const int32_t* indices, int64_t rows, int64_t cols, int64_t nnz,
                            unsigned int* bad, hipStream_t stream);

// ---------------------------------------------------------------------------
// Row-wise kernels.
// ---------------------------------------------------------------------------
// U[i][j] = exp(Z[i][j] - max_i) / sum_i - [j == y[i]];  out_bf16 selects the U dtype.
// blocked: Z is the tile-blocked array written by launch_mlr_forward_bf16 instead of a row-major [B][J].
// scratch: mlr_softmax_scratch_bytes(B, J) bytes (8-byte aligned; contents irrelevant) or null; with it, blocked
// logits of long rows are read once, by several workgroups per row that exchange their partial sums through it.
int64_t mlr_softmax_scratch_bytes(int64_t B, int64_t J);
// dev (needed with scratch): CU count for the grid of that kernel, and the polls of a partner's word before a
// workgroup does the partner's part itself.  Every such event is counted on the device (softmax_fallbacks).
hipError_t launch_mlr_softmax(const float* Z, const int32_t* y, void* U, bool out_bf16, int64_t B, int64_t J,
                              hipStream_t stream, bool blocked = false, void* scratch = nullptr,
                              const DeviceInfo* dev = nullptr);
// Partner pairs that workgroups of the one-read softmax computed themselves instead of receiving them, on the
// current device since the library was loaded (copies a device counter: the caller synchronises first).
hipError_t softmax_fallbacks(unsigned long long* count);
// V = X - Y (elementwise, n elements).
// V = X - Y over n floats; *counter (nullable, device) is set to 0 by the same launch.
hipError_t launch_diff(const float* X, const float* Y, float* V, int64_t n, int32_t* counter, hipStream_t stream);
// DML coefficient: d = ||Q_i||^2; c = +2 (sim>0), -2 (sim<=0 and d<margin), else 0; U_i = c Q_i.
// n_active (nullable) must have been zeroed; it is incremented once per active row.
hipError_t launch_dml_scale(const float* Q, const int8_t* sim, float* U, int32_t* n_active,
                            float margin, int64_t B, int64_t K, hipStream_t stream);
// Vs[i][d] = coef[i] * V[i][d] (N rows of D).
hipError_t launch_scale_rows(const float* V, const float* coef, float* Vs, int64_t N, int64_t D, hipStream_t stream);
// W[i] = Z[i] / lambda (n elements; W may alias Z).
hipError_t launch_div_scalar(const float* Z, float* W, float lambda, int64_t n, hipStream_t stream);
// Dual coordinate steps of l2-regularised multiclass logistic regression at the logits
// Zl[B][J] = X W^T: P[B][J] (the samples' dual points in the simplex) is advanced by
// dU = beta (p* - P), p* the coordinate minimiser with c_i = ||x_i||^2 / (lambda n_total).
hipError_t launch_sdca_mlr(const float* Zl, const float* X, float* P, float* dU, int64_t B, int64_t J, int64_t D,
                           float lambda, int64_t n_total, float beta, hipStream_t stream);
// Fill n 32-bit words with `value`.
hipError_t launch_fill_u32(void* p, uint32_t value, int64_t n, hipStream_t stream);
// Row projection / normalisation of W[J][D].
hipError_t launch_prox_rows(float* W, int64_t J, int64_t D, int mode, hipStream_t stream);
// Power iteration on W^T W: writes the norm estimate to *L_out (device).
// scratch: float[D (b) + J (c) + chunks*D (partials) + D (g)] with chunks = power_chunks(J).
int64_t power_chunks(int64_t J);
hipError_t launch_power_iteration(const float* W, int64_t J, int64_t D, int iters, float* scratch,
                                  float* L_out, hipStream_t stream);

}  // namespace sfb
