// fp32 MFMA GEMM family for gfx950 (v_mfma_f32_32x32x2_f32), used by every
// fp32 workload: MLR logits, DML projections, the two ISTA contractions of
// sparse coding, and the reconstruction + application of the SF sum.
//
//   acc[m][n] = sum_k A(m,k) * B(n,k)
//
// Either operand may be k-contiguous ([rows][k], e.g. W[J][D] against the
// feature index) or k-strided ([k][rows], e.g. the SF matrices U[N][J], V[N][D]
// against the SF index), so "U^T V" needs no transposed copy: a k-strided tile
// is kept in LDS as it sits in memory and each MFMA lane picks one float.
//
// Workgroup: 256 threads = 2x2 wavefronts, tile BT x BT x 32 (BT = 64 or 128),
// one LDS stage plus a register prefetch of the next k-slice.
//
// Shapes with few output tiles and a long k (the residual x - W^T a of sparse
// coding: 512 x 1024 over k = 4096; the DML projections) are split along k over
// several workgroups: each writes its partial sums to a scratch buffer and a
// second kernel adds them in a fixed order and applies the epilogue, so results
// stay bit-reproducible (no float atomics).
#include "kernels.h"

namespace sfb {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int NT = 256;
constexpr int BK = 32;
constexpr int KC_PITCH = BK + 4;  // floats; 144-byte rows keep 16-byte reads of 16 rows on distinct banks

template <int BT>
struct TileGeom {
    static constexpr int KS_PITCH = BT + 32;
    static constexpr int KC_FLOATS = BT * KC_PITCH;
    static constexpr int KS_FLOATS = BK * KS_PITCH;
    static constexpr int FLOATS = KC_FLOATS > KS_FLOATS ? KC_FLOATS : KS_FLOATS;
    static constexpr int UNITS = BT * BK / 4;  // float4 units per operand tile
    static constexpr int PER_THREAD = UNITS / NT;
};

struct Params {
    const float* A;
    const float* B;
    float* C;
    const float* aux;
    const float* L_ptr;
    int64_t lda, ldb, ldc;
    int64_t M, N, K;
    float eta, lambda;
    int vecA, vecB;
    int tiles_n;
    int split_k;       // > 1: workgroup z of a tile covers k-slices [z * slabs, (z + 1) * slabs) and writes partial[z]
    int64_t slabs;     // k-slices of BK per split
    float* partial;    // [split_k][M][N]
};

// Global -> registers for one operand tile.  `outer` is the strided index
// (rows for k-contiguous, k for k-strided), `inner` the contiguous one.
template <int BT, bool KS>
__device__ __forceinline__ void fetch_tile(floatx4 (&r)[TileGeom<BT>::PER_THREAD], const float* __restrict__ P,
                                           int64_t ld, int64_t row0, int64_t rows, int64_t k0, int64_t K,
                                           int vec, int tid)
{
    constexpr int INNER4 = KS ? BT / 4 : BK / 4;
#pragma unroll
    for (int i = 0; i < TileGeom<BT>::PER_THREAD; ++i) {
        const int u = tid + NT * i;
        const int o = u / INNER4;
        const int c = (u % INNER4) * 4;
        const int64_t outer = (KS ? k0 : row0) + o;
        const int64_t inner = (KS ? row0 : k0) + c;
        const int64_t outer_end = KS ? K : rows;
        const int64_t inner_end = KS ? rows : K;
        floatx4 v = {0.f, 0.f, 0.f, 0.f};
        if (outer < outer_end) {
            const float* src = P + outer * ld + inner;
            if (vec && inner + 3 < inner_end) {
                v = *reinterpret_cast<const floatx4*>(src);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (inner + e < inner_end) v[e] = src[e];
            }
        }
        r[i] = v;
    }
}

template <int BT, bool KS>
__device__ __forceinline__ void stash_tile(float* lds, const floatx4 (&r)[TileGeom<BT>::PER_THREAD], int tid)
{
    constexpr int INNER4 = KS ? BT / 4 : BK / 4;
    constexpr int PITCH = KS ? TileGeom<BT>::KS_PITCH : KC_PITCH;
#pragma unroll
    for (int i = 0; i < TileGeom<BT>::PER_THREAD; ++i) {
        const int u = tid + NT * i;
        const int o = u / INNER4;
        const int c = (u % INNER4) * 4;
        *reinterpret_cast<floatx4*>(lds + o * PITCH + c) = r[i];
    }
}

// MFMA operand values of one lane for k-group t (8 consecutive k): lane group g
// (lane / 32) owns k = 8t + 4g + e, e = 0..3; the e-th MFMA of the group
// consumes element e from both lane groups, i.e. two distinct k per MFMA.
template <int BT, bool KS, int TILES>
__device__ __forceinline__ void read_frags(float (&f)[TILES][4], const float* lds, int w0, int l32, int g, int t)
{
#pragma unroll
    for (int x = 0; x < TILES; ++x) {
        const int row = w0 + x * 32 + l32;
        if (KS) {
#pragma unroll
            for (int e = 0; e < 4; ++e) f[x][e] = lds[(8 * t + 4 * g + e) * TileGeom<BT>::KS_PITCH + row];
        } else {
            const floatx4 v = *reinterpret_cast<const floatx4*>(lds + row * KC_PITCH + 8 * t + 4 * g);
#pragma unroll
            for (int e = 0; e < 4; ++e) f[x][e] = v[e];
        }
    }
}

template <int EPI>
__device__ __forceinline__ void epilogue_elem(const Params& p, int64_t row, int64_t col, float acc, float invL)
{
    const int64_t idx = row * p.ldc + col;
    if (EPI == EPI_STORE) {
        p.C[idx] = acc;
    } else if (EPI == EPI_RMW) {
        p.C[idx] = p.C[idx] - p.eta * acc;
    } else if (EPI == EPI_RESID) {
        p.C[idx] = p.aux[idx] - acc;
    } else {
        const float t = p.aux[idx] + acc * invL;
        const float th = p.lambda * invL;
        p.C[idx] = t > th ? t - th : (t < -th ? t + th : 0.f);
    }
}

template <int BT, bool A_KS, bool B_KS, int EPI>
__global__ __launch_bounds__(NT) void gemm_f32_kernel(Params p)
{
    constexpr int TM = BT / 64;  // 32x32 MFMA tiles per wave along m (and n)
    __shared__ __attribute__((aligned(16))) float ldsA[TileGeom<BT>::FLOATS];
    __shared__ __attribute__((aligned(16))) float ldsB[TileGeom<BT>::FLOATS];

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int l32 = lane & 31;
    const int g = lane >> 5;
    const int wm0 = (wave >> 1) * (BT / 2);
    const int wn0 = (wave & 1) * (BT / 2);

    const int64_t tile = blockIdx.x;
    const int64_t m0 = (tile / p.tiles_n) * BT;
    const int64_t n0 = (tile % p.tiles_n) * BT;
    const int64_t z = blockIdx.y;

    floatx16 acc[TM][TM];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    floatx4 ra[TileGeom<BT>::PER_THREAD], rb[TileGeom<BT>::PER_THREAD];
    const int64_t nk_all = (p.K + BK - 1) / BK;
    const int64_t k_first = p.split_k > 1 ? z * p.slabs : 0;
    const int64_t nk = p.split_k > 1 ? (k_first + p.slabs < nk_all ? k_first + p.slabs : nk_all) : nk_all;
    if (k_first < nk) {
        fetch_tile<BT, A_KS>(ra, p.A, p.lda, m0, p.M, k_first * BK, p.K, p.vecA, tid);
        fetch_tile<BT, B_KS>(rb, p.B, p.ldb, n0, p.N, k_first * BK, p.K, p.vecB, tid);
    }
    for (int64_t kt = k_first; kt < nk; ++kt) {
        stash_tile<BT, A_KS>(ldsA, ra, tid);
        stash_tile<BT, B_KS>(ldsB, rb, tid);
        __syncthreads();
        if (kt + 1 < nk) {
            fetch_tile<BT, A_KS>(ra, p.A, p.lda, m0, p.M, (kt + 1) * BK, p.K, p.vecA, tid);
            fetch_tile<BT, B_KS>(rb, p.B, p.ldb, n0, p.N, (kt + 1) * BK, p.K, p.vecB, tid);
        }
#pragma unroll
        for (int t = 0; t < BK / 8; ++t) {
            float fa[TM][4], fb[TM][4];
            read_frags<BT, A_KS, TM>(fa, ldsA, wm0, l32, g, t);
            read_frags<BT, B_KS, TM>(fb, ldsB, wn0, l32, g, t);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int b = 0; b < TM; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a][e], fb[b][e], acc[a][b], 0, 0, 0);
        }
        __syncthreads();
    }

    float invL = 0.f;
    if (EPI == EPI_SHRINK) invL = 1.0f / p.L_ptr[0];
    // Accumulator layout of the 32x32 MFMA: register i of lane (g, l32) holds
    // row 8*(i/4) + 4*g + (i%4), column l32.
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b) {
            const int64_t col = n0 + wn0 + b * 32 + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t row = m0 + wm0 + a * 32 + 8 * (i / 4) + 4 * g + (i % 4);
                if (row < p.M && col < p.N) {
                    if (p.split_k > 1)
                        p.partial[(z * p.M + row) * p.N + col] = acc[a][b][i];
                    else
                        epilogue_elem<EPI>(p, row, col, acc[a][b][i], invL);
                }
            }
        }
}

// Sum of the k-splits in index order, then the epilogue.
template <int EPI>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(Params p)
{
    float invL = 0.f;
    if (EPI == EPI_SHRINK) invL = 1.0f / p.L_ptr[0];
    const int64_t total = p.M * p.N, stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
        float sum = p.partial[i];
        for (int z = 1; z < p.split_k; ++z) sum += p.partial[z * total + i];
        epilogue_elem<EPI>(p, i / p.N, i % p.N, sum, invL);
    }
}

template <int BT, bool A_KS, bool B_KS, int EPI>
hipError_t launch_one(Params p, hipStream_t stream)
{
    const int64_t tm = (p.M + BT - 1) / BT, tn = (p.N + BT - 1) / BT;
    p.tiles_n = (int)tn;
    if (tm * tn > 0x7fffffffLL) return hipErrorInvalidValue;
    const unsigned gz = p.split_k > 1 ? (unsigned)p.split_k : 1u;
    hipLaunchKernelGGL((gemm_f32_kernel<BT, A_KS, B_KS, EPI>), dim3((unsigned)(tm * tn), gz), dim3(NT), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.split_k <= 1) return e;
    int64_t g = (p.M * p.N + 255) / 256;
    if (g > 4096) g = 4096;
    hipLaunchKernelGGL((splitk_reduce_kernel<EPI>), dim3((unsigned)g), dim3(256), 0, stream, p);
    return hipGetLastError();
}

template <bool A_KS, bool B_KS, int EPI>
hipError_t launch_sized(Params p, hipStream_t stream)
{
    const int64_t t128 = ((p.M + 127) / 128) * ((p.N + 127) / 128);
    if (t128 >= 256) {
        p.split_k = 1;
        return launch_one<128, A_KS, B_KS, EPI>(p, stream);
    }
    return launch_one<64, A_KS, B_KS, EPI>(p, stream);
}

}  // namespace

// How many ways a contraction is split along k: only when 64 x 64 tiles leave
// most CUs idle and every split still gets at least 8 k-slices.
int gemm_f32_split_k(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0) return 1;
    const int64_t t128 = ((M + 127) / 128) * ((N + 127) / 128);
    if (t128 >= 256) return 1;
    const int64_t tiles = ((M + 63) / 64) * ((N + 63) / 64), nk = (K + BK - 1) / BK;
    if (tiles >= 256) return 1;
    int64_t s = (512 + tiles - 1) / tiles;
    if (s > nk / 8) s = nk / 8;
    if (s > 8) s = 8;
    return s < 2 ? 1 : (int)s;
}

int64_t gemm_f32_partial_bytes(int64_t M, int64_t N, int64_t K)
{
    const int s = gemm_f32_split_k(M, N, K);
    return s > 1 ? (int64_t)s * M * N * 4 : 0;
}

hipError_t launch_gemm_f32(const GemmF32Args& a, hipStream_t stream)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    Params p;
    p.split_k = a.partial ? gemm_f32_split_k(a.M, a.N, a.K) : 1;
    p.partial = a.partial;
    {
        const int64_t nk = (a.K + BK - 1) / BK;
        p.slabs = p.split_k > 1 ? (nk + p.split_k - 1) / p.split_k : nk;
    }
    p.A = a.A; p.B = a.B; p.C = a.C; p.aux = a.aux; p.L_ptr = a.L_ptr;
    p.lda = a.lda; p.ldb = a.ldb; p.ldc = a.ldc;
    p.M = a.M; p.N = a.N; p.K = a.K;
    p.eta = a.eta; p.lambda = a.lambda;
    p.vecA = ((a.lda % 4) == 0 && (reinterpret_cast<uintptr_t>(a.A) % 16) == 0) ? 1 : 0;
    p.vecB = ((a.ldb % 4) == 0 && (reinterpret_cast<uintptr_t>(a.B) % 16) == 0) ? 1 : 0;
    p.tiles_n = 0;
    const bool aks = a.a_kstrided, bks = a.b_kstrided;
    if (!aks && !bks && a.epilogue == EPI_STORE) return launch_sized<false, false, EPI_STORE>(p, stream);
    if (!aks && !bks && a.epilogue == EPI_SHRINK) return launch_sized<false, false, EPI_SHRINK>(p, stream);
    if (!aks && bks && a.epilogue == EPI_RESID) return launch_sized<false, true, EPI_RESID>(p, stream);
    if (aks && bks && a.epilogue == EPI_RMW) return launch_sized<true, true, EPI_RMW>(p, stream);
    return hipErrorInvalidValue;
}

}  // namespace sfb
