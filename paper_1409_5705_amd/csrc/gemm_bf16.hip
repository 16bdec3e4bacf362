// bf16 MFMA kernels (v_mfma_f32_32x32x16_bf16, fp32 accumulate) of the large
// multiclass-logistic path on gfx950:
//
//   forward:  Z[b][j]  = sum_d X[b][d] * bf16(W[j][d])          (logits W x, Figure 2 "predict")
//   apply:    W[j][d] -= eta * sum_i U[i][j] * V[i][d]          (SF sum of Section 3)
//
// Both stage BM x BK and BN x BK bf16 tiles in LDS as [row][k] (k contiguous,
// 16 bytes of padding per row) and differ only in how a tile gets there:
//   forward  X: straight 16-byte copies;  W: fp32 in HBM, rounded to bf16 (RNE)
//            in registers on the way in, so no bf16 copy of the 13 GB matrix exists;
//   apply    U, V: the contraction index (the SF index) is the strided one in
//            memory, so each thread loads an 8(k) x 8(col) block with eight
//            coalesced 16-byte loads, transposes it in registers and writes
//            eight 16-byte [col][k] rows.
// The apply epilogue is the only pass over W: read, subtract eta*acc, write.
#include "kernels.h"

namespace sfb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int NUM_XCD = 8;

template <int BM_, int BN_, int BK_, int WM_, int WN_>
struct Cfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
    static constexpr int NT = 64 * WM * WN;
    static constexpr int TM = BM / (WM * 32);  // 32x32 MFMA tiles per wave along m
    static constexpr int TN = BN / (WN * 32);
    static constexpr int PITCH = BK + 8;       // bf16 elements per LDS row
    static constexpr int LDS_BYTES = (BM + BN) * PITCH * 2;
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && BK % 16 == 0, "tile shape");
};

// Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2).
// Map them so that each XCD walks a contiguous range of logical tiles: tiles
// that share operand panels then run at the same time on the same L2.
__device__ __forceinline__ int64_t xcd_contiguous(int64_t id, int64_t total)
{
    const int64_t x = id % NUM_XCD, local = id / NUM_XCD;
    const int64_t q = total / NUM_XCD, r = total % NUM_XCD;
    return x * q + (x < r ? x : r) + local;
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    floatx2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);  // round to nearest even
    return __builtin_bit_cast(uint32_t, h);
}

// One BK-deep MFMA pass over the LDS tiles.
template <class C>
__device__ __forceinline__ void mfma_tile(floatx16 (&acc)[C::TM][C::TN], const uint16_t* ldsA, const uint16_t* ldsB,
                                          int wm0, int wn0, int l32, int g)
{
#pragma unroll
    for (int ks = 0; ks < C::BK / 16; ++ks) {
        bf16x8 fa[C::TM], fb[C::TN];
#pragma unroll
        for (int x = 0; x < C::TM; ++x)
            fa[x] = *reinterpret_cast<const bf16x8*>(ldsA + (wm0 + x * 32 + l32) * C::PITCH + ks * 16 + g * 8);
#pragma unroll
        for (int y = 0; y < C::TN; ++y)
            fb[y] = *reinterpret_cast<const bf16x8*>(ldsB + (wn0 + y * 32 + l32) * C::PITCH + ks * 16 + g * 8);
#pragma unroll
        for (int x = 0; x < C::TM; ++x)
#pragma unroll
            for (int y = 0; y < C::TN; ++y)
                acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[x], fb[y], acc[x][y], 0, 0, 0);
    }
}

// ---------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------
template <class C>
__global__ __launch_bounds__(C::NT) void mlr_forward_bf16_kernel(const uint16_t* __restrict__ X,
                                                                  const float* __restrict__ W, float* __restrict__ Z,
                                                                  int64_t B, int64_t J, int64_t D, int64_t tiles_b,
                                                                  int64_t tiles_total)
{
    extern __shared__ u32x4 smem[];
    uint16_t* ldsA = reinterpret_cast<uint16_t*>(smem);
    uint16_t* ldsB = ldsA + C::BM * C::PITCH;
    constexpr int CH = C::BK / 8;               // 8-element k chunks per row
    constexpr int UA = C::BM * CH / C::NT;      // chunks per thread, X tile
    constexpr int UB = C::BN * CH / C::NT;      // chunks per thread, W tile
    static_assert(C::BM * CH % C::NT == 0 && C::BN * CH % C::NT == 0, "loader split");

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    const int wm0 = (wave / C::WN) * (C::TM * 32), wn0 = (wave % C::WN) * (C::TN * 32);
    const int64_t t = xcd_contiguous(blockIdx.x, tiles_total);
    const int64_t m0 = (t % tiles_b) * C::BM;   // sample index
    const int64_t n0 = (t / tiles_b) * C::BN;   // class index

    floatx16 acc[C::TM][C::TN];
#pragma unroll
    for (int x = 0; x < C::TM; ++x)
#pragma unroll
        for (int y = 0; y < C::TN; ++y)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[x][y][i] = 0.f;

    u32x4 ra[UA];
    floatx4 rb[UB][2];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < UA; ++i) {
            const int u = tid + C::NT * i, row = u / CH, c = (u % CH) * 8;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (m0 + row < B && k0 + c < D)
                v = *reinterpret_cast<const u32x4*>(X + (m0 + row) * D + k0 + c);
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < UB; ++i) {
            const int u = tid + C::NT * i, row = u / CH, c = (u % CH) * 8;
            floatx4 v0 = {0.f, 0.f, 0.f, 0.f}, v1 = v0;
            if (n0 + row < J && k0 + c < D) {
                const float* src = W + (n0 + row) * D + k0 + c;
                v0 = *reinterpret_cast<const floatx4*>(src);
                v1 = *reinterpret_cast<const floatx4*>(src + 4);
            }
            rb[i][0] = v0;
            rb[i][1] = v1;
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < UA; ++i) {
            const int u = tid + C::NT * i, row = u / CH, c = (u % CH) * 8;
            *reinterpret_cast<u32x4*>(ldsA + row * C::PITCH + c) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < UB; ++i) {
            const int u = tid + C::NT * i, row = u / CH, c = (u % CH) * 8;
            u32x4 v;
            v[0] = pack_bf16(rb[i][0][0], rb[i][0][1]);
            v[1] = pack_bf16(rb[i][0][2], rb[i][0][3]);
            v[2] = pack_bf16(rb[i][1][0], rb[i][1][1]);
            v[3] = pack_bf16(rb[i][1][2], rb[i][1][3]);
            *reinterpret_cast<u32x4*>(ldsB + row * C::PITCH + c) = v;
        }
    };

    const int64_t nk = (D + C::BK - 1) / C::BK;
    fetch(0);
    for (int64_t kt = 0; kt < nk; ++kt) {
        stash();
        __syncthreads();
        if (kt + 1 < nk) fetch((kt + 1) * C::BK);
        mfma_tile<C>(acc, ldsA, ldsB, wm0, wn0, l32, g);
        __syncthreads();
    }

#pragma unroll
    for (int x = 0; x < C::TM; ++x)
#pragma unroll
        for (int y = 0; y < C::TN; ++y) {
            const int64_t col = n0 + wn0 + y * 32 + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t row = m0 + wm0 + x * 32 + 8 * (i / 4) + 4 * g + (i % 4);
                if (row < B && col < J) Z[row * J + col] = acc[x][y][i];
            }
        }
}

// ---------------------------------------------------------------------------
// apply
// ---------------------------------------------------------------------------
// 8x8 bf16 transpose in registers: r[k] holds columns 0..7 of row k (two per
// dword); o[c] receives rows 0..7 of column c.
__device__ __forceinline__ void transpose8x8_bf16(const u32x4 (&r)[8], u32x4 (&o)[8])
{
#pragma unroll
    for (int c = 0; c < 8; ++c) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t lo = r[2 * q][c / 2], hi = r[2 * q + 1][c / 2];
            o[c][q] = (c & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
        }
    }
}

template <class C>
__global__ __launch_bounds__(C::NT) void apply_bf16_kernel(float* __restrict__ W, const uint16_t* __restrict__ U,
                                                            const uint16_t* __restrict__ V, int64_t N, int64_t J,
                                                            int64_t D, float eta, int64_t tiles_j, int64_t tiles_d,
                                                            int64_t tiles_total, int group_j)
{
    extern __shared__ u32x4 smem[];
    uint16_t* ldsA = reinterpret_cast<uint16_t*>(smem);
    uint16_t* ldsB = ldsA + C::BM * C::PITCH;
    constexpr int RG = C::BK / 8;                 // 8-row groups along k
    constexpr int NA = RG * (C::BM / 8);          // 8x8 blocks in the U tile
    constexpr int NB = RG * (C::BN / 8);          // 8x8 blocks in the V tile
    constexpr int PB = (NA + NB) / C::NT;         // blocks per thread
    static_assert((NA + NB) % C::NT == 0 && NA % 64 == 0, "loader split");

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    const int wm0 = (wave / C::WN) * (C::TM * 32), wn0 = (wave % C::WN) * (C::TN * 32);

    // Raster: groups of `group_j` row-tiles of W; inside a group the row-tile
    // index runs fastest, so concurrently resident workgroups share V panels
    // and the group's U panels stay in L2 for the whole sweep over D.
    const int64_t t = xcd_contiguous(blockIdx.x, tiles_total);
    const int64_t per_group = (int64_t)group_j * tiles_d;
    const int64_t grp = t / per_group, r = t % per_group;
    const int64_t rem_j = tiles_j - grp * group_j;
    const int64_t gj = rem_j < group_j ? rem_j : group_j;
    const int64_t m0 = (grp * group_j + r % gj) * C::BM;  // row of W (class index j)
    const int64_t n0 = (r / gj) * C::BN;                  // column of W (feature index d)

    floatx16 acc[C::TM][C::TN];
#pragma unroll
    for (int x = 0; x < C::TM; ++x)
#pragma unroll
        for (int y = 0; y < C::TN; ++y)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[x][y][i] = 0.f;

    u32x4 rg[PB][8];
    auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            int v = tid + C::NT * i;
            const bool isA = v < NA;
            if (!isA) v -= NA;
            const int cols8 = isA ? C::BM / 8 : C::BN / 8;
            const int cg = v % cols8, kg = v / cols8;
            const uint16_t* P = isA ? U : V;
            const int64_t ld = isA ? J : D;
            const int64_t c0 = (isA ? m0 : n0) + cg * 8;
            const bool col_ok = c0 < ld;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int64_t k = k0 + kg * 8 + q;
                u32x4 x = {0u, 0u, 0u, 0u};
                if (col_ok && k < N) x = *reinterpret_cast<const u32x4*>(P + k * ld + c0);
                rg[i][q] = x;
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            int v = tid + C::NT * i;
            const bool isA = v < NA;
            if (!isA) v -= NA;
            const int cols8 = isA ? C::BM / 8 : C::BN / 8;
            const int cg = v % cols8, kg = v / cols8;
            uint16_t* dst = (isA ? ldsA : ldsB) + (cg * 8) * C::PITCH + kg * 8;
            u32x4 o[8];
            transpose8x8_bf16(rg[i], o);
#pragma unroll
            for (int c = 0; c < 8; ++c) *reinterpret_cast<u32x4*>(dst + c * C::PITCH) = o[c];
        }
    };

    const int64_t nk = (N + C::BK - 1) / C::BK;
    fetch(0);
    for (int64_t kt = 0; kt < nk; ++kt) {
        stash();
        __syncthreads();
        if (kt + 1 < nk) fetch((kt + 1) * C::BK);
        mfma_tile<C>(acc, ldsA, ldsB, wm0, wn0, l32, g);
        __syncthreads();
    }

#pragma unroll
    for (int x = 0; x < C::TM; ++x)
#pragma unroll
        for (int y = 0; y < C::TN; ++y) {
            const int64_t col = n0 + wn0 + y * 32 + l32;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t row = m0 + wm0 + x * 32 + 8 * (i / 4) + 4 * g + (i % 4);
                if (row < J && col < D) {
                    float* w = W + row * D + col;
                    *w = *w - eta * acc[x][y][i];
                }
            }
        }
}

int g_forward_variant = -1;
int g_apply_variant = -1;

template <class C>
hipError_t launch_forward(const uint16_t* X, const float* W, float* Z, int64_t B, int64_t J, int64_t D,
                          hipStream_t stream)
{
    const int64_t tb = (B + C::BM - 1) / C::BM, tj = (J + C::BN - 1) / C::BN;
    const int64_t total = tb * tj;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;
    static bool attr_done = false;
    if (!attr_done && C::LDS_BYTES > 65536) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&mlr_forward_bf16_kernel<C>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL((mlr_forward_bf16_kernel<C>), dim3((unsigned)total), dim3(C::NT), C::LDS_BYTES, stream, X, W,
                       Z, B, J, D, tb, total);
    return hipGetLastError();
}

template <class C>
hipError_t launch_apply(float* W, const uint16_t* U, const uint16_t* V, int64_t N, int64_t J, int64_t D, float eta,
                        int group_j, hipStream_t stream)
{
    const int64_t tj = (J + C::BM - 1) / C::BM, td = (D + C::BN - 1) / C::BN;
    const int64_t total = tj * td;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;
    static bool attr_done = false;
    if (!attr_done && C::LDS_BYTES > 65536) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&apply_bf16_kernel<C>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL((apply_bf16_kernel<C>), dim3((unsigned)total), dim3(C::NT), C::LDS_BYTES, stream, W, U, V, N,
                       J, D, eta, tj, td, total, group_j);
    return hipGetLastError();
}

}  // namespace

void set_bf16_variant(int forward_variant, int apply_variant)
{
    g_forward_variant = forward_variant;
    g_apply_variant = apply_variant;
}

hipError_t launch_mlr_forward_bf16(const uint16_t* X, const float* W, float* Z, int64_t B, int64_t J, int64_t D,
                                   hipStream_t stream)
{
    if (B <= 0 || J <= 0) return hipSuccess;
    switch (g_forward_variant) {
        default:
            return launch_forward<Cfg<128, 128, 64, 2, 2>>(X, W, Z, B, J, D, stream);
    }
}

hipError_t launch_apply_bf16(float* W, const uint16_t* U, const uint16_t* V, int64_t N, int64_t J, int64_t D,
                             float eta, hipStream_t stream)
{
    if (N <= 0 || J <= 0 || D <= 0) return hipSuccess;
    switch (g_apply_variant) {
        default:
            return launch_apply<Cfg<128, 128, 64, 2, 2>>(W, U, V, N, J, D, eta, 8, stream);
    }
}

}  // namespace sfb
