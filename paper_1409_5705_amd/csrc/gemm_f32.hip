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

#include <cmath>

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

// ---------------------------------------------------------------------------
// The pipelined kernel: operands whose rows are 16-byte aligned go from global
// memory straight into LDS (global_load_lds_dwordx4, 16 bytes a lane, no staging
// registers), three LDS stages of one k-slice (32 of k) each, one workgroup
// barrier per slice: at slice s the loads of slice s + 1 are in flight, those of
// slice s + 2 are issued right after the barrier into the stage slice s - 1 was
// read from (every wavefront has passed its reads of s - 1 before it arrives at
// the barrier).  256 threads = 2 x 2 wavefronts, tile BM x BN.
//   k-contiguous operand: LDS rows of 32 floats (128 bytes), the eight 16-byte
//     chunks of row r XOR-swizzled by r & 7 (applied on the global side: a lane
//     fetches the chunk that belongs in its slot), so that the 16-byte fragment
//     reads of 8 consecutive rows hit 8 different bank groups;
//   k-strided operand: LDS as in memory, [k][rows]; a fragment is four 4-byte reads.
// Rows past the end of the matrix are clamped (they feed accumulators that are not
// stored).  A last partial k-slice (K % 32 != 0) goes through registers with zero
// fill, like every slice of the plain kernel above.
// ---------------------------------------------------------------------------
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int DL_STAGES = 4;     // LDS stages: the loads of three k-slices are in flight while one is multiplied

struct DlParams {
    Params g;
    int num_xcd;
    int tiles_m;
    int group_m;    // raster: groups of group_m row-tiles, row-tile index fastest inside a group
};

__device__ __forceinline__ void dl_load_16(uint32_t lds_addr, uint64_t gbase, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(gbase) : "memory");
}
__device__ __forceinline__ uint64_t dl_uniform64(uint64_t a)
{
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    return ((uint64_t)hi << 32) | (uint64_t)lo;
}

template <int LX, bool KS, int ROWS_TILE>
__device__ __forceinline__ void dl_lane_offsets(uint32_t (&off)[LX], int wave, int lane, int64_t row0, int64_t rows, int64_t ld)
{
#pragma unroll
    for (int i = 0; i < LX; ++i) {
        if (!KS) {
            const int r = 8 * (LX * wave + i) + (lane >> 3);
            int64_t rr = row0 + r;
            if (rr >= rows) rr = rows - 1;
            off[i] = (uint32_t)((rr - row0) * ld * 4) + (uint32_t)((((lane & 7) ^ (r & 7)) << 4));
        } else {
            const int byte = 1024 * (LX * wave + i) + 16 * lane;
            const int k = byte / (ROWS_TILE * 4);
            int64_t m = row0 + (byte % (ROWS_TILE * 4)) / 4;
            if (m + 4 > rows) m = rows - 4;               // (rows % 4 == 0 and rows >= 4 on this path)
            off[i] = (uint32_t)(k * ld * 4) + (uint32_t)((m - row0) * 4);
        }
    }
}

template <int BM, int BN, bool A_KS, bool B_KS, int EPI>
__global__ __launch_bounds__(NT) void gemm_f32_dl_kernel(DlParams dp)
{
    const Params& p = dp.g;
    constexpr int TMA = BM / 64, TNB = BN / 64;          // 32 x 32 MFMA tiles per wavefront
    constexpr int A_BYTES = BM * BK * 4, B_BYTES = BN * BK * 4, STAGE = A_BYTES + B_BYTES, NS = DL_STAGES;
    constexpr int LA = A_BYTES / 1024 / 4, LB = B_BYTES / 1024 / 4;   // 1 KB loads per wavefront and slice
    extern __shared__ u32x4 dl_smem[];
    char* const lds = reinterpret_cast<char*>(dl_smem);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)dl_smem;

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);

    // tiles: each XCD (one L2) takes a contiguous range of a raster in which consecutive tiles form compact blocks
    // (group_m row-tiles x as many column-tiles): the workgroups of an XCD walk k together, so a line of an operand
    // panel is fetched into that L2 once and found there by the other tiles that share the panel
    const int64_t tiles = (int64_t)gridDim.x;
    int64_t m0, n0;
    {
        const int64_t x = blockIdx.x % dp.num_xcd, wi = blockIdx.x / dp.num_xcd;
        const int64_t q = tiles / dp.num_xcd, r = tiles % dp.num_xcd;
        const int64_t L = x * q + (x < r ? x : r) + wi;
        const int64_t per_group = (int64_t)dp.group_m * p.tiles_n;
        const int64_t grp = L / per_group, rr = L % per_group;
        const int64_t rem = dp.tiles_m - grp * dp.group_m;
        const int64_t gm = rem < dp.group_m ? rem : dp.group_m;
        m0 = (grp * dp.group_m + rr % gm) * BM;
        n0 = (rr / gm) * BN;
    }
    const int64_t z = blockIdx.y;
    const int64_t nk_full = p.K / BK;                     // whole slices
    const int64_t nk_all = (p.K + BK - 1) / BK;
    const int64_t k_first = p.split_k > 1 ? z * p.slabs : 0;
    const int64_t k_end = p.split_k > 1 ? (k_first + p.slabs < nk_all ? k_first + p.slabs : nk_all) : nk_all;
    const int64_t k_end_full = k_end < nk_full ? k_end : nk_full;     // direct loads cover [k_first, k_end_full)

    // ---- loader: per-lane byte offsets within a slice, relative to the operand's base of the slice ----
    // k-contiguous: load i of a wavefront fills LDS rows 8 (LX * wave + i) .. + 7; lane l fills slot l & 7 of row
    //   + (l >> 3), i.e. fetches chunk (l & 7) ^ (row & 7) of that row.
    // k-strided: the slice is BK rows of BM (BN) floats; 1 KB pieces in order.
    uint32_t offA[LA], offB[LB];
    dl_lane_offsets<LA, A_KS, BM>(offA, wave, lane, m0, p.M, p.lda);
    dl_lane_offsets<LB, B_KS, BN>(offB, wave, lane, n0, p.N, p.ldb);
    // base address of the operand's first element of slice kt (may be "before" the tile's clamped rows: offsets are >= 0)
    auto baseA = [&](int64_t kt) {
        return dl_uniform64(reinterpret_cast<uint64_t>(p.A) + (uint64_t)(A_KS ? (kt * BK * p.lda + m0) : (m0 * p.lda + kt * BK)) * 4);
    };
    auto baseB = [&](int64_t kt) {
        return dl_uniform64(reinterpret_cast<uint64_t>(p.B) + (uint64_t)(B_KS ? (kt * BK * p.ldb + n0) : (n0 * p.ldb + kt * BK)) * 4);
    };
    auto issue = [&](int64_t kt, int stage) {            // all loads of slice kt (clamped to the last whole slice)
        if (kt >= k_end_full) kt = k_end_full - 1;
        const uint64_t ga = baseA(kt), gb = baseB(kt);
        const uint32_t dst = lds_base + stage * STAGE;
#pragma unroll
        for (int i = 0; i < LA; ++i) dl_load_16(dst + (LA * wave + i) * 1024u, ga, offA[i]);
#pragma unroll
        for (int i = 0; i < LB; ++i) dl_load_16(dst + A_BYTES + (LB * wave + i) * 1024u, gb, offB[i]);
    };

    floatx16 acc[TMA][TNB];
#pragma unroll
    for (int a = 0; a < TMA; ++a)
#pragma unroll
        for (int b = 0; b < TNB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // one k-slice from stage `st`: 4 groups of 8 k, each 4 MFMAs per tile pair.  The fragments of group t + 1 are
    // read while the MFMAs of group t run (two register sets), a few reads after each MFMA; the order is pinned,
    // otherwise the compiler puts each 4-byte read of a k-strided operand right before the MFMA that uses it and
    // the wavefront waits out the LDS latency with an idle matrix pipe.
    constexpr int NRA = A_KS ? TMA * 4 : TMA, NRB = B_KS ? TNB * 4 : TNB, NR = NRA + NRB;   // LDS reads per group
    struct Frag {
        float a[TMA][4], b[TNB][4];
    };
    auto read_op = [&](const char* sa, const char* sb, int t, int q, Frag& f) {    // q: compile-time after unrolling
        if (q < NRA) {
            const int x = A_KS ? q / 4 : q, r = wm0 + 32 * x + l32;
            if (A_KS) {
                const int e = q % 4;
                f.a[x][e] = *reinterpret_cast<const float*>(sa + (8 * t + 4 * g + e) * (BM * 4) + r * 4);
            } else {
                const floatx4 v = *reinterpret_cast<const floatx4*>(sa + r * 128 + (((2 * t + g) ^ (r & 7)) << 4));
#pragma unroll
                for (int e = 0; e < 4; ++e) f.a[x][e] = v[e];
            }
        } else {
            const int qq = q - NRA, x = B_KS ? qq / 4 : qq, r = wn0 + 32 * x + l32;
            if (B_KS) {
                const int e = qq % 4;
                f.b[x][e] = *reinterpret_cast<const float*>(sb + (8 * t + 4 * g + e) * (BN * 4) + r * 4);
            } else {
                const floatx4 v = *reinterpret_cast<const floatx4*>(sb + r * 128 + (((2 * t + g) ^ (r & 7)) << 4));
#pragma unroll
                for (int e = 0; e < 4; ++e) f.b[x][e] = v[e];
            }
        }
    };
    Frag f[2];
    constexpr int NM = 4 * TMA * TNB;                                  // MFMAs per group
    // groups t0, t0 + 1 of the slice in stage `st`; the reads interleaved with the MFMAs of a group fetch the next
    // group, which for the slice's last group is group 0 of the slice in stage `st_next`
    auto compute_half = [&](int st, int st_next, int t0) {
        const char* sa = lds + st * STAGE;
        const char* sb = sa + A_BYTES;
        const char* na = lds + st_next * STAGE;
        const char* nb = na + A_BYTES;
#pragma unroll
        for (int t = t0; t < t0 + 2; ++t) {
            const bool last = t + 1 == BK / 8;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                const int e = i / (TMA * TNB), a = (i / TNB) % TMA, b = i % TNB;
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(f[t & 1].a[a][e], f[t & 1].b[b][e], acc[a][b], 0, 0, 0);
#pragma unroll
                for (int q = i * NR / NM; q < (i + 1) * NR / NM; ++q)
                    read_op(last ? na : sa, last ? nb : sb, last ? 0 : t + 1, q, f[(t + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    auto compute = [&](int st) {      // a whole slice on its own (the partial last slice)
        const char* sa = lds + st * STAGE;
        const char* sb = sa + A_BYTES;
#pragma unroll
        for (int q = 0; q < NR; ++q) read_op(sa, sb, 0, q, f[0]);
        compute_half(st, st, 0);
        compute_half(st, st, 2);
    };

    // The values the epilogue combines with (W, the samples, the previous codes): requested during the last
    // k-slice, so that their latency runs under its MFMAs.
    float old[TMA][TNB][16];
    auto load_old = [&]() {
        if (EPI == EPI_STORE || p.split_k > 1) return;
#pragma unroll
        for (int a = 0; a < TMA; ++a)
#pragma unroll
            for (int b = 0; b < TNB; ++b) {
                const int64_t col = n0 + wn0 + b * 32 + l32, row_first = m0 + wm0 + a * 32 + 4 * g;
                const float* src = (EPI == EPI_RMW ? p.C : p.aux) + row_first * p.ldc + col;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int dr = 8 * (i / 4) + (i % 4);
                    old[a][b][i] = (col < p.N && row_first + dr < p.M) ? src[(int64_t)dr * p.ldc] : 0.f;
                }
            }
    };
    const bool tail = k_end > k_end_full;
    if (k_first < k_end_full) {
        // Slice s lives in stage s % NS.  In the middle of slice s every wavefront waits until slice s + 1 has landed
        // and meets the others: after that barrier the stage of slice s - 1 is free (the loads of slice s + NS - 1
        // go there) and the second half of slice s can fetch the first fragments of slice s + 1, so that the MFMA
        // pipe does not drain at a slice boundary.  Loads complete in order: "slice s + 1 has landed" = at most the
        // loads of the NS - 3 slices after it are outstanding.
#pragma unroll
        for (int i = 0; i < NS - 1; ++i) issue(k_first + i, i);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * (LA + LB)) : "memory");
        __syncthreads();
        {
            const char* sa = lds;
            const char* sb = sa + A_BYTES;
#pragma unroll
            for (int q = 0; q < NR; ++q) read_op(sa, sb, 0, q, f[0]);
        }
        int st = 0;
        for (int64_t kt = k_first; kt < k_end_full; ++kt) {
            const int st_next = st + 1 == NS ? 0 : st + 1;
            compute_half(st, st_next, 0);
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 3) * (LA + LB)) : "memory");
            __syncthreads();
            issue(kt + NS - 1, st >= 1 ? st - 1 : NS - 1);    // into the stage slice kt - 1 was read from
            if (kt + 1 == k_end_full && !tail) load_old();
            compute_half(st, st_next, 2);
            st = st_next;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no direct load in flight when LDS is reused or released
        __syncthreads();
    }
    if (k_end > k_end_full) {
        // the partial last slice: through registers, zero-filled past K, into stage 0 in the layouts above
        const int64_t k0 = nk_full * BK;
        constexpr int PA = BM * BK / 4 / NT, PB = BN * BK / 4 / NT;
        auto stage_partial = [&](char* dst, const float* P, int64_t ld, bool ks, int rows_tile, int64_t row0, int64_t rows,
                                 int per) {
            for (int i = 0; i < per; ++i) {
                const int u = tid + NT * i;
                floatx4 v = {0.f, 0.f, 0.f, 0.f};
                if (!ks) {
                    const int r = u / 8, c = u % 8;           // row, 16-byte chunk
                    const int64_t rr = row0 + r, k = k0 + 4 * c;
                    if (rr < rows) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (k + e < p.K) v[e] = P[rr * ld + k + e];
                    }
                    *reinterpret_cast<floatx4*>(dst + r * 128 + ((c ^ (r & 7)) << 4)) = v;
                } else {
                    const int per_row = rows_tile / 4, kk = u / per_row, m4 = (u % per_row) * 4;
                    const int64_t k = k0 + kk;
                    if (k < p.K) {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (row0 + m4 + e < rows) v[e] = P[k * ld + row0 + m4 + e];
                    }
                    *reinterpret_cast<floatx4*>(dst + kk * (rows_tile * 4) + m4 * 4) = v;
                }
            }
        };
        stage_partial(lds, p.A, p.lda, A_KS, BM, m0, p.M, PA);
        stage_partial(lds + A_BYTES, p.B, p.ldb, B_KS, BN, n0, p.N, PB);
        __syncthreads();
        load_old();
        compute(0);
    } else if (k_first >= k_end_full) {
        load_old();
    }

    // Epilogue.  Register i of lane (g, l32) of MFMA tile (a, b) is row 32 a + 8 (i / 4) + 4 g + i % 4, column
    // 32 b + l32 of the wavefront's block: for fixed (a, b, i) a half-wave covers 128 contiguous bytes of one row.
    // The 16 values a tile combines with (W, the samples, the previous codes) are all requested before the first
    // is used.
    float invL = 0.f, th = 0.f;
    if (EPI == EPI_SHRINK) {
        invL = 1.0f / p.L_ptr[0];
        th = p.lambda * invL;
    }
#pragma unroll
    for (int a = 0; a < TMA; ++a)
#pragma unroll
        for (int b = 0; b < TNB; ++b) {
            const int64_t col = n0 + wn0 + b * 32 + l32;
            const int64_t row_first = m0 + wm0 + a * 32 + 4 * g;
            const bool col_ok = col < p.N;
            if (p.split_k > 1) {
                float* dst = p.partial + (z * p.M + row_first) * p.N + col;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int dr = 8 * (i / 4) + (i % 4);
                    if (col_ok && row_first + dr < p.M) dst[(int64_t)dr * p.N] = acc[a][b][i];
                }
                continue;
            }
            float* dst = p.C + row_first * p.ldc + col;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int dr = 8 * (i / 4) + (i % 4);
                float v = acc[a][b][i];
                if (EPI == EPI_RMW) {
                    v = old[a][b][i] - p.eta * v;
                } else if (EPI == EPI_RESID) {
                    v = old[a][b][i] - v;
                } else if (EPI == EPI_SHRINK) {
                    const float t = old[a][b][i] + v * invL;
                    v = t > th ? t - th : (t < -th ? t + th : 0.f);
                }
                if (col_ok && row_first + dr < p.M) dst[(int64_t)dr * p.ldc] = v;
            }
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

// ---- the pipelined kernel: tile shape and k-split by a small cost model ----
struct DlPlan {
    int bm, bn, split;
};

// Estimated duration (seconds) of a contraction as `rounds` of one workgroup per CU, each walking its k-slices at
// the fp32 MFMA rate of a CU times an efficiency that falls with the tile (smaller tiles move more operand bytes per
// flop through the L2), plus, when k is split, the second pass that adds the partial sums.
static DlPlan dl_plan(int64_t M, int64_t N, int64_t K, int cus, int max_split)
{
    static const int shapes[3][2] = {{128, 128}, {128, 64}, {64, 64}};
    static const double eff[3] = {0.85, 0.80, 0.70};
    const int64_t nk = (K + BK - 1) / BK;
    DlPlan best = {64, 64, 1};
    double best_t = 1e30;
    for (int sh = 0; sh < 3; ++sh) {
        const int bm = shapes[sh][0], bn = shapes[sh][1];
        const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
        for (int s = 1; s <= max_split; ++s) {
            if (s > 1 && nk / s < 8) break;
            const int64_t slabs = (nk + s - 1) / s;
            const double rounds = (double)((tiles * s + cus - 1) / cus);
            const double slice = 2.0 * bm * bn * BK / (157.3e12 / 256.0 * eff[sh]);      // one workgroup, one k-slice
            double t = rounds * ((double)slabs * slice + 4e-6);                             // + pipeline fill and epilogue of a round
            if (s > 1) t += 3e-6 + (double)(s + 1) * (double)M * (double)N * 4.0 / 3e12;
            if (t < best_t) {
                best_t = t;
                best = DlPlan{bm, bn, s};
            }
        }
    }
    return best;
}

template <int BM, int BN, bool A_KS, bool B_KS, int EPI>
hipError_t launch_dl_one(Params p, DeviceInfo& dev, int slot, hipStream_t stream)
{
    const int64_t tm = (p.M + BM - 1) / BM, tn = (p.N + BN - 1) / BN;
    p.tiles_n = (int)tn;
    if (tm * tn > 0x7fffffffLL) return hipErrorInvalidValue;
    constexpr int LDS = DL_STAGES * (BM + BN) * BK * 4;
    if (!dev.gemm_f32_lds_set[slot]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_f32_dl_kernel<BM, BN, A_KS, B_KS, EPI>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        dev.gemm_f32_lds_set[slot] = true;
    }
    DlParams dp;
    dp.g = p;
    dp.num_xcd = dev.xcds > 0 ? dev.xcds : 1;
    dp.tiles_m = (int)tm;
    {   // block of tiles per XCD with the fewest operand rows: group_m ~ sqrt(tiles per XCD * BN / BM)
        const double per_xcd = (double)(tm * tn) / dp.num_xcd;
        int gm = (int)(sqrt(per_xcd * BN / BM) + 0.5);
        if (gm < 1) gm = 1;
        if (gm > tm) gm = (int)tm;
        dp.group_m = gm;
    }
    const unsigned gz = p.split_k > 1 ? (unsigned)p.split_k : 1u;
    hipLaunchKernelGGL((gemm_f32_dl_kernel<BM, BN, A_KS, B_KS, EPI>), dim3((unsigned)(tm * tn), gz), dim3(NT), LDS, stream, dp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.split_k <= 1) return e;
    int64_t g = (p.M * p.N + 255) / 256;
    if (g > 4096) g = 4096;
    hipLaunchKernelGGL((splitk_reduce_kernel<EPI>), dim3((unsigned)g), dim3(256), 0, stream, p);
    return hipGetLastError();
}

template <bool A_KS, bool B_KS, int EPI>
hipError_t launch_dl(Params p, DeviceInfo& dev, int combo, int max_split, hipStream_t stream)
{
    const DlPlan plan = dl_plan(p.M, p.N, p.K, dev.cus > 0 ? dev.cus : 256, max_split);
    p.split_k = plan.split;
    const int64_t nk = (p.K + BK - 1) / BK;
    p.slabs = plan.split > 1 ? (nk + plan.split - 1) / plan.split : nk;
    if (plan.bm == 128 && plan.bn == 128) return launch_dl_one<128, 128, A_KS, B_KS, EPI>(p, dev, combo * 3 + 0, stream);
    if (plan.bm == 128) return launch_dl_one<128, 64, A_KS, B_KS, EPI>(p, dev, combo * 3 + 1, stream);
    return launch_dl_one<64, 64, A_KS, B_KS, EPI>(p, dev, combo * 3 + 2, stream);
}

}  // namespace

// How many ways a contraction may be split along k at most: only when there are few output tiles and every
// split still gets at least 8 k-slices.  The scratch is sized for this bound; the launcher picks the split.
static int gemm_f32_max_split(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0) return 1;
    const int64_t t128 = ((M + 127) / 128) * ((N + 127) / 128), nk = (K + BK - 1) / BK;
    if (t128 >= 256) return 1;
    int64_t s = nk / 8;
    if (s > 8) s = 8;
    return s < 2 ? 1 : (int)s;
}

// The plain kernel's split: only when 64 x 64 tiles leave most CUs idle.
int gemm_f32_split_k(int64_t M, int64_t N, int64_t K)
{
    const int max_split = gemm_f32_max_split(M, N, K);
    if (max_split <= 1) return 1;
    const int64_t tiles = ((M + 63) / 64) * ((N + 63) / 64);
    if (tiles >= 256) return 1;
    int64_t s = (512 + tiles - 1) / tiles;
    if (s > max_split) s = max_split;
    return s < 2 ? 1 : (int)s;
}

int64_t gemm_f32_partial_bytes(int64_t M, int64_t N, int64_t K)
{
    const int s = gemm_f32_max_split(M, N, K);
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
    // the pipelined kernel: 16-byte aligned operand rows, at least one whole k-slice, 32-bit in-tile offsets
    const bool dl = a.dev && p.vecA && p.vecB && a.K >= BK && (!aks || a.M % 4 == 0) && (!bks || a.N % 4 == 0) &&
                    a.lda * 4 * 128 < (1LL << 31) && a.ldb * 4 * 128 < (1LL << 31);
    if (dl) {
        const int max_split = a.partial ? gemm_f32_max_split(a.M, a.N, a.K) : 1;
        if (!aks && !bks && a.epilogue == EPI_STORE) return launch_dl<false, false, EPI_STORE>(p, *a.dev, 0, max_split, stream);
        if (!aks && !bks && a.epilogue == EPI_SHRINK) return launch_dl<false, false, EPI_SHRINK>(p, *a.dev, 1, max_split, stream);
        if (!aks && bks && a.epilogue == EPI_RESID) return launch_dl<false, true, EPI_RESID>(p, *a.dev, 2, max_split, stream);
        if (aks && bks && a.epilogue == EPI_RMW) return launch_dl<true, true, EPI_RMW>(p, *a.dev, 3, max_split, stream);
        return hipErrorInvalidValue;
    }
    if (!aks && !bks && a.epilogue == EPI_STORE) return launch_sized<false, false, EPI_STORE>(p, stream);
    if (!aks && !bks && a.epilogue == EPI_SHRINK) return launch_sized<false, false, EPI_SHRINK>(p, stream);
    if (!aks && bks && a.epilogue == EPI_RESID) return launch_sized<false, true, EPI_RESID>(p, stream);
    if (aks && bks && a.epilogue == EPI_RMW) return launch_sized<true, true, EPI_RMW>(p, stream);
    return hipErrorInvalidValue;
}

}  // namespace sfb
