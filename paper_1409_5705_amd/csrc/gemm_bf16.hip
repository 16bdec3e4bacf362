// bf16 MFMA kernel (v_mfma_f32_32x32x16_bf16, fp32 accumulate) of the large
// multiclass-logistic path on gfx950, and the small layout kernels around it:
//
//   forward:  Z[b][j]  = sum_d X[b][d] * bf16(W[j][d])          (logits W x, Figure 2 "predict")
//   apply:    W[j][d] -= eta * sum_i U[i][j] * V[i][d]          (SF sum of Section 3)
//
// One kernel serves both: C[m][n] = sum_k A[m][k] * B[n][k], both operands bf16,
// k-contiguous, with 128-byte-aligned rows and k zero-padded to a multiple of 64:
//   forward  A = X copied to an aligned pitch, B = the bf16 working copy of W
//            ("shadow": fp32 master weights + bf16 compute copy, kept current by
//            the apply epilogue), C = Z stored;
//   apply    A = U^T, B = V^T (transpose_bf16_kernel: each tile's operand panel
//            is one contiguous block), C = W read-modify-written in the epilogue
//            (the only pass over W), which also refreshes the shadow.
//
// What the measurements on MI355X dictated:
//   * A wavefront issues at most one instruction every four cycles and the
//     vector-memory path of a CU sustains ~110 outstanding 128-byte requests, so
//     the kernel is bound by requests per flop and by instructions per slice,
//     not by MFMA rate: hence large tiles, aligned bf16 operands only (every
//     request is a whole line), and a loader that runs nothing but loads, a
//     handful of address operations and LDS writes per k-slice.
//   * One-slice-deep prefetch left the MFMA pipe idle behind ~3 us tail
//     latencies: the kernel is persistent and warp-specialised, 512 threads =
//     4 consumer wavefronts (MFMA + epilogue, 128 x 64 or 64 x 128 each) + 4
//     producer wavefronts that keep the loads of two k-slices in flight in
//     registers and run ahead across tile boundaries, so an epilogue overlaps
//     the next tile's loads.  One workgroup barrier per k-slice, LDS
//     double-buffered.  (256 x 256 tiles with 8 consumer wavefronts would halve
//     the requests per flop again but do not fit the 168 registers a wavefront
//     gets at three per SIMD without spilling.)
//   * LDS rows are 128 bytes, the eight 16-byte chunks of a row XOR-swizzled by
//     a function of the row: conflict-free operand reads, no padding.
//   * Workgroup ids are dealt round-robin to the 8 XCDs (one L2 each): the 32
//     workgroups of an XCD walk 32 consecutive tiles of a raster in which tiles
//     sharing operand panels are neighbours.
#include "kernels.h"

#include <type_traits>

namespace sfb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int NUM_XCD = 8;
constexpr int BK = 64;            // k-slice: one 128-byte LDS row of bf16
constexpr int NPROD = 256;        // producer threads (the last four wavefronts)

// Workgroup tile BM x BN; consumer wavefronts in a WM x WN grid, each TM x TN
// MFMA tiles of 32 x 32.  WAVES_PER_SIMD bounds the registers of a wavefront.
template <int BM_, int BN_, int WM_, int WN_>
struct Cfg {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
    static constexpr int NCONS = WM * WN;
    static constexpr int NT = NCONS * 64 + NPROD;
    static constexpr int WAVES_PER_SIMD = NT / 256;
    static constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);
    static constexpr int UA = BM * 8 / NPROD, UB = BN * 8 / NPROD;   // 16-byte chunks per producer thread
    static constexpr int LDS_BYTES = 0x10000 + (BM + BN) * 128;      // stage 1 sits 64 KiB above stage 0
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && (BM + BN) * 128 <= 0x10000 && UA >= 2 && UB >= 2,
                  "tile shape");
};

enum Mode : int { MODE_FWD = 0, MODE_APPLY = 1 };

struct Params {
    const uint16_t* A;  // bf16 [M][lda], lda % 64 == 0, k zero-padded to K
    const uint16_t* B;  // bf16 [N][ldb]
    float* C;           // [M][ldc]
    uint16_t* shadow;   // apply: bf16 copy of C to refresh ([M][ld_shadow]), or null
    int64_t M, N, K;    // K % 64 == 0
    int64_t lda, ldb, ldc, ld_shadow;
    float eta;
    int tiles_m, tiles_n;
    int64_t tiles_total;
    int group_m;        // raster: groups of group_m row-tiles, row-tile index fastest inside a group
    int dbg;            // timing experiments: 2 = skip epilogue, 4 = skip MFMA, 8 = no shadow store
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    floatx2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);  // round to nearest even
    return __builtin_bit_cast(uint32_t, h);
}

// LDS byte offset of the 16-byte chunk c (0..7) of tile row r.  Rows are 128
// bytes, i.e. half of the 64 banks; the chunk slot is c ^ f(r) with
// f(r) = ((r >> 1) ^ (r >> 3)) & 7, so that 16 consecutive rows at one chunk
// index (an MFMA operand read) hit 16 distinct bank groups.
// Two identities keep the per-slice address arithmetic to one XOR:
//   f(r + 32) = f(r) ^ 4, f(r + 64) = f(r): rows 64 apart differ by a constant;
//   chunk (2 ks + g) of row r sits at lds_byte(r, g) ^ (32 ks).
// An LDS stage is [A tile 32 KiB][B tile 32 KiB]; stage 1 is at +64 KiB, so a
// stage flip is an XOR of the base offset with 0x10000.
__device__ __forceinline__ uint32_t lds_byte(int r, int c)
{
    return (uint32_t)(r * 128 + (((c ^ (r >> 1) ^ (r >> 3)) & 7) << 4));
}

template <class C>
struct Slice {  // registers of one k-slice in flight in a producer thread
    u32x4 a[C::UA];
    u32x4 b[C::UB];
};

template <int MODE, class C>
__global__ __launch_bounds__(C::NT, C::WAVES_PER_SIMD) void sf_gemm_kernel(Params p)
{
    constexpr int BM = C::BM, BN = C::BN, NCONS = C::NCONS, TM = C::TM, TN = C::TN;
    extern __shared__ u32x4 smem[];
    uint16_t* lds = reinterpret_cast<uint16_t*>(smem);

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    // the wavefront index as a scalar: the role branch below is then a uniform
    // (scalar) branch, never an exec-masked region around the barriers
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool producer = wave >= NCONS;
    static_assert(C::NT % 256 == 0, "whole wavefronts per SIMD");

    // ---- persistent schedule ------------------------------------------------
    const int64_t x = blockIdx.x % NUM_XCD, wi = blockIdx.x / NUM_XCD, per_xcd = gridDim.x / NUM_XCD;
    const int64_t q8 = p.tiles_total / NUM_XCD, r8 = p.tiles_total % NUM_XCD;
    const int64_t xcd_start = x * q8 + (x < r8 ? x : r8), xcd_cnt = q8 + (x < r8 ? 1 : 0);
    if (wi >= xcd_cnt) return;
    const int64_t n_my = (xcd_cnt - wi + per_xcd - 1) / per_xcd;   // tiles of this workgroup
    const int64_t nk = p.K / BK;
    const int64_t S = n_my * nk;                                    // k-slices of this workgroup, all tiles

    auto tile_origin = [&](int64_t ordinal, int64_t& m0, int64_t& n0) {
        const int64_t L = xcd_start + ordinal * per_xcd + wi;
        const int64_t per_group = (int64_t)p.group_m * p.tiles_n;
        const int64_t grp = L / per_group, r = L % per_group;
        const int64_t rem = p.tiles_m - grp * p.group_m;
        const int64_t gm = rem < p.group_m ? rem : p.group_m;
        m0 = (grp * p.group_m + r % gm) * BM;
        n0 = (r / gm) * BN;
    };

    // One barrier per k-slice step, executed by both roles (1 + 2 * ceil(S / 2)
    // barriers each).  At step s the consumers run the MFMAs of slice s out of
    // LDS stage s & 1 (and the epilogue when the slice ends a tile); the
    // producers move slice s+1 from register set (s+1) & 1 into LDS stage
    // (s+1) & 1 and then issue the loads of slice s+3 into the freed set.  The
    // roles are separate loops so that a wavefront's registers hold either
    // accumulators or slices, never both.
    if (producer) {
        // Every load is unconditional (rows outside the matrix are clamped to the
        // last row: they only feed accumulators that are never stored; k is
        // zero-padded), so the number of loads in flight is a compile-time fact
        // and the wait before staging a slice leaves the next slice's loads
        // outstanding.  Past the last slice the cursor stays on a valid tile and
        // the loads are simply never staged.
        const int ptid = tid - NCONS * 64;
        const int prow = ptid >> 3, pc = ptid & 7;
        const uint32_t pitchA = (uint32_t)p.lda * 2u, pitchB = (uint32_t)p.ldb * 2u;
        Slice<C> sl[2];
        int64_t iss_q = 0, iss_k = 0, iss_m0 = 0, iss_n0 = 0;
        const char* baseA = nullptr;   // address of (row 0, current k-slice) of the tile being loaded
        const char* baseB = nullptr;
        int lastA = 0, lastB = 0;      // last valid row of the tile
        auto enter_tile = [&]() {
            baseA = reinterpret_cast<const char*>(p.A) + iss_m0 * p.lda * 2;
            baseB = reinterpret_cast<const char*>(p.B) + iss_n0 * p.ldb * 2;
            lastA = (int)(p.M - iss_m0 < BM ? p.M - iss_m0 : BM) - 1;
            lastB = (int)(p.N - iss_n0 < BN ? p.N - iss_n0 : BN) - 1;
        };
        auto issue = [&](Slice<C>& s) {
#pragma unroll
            for (int i = 0; i < C::UA; ++i) {
                const int r = prow + 32 * i < lastA ? prow + 32 * i : lastA;
                s.a[i] = *reinterpret_cast<const u32x4*>(baseA + ((uint32_t)r * pitchA + (uint32_t)pc * 16u));
            }
#pragma unroll
            for (int i = 0; i < C::UB; ++i) {
                const int r = prow + 32 * i < lastB ? prow + 32 * i : lastB;
                s.b[i] = *reinterpret_cast<const u32x4*>(baseB + ((uint32_t)r * pitchB + (uint32_t)pc * 16u));
            }
            baseA += BK * 2;
            baseB += BK * 2;
            ++iss_q;
            if (++iss_k == nk) {
                iss_k = 0;
                if (iss_q < S) tile_origin(iss_q / nk, iss_m0, iss_n0);
                enter_tile();
            }
        };
        // LDS write offsets: rows prow + 32 i; even / odd i differ by the constant of
        // the swizzle, the rest is an immediate offset.
        char* const lds_bytes = reinterpret_cast<char*>(lds);
        uint32_t wr0 = lds_byte(prow, pc), wr1 = lds_byte(prow + 32, pc) - 32 * 128;
        auto stash = [&](const Slice<C>& s) {   // into the stage wr0 / wr1 currently point at, then flip them
#pragma unroll
            for (int i = 0; i < C::UA; ++i)
                *reinterpret_cast<u32x4*>(lds_bytes + ((i & 1) ? wr1 : wr0) + i * 32 * 128) = s.a[i];
#pragma unroll
            for (int i = 0; i < C::UB; ++i)
                *reinterpret_cast<u32x4*>(lds_bytes + ((i & 1) ? wr1 : wr0) + i * 32 * 128 + BM * 128) = s.b[i];
            wr0 ^= 0x10000u;
            wr1 ^= 0x10000u;
        };
        tile_origin(0, iss_m0, iss_n0);
        enter_tile();
        issue(sl[0]);
        issue(sl[1]);
        stash(sl[0]);                  // slice 0 -> stage 0
        issue(sl[0]);
        __syncthreads();
        for (int64_t s = 0; s < S; s += 2) {
            stash(sl[1]);              // slice s+1 -> stage 1
            issue(sl[1]);
            __syncthreads();
            stash(sl[0]);              // slice s+2 -> stage 0
            issue(sl[0]);
            __syncthreads();
        }
    } else {
        const int wm0 = (wave / C::WN) * (TM * 32), wn0 = (wave % C::WN) * (TN * 32);
        floatx16 acc[TM][TN];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
        int64_t con_k = 0, con_tile = 0, cur_m0 = 0, cur_n0 = 0;
        tile_origin(0, cur_m0, cur_n0);

        // LDS read offsets of this lane: chunk g of rows wm0 + l32 (+32) of the A
        // tile and wn0 + l32 (+32) of the B tile, in the stage being consumed.
        const char* const lds_bytes = reinterpret_cast<const char*>(lds);
        uint32_t ra0 = lds_byte(wm0 + l32, g), ra1 = lds_byte(wm0 + 32 + l32, g) - 32 * 128;
        uint32_t rb0 = lds_byte(wn0 + l32, g) + BM * 128, rb1 = lds_byte(wn0 + 32 + l32, g) - 32 * 128 + BM * 128;
        auto mfma_slice = [&]() {      // MFMAs of the stage ra / rb point at, then flip them
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                bf16x8 fa[TM], fb[TN];
#pragma unroll
                for (int a = 0; a < TM; ++a)
                    fa[a] = *reinterpret_cast<const bf16x8*>(lds_bytes + (((a & 1) ? ra1 : ra0) ^ (32u * ks)) +
                                                             a * 32 * 128);
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    fb[b] = *reinterpret_cast<const bf16x8*>(lds_bytes + (((b & 1) ? rb1 : rb0) ^ (32u * ks)) +
                                                             b * 32 * 128);
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
            }
        };
        auto flip_stage = [&]() {
            ra0 ^= 0x10000u;
            ra1 ^= 0x10000u;
            rb0 ^= 0x10000u;
            rb1 ^= 0x10000u;
        };

        // Epilogue of one tile.  Register i of lane (g, l32) of a 32x32 MFMA tile
        // is row 8*(i/4) + 4*g + i%4, column l32.  Two column-adjacent tiles are
        // first combined with v_permlane32_swap (upper half of one register <->
        // lower half of the other): afterwards one register holds ONE row across
        // 64 consecutive columns (lane = column), the other the row 4 below.  Every
        // access of C is then 256 contiguous bytes (128 for the bf16 copy) at a
        // uniform row address plus a per-lane column offset.
        static_assert(TN % 2 == 0, "tiles are paired along n");
        // C is addressed through a raw buffer descriptor based at this wave's corner
        // of the tile: row offsets are scalar, the column offset is one register per
        // lane, so no per-row address registers are live while loads are in flight.
        auto make_rsrc = [&](const void* base) {
            const uint64_t a = reinterpret_cast<uint64_t>(base);
            // (the builtin returns a signed int: narrow to 32 unsigned bits before widening)
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
            const uint64_t u = ((uint64_t)hi << 32) | (uint64_t)lo;
            return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(u), 0, 0xffffffff, 0x00020000);
        };
        auto epilogue_tile = [&](int64_t m0, int64_t n0, auto guard_tag) {
            constexpr bool GUARD = decltype(guard_tag)::value;
            const auto crs = make_rsrc(p.C + (m0 + wm0) * p.ldc + n0 + wn0);
            const bool has_shadow = p.shadow && !(p.dbg & 8);
            const auto srs = make_rsrc(has_shadow ? p.shadow + (m0 + wm0) * p.ld_shadow + n0 + wn0 : p.shadow);
            const int64_t rows_left = p.M - (m0 + wm0);
            const uint32_t row_c = (uint32_t)p.ldc * 4u, row_s = (uint32_t)p.ld_shadow * 2u;
            // One block = 32 rows x 64 columns (two column-adjacent MFMA tiles).  The loads of
            // block q+1 are in flight while block q is combined and stored.
            constexpr int NQ = TM * (TN / 2);
            float w[2][32];
            auto load_block = [&](int q, float* dst) {
                const int ta = q / (TN / 2), tp = q % (TN / 2);
                const bool col_ok = !GUARD || (n0 + wn0 + tp * 64 + lane < p.N);
                const uint32_t coff = (uint32_t)(tp * 64 + lane);
#pragma unroll
                for (int e = 0; e < 32; ++e) {
                    const int i = e / 2, dr = ta * 32 + 8 * (i / 4) + (i % 4) + 4 * (e & 1);
                    dst[e] = 0.f;
                    if (col_ok && (!GUARD || dr < rows_left))
                        dst[e] = __uint_as_float(
                            __builtin_amdgcn_raw_buffer_load_b32(crs, coff * 4u, (uint32_t)dr * row_c, 0));
                }
            };
            if (MODE == MODE_APPLY) load_block(0, w[0]);
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int ta = q / (TN / 2), tp = q % (TN / 2);
                if (MODE == MODE_APPLY && q + 1 < NQ) load_block(q + 1, w[(q + 1) & 1]);
                const bool col_ok = !GUARD || (n0 + wn0 + tp * 64 + lane < p.N);
                const uint32_t coff = (uint32_t)(tp * 64 + lane);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    // (element first into a scalar: bit-casting a vector element directly is
                    // miscompiled by this toolchain)
                    const float lo = acc[ta][2 * tp][i], hi = acc[ta][2 * tp + 1][i];
                    const auto sw =
                        __builtin_amdgcn_permlane32_swap(__float_as_uint(lo), __float_as_uint(hi), false, false);
                    const uint32_t s0 = sw[0], s1 = sw[1];
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        const float val = __uint_as_float(half ? s1 : s0);
                        const int dr = ta * 32 + 8 * (i / 4) + (i % 4) + 4 * half;
                        if (col_ok && (!GUARD || dr < rows_left)) {
                            if (MODE == MODE_FWD) {
                                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(val), crs, coff * 4u,
                                                                      (uint32_t)dr * row_c, 0);
                            } else {
                                const float nw = w[q & 1][2 * i + half] - p.eta * val;
                                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(nw), crs, coff * 4u,
                                                                      (uint32_t)dr * row_c, 0);
                                if (has_shadow)
                                    __builtin_amdgcn_raw_buffer_store_b16((uint16_t)(pack_bf16(nw, 0.f) & 0xffffu),
                                                                          srs, coff * 2u, (uint32_t)dr * row_s, 0);
                            }
                        }
                    }
                }
            }
        };
        auto epilogue = [&](int64_t m0, int64_t n0) {
            if ((m0 + BM <= p.M) && (n0 + BN <= p.N))
                epilogue_tile(m0, n0, std::false_type{});
            else
                epilogue_tile(m0, n0, std::true_type{});
        };

        auto consume = [&](int64_t s) {
            if (!(p.dbg & 4)) mfma_slice();
            flip_stage();
            if (++con_k == nk) {
                con_k = 0;
                if (!(p.dbg & 2)) epilogue(cur_m0, cur_n0);
                ++con_tile;
                if (con_tile < n_my) tile_origin(con_tile, cur_m0, cur_n0);
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
            }
        };
        __syncthreads();
        for (int64_t s = 0; s < S; s += 2) {
            consume(s);
            __syncthreads();
            if (s + 1 < S) consume(s + 1);
            __syncthreads();
        }
    }
}

// src[rows_src][cols] (bf16, row-major) -> dst[cols][pitch]; source rows
// rows_src..pitch-1 are taken as zero.  64x64 tiles through LDS, 256 threads.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t* __restrict__ src,
                                                             uint16_t* __restrict__ dst, int64_t rows_src,
                                                             int64_t cols, int64_t pitch)
{
    __shared__ uint16_t tile[64][64 + 2];
    const int64_t c0 = (int64_t)blockIdx.x * 64, k0 = (int64_t)blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < 64; r += 4) {
        const int64_t k = k0 + r, c = c0 + tx;
        tile[r][tx] = (k < rows_src && c < cols) ? src[k * cols + c] : (uint16_t)0;
    }
    __syncthreads();
    for (int r = ty; r < 64; r += 4) {
        const int64_t c = c0 + r, k = k0 + tx;
        if (c < cols && k < pitch) dst[c * pitch + k] = tile[tx][r];
    }
}

// dst[r][0..pitch) = bf16(src[r][0..cols)) followed by zeros; 8 elements a thread.
template <typename SrcT>
__global__ __launch_bounds__(256) void pad_rows_bf16_kernel(const SrcT* __restrict__ src, uint16_t* __restrict__ dst,
                                                            int64_t rows, int64_t cols, int64_t pitch)
{
    const int64_t chunks = pitch / 8;
    const int64_t total = rows * chunks;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int64_t r = idx / chunks, c = (idx % chunks) * 8;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (c < cols) {   // cols % 8 == 0: a chunk is entirely inside or outside
            if constexpr (sizeof(SrcT) == 4) {
                const floatx4 a = *reinterpret_cast<const floatx4*>(src + r * cols + c);
                const floatx4 b = *reinterpret_cast<const floatx4*>(src + r * cols + c + 4);
                v[0] = pack_bf16(a[0], a[1]);
                v[1] = pack_bf16(a[2], a[3]);
                v[2] = pack_bf16(b[0], b[1]);
                v[3] = pack_bf16(b[2], b[3]);
            } else {
                v = *reinterpret_cast<const u32x4*>(src + r * cols + c);
            }
        }
        *reinterpret_cast<u32x4*>(dst + r * pitch + c) = v;
    }
}

int g_forward_dbg = 0;   // timing experiments only: 2 = no epilogue, 4 = no MFMA
int g_apply_dbg = 0;

template <int MODE, class C>
hipError_t launch(Params p, hipStream_t stream)
{
    constexpr int BM = C::BM, BN = C::BN;
    p.tiles_m = (int)((p.M + BM - 1) / BM);
    p.tiles_n = (int)((p.N + BN - 1) / BN);
    p.tiles_total = (int64_t)p.tiles_m * p.tiles_n;
    if (p.group_m <= 0 || p.group_m > p.tiles_m) p.group_m = p.tiles_m;
    // 32-bit in-tile byte offsets in the loaders
    if (p.lda * 2 * BM >= (1LL << 31) || p.ldb * 2 * BN >= (1LL << 31) || p.ldc * 4 * BM >= (1LL << 31))
        return hipErrorInvalidValue;
    if (p.K % BK != 0 || p.lda % BK != 0 || p.ldb % BK != 0) return hipErrorInvalidValue;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sf_gemm_kernel<MODE, C>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    int64_t grid = 256;                      // one persistent workgroup per CU
    if (p.tiles_total < grid) grid = (p.tiles_total + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    hipLaunchKernelGGL((sf_gemm_kernel<MODE, C>), dim3((unsigned)grid), dim3(C::NT), C::LDS_BYTES, stream, p);
    return hipGetLastError();
}

unsigned grid_for(int64_t n)
{
    int64_t g = (n + 255) / 256;
    if (g > 16384) g = 16384;
    return (unsigned)(g < 1 ? 1 : g);
}

}  // namespace

void set_bf16_variant(int forward_variant, int apply_variant)
{
    g_forward_dbg = forward_variant < 0 ? 0 : forward_variant / 100;
    g_apply_dbg = apply_variant < 0 ? 0 : apply_variant / 100;
}

int64_t bf16_pitch(int64_t cols) { return (cols + BK - 1) / BK * BK; }

hipError_t launch_shadow_from_w(const float* W, uint16_t* shadow, int64_t J, int64_t D, hipStream_t stream)
{
    if (J <= 0 || D <= 0) return hipSuccess;
    const int64_t pitch = bf16_pitch(D);
    hipLaunchKernelGGL((pad_rows_bf16_kernel<float>), dim3(grid_for(J * (pitch / 8))), dim3(256), 0, stream, W, shadow,
                       J, D, pitch);
    return hipGetLastError();
}

hipError_t launch_mlr_forward_bf16(const uint16_t* X, const uint16_t* W_shadow, float* Z, uint16_t* X_aligned,
                                   int64_t B, int64_t J, int64_t D, hipStream_t stream)
{
    if (B <= 0 || J <= 0) return hipSuccess;
    const int64_t pitch = bf16_pitch(D);
    hipLaunchKernelGGL((pad_rows_bf16_kernel<uint16_t>), dim3(grid_for(B * (pitch / 8))), dim3(256), 0, stream, X,
                       X_aligned, B, D, pitch);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    Params p = {};
    p.A = X_aligned; p.lda = pitch; p.M = B;
    p.B = W_shadow; p.ldb = pitch; p.N = J;
    p.C = Z; p.ldc = J;
    p.K = pitch;
    p.group_m = 0;               // all batch tiles of one class tile are neighbours (they share the W tile)
    p.dbg = g_forward_dbg;
    return launch<MODE_FWD, Cfg<256, 128, 2, 2>>(p, stream);
}

int64_t apply_bf16_workspace_bytes(int64_t N, int64_t J, int64_t D) { return (J + D) * bf16_pitch(N) * 2; }

hipError_t launch_apply_bf16(float* W, uint16_t* W_shadow, const uint16_t* U, const uint16_t* V, int64_t N, int64_t J,
                             int64_t D, float eta, void* workspace, hipStream_t stream)
{
    if (N <= 0 || J <= 0 || D <= 0) return hipSuccess;
    const int64_t Np = bf16_pitch(N);
    uint16_t* Ut = static_cast<uint16_t*>(workspace);
    uint16_t* Vt = Ut + J * Np;
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)((J + 63) / 64), (unsigned)(Np / 64)), dim3(256), 0,
                       stream, U, Ut, N, J, Np);
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)((D + 63) / 64), (unsigned)(Np / 64)), dim3(256), 0,
                       stream, V, Vt, N, D, Np);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    Params p = {};
    p.A = Ut; p.lda = Np; p.M = J;
    p.B = Vt; p.ldb = Np; p.N = D;
    p.C = W; p.ldc = D;
    p.shadow = W_shadow; p.ld_shadow = bf16_pitch(D);
    p.K = Np;
    p.eta = eta;
    p.group_m = 8;               // 8 row-tiles x 4 column tiles under one L2 at a time
    p.dbg = g_apply_dbg;
    return launch<MODE_APPLY, Cfg<128, 256, 2, 2>>(p, stream);
}

}  // namespace sfb
