// bf16 MFMA kernels (v_mfma_f32_32x32x16_bf16, fp32 accumulate) of the large
// multiclass-logistic path on gfx950:
//
//   forward:  Z[b][j]  = sum_d X[b][d] * bf16(W[j][d])          (logits W x, Figure 2 "predict")
//   apply:    W[j][d] -= eta * sum_i U[i][j] * V[i][d]          (SF sum of Section 3)
//
// One kernel template serves both.  C[m][n] = sum_k A[m][k] * B[n][k] with both
// operands k-contiguous in memory:
//   forward  A = X (bf16), B = W (fp32 in HBM, rounded to bf16 in registers on
//            the way to LDS: no bf16 copy of the 13 GB matrix exists), C = Z stored;
//   apply    A = U^T, B = V^T (bf16, made by transpose_bf16_kernel: each tile's
//            operand panel is then one contiguous, line-aligned block), C = W
//            read-modify-written in the epilogue, the only pass over W.
//
// Structure (what the measurements asked for: the MFMA pipe sat idle behind
// one-slice-deep prefetches whose tail latency is ~3 us under load):
//   * persistent workgroups, 512 threads = 4 consumer + 4 producer wavefronts
//     (one of each per SIMD);
//   * producers keep the global loads of two k-slices in flight in registers,
//     convert and write the slice after next into a double-buffered LDS stage;
//     they run ahead across tile boundaries, so a tile's epilogue overlaps the
//     loads of the next tile;
//   * consumers only read LDS and issue MFMAs (128 x 64 or 64 x 128 per wave),
//     then run the epilogue;
//   * one workgroup barrier per k-slice;
//   * LDS rows are 128 bytes, the eight 16-byte chunks of a row XOR-swizzled by a
//     function of the row: conflict-free operand reads and writes, no padding;
//   * the workgroup -> tile schedule is XCD-aware (ids are dealt round-robin to
//     the 8 XCDs): the 32 workgroups of an XCD walk 32 consecutive tiles of a
//     raster in which tiles sharing operand panels are neighbours.
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
constexpr int BK = 64;          // k-slice, bf16 elements (one 128-byte LDS row)
constexpr int NT = 512;         // threads per workgroup
constexpr int NPROD = 256;      // producer threads (wavefronts 4..7)

enum Mode : int { MODE_FWD = 0, MODE_APPLY = 1 };

struct Params {
    const uint16_t* A;  // bf16 [M][lda]
    const void* B;      // forward: float [N][ldb]; apply: bf16 [N][ldb]
    float* C;           // [M][ldc]
    int64_t M, N, K;
    int64_t lda, ldb, ldc;
    float eta;
    int tiles_m, tiles_n;
    int64_t tiles_total;
    int group_m;        // raster: groups of group_m row-tiles, row-tile index fastest inside a group
    int dbg;            // timing experiments: 2 = skip epilogue, 4 = skip MFMA
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    floatx2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);  // round to nearest even
    return __builtin_bit_cast(uint32_t, h);
}

// LDS offset (in bf16 elements) of the 16-byte chunk c (0..7) of tile row r.
// Rows are 128 bytes, i.e. half of the 64 banks; the chunk slot is c ^ f(r) with
// f(r) = ((r >> 1) ^ (r >> 3)) & 7, so that 16 consecutive rows at one chunk
// index (an MFMA operand read) hit 16 distinct bank groups.
__device__ __forceinline__ int lds_off(int r, int c) { return r * 64 + (((c ^ (r >> 1) ^ (r >> 3)) & 7) << 3); }

template <int MODE, int BM_, int BN_>
struct Geom {
    static constexpr int BM = BM_, BN = BN_;
    static constexpr bool B_F32 = (MODE == MODE_FWD);
    static constexpr int NB = B_F32 ? 2 : 1;             // 16-byte loads per 8-element chunk of B
    static constexpr int WM = 2, WN = 2;                 // consumer wave grid
    static constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);
    static constexpr int UA = BM * 8 / NPROD;            // 16-byte chunks of the A tile per producer thread
    static constexpr int UB = BN * 8 / NPROD;            // 8-element chunks of the B tile per producer thread
    static constexpr int STAGE = (BM + BN) * BK;         // bf16 elements per LDS stage
    static constexpr int LDS_BYTES = 2 * STAGE * 2;
    static_assert(BM % 64 == 0 && BN % 64 == 0 && (BM * 8) % NPROD == 0 && (BN * 8) % NPROD == 0, "tile shape");
};

// Registers of one k-slice in flight in a producer thread.
template <bool F32> struct BChunk { u32x4 v[1]; };
template <> struct BChunk<true> { floatx4 v[2]; };
template <class G>
struct Slice {
    u32x4 a[G::UA];
    BChunk<G::B_F32> b[G::UB];
    uint32_t mask;   // bit i: chunk i of A is inside the matrix; bit 16 + i: chunk i of B
};

template <int MODE, int BM, int BN>
__global__ __launch_bounds__(NT, 2) void sf_gemm_kernel(Params p)
{
    using G = Geom<MODE, BM, BN>;
    extern __shared__ u32x4 smem[];
    uint16_t* lds = reinterpret_cast<uint16_t*>(smem);

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
    // the wavefront index as a scalar: the role branch below is then a uniform
    // (scalar) branch, never an exec-masked region around the barriers
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool producer = wave >= 4;
    const int ptid = tid - NPROD;

    // ---- persistent schedule ------------------------------------------------
    const int64_t x = blockIdx.x % NUM_XCD, wi = blockIdx.x / NUM_XCD, per_xcd = gridDim.x / NUM_XCD;
    const int64_t q8 = p.tiles_total / NUM_XCD, r8 = p.tiles_total % NUM_XCD;
    const int64_t xcd_start = x * q8 + (x < r8 ? x : r8), xcd_cnt = q8 + (x < r8 ? 1 : 0);
    if (wi >= xcd_cnt) return;
    const int64_t n_my = (xcd_cnt - wi + per_xcd - 1) / per_xcd;   // tiles of this workgroup
    const int64_t nk = (p.K + BK - 1) / BK;
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

    // ---- producer state -------------------------------------------------------
    // Every load of a slice is unconditional (rows outside the matrix and k past
    // the end are clamped to a valid address and zeroed through a mask when the
    // slice is staged), so the number of loads in flight is a compile-time fact
    // and the wait before staging a slice leaves the loads of the next slice
    // outstanding.  Past the last slice the state stays on a valid tile and the
    // loads are simply never staged.
    // A wavefront issues at most one instruction every four cycles, so the
    // per-slice instruction count of a producer is what bounds the kernel: an
    // address is a uniform 64-bit base (advanced by one k-slice per step) plus a
    // 32-bit per-thread byte offset computed once per tile (the host checks that
    // a tile spans less than 2 GiB), and the common case (interior tile, full
    // k-slice) runs nothing but loads, conversions and LDS writes.
    Slice<G> sl[2];
    bool sl_plain[2] = {true, true};   // slice needs no masking (interior tile, full k-slice)
    int64_t iss_q = 0;                 // next slice to issue loads for
    int64_t iss_k = 0;                 // its k-slice index inside its tile
    int64_t iss_m0 = 0, iss_n0 = 0;    // its tile origin
    const int prow = ptid >> 3, pc8 = (ptid & 7) * 8;
    constexpr int A_ESZ = 2, B_ESZ = G::B_F32 ? 4 : 2;
    const uint32_t pitchA = (uint32_t)p.lda * A_ESZ, pitchB = (uint32_t)p.ldb * B_ESZ;
    uint32_t offA[G::UA], offB[G::UB];  // byte offsets of this thread's chunks from the tile's (row 0, k0)
    uint32_t row_mask = 0;              // bit i: row of A chunk i inside the matrix; bit 16 + i: same for B
    bool tile_interior = true;
    const char* baseA = nullptr;        // address of (row 0, current k-slice) of the tile being loaded
    const char* baseB = nullptr;
    const bool k_has_tail = (p.K % BK) != 0;
    auto enter_tile = [&]() {           // per-tile bases, offsets and row masks
        baseA = reinterpret_cast<const char*>(p.A) + iss_m0 * p.lda * A_ESZ;
        baseB = reinterpret_cast<const char*>(p.B) + iss_n0 * p.ldb * B_ESZ;
        const int availA = (int)(p.M - iss_m0 < BM ? p.M - iss_m0 : BM);
        const int availB = (int)(p.N - iss_n0 < BN ? p.N - iss_n0 : BN);
        tile_interior = availA == BM && availB == BN;
        row_mask = 0;
#pragma unroll
        for (int i = 0; i < G::UA; ++i) {
            const int row = prow + 32 * i;
            const uint32_t r = row < availA ? (uint32_t)row : (uint32_t)(availA - 1);
            offA[i] = r * pitchA + pc8 * A_ESZ;
            row_mask |= (row < availA ? 1u : 0u) << i;
        }
#pragma unroll
        for (int i = 0; i < G::UB; ++i) {
            const int row = prow + 32 * i;
            const uint32_t r = row < availB ? (uint32_t)row : (uint32_t)(availB - 1);
            offB[i] = r * pitchB + pc8 * B_ESZ;
            row_mask |= (row < availB ? 1u : 0u) << (16 + i);
        }
    };
    if (producer) {
        tile_origin(0, iss_m0, iss_n0);
        enter_tile();
    }

    auto issue = [&](Slice<G>& s, bool& plain) {    // loads of slice iss_q into s, then advance
        const bool tail = k_has_tail && iss_k == nk - 1;
        if (__builtin_expect(!tail, 1)) {
#pragma unroll
            for (int i = 0; i < G::UA; ++i) s.a[i] = *reinterpret_cast<const u32x4*>(baseA + offA[i]);
#pragma unroll
            for (int i = 0; i < G::UB; ++i) {
                const char* src = baseB + offB[i];
                if constexpr (G::B_F32) {
                    s.b[i].v[0] = *reinterpret_cast<const floatx4*>(src);
                    s.b[i].v[1] = *reinterpret_cast<const floatx4*>(src + 16);
                } else {
                    s.b[i].v[0] = *reinterpret_cast<const u32x4*>(src);
                }
            }
            s.mask = row_mask;
            plain = tile_interior;
        } else {
            // partial last k-slice: chunks past the end re-read chunk 0 of their row and are masked off
            const bool k_ok = iss_k * BK + pc8 < p.K;
            const uint32_t backA = k_ok ? 0u : (uint32_t)(pc8 * A_ESZ), backB = k_ok ? 0u : (uint32_t)(pc8 * B_ESZ);
#pragma unroll
            for (int i = 0; i < G::UA; ++i) s.a[i] = *reinterpret_cast<const u32x4*>(baseA + (offA[i] - backA));
#pragma unroll
            for (int i = 0; i < G::UB; ++i) {
                const char* src = baseB + (offB[i] - backB);
                if constexpr (G::B_F32) {
                    s.b[i].v[0] = *reinterpret_cast<const floatx4*>(src);
                    s.b[i].v[1] = *reinterpret_cast<const floatx4*>(src + 16);
                } else {
                    s.b[i].v[0] = *reinterpret_cast<const u32x4*>(src);
                }
            }
            s.mask = k_ok ? row_mask : 0u;
            plain = false;
        }
        baseA += BK * A_ESZ;
        baseB += BK * B_ESZ;
        ++iss_q;
        if (++iss_k == nk) {
            iss_k = 0;
            if (iss_q < S) tile_origin(iss_q / nk, iss_m0, iss_n0);
            enter_tile();       // past the end: back to k = 0 of the last tile (valid addresses, never staged)
        }
    };
    auto stash = [&](const Slice<G>& s, bool plain, uint16_t* stage) {   // registers -> LDS stage (A tile, B tile)
        uint16_t* ldsA = stage;
        uint16_t* ldsB = stage + BM * BK;
        const int c = ptid & 7;
        if (__builtin_expect(plain, 1)) {
#pragma unroll
            for (int i = 0; i < G::UA; ++i)
                *reinterpret_cast<u32x4*>(ldsA + lds_off(prow + 32 * i, c)) = s.a[i];
#pragma unroll
            for (int i = 0; i < G::UB; ++i) {
                u32x4 v;
                if constexpr (G::B_F32) {
                    const floatx4 v0 = s.b[i].v[0], v1 = s.b[i].v[1];
                    v[0] = pack_bf16(v0[0], v0[1]);
                    v[1] = pack_bf16(v0[2], v0[3]);
                    v[2] = pack_bf16(v1[0], v1[1]);
                    v[3] = pack_bf16(v1[2], v1[3]);
                } else {
                    v = s.b[i].v[0];
                }
                *reinterpret_cast<u32x4*>(ldsB + lds_off(prow + 32 * i, c)) = v;
            }
        } else {
            const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < G::UA; ++i)
                *reinterpret_cast<u32x4*>(ldsA + lds_off(prow + 32 * i, c)) = ((s.mask >> i) & 1u) ? s.a[i] : zero;
#pragma unroll
            for (int i = 0; i < G::UB; ++i) {
                u32x4 v;
                if constexpr (G::B_F32) {
                    const floatx4 v0 = s.b[i].v[0], v1 = s.b[i].v[1];
                    v[0] = pack_bf16(v0[0], v0[1]);
                    v[1] = pack_bf16(v0[2], v0[3]);
                    v[2] = pack_bf16(v1[0], v1[1]);
                    v[3] = pack_bf16(v1[2], v1[3]);
                } else {
                    v = s.b[i].v[0];
                }
                *reinterpret_cast<u32x4*>(ldsB + lds_off(prow + 32 * i, c)) = ((s.mask >> (16 + i)) & 1u) ? v : zero;
            }
        }
    };

    // ---- consumer state -------------------------------------------------------
    const int wm0 = ((wave >> 1) & 1) * (G::TM * 32), wn0 = (wave & 1) * (G::TN * 32);
    floatx16 acc[G::TM][G::TN];
#pragma unroll
    for (int a = 0; a < G::TM; ++a)
#pragma unroll
        for (int b = 0; b < G::TN; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
    int64_t con_k = 0, con_tile = 0;

    auto mfma_slice = [&](const uint16_t* stage) {
        const uint16_t* ldsA = stage;
        const uint16_t* ldsB = stage + BM * BK;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[G::TM], fb[G::TN];
#pragma unroll
            for (int a = 0; a < G::TM; ++a)
                fa[a] = *reinterpret_cast<const bf16x8*>(ldsA + lds_off(wm0 + a * 32 + l32, ks * 2 + g));
#pragma unroll
            for (int b = 0; b < G::TN; ++b)
                fb[b] = *reinterpret_cast<const bf16x8*>(ldsB + lds_off(wn0 + b * 32 + l32, ks * 2 + g));
#pragma unroll
            for (int a = 0; a < G::TM; ++a)
#pragma unroll
                for (int b = 0; b < G::TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }
    };

    // Epilogue of one tile.  Register i of lane (g, l32) of a 32x32 MFMA tile is
    // row 8*(i/4) + 4*g + i%4, column l32: a wavefront access covers two
    // 128-byte row segments of C.
    auto epilogue = [&](int64_t m0, int64_t n0) {
        constexpr int T = G::TM * G::TN;
        const bool interior = (m0 + BM <= p.M) && (n0 + BN <= p.N);
        float* const cbase = p.C + (m0 + wm0 + 4 * g) * p.ldc + n0 + wn0 + l32;
        if (MODE == MODE_FWD) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                float* q = cbase + (int64_t)((t / G::TN) * 32) * p.ldc + (t % G::TN) * 32;
                const int64_t row0 = m0 + wm0 + 4 * g + (t / G::TN) * 32, col = n0 + wn0 + (t % G::TN) * 32 + l32;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int dr = 8 * (i / 4) + (i % 4);
                    if (interior || (row0 + dr < p.M && col < p.N))
                        q[(int64_t)dr * p.ldc] = acc[t / G::TN][t % G::TN][i];
                }
            }
        } else if (interior) {
            // read-modify-write, one MFMA tile at a time; the loads of the next
            // tile are issued before the stores of the current one
            float wv[2][16];
            auto load_tile = [&](int t, float (&dst)[16]) {
                const float* q = cbase + (int64_t)((t / G::TN) * 32) * p.ldc + (t % G::TN) * 32;
#pragma unroll
                for (int i = 0; i < 16; ++i) dst[i] = q[(int64_t)(8 * (i / 4) + (i % 4)) * p.ldc];
            };
            load_tile(0, wv[0]);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                if (t + 1 < T) load_tile(t + 1, wv[(t + 1) & 1]);
                float* q = cbase + (int64_t)((t / G::TN) * 32) * p.ldc + (t % G::TN) * 32;
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    q[(int64_t)(8 * (i / 4) + (i % 4)) * p.ldc] = wv[t & 1][i] - p.eta * acc[t / G::TN][t % G::TN][i];
            }
        } else {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                float* q = cbase + (int64_t)((t / G::TN) * 32) * p.ldc + (t % G::TN) * 32;
                const int64_t row0 = m0 + wm0 + 4 * g + (t / G::TN) * 32, col = n0 + wn0 + (t % G::TN) * 32 + l32;
                float wv[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int dr = 8 * (i / 4) + (i % 4);
                    wv[i] = 0.f;
                    if (row0 + dr < p.M && col < p.N) wv[i] = q[(int64_t)dr * p.ldc];
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int dr = 8 * (i / 4) + (i % 4);
                    if (row0 + dr < p.M && col < p.N)
                        q[(int64_t)dr * p.ldc] = wv[i] - p.eta * acc[t / G::TN][t % G::TN][i];
                }
            }
        }
    };

    // Step s (after the prologue's barrier): consumers run the MFMAs of slice s
    // out of LDS stage s & 1 (and the epilogue when the slice ends a tile);
    // producers move slice s+1 from register set (s+1) & 1 into LDS stage
    // (s+1) & 1 and then issue the loads of slice s+3 into the freed set.  One
    // barrier per step, executed by both roles (the two loops run the same
    // number of barriers, 1 + 2 * ceil(S / 2)).  The roles are kept in separate loops so that
    // a wavefront's registers hold either accumulators or slices, never both.
    if (producer) {
        // slices 0 and 1 in flight, slice 0 staged, slice 2 in flight
        issue(sl[0], sl_plain[0]);
        issue(sl[1], sl_plain[1]);
        stash(sl[0], sl_plain[0], lds);
        issue(sl[0], sl_plain[0]);
        __syncthreads();
        // Both half-steps always run (a slice past the end is staged into the
        // stage nobody reads): a body without conditionals lets the compiler
        // keep exact counts of the loads in flight.
        for (int64_t s = 0; s < S; s += 2) {
            stash(sl[1], sl_plain[1], lds + G::STAGE);
            issue(sl[1], sl_plain[1]);
            __syncthreads();
            stash(sl[0], sl_plain[0], lds);
            issue(sl[0], sl_plain[0]);
            __syncthreads();
        }
    } else {
        // L2 prefetch.  The consumers' vector-memory counter is idle during the
        // k-loop, so they touch (one dword per 128-byte line, value discarded) the
        // lines the workgroup will need from HBM a few microseconds later:
        //   forward: the fp32 W slice PF_AHEAD steps ahead of the producers' loads
        //            (every W line comes from HBM exactly once; without this each
        //            slice waits out an HBM round trip);
        //   apply:   the W tile of the epilogue, during the last steps of its k-loop.
        // The loads are inline asm writing one never-read register that stays live
        // to the end: the compiler's own vmcnt waits can only get stricter by them.
        uint32_t pf_sink = 0;
        auto touch = [&](const char* base, uint32_t off) {
            const char* addr = base + off;
            asm volatile("global_load_dword %0, %1, off" : "+v"(pf_sink) : "v"(addr) : "memory");
        };
        constexpr int PF_AHEAD = 8;
        constexpr int B_ESZ = G::B_F32 ? 4 : 2;
        const uint32_t pitchB = (uint32_t)p.ldb * B_ESZ;
        // forward cursor: slice pf_q = (tile pf_q / nk, k-slice pf_k)
        int64_t pf_q = PF_AHEAD < S ? PF_AHEAD : S, pf_k = 0, pf_n0 = 0;
        uint32_t pf_off = 0;
        auto pf_enter_tile = [&]() {
            int64_t m0;
            tile_origin(pf_q / nk, m0, pf_n0);
            const int availB = (int)(p.N - pf_n0 < BN ? p.N - pf_n0 : BN);
            const int row = wave * 32 + (lane >> 1);      // BN = 128: 4 wavefronts x 32 rows, 2 lines a row
            const uint32_t r = row < availB ? (uint32_t)row : (uint32_t)(availB - 1);
            pf_off = r * pitchB;
        };
        if (MODE == MODE_FWD && pf_q < S) {
            pf_k = pf_q % nk;
            pf_enter_tile();
        }
        // apply: origin of the tile being accumulated
        int64_t cur_m0 = 0, cur_n0 = 0;
        constexpr int PF_STEPS = BM * BN / 8192;          // steps to touch a C tile, 256 lines a step
        if (MODE == MODE_APPLY) tile_origin(0, cur_m0, cur_n0);

        auto consume = [&](int64_t s) {
            if (MODE == MODE_FWD) {
                if (false && pf_q < S && BN == 128) {   // measured: costs more L2 requests than it saves latency
                    const int64_t slice_bytes = (p.K - pf_k * BK < BK ? p.K - pf_k * BK : BK) * B_ESZ;
                    const uint32_t koff = ((lane & 1) * 128 < slice_bytes) ? (lane & 1) * 128 : 0;
                    touch(reinterpret_cast<const char*>(p.B) + (pf_n0 * p.ldb + pf_k * BK) * B_ESZ, pf_off + koff);
                    ++pf_q;
                    if (++pf_k == nk) {
                        pf_k = 0;
                        if (pf_q < S) pf_enter_tile();
                    }
                }
            } else if (nk >= PF_STEPS && con_k >= nk - PF_STEPS) {
                constexpr int LPR = BN / 32;                // 128-byte lines per row of the C tile
                const int u = ((int)(con_k - (nk - PF_STEPS)) * 4 + wave) * 64 + lane;
                int row = u / LPR, line = u % LPR;
                if (cur_m0 + row >= p.M) row = 0;
                if (cur_n0 + line * 32 >= p.N) line = 0;
                touch(reinterpret_cast<const char*>(p.C) + (cur_m0 * p.ldc + cur_n0) * 4,
                      (uint32_t)row * (uint32_t)p.ldc * 4u + (uint32_t)line * 128u);
            }
            if (!(p.dbg & 4)) mfma_slice(lds + (s & 1) * G::STAGE);
            if (++con_k == nk) {
                con_k = 0;
                if (!(p.dbg & 2)) {
                    int64_t m0, n0;
                    tile_origin(con_tile, m0, n0);
                    epilogue(m0, n0);
                }
                ++con_tile;
                if (MODE == MODE_APPLY && con_tile < n_my) tile_origin(con_tile, cur_m0, cur_n0);
#pragma unroll
                for (int a = 0; a < G::TM; ++a)
#pragma unroll
                    for (int b = 0; b < G::TN; ++b)
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
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        asm volatile("" ::"v"(pf_sink));
    }
}

// U[N][cols] (bf16, row-major) -> Ut[cols][Npad]; rows N..Npad-1 of the source
// are taken as zero.  64x64 tiles through LDS, 256 threads.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t* __restrict__ src,
                                                             uint16_t* __restrict__ dst, int64_t N, int64_t cols,
                                                             int64_t Npad)
{
    __shared__ uint16_t tile[64][64 + 2];
    const int64_t c0 = (int64_t)blockIdx.x * 64, k0 = (int64_t)blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
    for (int r = ty; r < 64; r += 4) {
        const int64_t k = k0 + r, c = c0 + tx;
        tile[r][tx] = (k < N && c < cols) ? src[k * cols + c] : (uint16_t)0;
    }
    __syncthreads();
#pragma unroll
    for (int r = ty; r < 64; r += 4) {
        const int64_t c = c0 + r, k = k0 + tx;
        if (c < cols && k < Npad) dst[c * Npad + k] = tile[tx][r];
    }
}

int g_forward_dbg = 0;   // timing experiments only: 2 = no epilogue, 4 = no MFMA
int g_apply_dbg = 0;
int g_forward_variant = -1, g_apply_variant = -1;

template <int MODE, int BM, int BN>
hipError_t launch(Params p, hipStream_t stream)
{
    using G = Geom<MODE, BM, BN>;
    p.tiles_m = (int)((p.M + BM - 1) / BM);
    p.tiles_n = (int)((p.N + BN - 1) / BN);
    p.tiles_total = (int64_t)p.tiles_m * p.tiles_n;
    if (p.group_m <= 0 || p.group_m > p.tiles_m) p.group_m = p.tiles_m;
    // 32-bit in-tile byte offsets in the loaders and the prefetcher
    if (p.lda * 2 * BM >= (1LL << 31) || p.ldb * (G::B_F32 ? 4 : 2) * BN >= (1LL << 31) ||
        p.ldc * 4 * BM >= (1LL << 31))
        return hipErrorInvalidValue;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sf_gemm_kernel<MODE, BM, BN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    int64_t grid = 256;                      // one persistent workgroup per CU
    if (p.tiles_total < grid) grid = (p.tiles_total + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    hipLaunchKernelGGL((sf_gemm_kernel<MODE, BM, BN>), dim3((unsigned)grid), dim3(NT), G::LDS_BYTES, stream, p);
    return hipGetLastError();
}

}  // namespace

void set_bf16_variant(int forward_variant, int apply_variant)
{
    g_forward_variant = forward_variant < 0 ? -1 : forward_variant % 100;
    g_apply_variant = apply_variant < 0 ? -1 : apply_variant % 100;
    g_forward_dbg = forward_variant < 0 ? 0 : forward_variant / 100;
    g_apply_dbg = apply_variant < 0 ? 0 : apply_variant / 100;
}

hipError_t launch_mlr_forward_bf16(const uint16_t* X, const float* W, float* Z, int64_t B, int64_t J, int64_t D,
                                   hipStream_t stream)
{
    if (B <= 0 || J <= 0) return hipSuccess;
    Params p = {};
    p.A = X; p.lda = D; p.M = B;
    p.B = W; p.ldb = D; p.N = J;
    p.C = Z; p.ldc = J;
    p.K = D;
    p.group_m = 0;               // all batch tiles of one class tile are neighbours (they share the W tile)
    p.dbg = g_forward_dbg;
    return launch<MODE_FWD, 256, 128>(p, stream);
}

int64_t apply_bf16_workspace_bytes(int64_t N, int64_t J, int64_t D)
{
    const int64_t Npad = (N + BK - 1) / BK * BK;
    return (J + D) * Npad * 2;
}

hipError_t launch_apply_bf16(float* W, const uint16_t* U, const uint16_t* V, int64_t N, int64_t J, int64_t D,
                             float eta, void* workspace, hipStream_t stream)
{
    if (N <= 0 || J <= 0 || D <= 0) return hipSuccess;
    const int64_t Npad = (N + BK - 1) / BK * BK;
    uint16_t* Ut = static_cast<uint16_t*>(workspace);
    uint16_t* Vt = Ut + J * Npad;
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)((J + 63) / 64), (unsigned)(Npad / 64)), dim3(256), 0,
                       stream, U, Ut, N, J, Npad);
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)((D + 63) / 64), (unsigned)(Npad / 64)), dim3(256), 0,
                       stream, V, Vt, N, D, Npad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    Params p = {};
    p.A = Ut; p.lda = Npad; p.M = J;
    p.B = Vt; p.ldb = Npad; p.N = D;
    p.C = W; p.ldc = D;
    p.K = Npad;
    p.eta = eta;
    p.group_m = 8;               // 8 row-tiles x 4 column tiles under one L2 at a time
    p.dbg = g_apply_dbg;
    switch (g_apply_variant) {
        case 1: return launch<MODE_APPLY, 256, 128>(p, stream);
        default: return launch<MODE_APPLY, 128, 256>(p, stream);
    }
}

}  // namespace sfb
