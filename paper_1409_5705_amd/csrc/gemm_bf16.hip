// bf16 MFMA kernel (v_mfma_f32_16x16x32_bf16, fp32 accumulate) of the large
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
//   * The vector-memory path of a CU sustains ~110 outstanding 128-byte requests
//     and a wavefront issues at most one instruction every four cycles, so the
//     kernel must be lean in requests and instructions per flop.
//     Hence the largest tile the register file holds, 256 x 256 per workgroup of
//     four wavefronts (one per SIMD, 128 x 128 = 256 accumulator registers
//     each), aligned bf16 operands only (every request is a whole line), and
//     operand tiles that go from global memory straight into LDS
//     (global_load_lds_dwordx4: no staging registers, no LDS write
//     instructions, 16 load instructions per wavefront and k-slice).
//   * The matrix pipes run at the clock the chip grants, and that clock falls with
//     the bits that toggle in them: on operands that change, the 16x16x32 form of
//     the MFMA keeps a higher clock than the 32x32x16 form for the same fragment
//     bytes from LDS (register-only loops: 1.92 against 1.78 PFLOP/s).  A wavefront's
//     128 x 128 block is therefore 8 x 8 tiles of 16 x 16, 64 MFMAs per 32 of k.
//   * LDS rows are 128 bytes, the eight 16-byte chunks of a row XOR-swizzled by
//     a function of the row: conflict-free operand reads, no padding.  A direct
//     load writes 64 lanes x 16 bytes = 8 consecutive LDS rows; the swizzle is
//     applied on the global side (each lane fetches the chunk that belongs in
//     its slot).
//   * Two LDS stages of 64 KiB, a slice being two k-steps of 32.  The loads of
//     slice s+2 may start as soon as every wavefront has read the last fragments
//     of slice s (after its first k-step: the second step's fragments are read
//     under the first step's MFMAs) and must have landed three quarters into slice
//     s+1; they are spread over the second half of slice s, one per four MFMAs (a
//     burst of loads blocks the wavefront in the memory-issue stage while the MFMA
//     pipe runs dry; loads issued later have too little time left).  Fragments are
//     double-buffered in registers across the barriers, so the MFMA pipe
//     does not drain at a slice boundary.  Two workgroup barriers per k-slice.
//   * The loader permutes the rows of the B tile inside LDS so that the eight
//     MFMA tiles of a lane hold eight consecutive columns of C (forward: two
//     groups of four): the epilogue reads and writes C and the 16-bit planes
//     with 16-byte accesses that cover whole lines, without any cross-lane shuffle.
//   * Workgroups are persistent (one per CU); ids are dealt round-robin to the
//     XCDs (one L2 each; 8 of 32 CUs on MI355X, both read from the device): the
//     workgroups of an XCD walk consecutive tiles of a raster in which tiles
//     sharing operand panels are neighbours.
#include "kernels.h"

#include <type_traits>

namespace sfb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 64;                   // k-slice: one 128-byte LDS row of bf16
constexpr int BM = 256, BN = 256;        // workgroup tile
constexpr int TM = 8, TN = 8;            // 16 x 16 MFMA tiles per wavefront: 128 x 128 (2 x 2 wavefronts)
constexpr int NT = 256;
constexpr uint32_t STAGE = 0x10000u;     // bytes of one LDS stage: [A tile 32 KiB][B tile 32 KiB]
constexpr uint32_t B_OFF = BM * 128;
constexpr int LDS_BYTES = 2 * STAGE;
// Cache policy of the accesses of C and of its bf16 copy: non-temporal (each
// line is touched once per launch; left at the default policy they sweep the
// operand panels, which ARE reused, out of the 4 MiB L2 of the XCD).
constexpr int C_POLICY = 2;
// Load schedule: of the 16 direct loads a wavefront issues per k-slice, N2B go out
// in the third quarter of the slice two before the one they fetch (as soon as its
// LDS stage is free), N3 in its last quarter, N0 in the first quarter of the next
// slice and N1 in its second quarter, evenly spaced between the MFMAs.  Measured at the
// headline shape, forward / apply in ms, interleaved on one box: 8,8,0,0 4.32 / 6.24,
// 7,7,2,0 and 10,6,0,0 4.30 / 6.24, 6,10,0,0 4.32 / 6.25, 8,6,2,0 and 6,8,2,0 4.31 / 6.27,
// 5,8,3,0 4.37 / 6.28, 6,5,5,0 4.43 / 6.29, 4,6,6,0 4.53 / 6.35, 3,6,7,0 4.62 / 6.37, 2,6,6,2
// 4.89 / 6.38, 4,4,4,4 4.97 / 6.54: what is issued in the first half of the next slice has
// too little time left before that slice's barrier B.
#ifndef SFB_SCHED
#define SFB_SCHED 8, 8, 0, 0
#endif
#ifndef SFB_APOS
#define SFB_APOS 64
#endif
#ifndef SFB_BPOS
#define SFB_BPOS 32
#endif
// Barrier A after APOS of the 64 MFMAs of a slice's first k-step, barrier B after BPOS of those of the second
// (A at 48, 56 or 64 and B at 16, 32 or 48: within 1 % of each other on both contractions; 64 / 32 is the best step).
constexpr int APOS = SFB_APOS, BPOS = SFB_BPOS;
constexpr int SCHED[4] = {SFB_SCHED};
constexpr int N2B = SCHED[0], N3 = SCHED[1], N0 = SCHED[2], N1 = SCHED[3];
static_assert(N2B + N3 + N0 + N1 == 16 && N2B >= 0 && N3 >= 0 && N0 >= 0 && N1 >= 0, "16 loads per slice");
static_assert(APOS >= 40 && APOS <= 64 && (APOS == 64 || N1 == 0) && BPOS >= 0 && BPOS <= 48 && (64 - BPOS) % 16 == 0, "barrier positions");
constexpr int EPD = 3;                   // epilogue: blocks of C loads in flight + the one being stored (2: the same; 4 spills)

// MODE_SPLIT: the apply on a matrix stored as two 16-bit planes (see split_from_w_kernel):
// `shadow` is the high plane, `lo` the low one, C is not touched.
enum Mode : int { MODE_FWD = 0, MODE_APPLY = 1, MODE_SPLIT = 2 };

struct Params {
    const uint16_t* A;  // bf16 in blocks of 256 rows x 64 columns (operand_index): block (m / 256, k / 64) at index (m / 256) * (K / 64) + k / 64; k zero-padded to K
    const uint16_t* B;  // bf16, the same layout ((n / 256) * (K / 64) + k / 64)
    float* C;           // [M][ldc]; forward: stored tile by tile (see c_blocked)
    int c_blocked;      // forward: C is an array of BM x BN tiles, tile (tm, tn) at index tn * tiles_m + tm, rows of BN floats
    uint16_t* shadow;   // apply: bf16 copy of C to refresh ([M][ld_shadow]), or null; split: high plane
    uint16_t* lo;       // split: low plane, stored tile by tile (BM x BN tiles, tile (tm, tn) at index tm * tiles_n + tn)
    int64_t M, N, K;    // K % 64 == 0
    int64_t lda, ldb, ldc, ld_shadow;
    float eta;
    int tiles_m, tiles_n;
    int64_t tiles_total;
    int group_m;        // raster: groups of group_m row-tiles, row-tile index fastest inside a group
    int num_xcd;        // XCDs of the device: consecutive workgroup ids go to consecutive XCDs
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    floatx2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);  // round to nearest even
    return __builtin_bit_cast(uint32_t, h);
}

// A parameter matrix kept as two 16-bit planes: the halves of word = bits + 0x8000 (modulo 2^32).  hi = word >> 16
// is the value rounded to bf16 (to nearest, ties away from zero), lo = word & 0xffff; bits = ((hi << 16) | lo) -
// 0x8000, exactly.  Two elements a dword in both planes: split_pair / join_pair move between the packed halves and
// the two words with one byte permute each.
__device__ __forceinline__ uint32_t split_word(float v) { return __float_as_uint(v) + 0x8000u; }
__device__ __forceinline__ float split_value(uint32_t word) { return __uint_as_float(word - 0x8000u); }
// words of elements 0 and 1 from their packed high halves h = [h1 : h0] and low halves l = [l1 : l0]
__device__ __forceinline__ uint32_t join_pair0(uint32_t h, uint32_t l) { return __builtin_amdgcn_perm(h, l, 0x05040100u); }
__device__ __forceinline__ uint32_t join_pair1(uint32_t h, uint32_t l) { return __builtin_amdgcn_perm(h, l, 0x07060302u); }
// packed high halves [w1 >> 16 : w0 >> 16] and low halves [w1 & 0xffff : w0 & 0xffff] of two words
__device__ __forceinline__ uint32_t pack_hi(uint32_t w0, uint32_t w1) { return __builtin_amdgcn_perm(w1, w0, 0x07060302u); }
__device__ __forceinline__ uint32_t pack_lo(uint32_t w0, uint32_t w1) { return __builtin_amdgcn_perm(w1, w0, 0x05040100u); }

// Element (r, c) of a bf16 operand of sf_gemm_kernel (and of the high plane): blocks of BM rows x BK columns
// (one k-slice of a row tile, 32 KB in one piece), block (r / BM, c / BK) at index (r / BM) * (pitch / BK) + c / BK.
__device__ __forceinline__ int64_t operand_index(int64_t r, int64_t c, int64_t pitch)
{
    return ((r / BM) * (pitch / BK) + c / BK) * (int64_t)(BM * BK) + (r % BM) * BK + c % BK;
}
// Chunk-slot swizzle of tile row r: chunk c of the row sits in slot c ^ swz(r).
// Chosen by measurement: an MFMA operand read (runs of 16 consecutive rows at one
// chunk, 16 bytes a lane: rows of either parity meet the eight slots once each)
// costs 26.9 cycles with this function, as little as with padded rows, against
// 32.2 with r & 7 or (r >> 1) ^ (r >> 3) and 128 without a swizzle.
// swz(r + 16) = swz(r) ^ 2, swz(r + 32) = swz(r) ^ 4 and swz(r + 64) = swz(r).
__device__ __forceinline__ int swz(int r) { return (r ^ (r >> 3)) & 7; }
// LDS byte offset of chunk c (0..7) of tile row r (128-byte rows).  Chunk
// (4 ks + q), q < 4, of row r sits at lds_byte(r, q) ^ (64 ks).
__device__ __forceinline__ uint32_t lds_byte(int r, int c) { return (uint32_t)(r * 128 + ((c ^ swz(r)) << 4)); }

// f(integral_constant<int, B>), ..., f(integral_constant<int, E - 1>): a loop that is unrolled by construction (the
// 64-MFMA steps of the slice are beyond what the unroller accepts under a pragma, and an index that is not a
// constant would put the accumulators in scratch memory).
template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// The i-th of n loads goes after MFMA (2 i + 1) m / (2 n) of the m MFMAs of a window; -1: no load after MFMA j.
constexpr int slot(int j, int n, int m)
{
    for (int i = 0; i < n; ++i)
        if (j == (2 * i + 1) * m / (2 * n)) return i;
    return -1;
}

// A wave-uniform 64-bit value as the compiler can see it (scalar registers).
__device__ __forceinline__ uint64_t uniform64(uint64_t a)
{
    // (the builtin returns a signed int: narrow to 32 unsigned bits before widening)
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    return ((uint64_t)hi << 32) | (uint64_t)lo;
}

// 16 bytes per lane from global memory straight into LDS: lane l's bytes land at
// LDS address lds_addr + 16 l (lds_addr wave-uniform, in M0); the global address
// is gbase (uniform) + voff (per lane).  Issued as inline assembly so that the
// compiler's wait-count insertion does not tie every later LDS read to it; the
// caller waits (vmcnt) before the barrier that publishes the data.
// NT: non-temporal, for an operand whose lines are used by a few CUs at about the
// same time and never again (the class panel of the forward contraction: 6.5 GB
// streaming past a 4 MiB L2 in which the sample panels should stay; forward
// 4.78 -> 4.72 ms).  On an operand that IS reused it is ruinous (sample panel of
// the forward +20 %, either operand of the apply +25 %).
template <bool NT>
__device__ __forceinline__ void load_to_lds_16(uint32_t lds_addr, uint64_t gbase, uint32_t voff)
{
    if (NT)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_addr), "v"(voff), "s"(gbase)
                     : "memory");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(gbase)
                     : "memory");
}
// One accumulator element out of the accumulation registers.  Written as
// assembly because the compiler otherwise copies whole 16-register tiles (64
// registers per block of the epilogue) to ordinary registers up front.  The
// caller guarantees that the MFMA that wrote the element has retired
// (mfma_results_settle).
__device__ __forceinline__ float acc_read(float element)
{
    float v;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(element));
    return v;
}
// More wait states than the longest MFMA needs to write back its result.
__device__ __forceinline__ void mfma_results_settle()
{
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
}
__device__ __forceinline__ void wait_all_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <int MODE>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(1, 1))) void sf_gemm_kernel(Params p)
{
    extern __shared__ u32x4 smem[];
    const char* const lds_bytes = reinterpret_cast<const char*>(smem);
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar
    const int wm0 = (wave >> 1) * (TM * 16), wn0 = (wave & 1) * (TN * 16);

    // ---- persistent schedule ------------------------------------------------
    const int64_t x = blockIdx.x % p.num_xcd, wi = blockIdx.x / p.num_xcd, per_xcd = gridDim.x / p.num_xcd;
    const int64_t q8 = p.tiles_total / p.num_xcd, r8 = p.tiles_total % p.num_xcd;
    const int64_t xcd_start = x * q8 + (x < r8 ? x : r8), xcd_cnt = q8 + (x < r8 ? 1 : 0);
    if (wi >= xcd_cnt) return;
    const int64_t n_my = (xcd_cnt - wi + per_xcd - 1) / per_xcd;   // tiles of this workgroup
    const int64_t nk = p.K / BK;
    const int64_t S = n_my * nk;                                    // k-slices of this workgroup, all tiles
    // Order of the 64 MFMAs of a k-step: the outer operand's fragment stays for eight MFMAs, the inner one's changes
    // with every MFMA.  The operand that is mostly zeros (the samples: A of the forward, B of the apply) is the one
    // that changes: fewer bits toggle at the matrix pipes' inputs.
    // (forward 4.24 -> 4.20 ms against the other order, interleaved; the apply does not care)
    constexpr bool B_OUTER = MODE == MODE_FWD;
    auto tile_a = [](int j) { return B_OUTER ? j % TM : j / TN; };
    auto tile_b = [](int j) { return B_OUTER ? j / TM : j % TN; };

    auto tile_origin = [&](int64_t ordinal, int64_t& m0, int64_t& n0) {
        const int64_t L = xcd_start + ordinal * per_xcd + wi;
        const int64_t per_group = (int64_t)p.group_m * p.tiles_n;
        const int64_t grp = L / per_group, r = L % per_group;
        const int64_t rem = p.tiles_m - grp * p.group_m;
        const int64_t gm = rem < p.group_m ? rem : p.group_m;
        m0 = (grp * p.group_m + r % gm) * BM;
        n0 = (r / gm) * BN;
    };

    // Which row of the B tile sits in LDS row r.  MFMA tile tb of a wavefront takes
    // its 16 columns from LDS rows 16 tb .. 16 tb + 15 of the wavefront's 128; those
    // rows hold tile rows 8 c + tb (c = 0..15), so that a lane ends up with eight
    // CONSECUTIVE columns of C in its eight tiles (16-byte accesses of the 16-bit
    // planes, two of C per row in the epilogue, no cross-lane shuffles).  The loader
    // is free to do this: each lane of a direct load supplies its own global address.
    // (Where C is fp32 — the logits of the forward, W as an fp32 array — a lane's eight columns are 32 bytes of a
    // row.  There they are two groups of four, 64 columns apart, so that each of the two 16-byte accesses of a row
    // covers whole lines: tile rows 4 c + tb % 4 + 64 (tb / 4); the bf16 copy is then accessed 8 bytes at a time.)
    constexpr bool SPLIT8 = MODE != MODE_SPLIT;
    auto b_row_of = [](int r) {
        return SPLIT8 ? (r & ~127) | ((r & 15) << 2) | ((r >> 4) & 3) | (((r >> 6) & 1) << 6)
                      : (r & ~127) | ((r & 15) << 3) | ((r >> 4) & 7);
    };

    // ---- loader ---------------------------------------------------------------
    // A k-slice of a tile is 32 blocks of 8 rows for each operand; wavefront w
    // loads blocks 8w..8w+7 of both.  Lane l of block b fills slot l & 7 of row
    // 8b + (l >> 3), i.e. fetches chunk (l & 7) ^ swz(row).  Rows past the end of
    // the matrix are clamped to its last row: they only feed accumulators that
    // are never stored; k is zero-padded.
    const uint32_t pitchA = (uint32_t)BK * 2u, pitchB = (uint32_t)BK * 2u;   // a row of a block is one 128-byte line
    const uint64_t stepA = (uint64_t)BM * BK * 2, stepB = (uint64_t)BN * BK * 2;   // bytes from a k-slice to the next
    uint32_t offA[8], offB[8];
    uint64_t gA = 0, gB = 0;           // address of (row 0, current k-slice) of the tile being loaded
    int64_t iss_q = 0, iss_k = 0;
    uint32_t iss_stage = 0;
    auto enter_tile = [&](int64_t ordinal) {
        int64_t m0, n0;
        tile_origin(ordinal, m0, n0);
        gA = uniform64(reinterpret_cast<uint64_t>(p.A) + (uint64_t)(m0 / BM) * (uint64_t)nk * stepA);
        gB = uniform64(reinterpret_cast<uint64_t>(p.B) + (uint64_t)(n0 / BN) * (uint64_t)nk * stepB);
        const int lastA = (int)(p.M - m0 < BM ? p.M - m0 : BM) - 1;
        const int lastB = (int)(p.N - n0 < BN ? p.N - n0 : BN) - 1;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = 8 * (8 * wave + i) + (lane >> 3);   // LDS row
            const uint32_t c16 = (uint32_t)(((lane & 7) ^ swz(r)) << 4);
            offA[i] = (uint32_t)(r < lastA ? r : lastA) * pitchA + c16;
            const int rb = b_row_of(r);                        // tile row of B kept in that LDS row
            offB[i] = (uint32_t)(rb < lastB ? rb : lastB) * pitchB + c16;
        }
    };
    // The 16 loads of a slice are issued one at a time (issue_one(0..15)) so that
    // they can be interleaved with MFMAs: a burst of loads blocks the wavefront in
    // the memory-issue stage while the MFMA pipe runs dry.
    auto issue_one = [&](int j) {
        const uint32_t dst = lds_base + iss_stage + (uint32_t)(8 * wave) * 1024u;
        if (j < 8)
            load_to_lds_16<false>(dst + j * 1024u, gA, offA[j & 7]);
        else
            load_to_lds_16<MODE == MODE_FWD>(dst + B_OFF + (j - 8) * 1024u, gB, offB[j & 7]);
    };
    auto issue_done = [&]() {   // advance the load cursor by one slice
        gA += stepA;
        gB += stepB;
        iss_stage ^= STAGE;
        ++iss_q;
        if (++iss_k == nk) {
            iss_k = 0;
            if (iss_q < S) {
                enter_tile(iss_q / nk);
            } else {   // past the last slice: stay on the last tile (such loads are never read)
                gA -= (uint64_t)nk * stepA;
                gB -= (uint64_t)nk * stepB;
            }
        }
    };
    auto issue = [&]() {
#pragma unroll
        for (int j = 0; j < 16; ++j) issue_one(j);
        issue_done();
    };

    // ---- MFMA side ------------------------------------------------------------
    // 16x16x32 MFMAs: on operands that change, the chip keeps a higher clock with them than with the 32x32x16 form
    // (register-only loops on pseudo-random bf16 data, sfb_peaks: 1.92 against 1.78 PFLOP/s), for
    // the same fragment bytes from LDS: eight A and eight B fragments per 32 of k, 64 MFMAs.
    floatx4 acc[TM][TN];    // defined by the first MFMAs of each tile (zero addend)

    // Lane l = (quad q = l >> 4, l16 = l & 15) supplies row l16 of a fragment's 16 rows and the 8 values
    // k = 8 q .. 8 q + 7 of the 32 of a k-step (the same assignment for both operands: any is right).
    // LDS byte offsets of chunk q of rows wm0 + 16 t + l16 (t = 0..3; t + 4 is 64 rows = 8 KiB further: swz(r + 64)
    // = swz(r)) of the A tile and of wn0 + 16 t + l16 of the B tile, in the stage being read; k-step ks of the
    // slice is chunk 4 ks + q: the offset XOR 64 ks.
    const int l16 = lane & 15, quad = lane >> 4;
    uint32_t ra[4], rb[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        ra[t] = lds_byte(wm0 + 16 * t + l16, quad);
        rb[t] = lds_byte(wn0 + 16 * t + l16, quad) + B_OFF;
    }
    struct Frags {
        bf16x8 a[TM], b[TN];
    };
    // The i-th fragment read of a k-step, in the order the MFMAs want them: the first fragment of the outer
    // operand, the eight of the inner one, the other seven of the outer one.
    auto read_one = [&](Frags& f, int ks, int i) {
        const bool outer = i == 0 || i > TN;            // a fragment of the operand of the MFMAs' outer loop
        const int t = i == 0 ? 0 : (i > TN ? i - TN : i - 1);
        if (outer != B_OUTER)
            f.a[t] = *reinterpret_cast<const bf16x8*>(lds_bytes + (ra[t & 3] ^ (64u * ks)) + (t >> 2) * 64 * 128);
        else
            f.b[t] = *reinterpret_cast<const bf16x8*>(lds_bytes + (rb[t & 3] ^ (64u * ks)) + (t >> 2) * 64 * 128);
    };
    auto read_frags = [&](Frags& f, int ks) {   // k-step ks (32 of k) of the stage ra / rb point at
#pragma unroll
        for (int i = 0; i < TM + TN; ++i) read_one(f, ks, i);
    };
    auto flip_stage = [&]() {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            ra[t] ^= STAGE;
            rb[t] ^= STAGE;
        }
    };

    // Epilogue of one tile.  Register i of lane (quad, l16) of MFMA tile (ta, tb) is
    // row 16 ta + 4 quad + i, column 8 l16 + tb of the wavefront's 128 x 128 block
    // (see b_row_of): for fixed (ta, i) a lane owns 8 consecutive columns, the 16
    // lanes of a quad 512 contiguous bytes of one row of C (256 of a 16-bit plane),
    // the other quads the rows 4, 8 and 12 below.  C is addressed through a raw buffer
    // descriptor based at the wavefront's corner of the tile: the row offset is
    // scalar, the lane offset one register, so no address registers are live
    // while loads are in flight.  Rows of C, of its bf16 copy and of the planes are
    // 16-byte aligned (checked by the launcher).
    auto make_rsrc = [&](const void* base) {
        return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(uniform64(reinterpret_cast<uint64_t>(base))),
                                                 0, 0xffffffff, 0x00020000);
    };
    auto epilogue_tile = [&](int64_t m0, int64_t n0, auto guard_tag) {
        constexpr bool GUARD = decltype(guard_tag)::value;
        const auto crs = make_rsrc(MODE == MODE_SPLIT ? p.C
                                   : (MODE == MODE_FWD && p.c_blocked)
                                       ? p.C + ((n0 / BN) * p.tiles_m + m0 / BM) * (int64_t)(BM * BN) + wm0 * BN + wn0
                                       : p.C + (m0 + wm0) * p.ldc + n0 + wn0);
        const bool has_shadow = p.shadow != nullptr;
        // (the bf16 copy / high plane is stored in the operand layout: blocks of BM rows x 64 columns)
        const auto srs = make_rsrc((MODE == MODE_SPLIT || has_shadow)
                                       ? p.shadow + ((m0 / BM) * (p.ld_shadow / BK) + (n0 + wn0) / BK) * (int64_t)(BM * BK) + wm0 * BK
                                       : p.shadow);
        const auto lrs = make_rsrc(MODE == MODE_SPLIT
                                       ? p.lo + ((m0 / BM) * p.tiles_n + n0 / BN) * (int64_t)(BM * BN) + wm0 * BN + wn0
                                       : p.lo);
        const uint32_t row_l = (uint32_t)BN * 2u, lane_l = (uint32_t)(4 * quad) * row_l + (uint32_t)l16 * 16u;
        const int rows_left = (int)(p.M - (m0 + wm0) < 4 * BM ? p.M - (m0 + wm0) : 4 * BM) - 4 * quad;   // for this lane
        const uint32_t row_c = (MODE == MODE_FWD && p.c_blocked) ? (uint32_t)BN * 4u : (uint32_t)p.ldc * 4u;
        const uint32_t row_s = (uint32_t)BK * 2u;
        const uint32_t lane_c = (uint32_t)(4 * quad) * row_c + (uint32_t)l16 * (SPLIT8 ? 16u : 32u);
        const uint32_t half_c = SPLIT8 ? 256u : 16u;        // bytes from a lane's first four columns to its other four
        const uint32_t lane_s = SPLIT8 ? (uint32_t)(4 * quad) * row_s + (uint32_t)l16 * 8u
                                       : (uint32_t)(l16 >> 3) * (uint32_t)(BM * BK * 2) + (uint32_t)(4 * quad) * row_s + (uint32_t)(l16 & 7) * 16u;
        const bool col_ok = !GUARD || (n0 + wn0 + (SPLIT8 ? 4 : 8) * l16 < p.N);   // N % 8 == 0: all eight (four) columns or none
        const bool col_ok1 = !GUARD || !SPLIT8 || (n0 + wn0 + 64 + 4 * l16 < p.N);    // (forward: the second group of four)
        // One block = the 16 rows of one ta: 4 rows per lane, 8 columns each (two 16-byte accesses per row: both
        // planes, or the two halves of the fp32 row segment).  The loads of the next EPD - 1 blocks are in flight
        // while a block is combined and stored.
        constexpr int NQ = TM;
        u32x4 w[EPD][4][2];
        mfma_results_settle();
        auto load_block = [&](int q, u32x4 (*dst)[2]) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int dr = q * 16 + e;
                dst[e][0] = u32x4{0u, 0u, 0u, 0u};
                dst[e][1] = u32x4{0u, 0u, 0u, 0u};
                if (col_ok && (!GUARD || dr < rows_left)) {
                    if (MODE == MODE_SPLIT) {   // eight columns of the high plane, eight of the low plane
                        dst[e][0] = __builtin_amdgcn_raw_buffer_load_b128(srs, lane_s, (uint32_t)dr * row_s, C_POLICY);
                        dst[e][1] = __builtin_amdgcn_raw_buffer_load_b128(lrs, lane_l, (uint32_t)dr * row_l, C_POLICY);
                    } else {
                        dst[e][0] = __builtin_amdgcn_raw_buffer_load_b128(crs, lane_c, (uint32_t)dr * row_c, C_POLICY);
                        if (col_ok1)
                            dst[e][1] = __builtin_amdgcn_raw_buffer_load_b128(crs, lane_c + half_c, (uint32_t)dr * row_c, C_POLICY);
                    }
                }
            }
        };
        if (MODE != MODE_FWD) {
#pragma unroll
            for (int q = 0; q < EPD - 1 && q < NQ; ++q) load_block(q, w[q % EPD]);
        }
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            if (MODE != MODE_FWD && q + EPD - 1 < NQ) load_block(q + EPD - 1, w[(q + EPD - 1) % EPD]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int dr = q * 16 + e;
                float v[TN];
#pragma unroll
                for (int tb = 0; tb < TN; ++tb) v[tb] = acc_read(acc[q][tb][e]);
                if (col_ok && (!GUARD || dr < rows_left)) {
                    if (MODE == MODE_FWD) {
                        const u32x4 out0 = {__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
                        const u32x4 out1 = {__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7])};
                        __builtin_amdgcn_raw_buffer_store_b128(out0, crs, lane_c, (uint32_t)dr * row_c, C_POLICY);
                        if (col_ok1)
                            __builtin_amdgcn_raw_buffer_store_b128(out1, crs, lane_c + half_c, (uint32_t)dr * row_c, C_POLICY);
                    } else if (MODE == MODE_SPLIT) {
                        uint32_t oh[4], ol[4];
                        bool changed = false;
#pragma unroll
                        for (int k = 0; k < 4; ++k) {      // dword k of both planes: columns 2 k, 2 k + 1
                            const uint32_t hk = w[q % EPD][e][0][k], lk = w[q % EPD][e][1][k];
                            const uint32_t w0 = split_word(split_value(join_pair0(hk, lk)) - p.eta * v[2 * k]);
                            const uint32_t w1 = split_word(split_value(join_pair1(hk, lk)) - p.eta * v[2 * k + 1]);
                            oh[k] = pack_hi(w0, w1);
                            ol[k] = pack_lo(w0, w1);
                            changed = changed || oh[k] != hk;
                        }
                        // the high halves change only where the update crosses a bf16 rounding boundary: lanes
                        // whose eight are unchanged leave the plane as it is (the same bits, fewer bytes written)
                        if (changed)
                            __builtin_amdgcn_raw_buffer_store_b128(u32x4{oh[0], oh[1], oh[2], oh[3]}, srs, lane_s,
                                                                   (uint32_t)dr * row_s, C_POLICY);
                        __builtin_amdgcn_raw_buffer_store_b128(u32x4{ol[0], ol[1], ol[2], ol[3]}, lrs, lane_l,
                                                               (uint32_t)dr * row_l, C_POLICY);
                    } else {
                        float nf[TN];
                        uint32_t sh[4];
                        bool changed[2] = {false, false};
#pragma unroll
                        for (int k = 0; k < 4; ++k) {      // (k / 2 is the group of four columns)
                            const uint32_t oa = w[q % EPD][e][k >> 1][(2 * k) & 3], ob = w[q % EPD][e][k >> 1][(2 * k + 1) & 3];
                            nf[2 * k] = __uint_as_float(oa) - p.eta * v[2 * k];
                            nf[2 * k + 1] = __uint_as_float(ob) - p.eta * v[2 * k + 1];
                            sh[k] = pack_bf16(nf[2 * k], nf[2 * k + 1]);
                            changed[k >> 1] = changed[k >> 1] || sh[k] != pack_bf16(__uint_as_float(oa), __uint_as_float(ob));
                        }
                        const u32x4 out0 = {__float_as_uint(nf[0]), __float_as_uint(nf[1]), __float_as_uint(nf[2]), __float_as_uint(nf[3])};
                        const u32x4 out1 = {__float_as_uint(nf[4]), __float_as_uint(nf[5]), __float_as_uint(nf[6]), __float_as_uint(nf[7])};
                        __builtin_amdgcn_raw_buffer_store_b128(out0, crs, lane_c, (uint32_t)dr * row_c, C_POLICY);
                        if (col_ok1)
                            __builtin_amdgcn_raw_buffer_store_b128(out1, crs, lane_c + half_c, (uint32_t)dr * row_c, C_POLICY);
                        // the copy is current on entry: rewrite it only where its bits change (the second group of
                        // four columns lies in the next block of 64 columns of the operand layout)
                        if (has_shadow && changed[0])
                            __builtin_amdgcn_raw_buffer_store_b64(u32x2{sh[0], sh[1]}, srs, lane_s, (uint32_t)dr * row_s, C_POLICY);
                        if (has_shadow && changed[1] && col_ok1)
                            __builtin_amdgcn_raw_buffer_store_b64(u32x2{sh[2], sh[3]}, srs, lane_s + (uint32_t)(BM * BK * 2),
                                                                  (uint32_t)dr * row_s, C_POLICY);
                    }
                }
            }
        }
    };

    // ---- pipeline ---------------------------------------------------------------
    // Slice s lives in stage s & 1 and is two k-steps of 32: f0 holds the fragments of the first, f1 of the second.
    // The second step's fragments are read under the first step's MFMAs, so after the first step every wavefront is
    // done with stage s & 1 (barrier A: the loads of slice s+2 start); half way through the second step the loads
    // of slice s+1 must have landed (barrier B), and its first fragments are read under the rest of that step.
    Frags f0, f1;
    enter_tile(0);
    issue();
    wait_all_vmem();
    __syncthreads();
    // (the first k-step of the loop issues the rest of slice 1)
#pragma unroll
    for (int j = 0; j < 16; ++j)
        if (j < N2B + N3) issue_one(j);
    read_frags(f0, 0);
    // One k-slice (slice s, living in stage s & 1; f0 holds its first fragments).
    // The direct loads are unconditional (past the last slice they re-fetch the
    // last tile into a stage nobody reads).  vmcnt counts in order, so at barrier B
    // only the N2B loads issued since A may still be in flight.
    // The instruction order of a slice is fixed by hand (a scheduling barrier after
    // every MFMA): left to itself the compiler sinks the fragment reads of the next
    // k-step to just before their first use, and the wavefront then waits out the
    // LDS latency with an idle MFMA pipe.  The sixteen reads of the next k-step
    // follow every second of the first 32 MFMAs of the current one (one per MFMA
    // would ask more of the LDS than it delivers while the direct loads write it).
    auto slice_body = [&](auto first_tag) {
        const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
        constexpr int STEP = TM * TN;          // MFMAs of a k-step
        // MFMAs 0 .. APOS-1: k-step 0 on f0 (the reads of k-step 1 into f1 behind every second of the first 32)
        static_for<0, APOS>([&](auto J) {
            constexpr int j = decltype(J)::value;
            if constexpr (decltype(first_tag)::value)
                acc[tile_a(j)][tile_b(j)] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0.a[tile_a(j)], f0.b[tile_b(j)], zero, 0, 0, 0);
            else
                acc[tile_a(j)][tile_b(j)] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0.a[tile_a(j)], f0.b[tile_b(j)], acc[tile_a(j)][tile_b(j)], 0, 0, 0);
            if constexpr (j < 32 && (j & 1) == 0) read_one(f1, 1, j >> 1);
            if constexpr (j < 32) {
                if constexpr (slot(j, N0, 32) >= 0) issue_one(N2B + N3 + slot(j, N0, 32));
            } else {
                if constexpr (slot(j - 32, N1, 32) >= 0) issue_one(N2B + N3 + N0 + slot(j - 32, N1, 32));
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        issue_done();
        __syncthreads();                                   // A
        // MFMAs APOS .. STEP+BPOS-1: the rest of k-step 0, the first BPOS of k-step 1 on f1; the first loads of slice s+2
        static_for<APOS, STEP + BPOS>([&](auto J) {
            constexpr int m = decltype(J)::value, j = m % STEP;
            if constexpr (m < STEP) {
                if constexpr (decltype(first_tag)::value)
                    acc[tile_a(j)][tile_b(j)] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0.a[tile_a(j)], f0.b[tile_b(j)], zero, 0, 0, 0);
                else
                    acc[tile_a(j)][tile_b(j)] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f0.a[tile_a(j)], f0.b[tile_b(j)], acc[tile_a(j)][tile_b(j)], 0, 0, 0);
            } else {
                acc[tile_a(j)][tile_b(j)] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f1.a[tile_a(j)], f1.b[tile_b(j)], acc[tile_a(j)][tile_b(j)], 0, 0, 0);
            }
            if constexpr (slot(m - APOS, N2B, STEP + BPOS - APOS) >= 0) issue_one(slot(m - APOS, N2B, STEP + BPOS - APOS));
            __builtin_amdgcn_sched_barrier(0);
        });
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N2B) : "memory");   // everything but those: slice s+1 is in LDS
        __syncthreads();                                   // B
        flip_stage();
        // the rest of k-step 1: reads of the next slice's k-step 0 into f0 (after the last slice: of a stage nobody uses)
        static_for<BPOS, STEP>([&](auto J) {
            constexpr int j = decltype(J)::value;
            constexpr int every = (STEP - BPOS) / (TM + TN);
            acc[tile_a(j)][tile_b(j)] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f1.a[tile_a(j)], f1.b[tile_b(j)], acc[tile_a(j)][tile_b(j)], 0, 0, 0);
            if constexpr ((j - BPOS) % every == 0 && (j - BPOS) / every < TM + TN) read_one(f0, 0, (j - BPOS) / every);
            if constexpr (slot(j - BPOS, N3, STEP - BPOS) >= 0) issue_one(N2B + slot(j - BPOS, N3, STEP - BPOS));
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    for (int64_t t = 0; t < n_my; ++t) {
        int64_t m0, n0;
        tile_origin(t, m0, n0);
        slice_body(std::true_type{});
        for (int64_t k = 1; k < nk; ++k) slice_body(std::false_type{});
        if ((m0 + BM <= p.M) && (n0 + BN <= p.N))
            epilogue_tile(m0, n0, std::false_type{});
        else
            epilogue_tile(m0, n0, std::true_type{});
    }
    wait_all_vmem();   // no direct load may be in flight when the workgroup's LDS is released
}

// src[rows_src][cols] (bf16, row-major) -> dst = its transpose [cols][pitch] in the blocked operand layout of
// sf_gemm_kernel; source rows rows_src..pitch-1 are taken as zero.  cols % 8 == 0, pitch % 64 == 0.
// 64x64 tiles through LDS, 256 threads, 16-byte global accesses on both sides
// (8 lanes cover one 128-byte row segment).
// coef (nullable): source row k is scaled by coef[k] (product in fp32, rounded to
// bf16 to nearest even).
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const uint16_t* __restrict__ src,
                                                             uint16_t* __restrict__ dst, int64_t rows_src,
                                                             int64_t cols, int64_t pitch,
                                                             const float* __restrict__ coef)
{
    constexpr int LP = 72;   // LDS row pitch in elements: 144 bytes, rows stay 16-byte aligned
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * LP];
    const int64_t c0 = (int64_t)blockIdx.x * 64, k0 = (int64_t)blockIdx.y * 64;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int id = threadIdx.x + 256 * it, r = id >> 3, cc = (id & 7) * 8;
        const int64_t k = k0 + r, c = c0 + cc;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (k < rows_src && c < cols) {
            v = *reinterpret_cast<const u32x4*>(src + k * cols + c);
            if (coef) {
                const float ck = coef[k];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t w = v[e];   // (element first into a scalar, see pack_bf16's callers)
                    v[e] = pack_bf16(ck * __uint_as_float(w << 16), ck * __uint_as_float(w & 0xffff0000u));
                }
            }
        }
        *reinterpret_cast<u32x4*>(&tile[r * LP + cc]) = v;
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int id = threadIdx.x + 256 * it, cr = id >> 3, kc = (id & 7) * 8;
        const int64_t c = c0 + cr;
        uint32_t o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            o[i] = (uint32_t)tile[(kc + 2 * i) * LP + cr] | ((uint32_t)tile[(kc + 2 * i + 1) * LP + cr] << 16);
        // (dst is stored in blocks of 256 rows x 64 columns, block (c / 256, k / 64) at index (c / 256) * (pitch / 64) + k / 64)
        if (c < cols)
            *reinterpret_cast<u32x4*>(dst + operand_index(c, k0 + kc, pitch)) = u32x4{o[0], o[1], o[2], o[3]};
    }
}

// dst(r, 0..pitch) = bf16(src[r][0..cols)) followed by zeros, in the operand layout; 8 elements a thread.
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
        *reinterpret_cast<u32x4*>(dst + operand_index(r, c, pitch)) = v;
    }
}

// W[J][D] fp32 -> the two planes ([J][pitch], columns D.. zero), 8 elements a thread; and back.
// Element (r, c) of the low plane: the plane is an array of BM x BN tiles in row-major tile order.
__device__ __forceinline__ int64_t split_lo_index(int64_t r, int64_t c, int64_t tiles_n)
{
    return ((r / BM) * tiles_n + c / BN) * (int64_t)(BM * BN) + (r % BM) * BN + c % BN;
}

__global__ __launch_bounds__(256) void split_from_w_kernel(const float* __restrict__ W, uint16_t* __restrict__ hi,
                                                           uint16_t* __restrict__ lo, int64_t rows, int64_t cols,
                                                           int64_t pitch, int64_t tiles_n)
{
    const int64_t chunks = pitch / 8, total = rows * chunks;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int64_t r = idx / chunks, c = (idx % chunks) * 8;
        u32x4 h = {0u, 0u, 0u, 0u}, l = {0u, 0u, 0u, 0u};
        if (c < cols) {   // cols % 8 == 0
            const floatx4 a = *reinterpret_cast<const floatx4*>(W + r * cols + c);
            const floatx4 b = *reinterpret_cast<const floatx4*>(W + r * cols + c + 4);
            const float a0 = a[0], a1 = a[1], a2 = a[2], a3 = a[3], b0 = b[0], b1 = b[1], b2 = b[2], b3 = b[3];
            const uint32_t w0 = split_word(a0), w1 = split_word(a1), w2 = split_word(a2), w3 = split_word(a3);
            const uint32_t w4 = split_word(b0), w5 = split_word(b1), w6 = split_word(b2), w7 = split_word(b3);
            h = u32x4{pack_hi(w0, w1), pack_hi(w2, w3), pack_hi(w4, w5), pack_hi(w6, w7)};
            l = u32x4{pack_lo(w0, w1), pack_lo(w2, w3), pack_lo(w4, w5), pack_lo(w6, w7)};
        }
        *reinterpret_cast<u32x4*>(hi + operand_index(r, c, pitch)) = h;
        if (c < cols) *reinterpret_cast<u32x4*>(lo + split_lo_index(r, c, tiles_n)) = l;
    }
}

__global__ __launch_bounds__(256) void w_from_split_kernel(const uint16_t* __restrict__ hi, const uint16_t* __restrict__ lo,
                                                           float* __restrict__ W, int64_t rows, int64_t cols,
                                                           int64_t pitch, int64_t tiles_n)
{
    const int64_t chunks = cols / 8, total = rows * chunks;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int64_t r = idx / chunks, c = (idx % chunks) * 8;
        const u32x4 h = *reinterpret_cast<const u32x4*>(hi + operand_index(r, c, pitch));
        const u32x4 l = *reinterpret_cast<const u32x4*>(lo + split_lo_index(r, c, tiles_n));
        const uint32_t h0 = h[0], h1 = h[1], h2 = h[2], h3 = h[3], l0 = l[0], l1 = l[1], l2 = l[2], l3 = l[3];
        const floatx4 a = {split_value(join_pair0(h0, l0)), split_value(join_pair1(h0, l0)),
                           split_value(join_pair0(h1, l1)), split_value(join_pair1(h1, l1))};
        const floatx4 b = {split_value(join_pair0(h2, l2)), split_value(join_pair1(h2, l2)),
                           split_value(join_pair0(h3, l3)), split_value(join_pair1(h3, l3))};
        *reinterpret_cast<floatx4*>(W + r * cols + c) = a;
        *reinterpret_cast<floatx4*>(W + r * cols + c + 4) = b;
    }
}

template <int MODE>
hipError_t launch(Params p, DeviceInfo& dev, hipStream_t stream)
{
    if (dev.cus <= 0 || dev.xcds <= 0) return hipErrorInvalidDevice;
    p.tiles_m = (int)((p.M + BM - 1) / BM);
    p.tiles_n = (int)((p.N + BN - 1) / BN);
    p.tiles_total = (int64_t)p.tiles_m * p.tiles_n;
    if (p.group_m <= 0 || p.group_m > p.tiles_m) p.group_m = p.tiles_m;
    // 32-bit in-tile byte offsets in the loaders and in the epilogue
    if (p.lda * 2 * BM >= (1LL << 31) || p.ldb * 2 * BN >= (1LL << 31) || p.ldc * 4 * BM >= (1LL << 31))
        return hipErrorInvalidValue;
    // 16-byte accesses of C, of its bf16 copy and of the two planes; a lane owns eight consecutive columns
    if (p.N % 8 != 0) return hipErrorInvalidValue;
    if (MODE != MODE_SPLIT && (reinterpret_cast<uintptr_t>(p.C) % 16 != 0 || p.ldc % 4 != 0)) return hipErrorInvalidValue;
    if (p.shadow && (reinterpret_cast<uintptr_t>(p.shadow) % 16 != 0 || p.ld_shadow % 8 != 0))
        return hipErrorInvalidValue;
    if (MODE == MODE_SPLIT && (!p.shadow || !p.lo || reinterpret_cast<uintptr_t>(p.lo) % 16 != 0 || p.ld_shadow < p.N ||
                               p.ld_shadow * 2 * BM >= (1LL << 31)))
        return hipErrorInvalidValue;
    if (p.K <= 0 || p.K % BK != 0 || p.lda % BK != 0 || p.ldb % BK != 0 || p.lda < p.K || p.ldb < p.K)
        return hipErrorInvalidValue;
    if (!dev.gemm_bf16_lds_set[MODE]) {       // (per device: the caller's context holds the flag)
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sf_gemm_kernel<MODE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        dev.gemm_bf16_lds_set[MODE] = true;
    }
    p.num_xcd = dev.xcds;
    int64_t grid = dev.cus / dev.xcds * dev.xcds;      // one persistent workgroup per CU, the same number per XCD
    if (grid <= 0) {
        grid = dev.cus;
        p.num_xcd = 1;
    }
    if (p.tiles_total < grid) grid = (p.tiles_total + p.num_xcd - 1) / p.num_xcd * p.num_xcd;
    hipLaunchKernelGGL((sf_gemm_kernel<MODE>), dim3((unsigned)grid), dim3(NT), LDS_BYTES, stream, p);
    return hipGetLastError();
}

unsigned grid_for(int64_t n)
{
    int64_t g = (n + 255) / 256;
    if (g > 16384) g = 16384;
    return (unsigned)(g < 1 ? 1 : g);
}

}  // namespace

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
                                   int64_t B, int64_t J, int64_t D, DeviceInfo& dev, hipStream_t stream)
{
    if (B <= 0 || J <= 0) return hipSuccess;
    const int64_t pitch = bf16_pitch(D);
    if (X) {   // null: the caller has already written X_aligned (rows of `pitch` elements, zero padded)
        hipLaunchKernelGGL((pad_rows_bf16_kernel<uint16_t>), dim3(grid_for(B * (pitch / 8))), dim3(256), 0, stream, X,
                           X_aligned, B, D, pitch);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    Params p = {};
    p.A = X_aligned; p.lda = pitch; p.M = B;
    p.B = W_shadow; p.ldb = pitch; p.N = J;
    p.C = Z; p.ldc = J;
    p.c_blocked = 1;             // logits tile by tile: a workgroup writes 256 KB in one piece (see mlr_logits_floats)
    p.K = pitch;
    p.group_m = 0;               // all batch tiles of one class tile are neighbours (they share the W tile)
    return launch<MODE_FWD>(p, dev, stream);
}

// Floats of the tile-blocked logits array of launch_mlr_forward_bf16.
int64_t mlr_logits_floats(int64_t B, int64_t J) { return ((B + BM - 1) / BM) * ((J + BN - 1) / BN) * (int64_t)(BM * BN); }

// Bytes of a rows x cols bf16 operand in the blocked layout (whole blocks of 256 rows, cols padded to 64).
int64_t bf16_operand_bytes(int64_t rows, int64_t cols) { return ((rows + BM - 1) / BM) * (int64_t)BM * bf16_pitch(cols) * 2; }
// Bytes of the low plane of a J x D matrix kept as two planes (whole 256 x 256 tiles).
int64_t split_lo_bytes(int64_t J, int64_t D) { return ((J + BM - 1) / BM) * ((D + BN - 1) / BN) * (int64_t)(BM * BN) * 2; }

// U^T (J x N) and V^T (D x N) in the operand layout, one after the other.
int64_t apply_bf16_workspace_bytes(int64_t N, int64_t J, int64_t D) { return bf16_operand_bytes(J, N) + bf16_operand_bytes(D, N); }

uint16_t* apply_bf16_vt(void* workspace, int64_t N, int64_t J)
{
    return static_cast<uint16_t*>(workspace) + bf16_operand_bytes(J, N) / 2;
}

hipError_t launch_apply_bf16_transpose(const uint16_t* U, const uint16_t* V, const float* coef, int64_t N, int64_t J,
                                       int64_t D, void* workspace, hipStream_t stream)
{
    if (N <= 0 || J <= 0 || D <= 0) return hipSuccess;
    const int64_t Np = bf16_pitch(N);
    uint16_t* Ut = static_cast<uint16_t*>(workspace);
    uint16_t* Vt = apply_bf16_vt(workspace, N, J);
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)((J + 63) / 64), (unsigned)(Np / 64)), dim3(256), 0,
                       stream, U, Ut, N, J, Np, static_cast<const float*>(nullptr));
    if (V)     // null: the caller writes V^T itself (apply_bf16_vt)
        hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)((D + 63) / 64), (unsigned)(Np / 64)), dim3(256), 0,
                           stream, V, Vt, N, D, Np, coef);
    return hipGetLastError();
}

hipError_t launch_split_from_w(const float* W, uint16_t* hi, uint16_t* lo, int64_t J, int64_t D, hipStream_t stream)
{
    if (J <= 0 || D <= 0) return hipSuccess;
    const int64_t pitch = bf16_pitch(D);
    hipLaunchKernelGGL(split_from_w_kernel, dim3(grid_for(J * (pitch / 8))), dim3(256), 0, stream, W, hi, lo, J, D, pitch, (D + BN - 1) / BN);
    return hipGetLastError();
}

hipError_t launch_w_from_split(const uint16_t* hi, const uint16_t* lo, float* W, int64_t J, int64_t D, hipStream_t stream)
{
    if (J <= 0 || D <= 0) return hipSuccess;
    hipLaunchKernelGGL(w_from_split_kernel, dim3(grid_for(J * (D / 8))), dim3(256), 0, stream, hi, lo, W, J, D,
                       bf16_pitch(D), (D + BN - 1) / BN);
    return hipGetLastError();
}

hipError_t launch_apply_bf16(float* W, uint16_t* W_shadow, uint16_t* W_lo, int64_t N, int64_t J, int64_t D, float eta,
                             const void* workspace, DeviceInfo& dev, hipStream_t stream)
{
    if (N <= 0 || J <= 0 || D <= 0) return hipSuccess;
    const int64_t Np = bf16_pitch(N);
    const uint16_t* Ut = static_cast<const uint16_t*>(workspace);
    const uint16_t* Vt = apply_bf16_vt(const_cast<void*>(workspace), N, J);
    Params p = {};
    p.A = Ut; p.lda = Np; p.M = J;
    p.B = Vt; p.ldb = Np; p.N = D;
    p.C = W; p.ldc = D;
    p.shadow = W_shadow; p.ld_shadow = bf16_pitch(D);
    p.K = Np;
    p.eta = eta;
    p.group_m = 8;               // 8 row-tiles x 4 column tiles under one L2 at a time (measured best of 1..32)
    if (W_lo) {
        p.lo = W_lo;
        return launch<MODE_SPLIT>(p, dev, stream);
    }
    return launch<MODE_APPLY>(p, dev, stream);
}

}  // namespace sfb
