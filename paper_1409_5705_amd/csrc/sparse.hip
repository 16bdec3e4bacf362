// Sparse (CSR) samples and second factors: validation, conversion into the
// dense, tile-aligned operand layouts the MFMA contractions read, and a forward
// contraction over the stored non-zeros only.
//
// Two routes for the logits z = W x of samples given as CSR rows:
//   * dense: at about 10 % non-zeros and hundreds of samples every 32-wide block
//     of every operand tile holds non-zeros, so the contraction stays a dense
//     MFMA product; the aligned copy of X is written directly from the CSR rows
//     (csr_scatter_kernel);
//   * gather (csr_forward_kernel): at the densities of tf-idf features (a
//     fraction of a per cent) the MFMA product is almost all multiplications by
//     zero.  Here W is streamed once, a few rows at a time, into LDS with the
//     rows interleaved (one 16-byte word per column holds that column's element
//     of every staged row), each lane owns one sample and walks its stored
//     entries: one LDS read per entry fetches the column for all staged rows.
//     Work is proportional to the number of stored entries times J; the floor is
//     one pass over W.
#include "kernels.h"

namespace sfb {
namespace {

__device__ __forceinline__ uint16_t f32_to_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);                                              // round to nearest even
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// One wavefront per CSR row: dst[r * row_stride + c * col_stride] = value (times
// coef[r] if given).  Entries whose column is outside [0, cols) and row ranges
// outside [0, nnz] are skipped, so malformed input cannot write out of bounds.
template <typename T>
__global__ __launch_bounds__(256) void csr_scatter_kernel(const int64_t* __restrict__ indptr,
                                                          const int32_t* __restrict__ indices,
                                                          const T* __restrict__ values,
                                                          const float* __restrict__ coef, T* __restrict__ dst,
                                                          int64_t rows, int64_t cols, int64_t nnz,
                                                          int64_t row_stride, int64_t col_stride)
{
    const int lane = threadIdx.x & 63;
    const int64_t waves = (int64_t)gridDim.x * 4;
    for (int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); r < rows; r += waves) {
        int64_t lo = indptr[r], hi = indptr[r + 1];
        if (lo < 0) lo = 0;
        if (hi > nnz) hi = nnz;
        const float c = coef ? coef[r] : 1.0f;
        for (int64_t t = lo + lane; t < hi; t += 64) {
            const int64_t col = indices[t];
            if (col < 0 || col >= cols) continue;
            T v = values[t];
            if (coef) {
                if constexpr (sizeof(T) == 2)
                    v = f32_to_bf16(c * bf16_to_f32(v));
                else
                    v = c * v;
            }
            // negative strides: blocks of 256 rows x 64 columns (the operand layout of the bf16 contractions);
            // col_stride = -pitch: the transpose, row_stride = -pitch: the matrix itself
            const int64_t at = col_stride < 0   ? ((col / 256) * (-col_stride / 64) + r / 64) * 16384 + (col % 256) * 64 + r % 64
                               : row_stride < 0 ? ((r / 256) * (-row_stride / 64) + col / 64) * 16384 + (r % 256) * 64 + col % 64
                                                : r * row_stride + col * col_stride;
            dst[at] = v;
        }
    }
}

// Counts violations of the format: indptr[0] == 0, indptr non-decreasing,
// indptr[rows] == nnz, column indices in [0, cols) and strictly increasing
// within a row.
__global__ __launch_bounds__(256) void csr_check_kernel(const int64_t* __restrict__ indptr,
                                                        const int32_t* __restrict__ indices, int64_t rows,
                                                        int64_t cols, int64_t nnz, unsigned int* __restrict__ bad)
{
    const int lane = threadIdx.x & 63;
    const int64_t waves = (int64_t)gridDim.x * 4;
    unsigned int mine = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (indptr[0] != 0) ++mine;
        if (indptr[rows] != nnz) ++mine;
    }
    for (int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); r < rows; r += waves) {
        const int64_t lo = indptr[r], hi = indptr[r + 1];
        if (lo < 0 || hi < lo || hi > nnz) {
            if (lane == 0) ++mine;
            continue;
        }
        for (int64_t t = lo + lane; t < hi; t += 64) {
            const int64_t col = indices[t];
            if (col < 0 || col >= cols) ++mine;
            else if (t > lo && (int64_t)indices[t - 1] >= col) ++mine;
        }
    }
    if (mine) atomicAdd(bad, mine);
}

// ---------------------------------------------------------------------------
// Forward contraction over stored non-zeros.
//
// Samples are taken in groups of 1024 (one workgroup of 256 threads covers a
// group: thread t owns samples 64 (t / 64 + 4 s) + t % 64, s = 0..3), classes in
// groups of 32 (a workgroup produces one 128-byte line of fp32 logits per
// sample), columns in chunks of C = 1024 (bf16) or 512 (fp32): a chunk of all 32
// rows is 64 KB of LDS, laid out per column as NW 16-byte words (word g holds the
// column's element of rows 8 g .. 8 g + 7 in bf16, 4 g .. 4 g + 3 in fp32).
// The CSR rows are first re-laid per (group, chunk, slice of 64 samples): entry t
// of lane l at [t][l], every lane padded to the longest of the slice with entries
// of value zero, so that a wavefront reads its entries with one coalesced load
// per step, once per chunk, and each entry is used for all 32 rows.  An entry
// holds the LDS byte offset of its column's word 0 (gf_word0) and the value.
// ---------------------------------------------------------------------------
constexpr int GF_THREADS = 256;
constexpr int GF_SPT = 4;                        // samples per thread
constexpr int GF_GROUP = GF_THREADS * GF_SPT;    // samples per workgroup pass
constexpr int GF_SLICES = GF_GROUP / 64;         // 64-sample slices per group
constexpr int GF_ROWS = 32;                      // classes per workgroup
constexpr int GF_MAX_CHUNKS = 32;
constexpr int GF_LDS_BYTES = 65536;

// LDS placement of chunk column c.  A column occupies NW consecutive 16-byte words; the staging threads write,
// and the lanes of a gather read, 16 bytes each, a quarter-wave (16 lanes) at a time over a 256-byte window of
// the banks that holds 16 / NW columns.  A staging thread handles G consecutive columns of one word index g, its
// neighbours the next G columns: left alone, the 16 lanes of a write would hit one 16-byte column of the banks.
// So the column's position among the 16 / NW of its window is XORed with the low bits of c / G and the word
// index with the next bits of c / G: 16 neighbouring threads write 16 different bank columns, and random
// gathers spread likewise.  Byte offset of word g of column c: gf_word0(c) ^ (g << 4).
template <int NW, int G>
__device__ __forceinline__ uint32_t gf_word0(uint32_t c)
{
    constexpr uint32_t CPW = 16 / NW;                                   // columns per 256-byte window
    const uint32_t l = c / G;
    const uint32_t col = c ^ (l & (CPW - 1));
    const uint32_t rot = (l / CPW) & (NW - 1);
    return col * (NW * 16u) + rot * 16u;
}

// Pass 1: longest lane of every (group, chunk, slice).  One wavefront per slice, lane = sample.
__global__ __launch_bounds__(256) void csr_slice_count_kernel(const int64_t* __restrict__ indptr,
                                                              const int32_t* __restrict__ indices, int64_t rows,
                                                              int64_t cols, int64_t nnz, int chunk_cols, int nchunks,
                                                              uint32_t* __restrict__ slen)
{
    __shared__ uint32_t cnt[GF_MAX_CHUNKS][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t slice = (int64_t)blockIdx.x * 4 + wave;            // global slice index
    const int64_t r = slice * 64 + lane;
    for (int c = 0; c < nchunks; ++c) cnt[c][threadIdx.x] = 0;
    if (r < rows) {
        int64_t lo = indptr[r], hi = indptr[r + 1];
        if (lo < 0) lo = 0;
        if (hi > nnz) hi = nnz;
        for (int64_t t = lo; t < hi; ++t) {
            const int64_t col = indices[t];
            if (col < 0 || col >= cols) continue;
            cnt[col / chunk_cols][threadIdx.x] += 1;
        }
    }
    if (slice * 64 >= rows) return;                                   // (whole wavefronts leave; no barrier below)
    const int64_t y = slice / GF_SLICES, w = slice % GF_SLICES;
    for (int c = 0; c < nchunks; ++c) {
        uint32_t m = cnt[c][threadIdx.x];
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) {
            const uint32_t other = (uint32_t)__shfl_xor((int)m, o, 64);
            m = other > m ? other : m;
        }
        if (lane == 0) slen[(y * nchunks + c) * GF_SLICES + w] = m;
    }
}

// Pass 2: soff = exclusive prefix sum of slen (units of 64 entries).  One workgroup.
__global__ __launch_bounds__(1024) void csr_slice_scan_kernel(const uint32_t* __restrict__ slen,
                                                              uint32_t* __restrict__ soff, int64_t n)
{
    __shared__ uint32_t part[1024];
    const int tid = threadIdx.x;
    const int64_t per = (n + 1023) / 1024, a = tid * per, b = a + per < n ? a + per : n;
    uint32_t sum = 0;
    for (int64_t i = a; i < b; ++i) sum += slen[i];
    part[tid] = sum;
    __syncthreads();
    if (tid == 0) {
        uint32_t run = 0;
        for (int i = 0; i < 1024; ++i) {
            const uint32_t v = part[i];
            part[i] = run;
            run += v;
        }
    }
    __syncthreads();
    uint32_t run = part[tid];
    for (int64_t i = a; i < b; ++i) {
        soff[i] = run;
        run += slen[i];
    }
}

// Pass 3: the entries.  Same mapping as pass 1; a lane walks its row again and appends to its column of every
// (chunk, slice) block, then pads that column to the block's length with zero entries.
template <bool BF16>
__global__ __launch_bounds__(256) void csr_slice_fill_kernel(const int64_t* __restrict__ indptr,
                                                             const int32_t* __restrict__ indices,
                                                             const void* __restrict__ values, int64_t rows,
                                                             int64_t cols, int64_t nnz, int chunk_cols, int nchunks,
                                                             const uint32_t* __restrict__ slen,
                                                             const uint32_t* __restrict__ soff,
                                                             uint32_t* __restrict__ entries)
{
    __shared__ uint32_t cur[GF_MAX_CHUNKS][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t slice = (int64_t)blockIdx.x * 4 + wave;
    if (slice * 64 >= rows) return;
    const int64_t r = slice * 64 + lane;
    const int64_t y = slice / GF_SLICES, w = slice % GF_SLICES;
    for (int c = 0; c < nchunks; ++c) cur[c][threadIdx.x] = 0;
    constexpr int EW = BF16 ? 1 : 2;                                  // 32-bit words per entry
    if (r < rows) {
        int64_t lo = indptr[r], hi = indptr[r + 1];
        if (lo < 0) lo = 0;
        if (hi > nnz) hi = nnz;
        for (int64_t t = lo; t < hi; ++t) {
            const int64_t col = indices[t];
            if (col < 0 || col >= cols) continue;
            const int c = (int)(col / chunk_cols);
            const uint32_t cc = (uint32_t)(col - (int64_t)c * chunk_cols);
            const uint32_t at = BF16 ? gf_word0<4, 8>(cc) : gf_word0<8, 4>(cc);
            const uint32_t k = cur[c][threadIdx.x]++;
            const int64_t idx = (y * nchunks + c) * GF_SLICES + w;
            const int64_t pos = ((int64_t)soff[idx] + k) * 64 + lane;
            if (BF16) {
                entries[pos] = ((uint32_t)static_cast<const uint16_t*>(values)[t] << 16) | at;      // at < 2^16
            } else {
                entries[2 * pos] = at;
                entries[2 * pos + 1] = __float_as_uint(static_cast<const float*>(values)[t]);
            }
        }
    }
    for (int c = 0; c < nchunks; ++c) {
        const int64_t idx = (y * nchunks + c) * GF_SLICES + w;
        const uint32_t len = slen[idx];
        for (uint32_t k = cur[c][threadIdx.x]; k < len; ++k) {
            const int64_t pos = ((int64_t)soff[idx] + k) * 64 + lane;
            for (int e = 0; e < EW; ++e) entries[EW * pos + e] = 0u;  // value zero at offset 0 of the chunk
        }
    }
}

// z(b, j) = sum over the stored entries (d, x) of sample b of W(j, d) x.
// BF16: W is a bf16 operand in blocks of 256 rows x 64 columns (pitch P, columns D.. zero); products through
//       v_dot2c_f32_bf16 with the other half of the pair zero (bf16 x bf16 is exact in fp32; fp32 accumulation);
//       Z is written as 256 x 256 tiles (tile (b / 256, j / 256) at index (j / 256) * tiles_b + b / 256), the
//       layout the softmax of this path reads.
// fp32: W row-major [J][D], Z row-major [B][J].
template <bool BF16>
__global__ __launch_bounds__(GF_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void csr_forward_kernel(
    const void* __restrict__ Wv, float* __restrict__ Z, const uint32_t* __restrict__ slen,
    const uint32_t* __restrict__ soff, const uint32_t* __restrict__ entries, int64_t B, int64_t J, int64_t D, int64_t P,
    int chunk_cols, int nchunks)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    extern __shared__ u32x4 gf_lds[];                                  // chunk_cols columns of NW words
    char* const lds = reinterpret_cast<char*>(gf_lds);
    constexpr int R = BF16 ? 8 : 4;                                    // rows per 16-byte word
    constexpr int G = BF16 ? 8 : 4;                                    // columns of a 16-byte load from a row of W
    constexpr int NW = GF_ROWS / R;                                    // words per column
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t y = blockIdx.y, jg = (int64_t)blockIdx.x * GF_ROWS;
    float acc[GF_SPT][GF_ROWS];
#pragma unroll
    for (int s = 0; s < GF_SPT; ++s)
#pragma unroll
        for (int i = 0; i < GF_ROWS; ++i) acc[s][i] = 0.f;
    // lengths and offsets of this group's (chunk, slice) blocks: read once, not once per chunk on the critical path
    __shared__ uint32_t s_len[GF_MAX_CHUNKS * GF_SLICES], s_off[GF_MAX_CHUNKS * GF_SLICES];
    for (int i = tid; i < nchunks * GF_SLICES; i += GF_THREADS) {
        s_len[i] = slen[y * nchunks * GF_SLICES + i];
        s_off[i] = soff[y * nchunks * GF_SLICES + i];
    }
    __syncthreads();

    constexpr int TB = BF16 ? 4 : 2, EW = BF16 ? 1 : 2;
    uint32_t len[GF_SPT];
    const uint32_t* ep[GF_SPT];
    uint32_t cur[GF_SPT][TB][EW], nxt[GF_SPT][TB][EW];
    auto fetch = [&](uint32_t t0, uint32_t (*dst)[TB][EW]) {
#pragma unroll
        for (int s = 0; s < GF_SPT; ++s)
#pragma unroll
            for (int u = 0; u < TB; ++u)
#pragma unroll
                for (int k = 0; k < EW; ++k)
                    dst[s][u][k] = t0 + u < len[s] ? ep[s][(int64_t)(t0 + u) * 64 * EW + k] : 0u;   // past the end: value zero
    };

    // Staging tasks of this thread: task n = word g (R rows) x group l (G columns) of a full chunk, the same in
    // every chunk.  task_src: element offset of (first row, first column of the group) in chunk 0; task_rows: how
    // many of the R rows exist; task_dst: LDS byte offset of the group's first column (the G columns of a group
    // are its G consecutive column slots, XORed with the group's position: gf_word0).
    constexpr int FULL = BF16 ? 1024 : 512, GROUPS = FULL / G, NT = GROUPS * NW / GF_THREADS;
    int task_l[NT], task_rows[NT];
    int64_t task_src[NT];
    uint32_t task_dst[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int task = tid + n * GF_THREADS, g = task / GROUPS, l = task % GROUPS;
        const int64_t j = jg + g * R;
        task_l[n] = l;
        task_rows[n] = j >= J ? 0 : (J - j < R ? (int)(J - j) : R);
        task_src[n] = BF16 ? ((j / 256) * (P / 64) + l / 8) * 16384 + (j % 256) * 64 + (l % 8) * 8 : j * D;
        task_dst[n] = gf_word0<NW, G>((uint32_t)(l * G)) ^ ((uint32_t)g << 4);
    }

    for (int c = 0; c < nchunks; ++c) {
        const int64_t c0 = (int64_t)c * chunk_cols;
        int64_t width = P - c0;
        if (width > chunk_cols) width = chunk_cols;
        // the first entries of this chunk are requested before its rows of W, so that both latencies run together
        uint32_t longest = 0;
#pragma unroll
        for (int s = 0; s < GF_SPT; ++s) {
            const int w = wave + 4 * s;
            len[s] = 0;
            ep[s] = entries;
            if ((y * GF_SLICES + w) * 64 < B) {                        // (wave-uniform)
                len[s] = __builtin_amdgcn_readfirstlane(s_len[c * GF_SLICES + w]);
                ep[s] = entries + ((int64_t)__builtin_amdgcn_readfirstlane(s_off[c * GF_SLICES + w]) * 64 + lane) * EW;
            }
            longest = len[s] > longest ? len[s] : longest;
        }
        fetch(0, nxt);
        __syncthreads();                                               // the previous chunk is no longer read
        // ---- stage the 32 rows x `width` columns ----
        // All loads of the thread's NT tasks are issued before the first is used, so that a thread waits out
        // the latency of W (it streams from HBM) once per chunk, not once per task.
#pragma unroll
        for (int n0 = 0; n0 < NT; n0 += 2) {     // (two tasks' rows in registers at a time)
        u32x4 in[NT][R];
#pragma unroll
        for (int n = n0; n < n0 + 2; ++n) {
#pragma unroll
            for (int i = 0; i < R; ++i) {
                in[n][i] = u32x4{0u, 0u, 0u, 0u};
                if (!task_rows[n] || task_l[n] * G >= width) continue;
                if (BF16) {      // the R rows of a word are R consecutive 128-byte lines of one 256 x 64 block
                    in[n][i] = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(Wv) + task_src[n] +
                                                               (int64_t)c * (chunk_cols / 64) * 16384 + i * 64);
                } else {
                    const int64_t col = c0 + task_l[n] * G;
                    const float* Wf = static_cast<const float*>(Wv) + task_src[n] + (i < task_rows[n] ? i : task_rows[n] - 1) * D + col;
                    if (col + 3 < D && (reinterpret_cast<uintptr_t>(Wf) & 15) == 0) {
                        in[n][i] = *reinterpret_cast<const u32x4*>(Wf);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < D) in[n][i][e] = __float_as_uint(Wf[e]);
                    }
                }
            }
        }
#pragma unroll
        for (int n = n0; n < n0 + 2; ++n) {
            if (task_l[n] * G >= width) continue;
#pragma unroll
            for (int e = 0; e < G; ++e) {
                u32x4 out;
                if (BF16) {      // column e of the 8 x 8 block: halves e & 1 of dword e / 2 of every row
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const uint32_t a = in[n][2 * k][e >> 1], b = in[n][2 * k + 1][e >> 1];
                        out[k] = __builtin_amdgcn_perm(b, a, (e & 1) ? 0x07060302u : 0x05040100u);
                    }
                } else {
                    const uint32_t a0 = in[n][0][e], a1 = in[n][1][e], a2 = in[n][2][e], a3 = in[n][3][e];
                    out = u32x4{a0, a1, a2, a3};
                }
                *reinterpret_cast<u32x4*>(lds + (task_dst[n] ^ (uint32_t)(e * NW * 16))) = out;
            }
        }
        }
        __syncthreads();
        // ---- every lane walks the entries of its samples in this chunk ----
        // The thread's four slices advance in lockstep, TB steps at a time, and the entries of the next TB steps
        // are requested before those of the current ones are used: the latency of the entry stream (it comes
        // from the L2) is hidden behind the NW LDS reads and 32 multiply-adds of each entry.
        for (uint32_t t0 = 0; t0 < longest; t0 += TB) {
#pragma unroll
            for (int s = 0; s < GF_SPT; ++s)
#pragma unroll
                for (int u = 0; u < TB; ++u)
#pragma unroll
                    for (int k = 0; k < EW; ++k) cur[s][u][k] = nxt[s][u][k];
            fetch(t0 + TB, nxt);
#pragma unroll
            for (int s = 0; s < GF_SPT; ++s) {
#pragma unroll
                for (int u = 0; u < TB; ++u) {
                    const uint32_t at = BF16 ? (cur[s][u][0] & 0xffffu) : cur[s][u][0];
                    if (BF16) {
                        const uint32_t ew = cur[s][u][0];
                        const bf16x2 xlo = __builtin_bit_cast(bf16x2, ew >> 16);           // [0 : x]
                        const bf16x2 xhi = __builtin_bit_cast(bf16x2, ew & 0xffff0000u);   // [x : 0]
#pragma unroll
                        for (int g = 0; g < NW; ++g) {
                            const u32x4 q = *reinterpret_cast<const u32x4*>(lds + (at ^ ((uint32_t)g << 4)));
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const uint32_t qk = q[k];
                                const bf16x2 wk = __builtin_bit_cast(bf16x2, qk);
                                float& a0 = acc[s][g * R + 2 * k];
                                float& a1 = acc[s][g * R + 2 * k + 1];
                                a0 = __builtin_amdgcn_fdot2_f32_bf16(xlo, wk, a0, false);
                                a1 = __builtin_amdgcn_fdot2_f32_bf16(xhi, wk, a1, false);
                            }
                        }
                    } else {
                        const float x = __uint_as_float(cur[s][u][EW - 1]);
#pragma unroll
                        for (int g = 0; g < NW; ++g) {
                            const u32x4 q = *reinterpret_cast<const u32x4*>(lds + (at ^ ((uint32_t)g << 4)));
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const uint32_t qk = q[k];
                                acc[s][g * R + k] = __builtin_fmaf(x, __uint_as_float(qk), acc[s][g * R + k]);
                            }
                        }
                    }
                }
            }
        }
    }
    // ---- store: 32 consecutive classes (one 128-byte line) of each of the thread's samples ----
    // A lane holds a whole line; stored from there, a wavefront's store would touch 64 lines with 16 bytes each.
    // The lines of a slice go through LDS instead (rows padded to 144 bytes: conflict-free both ways), so that 8
    // neighbouring lanes store one line together.
    __syncthreads();                                                   // the last chunk is no longer read
    char* const mine = lds + wave * (64 * 144);
#pragma unroll
    for (int s = 0; s < GF_SPT; ++s) {
#pragma unroll
        for (int i = 0; i < GF_ROWS; i += 4)
            *reinterpret_cast<u32x4*>(mine + lane * 144 + i * 4) =
                u32x4{__float_as_uint(acc[s][i]), __float_as_uint(acc[s][i + 1]), __float_as_uint(acc[s][i + 2]),
                      __float_as_uint(acc[s][i + 3])};
        __syncthreads();
        const int64_t b0 = (y * GF_SLICES + wave + 4 * s) * 64;
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int r = it * 8 + (lane >> 3), part = lane & 7;
            const int64_t b = b0 + r, j = jg + part * 4;
            const u32x4 v = *reinterpret_cast<const u32x4*>(mine + r * 144 + part * 16);
            if (b >= B || j >= J) continue;
            if (BF16) {      // J % 8 == 0 on this path: groups of four classes are inside or outside
                float* zt = Z + ((jg / 256) * ((B + 255) / 256) + b / 256) * 65536 + (b % 256) * 256 + jg % 256 + part * 4;
                *reinterpret_cast<u32x4*>(zt) = v;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (j + e < J) Z[b * J + j + e] = __uint_as_float(v[e]);
            }
        }
        __syncthreads();
    }
}

unsigned wave_grid(int64_t rows)
{
    int64_t g = (rows + 3) / 4;
    if (g > 65536) g = 65536;
    return (unsigned)(g < 1 ? 1 : g);
}

}  // namespace

hipError_t launch_csr_scatter(const int64_t* indptr, const int32_t* indices, const void* values, bool bf16,
                              const float* coef, void* dst, int64_t rows, int64_t cols, int64_t nnz,
                              int64_t row_stride, int64_t col_stride, hipStream_t stream)
{
    if (rows <= 0 || nnz <= 0) return hipSuccess;
    if (bf16)
        hipLaunchKernelGGL((csr_scatter_kernel<uint16_t>), dim3(wave_grid(rows)), dim3(256), 0, stream, indptr, indices,
                           static_cast<const uint16_t*>(values), coef, static_cast<uint16_t*>(dst), rows, cols, nnz,
                           row_stride, col_stride);
    else
        hipLaunchKernelGGL((csr_scatter_kernel<float>), dim3(wave_grid(rows)), dim3(256), 0, stream, indptr, indices,
                           static_cast<const float*>(values), coef, static_cast<float*>(dst), rows, cols, nnz,
                           row_stride, col_stride);
    return hipGetLastError();
}

// Columns per LDS chunk and number of chunks for rows of P staged columns.
static void gather_chunks(int64_t P, bool bf16, int* chunk_cols, int* nchunks)
{
    // all 32 rows of a chunk in 64 KB of LDS: 1024 columns of bf16, 512 of fp32; chunks of equal width
    const int64_t blocks = (P + 63) / 64, max_blocks = (bf16 ? 1024 : 512) / 64;
    const int64_t n = (blocks + max_blocks - 1) / max_blocks;
    *nchunks = (int)n;
    *chunk_cols = (int)((blocks + n - 1) / n * 64);
}

bool csr_gather_supported(int64_t B, int64_t J, int64_t D)
{
    if (B <= 0 || J <= 0 || D <= 0) return false;
    int cc, nc;
    gather_chunks((D + 63) / 64 * 64, false, &cc, &nc);               // (the fp32 chunks are the smaller ones)
    const int64_t groups = (B + GF_GROUP - 1) / GF_GROUP;
    return nc <= GF_MAX_CHUNKS && groups <= 65535 && (J + GF_ROWS - 1) / GF_ROWS <= 0x7fffffffLL &&
           ((B + 63) / 64) * ((D + 63) / 64 * 64) < (1LL << 31);      // 32-bit offsets in units of 64 entries
}

int64_t csr_gather_workspace_bytes(int64_t B, int64_t D, bool bf16)
{
    int cc, nc;
    const int64_t P = (D + 63) / 64 * 64;
    gather_chunks(P, bf16, &cc, &nc);
    const int64_t n_sl = (B + GF_GROUP - 1) / GF_GROUP * nc * GF_SLICES;
    const int64_t lens = (n_sl * 4 + 255) / 256 * 256;
    // every (chunk, slice) block is padded to its longest lane: at most every column of the chunk
    const int64_t ent = ((B + 63) / 64) * 64 * P * (bf16 ? 4 : 8);
    return 2 * lens + ent;
}

hipError_t launch_csr_forward_gather(const int64_t* indptr, const int32_t* indices, const void* values, bool bf16,
                                     const void* W, float* Z, int64_t B, int64_t J, int64_t D, int64_t nnz,
                                     void* workspace, hipStream_t stream)
{
    if (B <= 0 || J <= 0) return hipSuccess;
    if (!csr_gather_supported(B, J, D)) return hipErrorInvalidValue;
    int cc, nc;
    const int64_t P = (D + 63) / 64 * 64;
    gather_chunks(P, bf16, &cc, &nc);
    const int64_t groups = (B + GF_GROUP - 1) / GF_GROUP, n_sl = groups * nc * GF_SLICES;
    const int64_t lens = (n_sl * 4 + 255) / 256 * 256;
    uint32_t* slen = static_cast<uint32_t*>(workspace);
    uint32_t* soff = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + lens);
    uint32_t* entries = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + 2 * lens);
    const unsigned sgrid = (unsigned)(((B + 63) / 64 + 3) / 4);
    hipError_t e = launch_fill_u32(slen, 0u, n_sl, stream);            // slices past the last sample have length 0
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(csr_slice_count_kernel, dim3(sgrid), dim3(256), 0, stream, indptr, indices, B, D, nnz, cc, nc, slen);
    hipLaunchKernelGGL(csr_slice_scan_kernel, dim3(1), dim3(1024), 0, stream, slen, soff, n_sl);
    const dim3 grid((unsigned)((J + GF_ROWS - 1) / GF_ROWS), (unsigned)groups);
    size_t lds = (size_t)cc * (bf16 ? 64 : 128);                       // the chunk; the logits of four slices on the way out
    if (lds < 4 * 64 * 144) lds = 4 * 64 * 144;
    if (bf16) {
        hipLaunchKernelGGL((csr_slice_fill_kernel<true>), dim3(sgrid), dim3(256), 0, stream, indptr, indices, values, B,
                           D, nnz, cc, nc, slen, soff, entries);
        hipLaunchKernelGGL((csr_forward_kernel<true>), grid, dim3(GF_THREADS), lds, stream, W, Z, slen, soff, entries, B, J,
                           D, P, cc, nc);
    } else {
        hipLaunchKernelGGL((csr_slice_fill_kernel<false>), dim3(sgrid), dim3(256), 0, stream, indptr, indices, values, B,
                           D, nnz, cc, nc, slen, soff, entries);
        hipLaunchKernelGGL((csr_forward_kernel<false>), grid, dim3(GF_THREADS), lds, stream, W, Z, slen, soff, entries, B, J,
                           D, P, cc, nc);
    }
    return hipGetLastError();
}

hipError_t launch_csr_check(const int64_t* indptr, const int32_t* indices, int64_t rows, int64_t cols, int64_t nnz,
                            unsigned int* bad, hipStream_t stream)
{
    hipLaunchKernelGGL(csr_check_kernel, dim3(wave_grid(rows)), dim3(256), 0, stream, indptr, indices, rows, cols, nnz,
                       bad);
    return hipGetLastError();
}

}  // namespace sfb
