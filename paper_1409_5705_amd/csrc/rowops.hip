// Row-wise and elementwise kernels around the GEMMs: the softmax/label step of
// multiclass logistic regression, the pair difference and hinge coefficient of
// distance metric learning, the power iteration and the row projection of
// sparse coding.  All are HBM-bound streaming kernels with wavefront (64-lane)
// shuffle reductions.
#include "kernels.h"

namespace sfb {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
// Block reductions; `sm` has NT/64 floats.  Every thread gets the result.
template <int NT>
__device__ __forceinline__ float block_sum(float v, float* sm)
{
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = 0.f;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) r += sm[w];
    return r;
}
template <int NT>
__device__ __forceinline__ float block_max(float v, float* sm)
{
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = sm[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) r = fmaxf(r, sm[w]);
    return r;
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    floatx2 f = {a, b};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
}

// ---------------------------------------------------------------------------
// MLR: u = softmax(z) - onehot(y).  One workgroup per sample; two passes over
// the row: (1) running maximum and sum of exponentials together (the sum is
// rescaled whenever the maximum grows), read from HBM; (2) normalise + label +
// store, re-read from L2 (a row of the headline size is 1.3 MB).  Four 16-byte
// loads per thread are in flight in both passes.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void online_update(float& m, float& s, const floatx4 v)
{
    const float mn = fmaxf(fmaxf(m, fmaxf(v[0], v[1])), fmaxf(v[2], v[3]));
    s = s * expf(m - mn) + ((expf(v[0] - mn) + expf(v[1] - mn)) + (expf(v[2] - mn) + expf(v[3] - mn)));
    m = mn;
}

// tiles_m > 0: Z is not row-major but an array of 256 x 256 tiles, tile (row / 256, j / 256) at index
// (j / 256) * tiles_m + row / 256 (the layout the bf16 forward contraction writes: one piece per workgroup).
template <int NT, bool OUT_BF16>
__global__ __launch_bounds__(NT) void mlr_softmax_kernel(const float* __restrict__ Z, const int32_t* __restrict__ y,
                                                         void* __restrict__ Uv, int64_t J, int vec, int64_t tiles_m)
{
    __shared__ float sm[NT / 64];
    const int64_t row = blockIdx.x;
    const bool blocked = tiles_m > 0;
    const float* z = blocked ? Z + (row / 256) * 65536 + (row % 256) * 256 : Z + row * J;
    const int64_t tile_stride = tiles_m * 65536;          // floats from a tile to the next one along j
    struct View {   // logits of this row by class index (at1) or by group of four classes (at4)
        const float* z;
        int64_t ts;
        bool blocked;
        __device__ floatx4 at4(int64_t q) const
        {
            const int64_t o = blocked ? (q >> 6) * (ts >> 2) + (q & 63) : q;
            return reinterpret_cast<const floatx4*>(z)[o];
        }
        __device__ float at1(int64_t j) const { return z[blocked ? (j >> 8) * ts + (j & 255) : j]; }
    };
    const View zv = {z, tile_stride, blocked};
    const int tid = threadIdx.x;
    const int64_t J4 = vec ? J / 4 : 0;

    float m = -INFINITY, s = 0.f;
    int64_t q = tid;
    for (; q + 3 * NT < J4; q += 4 * NT) {
        const floatx4 a = zv.at4(q), b = zv.at4(q + NT), c = zv.at4(q + 2 * NT), d = zv.at4(q + 3 * NT);
        online_update(m, s, a);
        online_update(m, s, b);
        online_update(m, s, c);
        online_update(m, s, d);
    }
    for (; q < J4; q += NT) online_update(m, s, zv.at4(q));
    for (int64_t j = J4 * 4 + tid; j < J; j += NT) {
        const float v = zv.at1(j), mn = fmaxf(m, v);
        s = s * expf(m - mn) + expf(v - mn);
        m = mn;
    }
    // (a thread that saw no element has m = -inf, s = 0: its term is 0 * exp(-inf) = 0)
    const float M = block_max<NT>(m, sm);
    s = block_sum<NT>(s * expf(m - M), sm);
    const float inv = 1.0f / s;

    const int64_t lab = y[row];
    auto emit = [&](int64_t qq, const floatx4 v) {
        floatx4 p;
#pragma unroll
        for (int e = 0; e < 4; ++e) p[e] = expf(v[e] - M) * inv - ((qq * 4 + e == lab) ? 1.0f : 0.0f);
        if (OUT_BF16) {
            uint2 o;
            o.x = pack_bf16(p[0], p[1]);
            o.y = pack_bf16(p[2], p[3]);
            reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(Uv) + row * J)[qq] = o;
        } else {
            reinterpret_cast<floatx4*>(reinterpret_cast<float*>(Uv) + row * J)[qq] = p;
        }
    };
    q = tid;
    for (; q + 3 * NT < J4; q += 4 * NT) {
        const floatx4 a = zv.at4(q), b = zv.at4(q + NT), c = zv.at4(q + 2 * NT), d = zv.at4(q + 3 * NT);
        emit(q, a);
        emit(q + NT, b);
        emit(q + 2 * NT, c);
        emit(q + 3 * NT, d);
    }
    for (; q < J4; q += NT) emit(q, zv.at4(q));
    for (int64_t j = J4 * 4 + tid; j < J; j += NT) {
        const float p = expf(zv.at1(j) - M) * inv - ((j == lab) ? 1.0f : 0.0f);
        if (OUT_BF16) {
            reinterpret_cast<uint16_t*>(Uv)[row * J + j] = (uint16_t)(pack_bf16(p, 0.f) & 0xffffu);
        } else {
            reinterpret_cast<float*>(Uv)[row * J + j] = p;
        }
    }
}

// ---------------------------------------------------------------------------
// The same for long rows of tile-blocked logits, reading them once.  A row of
// the headline size (1.3 MB) outlives every cache between the two passes above,
// so the second pass is a second trip to memory.  Here CL workgroups share a
// row: each keeps its 1/CL of the row in registers (up to CHUNKS x 16 bytes a
// thread), reduces it to (max, sum of exponentials relative to that max),
// publishes the pair in one 64-bit word and collects the CL words of the row;
// the stored values become exp(z - max_own) and are rescaled on output.
//
// The grid is one workgroup per CU (1024 threads at no more than 128 registers), so
// the CL partners of a row normally run at the same time, and they execute the
// same number of row iterations.  Nothing depends on that, though: the wait for a
// partner's word is bounded (spin_limit polls), and a workgroup whose partner has
// not published in time (kernels of other streams can keep it off the chip)
// computes that partner's pair itself from the logits, and no longer waits for that
// partner in later rows.  So every workgroup finishes whatever the others do; the
// price of a missing partner is reading its part of the row a second time.
// `slots`: [B][CL] 64-bit words, all zero before the launch (a published word
// has a non-zero high half: the bits of a sum that is at least 1).
// ---------------------------------------------------------------------------
constexpr int CLUSTER_CHUNKS = 10;        // 16-byte chunks of a row per thread
// Cache policy of the logits read and of the factors written here: non-temporal, both are touched once (measured
// at the headline size, interleaved: 0.460 -> 0.434 ms; with only the loads non-temporal the transposes that read
// the factors next slow down by as much, with both they do not).
constexpr int STREAM_POLICY = 2;
// partner pairs computed by the waiting workgroup itself (one count per workgroup, row and partner)
__device__ unsigned long long g_softmax_fallbacks = 0;

__global__ __launch_bounds__(1024) void mlr_softmax_cluster_kernel(const float* __restrict__ Z,
                                                                  const int32_t* __restrict__ y,
                                                                  uint16_t* __restrict__ U, int64_t B, int64_t J,
                                                                  int64_t tiles_m, int CL, int tiles_per_wg,
                                                                  unsigned long long* __restrict__ slots, int spin_limit)
{
    constexpr int NT = 1024, R = CLUSTER_CHUNKS;
    __shared__ float sm[NT / 64];
    __shared__ float part_m[32], part_s[32];
    __shared__ int part_ok[32], gone[32];       // gone: partners this workgroup has stopped waiting for
    if (threadIdx.x < 32) gone[threadIdx.x] = 0;
    const int tid = threadIdx.x;
    const int groups = (int)gridDim.x / CL, grp = (int)blockIdx.x / CL, w = (int)blockIdx.x % CL;
    if (grp >= groups) return;                      // (a grid that is not a multiple of CL: the rest has no row)
    const int64_t tn = (J + 255) / 256;
    const int64_t t0 = (int64_t)w * tiles_per_wg;
    int64_t t1 = t0 + tiles_per_wg;
    if (t1 > tn) t1 = tn;
    const int64_t my_chunks = t1 > t0 ? (t1 - t0) * 64 : 0;      // 64 chunks of four classes per tile row

    // Chunk i of this thread: tile t0 + 16 i + tid / 64, classes 4 (tid % 64) .. + 3 of it.  Addresses are a
    // uniform part (row, i) plus a 32-bit part of the thread; which chunks exist does not depend on the row.
    const uint32_t t_tile = (uint32_t)tid >> 6, t_col = ((uint32_t)tid & 63u) * 4u;
    const uint32_t z_thread = t_tile * (uint32_t)(tiles_m * 65536) + t_col;        // floats; B <= 65536 (host check): < 2^28
    const uint32_t j_thread = t_tile * 256u + t_col;
    const int64_t z_step = 16 * tiles_m * 65536;                                   // floats from chunk i to i + 1
    uint32_t have = 0;
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int64_t c = (int64_t)i * NT + tid;
        if (c < my_chunks && (t0 + (c >> 6)) * 256 + (c & 63) * 4 < J) have |= 1u << i;
    }
    // (buffer accesses: a uniform 64-bit base in scalar registers plus one 32-bit offset register per thread,
    // instead of a 64-bit address pair per chunk)
    auto rsrc = [](const void* base) {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0xffffffff, 0x00020000);
    };
    auto load_row = [&](int64_t row, floatx4* v) {
        const float* base = Z + (row / 256) * 65536 + (row % 256) * 256 + t0 * tiles_m * 65536;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            v[i] = floatx4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            if (have & (1u << i)) {
                const u32x4 r = __builtin_amdgcn_raw_buffer_load_b128(rsrc(base + i * z_step), z_thread * 4u, 0, STREAM_POLICY);
                const uint32_t r0 = r[0], r1 = r[1], r2 = r[2], r3 = r[3];
                v[i] = floatx4{__uint_as_float(r0), __uint_as_float(r1), __uint_as_float(r2), __uint_as_float(r3)};
            }
        }
    };

    floatx4 v[R], vn[R];
    int64_t row = grp;
    if (row < B) load_row(row, v);
    for (; row < B; row += groups) {
        // own part: maximum, then exponentials relative to it (kept in v) and their sum
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < R; ++i) m = fmaxf(m, fmaxf(fmaxf(v[i][0], v[i][1]), fmaxf(v[i][2], v[i][3])));
        const float m_own = block_max<NT>(m, sm);
        // (2^(z log2 e - m log2 e) through the hardware exponential: one multiply-add and one v_exp per class instead
        // of the library routine's dozen instructions, which made this kernel ALU-bound; the result differs from
        // exp(z - m) by a few 1e-6 relative for |m| up to 60, far below the bf16 spacing of the output)
        const float LOG2E = 1.4426950408889634f;
        const float mb = -m_own * LOG2E;
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < R; ++i) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[i][e] = m_own == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(__builtin_fmaf(v[i][e], LOG2E, mb));
                s += v[i][e];
            }
        }
        float s_own = block_sum<NT>(s, sm);
        if (m_own == -INFINITY) s_own = 1.0f;       // no class at all in this part: counts as 1 * exp(-inf) = 0
        if (tid == 0) {
            const unsigned long long word = ((unsigned long long)__float_as_uint(s_own) << 32) | __float_as_uint(m_own);
            __hip_atomic_store(&slots[row * CL + w], word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // the next row's loads travel while the partners' words are awaited and this row is written
        const int64_t next = row + groups;
        if (next < B) load_row(next, vn);
        if (tid < CL) {
            if (tid == w) {
                part_m[tid] = m_own;
                part_s[tid] = s_own;
                part_ok[tid] = 1;
            } else {
                unsigned long long word = 0;
                const int polls = gone[tid] ? 1 : spin_limit;
                for (int spin = 0; spin < polls; ++spin) {
                    word = __hip_atomic_load(&slots[row * CL + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (word >> 32) break;
                    __builtin_amdgcn_s_sleep(8);
                }
                const int ok = (word >> 32) != 0;
                part_m[tid] = __uint_as_float((uint32_t)word);
                part_s[tid] = __uint_as_float((uint32_t)(word >> 32));
                part_ok[tid] = ok;
                if (!ok) gone[tid] = 1;
            }
        }
        __syncthreads();
        for (int k = 0; k < CL; ++k) {
            if (part_ok[k]) continue;               // (the same for every thread: read from LDS after the barrier)
            // partner k has not published: its pair from the logits themselves
            const int64_t k0 = (int64_t)k * tiles_per_wg;
            int64_t k1 = k0 + tiles_per_wg;
            if (k1 > tn) k1 = tn;
            const float* base = Z + (row / 256) * 65536 + (row % 256) * 256;
            float mk = -INFINITY, sk = 0.f;
            for (int64_t c = tid; c < (k1 - k0) * 64; c += NT) {
                const int64_t tile = k0 + (c >> 6);
                if (tile * 256 + (c & 63) * 4 < J)
                    online_update(mk, sk, *reinterpret_cast<const floatx4*>(base + tile * tiles_m * 65536 + (c & 63) * 4));
            }
            const float Mk = block_max<NT>(mk, sm);
            float Sk = block_sum<NT>(mk == -INFINITY ? 0.f : sk * expf(mk - Mk), sm);
            if (Mk == -INFINITY) Sk = 1.0f;
            if (tid == 0) {
                part_m[k] = Mk;
                part_s[k] = Sk;
                atomicAdd(&g_softmax_fallbacks, 1ull);
            }
            __syncthreads();
        }
        float M = part_m[0];
        for (int k = 1; k < CL; ++k) M = fmaxf(M, part_m[k]);
        float S = 0.f;
        for (int k = 0; k < CL; ++k) S += part_s[k] * expf(part_m[k] - M);
        const float scale = expf(m_own - M) / S;

        const int64_t out0 = row * J + t0 * 256;          // U index of class t0 * 256 of this row
        // the label relative to this thread's first class of chunk 0 (|.| < 2^31: labels and J are 32-bit)
        const int32_t lab_t = (int32_t)((int64_t)y[row] - t0 * 256) - (int32_t)j_thread;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            if (have & (1u << i)) {
                floatx4 p = v[i] * scale;
                const uint32_t at = (uint32_t)(lab_t - i * 4096);      // 0..3: the label is one of these four
                if (at < 4u) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) p[e] -= (at == (uint32_t)e) ? 1.0f : 0.0f;
                }
                const u32x2 o = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3])};
                __builtin_amdgcn_raw_buffer_store_b64(o, rsrc(U + out0 + i * 4096), j_thread * 2u, 0, STREAM_POLICY);
            }
        }
#pragma unroll
        for (int i = 0; i < R; ++i) v[i] = vn[i];
        __syncthreads();                            // part_m / part_s are rewritten in the next iteration
    }
}

// V = X - Y; also clears *counter (nullable): the count of active pairs a later kernel of the same call adds to.
__global__ __launch_bounds__(256) void diff_kernel(const float* __restrict__ X, const float* __restrict__ Y,
                                                   float* __restrict__ V, int64_t n, int32_t* __restrict__ counter)
{
    if (counter && blockIdx.x == 0 && threadIdx.x == 0) *counter = 0;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) V[i] = X[i] - Y[i];
}

__global__ __launch_bounds__(256) void scale_rows_kernel(const float* __restrict__ V, const float* __restrict__ coef,
                                                         float* __restrict__ Vs, int64_t N, int64_t D)
{
    const int64_t total = N * D, stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) Vs[i] = coef[i / D] * V[i];
}

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t* __restrict__ p, uint32_t value, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) p[i] = value;
}

// W = Z / lambda: the primal matrix from the auxiliary one for the squared l2
// regulariser (W = grad h^*(Z), Section 2.1, Stochastic DCA).
__global__ __launch_bounds__(256) void div_scalar_kernel(const float* __restrict__ Z, float* __restrict__ W,
                                                         float lambda, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) W[i] = Z[i] / lambda;
}

// w > 0 with w + log w = L (w = W0(e^L), the principal Lambert function).  The
// start is a lower bound of the root (e^L / (1 + e^L) for L < 1, L - log L
// otherwise), from which Newton's iteration on the concave left side rises
// monotonically; three steps reach fp32 accuracy over the whole range, four are
// taken.  Below L = -15 the series w = y - y^2 of y = e^L is exact in fp32.
__device__ __forceinline__ float lambert_w_exp(float L)
{
    if (L < -15.f) {
        const float y = expf(L);
        return y - y * y;
    }
    float w;
    if (L >= 1.f) {
        w = L - __logf(L);
    } else {
        const float y = __expf(L);
        w = y / (1.f + y);
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) w = w * (1.f + L - logf(w)) / (1.f + w);
    return w;
}

// Dual coordinate step of l2-regularised multiclass logistic regression, one
// workgroup per sample.  With z = W a_i (the row of Zl), c = ||a_i||^2 / (lambda N)
// and the sample's dual point p_old in the simplex, the minimiser p of the dual
// over this sample's variable solves
//     log p_j + c p_j = z_j + c p_old_j - nu  (every class j),   sum_j p_j = 1.
// Each class equation is p_j = W0(c e^{t_j}) / c; sum_j p_j is decreasing in nu
// and the root lies in [lse(theta) - c, lse(theta)], theta = z + c p_old.  nu is
// found by Newton's iteration on log(sum p) kept inside that bracket (bisection
// when a step leaves it).  Outputs: dU = beta (p - p_old), P += dU.
__global__ __launch_bounds__(256) void sdca_mlr_kernel(const float* __restrict__ Zl, const float* __restrict__ X,
                                                       float* __restrict__ P, float* __restrict__ dU, int64_t J,
                                                       int64_t D, float inv_lambda_n, float beta)
{
    __shared__ float sm[4];
    const int64_t i = blockIdx.x;
    const float* z = Zl + i * J;
    float* p_old = P + i * J;
    float* du = dU + i * J;
    const int tid = threadIdx.x;

    float acc = 0.f;
    for (int64_t d = tid; d < D; d += 256) {
        const float x = X[i * D + d];
        acc += x * x;
    }
    const float c = block_sum<256>(acc, sm) * inv_lambda_n;

    float m = -INFINITY;
    for (int64_t j = tid; j < J; j += 256) m = fmaxf(m, z[j] + c * p_old[j]);
    m = block_max<256>(m, sm);
    float s = 0.f;
    for (int64_t j = tid; j < J; j += 256) s += expf(z[j] + c * p_old[j] - m);
    s = block_sum<256>(s, sm);
    const float lse = m + logf(s);

    if (!(c > 1e-30f)) {   // a zero sample: the class equations decouple, p = softmax(z)
        for (int64_t j = tid; j < J; j += 256) {
            const float po = p_old[j], d = beta * (expf(z[j] - lse) - po);
            du[j] = d;
            p_old[j] = po + d;
        }
        return;
    }
    const float logc = logf(c), inv_c = 1.f / c;
    float lo = lse - c, hi = lse, nu = lo;
    for (int it = 0; it < 32; ++it) {
        float S = 0.f, T = 0.f;
        for (int64_t j = tid; j < J; j += 256) {
            const float w = lambert_w_exp(logc + (z[j] + c * p_old[j] - nu));
            S += w;                 // c p_j
            T += w / (1.f + w);     // c p_j / (1 + c p_j)
        }
        S = block_sum<256>(S, sm) * inv_c;
        T = block_sum<256>(T, sm) * inv_c;
        if (fabsf(S - 1.f) <= 1e-6f) break;          // (every thread holds the same S: a uniform exit)
        if (S > 1.f) lo = nu; else hi = nu;
        float cand = nu + S * logf(S) / T;
        if (!(cand > lo && cand < hi)) cand = 0.5f * (lo + hi);
        if (cand == nu) break;                        // bracket exhausted at fp32 resolution
        nu = cand;
    }
    for (int64_t j = tid; j < J; j += 256) {
        const float po = p_old[j];
        const float p = lambert_w_exp(logc + (z[j] + c * po - nu)) * inv_c;
        const float d = beta * (p - po);
        du[j] = d;
        p_old[j] = po + d;
    }
}

// DML: one workgroup per pair.
__global__ __launch_bounds__(256) void dml_scale_kernel(const float* __restrict__ Q, const int8_t* __restrict__ sim,
                                                        float* __restrict__ U, int32_t* __restrict__ n_active,
                                                        float margin, int64_t K)
{
    __shared__ float sm[4];
    const int64_t row = blockIdx.x;
    const float* q = Q + row * K;
    float d = 0.f;
    for (int64_t k = threadIdx.x; k < K; k += 256) d += q[k] * q[k];
    d = block_sum<256>(d, sm);
    float c;
    if (sim[row] > 0)
        c = 2.0f;
    else
        c = (d < margin) ? -2.0f : 0.0f;
    for (int64_t k = threadIdx.x; k < K; k += 256) U[row * K + k] = c * q[k];
    if (threadIdx.x == 0 && c != 0.0f && n_active) atomicAdd(n_active, 1);
}

// Prox of the unit-ball constraint on each row.
__global__ __launch_bounds__(256) void prox_rows_kernel(float* __restrict__ W, int64_t D, int mode)
{
    __shared__ float sm[4];
    float* w = W + (int64_t)blockIdx.x * D;
    float nn = 0.f;
    for (int64_t d = threadIdx.x; d < D; d += 256) nn += w[d] * w[d];
    nn = block_sum<256>(nn, sm);
    const float nrm = sqrtf(nn);
    const bool scale = (mode == 0) ? (nrm > 1.0f) : (nrm > 0.0f);
    if (scale)
        for (int64_t d = threadIdx.x; d < D; d += 256) w[d] = w[d] / nrm;
}

// ---------------------------------------------------------------------------
// Power iteration on W^T W: two kernels per iteration, W read from memory once.
// ---------------------------------------------------------------------------
// One workgroup per chunk of `rows` rows of W.  With b = g / ||g|| (g the raw vector of the previous iteration;
// every workgroup takes the norm itself while it reads g anyway):
//   c_j = W_j . b  for its rows (one wavefront per row at a time), then
//   part[chunk][d] = sum over its rows of W[j][d] c_j   (the rows come from the cache the second time).
constexpr int POWER_MAX_ROWS = 1024;
__global__ __launch_bounds__(256) void power_step_kernel(const float* __restrict__ W, const float* __restrict__ g,
                                                         float* __restrict__ part, int64_t J, int64_t D, int rows)
{
    __shared__ float sm[16];
    __shared__ float c[POWER_MAX_ROWS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float nn = 0.f;
    for (int64_t d = tid; d < D; d += 256) nn += g[d] * g[d];
    const float inv = 1.0f / sqrtf(block_sum<256>(nn, sm));
    const int64_t j0 = (int64_t)blockIdx.x * rows;
    for (int r = wave; r < rows; r += 4) {
        const int64_t j = j0 + r;
        float s = 0.f;
        if (j < J)
            for (int64_t d = lane; d < D; d += 64) s += W[j * D + d] * g[d];
        s = wave_sum(s);
        if (lane == 0) c[r] = s * inv;
    }
    __syncthreads();
    const int64_t j1 = j0 + rows < J ? j0 + rows : J;
    for (int64_t d = tid; d < D; d += 256) {
        float s = 0.f;
        for (int64_t j = j0; j < j1; ++j) s += W[j * D + d] * c[j - j0];
        part[(int64_t)blockIdx.x * D + d] = s;
    }
}
// The same for rows of at most 1024 floats, 16-byte aligned (D % 4 == 0): a workgroup keeps its 16 rows in
// registers (thread t holds columns 4 t .. 4 t + 3 of every row: one 16-byte load per row, all in flight
// together), so W is read once and nothing waits on a chain of dependent loads.
__global__ __launch_bounds__(256) void power_step16_kernel(const float* __restrict__ W, const float* __restrict__ g,
                                                           float* __restrict__ part, int64_t J, int64_t D)
{
    __shared__ float sm[16];
    __shared__ float cw[16][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t d0 = 4 * (int64_t)tid, j0 = (int64_t)blockIdx.x * 16;
    const bool have = d0 < D;
    floatx4 w[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        w[r] = floatx4{0.f, 0.f, 0.f, 0.f};
        if (have && j0 + r < J) w[r] = *reinterpret_cast<const floatx4*>(W + (j0 + r) * D + d0);
    }
    floatx4 g4 = {0.f, 0.f, 0.f, 0.f};
    if (have) g4 = *reinterpret_cast<const floatx4*>(g + d0);
    const float inv = 1.0f / sqrtf(block_sum<256>(g4[0] * g4[0] + g4[1] * g4[1] + g4[2] * g4[2] + g4[3] * g4[3], sm));
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float s = wave_sum(w[r][0] * g4[0] + w[r][1] * g4[1] + w[r][2] * g4[2] + w[r][3] * g4[3]);
        if (lane == 0) cw[r][wave] = s;
    }
    __syncthreads();
    floatx4 out = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float c = (((cw[r][0] + cw[r][1]) + cw[r][2]) + cw[r][3]) * inv;
        out += w[r] * c;
    }
    if (have) *reinterpret_cast<floatx4*>(part + (int64_t)blockIdx.x * D + d0) = out;
}
// g[d] = sum of the chunks' partials in a fixed order: 16 columns a workgroup, 16 interleaved groups of chunks
// per column (eight loads in flight per thread), combined in order.
__global__ __launch_bounds__(256) void power_reduce_kernel(const float* __restrict__ part, float* __restrict__ g,
                                                           int64_t D, int64_t chunks)
{
    __shared__ float sm[16][17];
    const int col = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int64_t d = (int64_t)blockIdx.x * 16 + col;
    float s = 0.f;
    if (d < D) {
        int64_t ch = grp;
        for (; ch + 7 * 16 < chunks; ch += 8 * 16) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = part[(ch + 16 * u) * D + d];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; ch < chunks; ch += 16) s += part[ch * D + d];
    }
    sm[grp][col] = s;
    __syncthreads();
    if (grp == 0 && d < D) {
        float t = sm[0][col];
#pragma unroll
        for (int k = 1; k < 16; ++k) t += sm[k][col];
        g[d] = t;
    }
}
// L = ||g||.  One workgroup.
__global__ __launch_bounds__(1024) void vec_norm_kernel(const float* __restrict__ g, float* __restrict__ L_out, int64_t D)
{
    __shared__ float sm[16];
    float nn = 0.f;
    for (int64_t d = threadIdx.x; d < D; d += 1024) nn += g[d] * g[d];
    nn = block_sum<1024>(nn, sm);
    if (threadIdx.x == 0) L_out[0] = sqrtf(nn);
}

unsigned grid_for(int64_t n)
{
    int64_t g = (n + 255) / 256;
    if (g > 65536) g = 65536;
    if (g < 1) g = 1;
    return (unsigned)g;
}

}  // namespace

// Cluster size of the one-read softmax for rows of J classes (tile-blocked logits), or 0 where the two-pass
// kernel is used: short rows (the second pass then comes from the L2), J not a multiple of 4, rows too long for
// 32 workgroups to hold.
static int softmax_cluster(int64_t J)
{
    if (J < 65536 || J % 4 != 0) return 0;
    const int64_t tn = (J + 255) / 256, per_wg = CLUSTER_CHUNKS * 1024 / 64;      // tile rows one workgroup holds
    for (int cl = 2; cl <= 32; cl *= 2)
        if ((tn + cl - 1) / cl <= per_wg) return cl;
    return 0;
}

hipError_t softmax_fallbacks(unsigned long long* count)
{
    return hipMemcpyFromSymbol(count, HIP_SYMBOL(g_softmax_fallbacks), sizeof(*count), 0, hipMemcpyDeviceToHost);
}

int64_t mlr_softmax_scratch_bytes(int64_t B, int64_t J) { return softmax_cluster(J) ? B * softmax_cluster(J) * 8 : 0; }

hipError_t launch_mlr_softmax(const float* Z, const int32_t* y, void* U, bool out_bf16, int64_t B, int64_t J,
                              hipStream_t stream, bool blocked, void* scratch, const DeviceInfo* dev)
{
    if (B <= 0 || J <= 0) return hipSuccess;
    const int cl = (blocked && out_bf16 && B <= 65536) ? softmax_cluster(J) : 0;   // (32-bit offsets of a thread)
    if (cl && scratch && dev && reinterpret_cast<uintptr_t>(Z) % 16 == 0 && reinterpret_cast<uintptr_t>(U) % 16 == 0) {
        // one workgroup per CU so that all are resident together; whole clusters only
        int grid = dev->cus / cl * cl;
        if (grid < cl) return hipErrorInvalidValue;
        if ((int64_t)grid / cl > B) grid = (int)B * cl;
        const int64_t tn = (J + 255) / 256;
        const int tiles_per_wg = (int)((tn + cl - 1) / cl);
        hipError_t e = launch_fill_u32(scratch, 0u, B * cl * 2, stream);
        if (e != hipSuccess) return e;
        unsigned long long* slots = static_cast<unsigned long long*>(scratch);
        hipLaunchKernelGGL(mlr_softmax_cluster_kernel, dim3((unsigned)grid), dim3(1024), 0, stream, Z, y,
                           static_cast<uint16_t*>(U), B, J, (B + 255) / 256, cl, tiles_per_wg, slots, dev->softmax_wait_polls);
        return hipGetLastError();
    }
    // Vector path: rows of Z (and of U) must start 16-byte (8-byte for bf16 U) aligned.
    const int vec = (J % 4 == 0) && (reinterpret_cast<uintptr_t>(Z) % 16 == 0) &&
                    (reinterpret_cast<uintptr_t>(U) % 16 == 0);
    const dim3 grid((unsigned)B);
    const int64_t tiles_m = blocked ? (B + 255) / 256 : 0;
    if (J > 16384) {
        if (out_bf16)
            hipLaunchKernelGGL((mlr_softmax_kernel<1024, true>), grid, dim3(1024), 0, stream, Z, y, U, J, vec, tiles_m);
        else
            hipLaunchKernelGGL((mlr_softmax_kernel<1024, false>), grid, dim3(1024), 0, stream, Z, y, U, J, vec, tiles_m);
    } else {
        if (out_bf16)
            hipLaunchKernelGGL((mlr_softmax_kernel<256, true>), grid, dim3(256), 0, stream, Z, y, U, J, vec, tiles_m);
        else
            hipLaunchKernelGGL((mlr_softmax_kernel<256, false>), grid, dim3(256), 0, stream, Z, y, U, J, vec, tiles_m);
    }
    return hipGetLastError();
}

hipError_t launch_diff(const float* X, const float* Y, float* V, int64_t n, int32_t* counter, hipStream_t stream)
{
    if (n <= 0) return counter ? launch_fill_u32(counter, 0u, 1, stream) : hipSuccess;
    hipLaunchKernelGGL(diff_kernel, dim3(grid_for(n)), dim3(256), 0, stream, X, Y, V, n, counter);
    return hipGetLastError();
}

hipError_t launch_scale_rows(const float* V, const float* coef, float* Vs, int64_t N, int64_t D, hipStream_t stream)
{
    if (N <= 0 || D <= 0) return hipSuccess;
    hipLaunchKernelGGL(scale_rows_kernel, dim3(grid_for(N * D)), dim3(256), 0, stream, V, coef, Vs, N, D);
    return hipGetLastError();
}

hipError_t launch_div_scalar(const float* Z, float* W, float lambda, int64_t n, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(div_scalar_kernel, dim3(grid_for(n)), dim3(256), 0, stream, Z, W, lambda, n);
    return hipGetLastError();
}

hipError_t launch_sdca_mlr(const float* Zl, const float* X, float* P, float* dU, int64_t B, int64_t J, int64_t D,
                           float lambda, int64_t n_total, float beta, hipStream_t stream)
{
    if (B <= 0 || J <= 0) return hipSuccess;
    if (B > 0x7fffffffLL) return hipErrorInvalidValue;
    const float inv_lambda_n = (float)(1.0 / ((double)lambda * (double)n_total));
    hipLaunchKernelGGL(sdca_mlr_kernel, dim3((unsigned)B), dim3(256), 0, stream, Zl, X, P, dU, J, D, inv_lambda_n, beta);
    return hipGetLastError();
}

hipError_t launch_fill_u32(void* p, uint32_t value, int64_t n, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_u32_kernel, dim3(grid_for(n)), dim3(256), 0, stream, reinterpret_cast<uint32_t*>(p),
                       value, n);
    return hipGetLastError();
}

hipError_t launch_dml_scale(const float* Q, const int8_t* sim, float* U, int32_t* n_active, float margin, int64_t B,
                            int64_t K, hipStream_t stream)
{
    if (B <= 0) return hipSuccess;
    hipLaunchKernelGGL(dml_scale_kernel, dim3((unsigned)B), dim3(256), 0, stream, Q, sim, U, n_active, margin, K);
    return hipGetLastError();
}

hipError_t launch_prox_rows(float* W, int64_t J, int64_t D, int mode, hipStream_t stream)
{
    if (J <= 0 || D <= 0) return hipSuccess;
    hipLaunchKernelGGL(prox_rows_kernel, dim3((unsigned)J), dim3(256), 0, stream, W, D, mode);
    return hipGetLastError();
}

// Rows of W per workgroup of the power iteration: 16, more where that would be over 1024 workgroups.
static int power_rows(int64_t J)
{
    int64_t r = (J + 1023) / 1024;
    if (r < 16) r = 16;
    return (int)r;
}

int64_t power_chunks(int64_t J)
{
    const int64_t ch = (J + power_rows(J) - 1) / power_rows(J);
    return ch < 1 ? 1 : ch;
}

hipError_t launch_power_iteration(const float* W, int64_t J, int64_t D, int iters, float* scratch, float* L_out,
                                  hipStream_t stream)
{
    const int rows = power_rows(J);
    if (rows > POWER_MAX_ROWS) return hipErrorInvalidValue;
    const int64_t chunks = power_chunks(J);
    float* b = scratch;                     // the start vector, then unused
    float* part = b + D + J;
    float* g = part + chunks * D;
    const float b0 = 1.0f / sqrtf((float)D);
    hipError_t e = launch_fill_u32(b, __builtin_bit_cast(uint32_t, b0), D, stream);
    if (e != hipSuccess) return e;
    const bool in_registers = rows == 16 && D <= 1024 && D % 4 == 0 && reinterpret_cast<uintptr_t>(W) % 16 == 0 &&
                              reinterpret_cast<uintptr_t>(scratch) % 16 == 0 && J % 4 == 0;
    for (int it = 0; it < iters; ++it) {
        if (in_registers)
            hipLaunchKernelGGL(power_step16_kernel, dim3((unsigned)chunks), dim3(256), 0, stream, W, it == 0 ? b : g, part, J, D);
        else
            hipLaunchKernelGGL(power_step_kernel, dim3((unsigned)chunks), dim3(256), 0, stream, W, it == 0 ? b : g, part, J, D, rows);
        hipLaunchKernelGGL(power_reduce_kernel, dim3((unsigned)((D + 15) / 16)), dim3(256), 0, stream, part, g, D, chunks);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(vec_norm_kernel, dim3(1), dim3(1024), 0, stream, g, L_out, D);
    return hipGetLastError();
}

}  // namespace sfb
