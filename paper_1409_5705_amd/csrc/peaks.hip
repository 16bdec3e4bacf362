// Stand-alone probe of what this GPU sustains on the two resources the
// roofline fractions are quoted against: the MFMA pipes (a register-only loop of
// bf16 32x32x16 and fp32 32x32x2 MFMAs, one and two wavefronts per SIMD; bf16 MFMAs of both
// shapes on operands that change) and HBM
// (streaming read, copy and read-modify-write of buffers far larger than the
// caches, 16 bytes per lane), and what ONE compute unit can pull through its
// vector-memory path when a quarter of the CUs stream alone (one workgroup each:
// lines that miss every cache against lines that stay in the L2, 4 and 16
// wavefronts, 8 and 16 bytes per lane; and the same for a stream of stores).  Prints one JSON object.  Used by
// `bench.py --peaks`; not part of the library.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#define CK(x)                                                                          \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                                  \
        }                                                                              \
    } while (0)

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <bool BF16>
__global__ __launch_bounds__(512) void mfma_loop(float* out, int iters)
{
    floatx16 acc[4];
    for (int a = 0; a < 4; ++a)
        for (int i = 0; i < 16; ++i) acc[a][i] = 0.f;
    const float x = 1.0f + threadIdx.x * 1e-6f, y = 0.5f;
    bf16x8 xb, yb;
    for (int i = 0; i < 8; ++i) {
        xb[i] = (__bf16)x;
        yb[i] = (__bf16)y;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                if (BF16)
                    acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xb, yb, acc[a], 0, 0, 0);
                else
                    acc[a] = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, acc[a], 0, 0, 0);
            }
    }
    float s = 0.f;
    for (int a = 0; a < 4; ++a)
        for (int i = 0; i < 16; ++i) s += acc[a][i];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The same bf16 work fed like a real contraction: a wavefront's 128 x 128 block, eight A and eight B fragments of
// pseudo-random values (|x| in [1/2, 2), random signs and mantissas) covering 32 of k, every fragment used by
// several MFMAs, and sign and mantissa bits of all fragments flipped by a new pattern after every 1.05 MFLOP
// (64 vector instructions: what the fragment reads of a kernel cost in issue slots).  SHAPE 32: 4 x 4 tiles of
// 32 x 32, two 32x32x16 MFMAs each; SHAPE 16: 8 x 8 tiles of 16 x 16, one 16x16x32 MFMA each.  The clock the
// chip grants depends on how many bits toggle: this is the matrix-pipe rate with operands that change, against
// mfma_loop's with operands that never do (flip_bits = 0 runs the identical instruction stream on operands that
// stay as they are, value_bits = 0 makes every element 0.5: the controls).
template <int SHAPE>
__global__ __launch_bounds__(256) void mfma_random_loop(float* out, int iters, uint32_t flip_bits, uint32_t value_bits)
{
    typedef uint32_t u32x4v __attribute__((ext_vector_type(4)));
    u32x4v fa[8], fb[8];
    uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    auto next = [&]() {
        h ^= h << 13;
        h ^= h >> 17;
        h ^= h << 5;
        return h;
    };
    for (int f = 0; f < 8; ++f)
        for (int e = 0; e < 4; ++e) {
            // two bf16 per word: exponent 126 or 127 (0.5 <= |x| < 2), random sign and mantissa
            fa[f][e] = (next() & value_bits) | 0x3f003f00u;
            fb[f][e] = (next() & value_bits) | 0x3f003f00u;
        }
    uint32_t flip = next();
    auto flip_all = [&]() {
        flip = flip * 1664525u + 1013904223u;
        const uint32_t m = flip & flip_bits;       // 0x807f807f: signs and mantissas only (no infinities, no NaNs)
#pragma unroll
        for (int f = 0; f < 8; ++f)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                fa[f][e] ^= m;
                fb[f][e] ^= (m >> 1) & flip_bits;
            }
    };
    float sum = 0.f;
    if (SHAPE == 32) {
        floatx16 acc[4][4];
        for (int a = 0; a < 4; ++a)
            for (int b = 0; b < 4; ++b)
                for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[a + 4 * ks]),
                                                                            __builtin_bit_cast(bf16x8, fb[b + 4 * ks]), acc[a][b], 0, 0, 0);
            flip_all();
        }
        for (int a = 0; a < 4; ++a)
            for (int b = 0; b < 4; ++b)
                for (int i = 0; i < 16; ++i) sum += acc[a][b][i];
    } else {
        floatx4 acc[8][8];
        for (int a = 0; a < 8; ++a)
            for (int b = 0; b < 8; ++b)
                for (int i = 0; i < 4; ++i) acc[a][b][i] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int a = 0; a < 8; ++a)
#pragma unroll
                for (int b = 0; b < 8; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fa[a]), __builtin_bit_cast(bf16x8, fb[b]),
                                                                        acc[a][b], 0, 0, 0);
            flip_all();
        }
        for (int a = 0; a < 8; ++a)
            for (int b = 0; b < 8; ++b)
                for (int i = 0; i < 4; ++i) sum += acc[a][b][i];
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

// MODE 0: read only (sum kept in a register, one store per thread); 1: copy; 2: read-modify-write in place.
// Four independent 16-byte accesses per lane and iteration.
template <int MODE>
__global__ __launch_bounds__(256) void stream_kernel(const floatx4* __restrict__ src, floatx4* __restrict__ dst,
                                                     size_t n4, float* sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n4; i += 4 * stride) {
        floatx4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (MODE == 0) acc += v[u];
            if (MODE == 1) __builtin_nontemporal_store(v[u], dst + i + u * stride);
            if (MODE == 2) __builtin_nontemporal_store(v[u] * 0.999f, dst + i + u * stride);
        }
    }
    for (; i < n4; i += stride) {
        const floatx4 v = __builtin_nontemporal_load(src + i);
        if (MODE == 0) acc += v;
        if (MODE == 1) __builtin_nontemporal_store(v, dst + i);
        if (MODE == 2) __builtin_nontemporal_store(v * 0.999f, dst + i);
    }
    if (MODE == 0) sink[(size_t)blockIdx.x * 256 + threadIdx.x] = acc[0] + acc[1] + acc[2] + acc[3];
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// One workgroup of T threads reads its own contiguous region of `footprint` bytes `passes` times, 16 accesses
// of W bytes per lane in flight.  footprint and the region are multiples of 16 * T * W.
template <int W, int T>
__global__ __launch_bounds__(T) void cu_read_kernel(const char* __restrict__ p, uint32_t* __restrict__ sink, size_t region,
                                                    uint32_t footprint, int passes)
{
    const char* base = p + (size_t)blockIdx.x * region;
    const auto rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, footprint, 0x00020000);
    const uint32_t lane_off = threadIdx.x * W, step = T * W;
    uint32_t acc = 0;
    for (int ps = 0; ps < passes; ++ps)
        for (uint32_t soff = 0; soff < footprint; soff += 16 * step) {
            if (W == 16) {
                u32x4 v[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, soff + i * step, 0);
#pragma unroll
                for (int i = 0; i < 16; ++i) acc += v[i][0] ^ v[i][1] ^ v[i][2] ^ v[i][3];
            } else {
                u32x2 v[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] = __builtin_amdgcn_raw_buffer_load_b64(rs, lane_off, soff + i * step, 0);
#pragma unroll
                for (int i = 0; i < 16; ++i) acc += v[i][0] ^ v[i][1];
            }
        }
    if (acc == 0x12345678u) sink[threadIdx.x] = acc;   // never true for a zeroed buffer: keeps the loads alive
}

// The same for stores: each workgroup fills its own region with 16-byte non-temporal stores, 16 per lane back to back.
template <int T>
__global__ __launch_bounds__(T) void cu_write_kernel(char* __restrict__ p, size_t region, uint32_t footprint)
{
    char* base = p + (size_t)blockIdx.x * region;
    const auto rs = __builtin_amdgcn_make_buffer_rsrc(base, 0, footprint, 0x00020000);
    const uint32_t lane_off = threadIdx.x * 16, step = T * 16;
    const u32x4 v = {threadIdx.x, blockIdx.x, 0u, 0u};
    for (uint32_t soff = 0; soff < footprint; soff += 16 * step) {
#pragma unroll
        for (int i = 0; i < 16; ++i) __builtin_amdgcn_raw_buffer_store_b128(v, rs, lane_off, soff + i * step, 2);
    }
}

template <typename F>
int time_ms(F launch, int reps, float* ms_out)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    launch();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0, 0));
    for (int r = 0; r < reps; ++r) launch();
    CK(hipEventRecord(e1, 0));
    CK(hipGetLastError());
    CK(hipDeviceSynchronize());
    CK(hipEventElapsedTime(ms_out, e0, e1));
    *ms_out /= reps;
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return 0;
}

int main()
{
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount;
    float* out;
    CK(hipMalloc(&out, (size_t)cus * 512 * 4));
    const int iters = 4000;
    float ms;
    double tf[4];
    int k = 0;
    for (int bf16 = 1; bf16 >= 0; --bf16)
        for (int threads = 256; threads <= 512; threads += 256) {
            if (bf16) {
                if (time_ms([&] { hipLaunchKernelGGL(mfma_loop<true>, dim3(cus), dim3(threads), 0, 0, out, iters); }, 3, &ms))
                    return 1;
            } else {
                if (time_ms([&] { hipLaunchKernelGGL(mfma_loop<false>, dim3(cus), dim3(threads), 0, 0, out, iters); }, 3, &ms))
                    return 1;
            }
            const double mfmas = (double)iters * 32 * (threads / 64) * cus;
            tf[k++] = mfmas * (bf16 ? 32768.0 : 4096.0) / (ms * 1e-3) / 1e12;
        }
    double tf_random = 0.0, tf_control = 0.0, tf_const = 0.0, tf_random16 = 0.0;
    {
        const int it2 = 60000;      // x 1.05 MFLOP per wavefront: about 35 ms, long enough for the clock to settle
        const double fl = (double)it2 * 1048576.0 * 4 * cus;
        if (time_ms([&] { hipLaunchKernelGGL(mfma_random_loop<32>, dim3(cus), dim3(256), 0, 0, out, it2, 0x807f807fu, 0x80ff80ffu); }, 3, &ms)) return 1;
        tf_random = fl / (ms * 1e-3) / 1e12;
        if (time_ms([&] { hipLaunchKernelGGL(mfma_random_loop<32>, dim3(cus), dim3(256), 0, 0, out, it2, 0u, 0x80ff80ffu); }, 3, &ms)) return 1;
        tf_control = fl / (ms * 1e-3) / 1e12;
        if (time_ms([&] { hipLaunchKernelGGL(mfma_random_loop<32>, dim3(cus), dim3(256), 0, 0, out, it2, 0u, 0u); }, 3, &ms)) return 1;
        tf_const = fl / (ms * 1e-3) / 1e12;
        if (time_ms([&] { hipLaunchKernelGGL(mfma_random_loop<16>, dim3(cus), dim3(256), 0, 0, out, it2, 0x807f807fu, 0x80ff80ffu); }, 3, &ms)) return 1;
        tf_random16 = fl / (ms * 1e-3) / 1e12;
    }
    CK(hipFree(out));

    const size_t bytes = (size_t)4 << 30;   // 4 GiB per buffer
    floatx4 *a, *b;
    float* sink;
    CK(hipMalloc(&a, bytes));
    CK(hipMalloc(&b, bytes));
    CK(hipMalloc(&sink, (size_t)cus * 32 * 256 * 4));
    CK(hipMemset(a, 0, bytes));
    CK(hipMemset(b, 0, bytes));
    const size_t n4 = bytes / 16;
    double gbs[3] = {0.0, 0.0, 0.0};
    for (unsigned per_cu = 4; per_cu <= 32; per_cu *= 2) {   // best of several grid sizes
        const unsigned grid = (unsigned)cus * per_cu;
        if (time_ms([&] { hipLaunchKernelGGL(stream_kernel<0>, dim3(grid), dim3(256), 0, 0, a, b, n4, sink); }, 5, &ms)) return 1;
        if (bytes / (ms * 1e-3) / 1e9 > gbs[0]) gbs[0] = bytes / (ms * 1e-3) / 1e9;
        if (time_ms([&] { hipLaunchKernelGGL(stream_kernel<1>, dim3(grid), dim3(256), 0, 0, a, b, n4, sink); }, 5, &ms)) return 1;
        if (2.0 * bytes / (ms * 1e-3) / 1e9 > gbs[1]) gbs[1] = 2.0 * bytes / (ms * 1e-3) / 1e9;
        if (time_ms([&] { hipLaunchKernelGGL(stream_kernel<2>, dim3(grid), dim3(256), 0, 0, a, a, n4, sink); }, 5, &ms)) return 1;
        if (2.0 * bytes / (ms * 1e-3) / 1e9 > gbs[2]) gbs[2] = 2.0 * bytes / (ms * 1e-3) / 1e9;
    }
    // One CU's read rate: a quarter of the CUs, one workgroup each, so that neither HBM nor an L2 is the limit.
    // "miss": 32 MiB per workgroup read once; "l2": 256 KiB per workgroup read 128 times.
    double cu[6];
    {
        const int wgs = cus / 4;
        const size_t region = (size_t)32 << 20;
        const char* pa = reinterpret_cast<const char*>(a);
        uint32_t* sk = reinterpret_cast<uint32_t*>(sink);
        const uint32_t big = (uint32_t)region, small = 256u << 10;
        int c = 0;
        if (time_ms([&] { hipLaunchKernelGGL((cu_read_kernel<16, 256>), dim3(wgs), dim3(256), 0, 0, pa, sk, region, big, 1); }, 3, &ms)) return 1;
        cu[c++] = (double)big / (ms * 1e-3) / 1e9;
        if (time_ms([&] { hipLaunchKernelGGL((cu_read_kernel<16, 1024>), dim3(wgs), dim3(1024), 0, 0, pa, sk, region, big, 1); }, 3, &ms)) return 1;
        cu[c++] = (double)big / (ms * 1e-3) / 1e9;
        if (time_ms([&] { hipLaunchKernelGGL((cu_read_kernel<16, 256>), dim3(wgs), dim3(256), 0, 0, pa, sk, region, small, 128); }, 3, &ms)) return 1;
        cu[c++] = 128.0 * small / (ms * 1e-3) / 1e9;
        if (time_ms([&] { hipLaunchKernelGGL((cu_read_kernel<16, 1024>), dim3(wgs), dim3(1024), 0, 0, pa, sk, region, small, 128); }, 3, &ms)) return 1;
        cu[c++] = 128.0 * small / (ms * 1e-3) / 1e9;
        if (time_ms([&] { hipLaunchKernelGGL((cu_read_kernel<8, 256>), dim3(wgs), dim3(256), 0, 0, pa, sk, region, small, 128); }, 3, &ms)) return 1;
        cu[c++] = 128.0 * small / (ms * 1e-3) / 1e9;
        if (time_ms([&] { hipLaunchKernelGGL((cu_read_kernel<8, 1024>), dim3(wgs), dim3(1024), 0, 0, pa, sk, region, small, 128); }, 3, &ms)) return 1;
        cu[c++] = 128.0 * small / (ms * 1e-3) / 1e9;
    }
    double cuw[2];
    {
        const int wgs = cus / 4;
        const size_t region = (size_t)32 << 20;
        char* pb = reinterpret_cast<char*>(b);
        if (time_ms([&] { hipLaunchKernelGGL((cu_write_kernel<256>), dim3(wgs), dim3(256), 0, 0, pb, region, (uint32_t)region); }, 3, &ms)) return 1;
        cuw[0] = (double)region / (ms * 1e-3) / 1e9;
        if (time_ms([&] { hipLaunchKernelGGL((cu_write_kernel<1024>), dim3(wgs), dim3(1024), 0, 0, pb, region, (uint32_t)region); }, 3, &ms)) return 1;
        cuw[1] = (double)region / (ms * 1e-3) / 1e9;
    }
    CK(hipFree(a));
    CK(hipFree(b));
    CK(hipFree(sink));
    printf("{\"device\": \"%s\", \"compute_units\": %d, \"clock_mhz\": %d, "
           "\"mfma_bf16_tflops\": {\"one_wave_per_simd\": %.1f, \"two_waves_per_simd\": %.1f, \"one_wave_changing_operands\": %.1f, \"same_loop_operands_kept\": %.1f, \"same_loop_all_elements_equal\": %.1f, "
           "\"one_wave_changing_operands_16x16x32\": %.1f}, "
           "\"mfma_f32_tflops\": {\"one_wave_per_simd\": %.1f, \"two_waves_per_simd\": %.1f}, "
           "\"hbm_gbs\": {\"read\": %.0f, \"copy_read_plus_write\": %.0f, \"read_modify_write\": %.0f}, "
           "\"one_cu_read_gbs\": {\"miss_4_waves\": %.1f, \"miss_16_waves\": %.1f, \"l2_4_waves\": %.1f, \"l2_16_waves\": %.1f, "
           "\"l2_4_waves_8_byte\": %.1f, \"l2_16_waves_8_byte\": %.1f}, "
           "\"one_cu_write_gbs\": {\"4_waves\": %.1f, \"16_waves\": %.1f}, "
           "\"buffer_gib\": 4}\n",
           prop.gcnArchName, cus, prop.clockRate / 1000, tf[0], tf[1], tf_random, tf_control, tf_const, tf_random16, tf[2], tf[3], gbs[0], gbs[1], gbs[2], cu[0], cu[1], cu[2],
           cu[3], cu[4], cu[5], cuw[0], cuw[1]);
    return 0;
}
