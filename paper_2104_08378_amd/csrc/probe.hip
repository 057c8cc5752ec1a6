// sp24_probe: what this chip delivers for the pieces the sparse product is made of.
// Not part of the library: a stand-alone executable that prints
//   - issue rate of the dense and 2:4-sparse matrix-core instructions in a register-only loop on every
//     compute unit, with trivial operands (small integers: few bits toggle) and with random operands, together
//     with the shader clock the loop ran at (cycle counter over the 100 MHz real-time counter);
//   - streaming read / write / copy bandwidth on buffers far larger than the last-level cache.
// These are the measured ceilings that the roofline fractions of the product kernels are set against:
// the published peaks assume the nominal clock, which the part does not hold under real toggle rates.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <type_traits>
#include <vector>

#define CK(x)                                                                                          \
    do {                                                                                               \
        hipError_t e_ = (x);                                                                           \
        if (e_ != hipSuccess) {                                                                        \
            printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__);              \
            exit(1);                                                                                   \
        }                                                                                              \
    } while (0)

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16 __attribute__((ext_vector_type(16)));
typedef __bf16 b8 __attribute__((ext_vector_type(8)));
typedef __bf16 b16 __attribute__((ext_vector_type(16)));
typedef int i4 __attribute__((ext_vector_type(4)));
typedef int i8v __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef int i16v __attribute__((ext_vector_type(16)));

enum { D16_F16, D16_BF16, D16_I8, D32_F16, D32_BF16, D32_I8, S16_F16, S16_BF16, S16_I8, S32_F16, S32_BF16, S32_I8, NVAR };
static const char* kNames[NVAR] = {"v_mfma_f32_16x16x32_f16",    "v_mfma_f32_16x16x32_bf16",    "v_mfma_i32_16x16x64_i8",
                                   "v_mfma_f32_32x32x16_f16",    "v_mfma_f32_32x32x16_bf16",    "v_mfma_i32_32x32x32_i8",
                                   "v_smfmac_f32_16x16x64_f16",  "v_smfmac_f32_16x16x64_bf16",  "v_smfmac_i32_16x16x128_i8",
                                   "v_smfmac_f32_32x32x32_f16",  "v_smfmac_f32_32x32x32_bf16",  "v_smfmac_i32_32x32x64_i8"};
// dense-equivalent operations per instruction (2 per multiply-add of the full, uncompressed shape)
static const double kOps[NVAR] = {2. * 16 * 16 * 32, 2. * 16 * 16 * 32, 2. * 16 * 16 * 64,  2. * 32 * 32 * 16, 2. * 32 * 32 * 16, 2. * 32 * 32 * 32,
                                  2. * 16 * 16 * 64, 2. * 16 * 16 * 64, 2. * 16 * 16 * 128, 2. * 32 * 32 * 32, 2. * 32 * 32 * 32, 2. * 32 * 32 * 64};

template <int V, typename ACC>
__device__ __forceinline__ void issue(ACC& c, const i4& a, const i8v& b, int idx)
{
    if constexpr (V == D16_F16) c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, a), c, 0, 0, 0);
    if constexpr (V == D16_BF16) c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(b8, a), __builtin_bit_cast(b8, a), c, 0, 0, 0);
    if constexpr (V == D16_I8) c = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, a, c, 0, 0, 0);
    if constexpr (V == D32_F16) c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, a), c, 0, 0, 0);
    if constexpr (V == D32_BF16) c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(b8, a), __builtin_bit_cast(b8, a), c, 0, 0, 0);
    if constexpr (V == D32_I8) c = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, a, c, 0, 0, 0);
    if constexpr (V == S16_F16) c = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, b), c, idx, 0, 0);
    if constexpr (V == S16_BF16) c = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(b8, a), __builtin_bit_cast(b16, b), c, idx, 0, 0);
    if constexpr (V == S16_I8) c = __builtin_amdgcn_smfmac_i32_16x16x128_i8(a, b, c, idx, 0, 0);
    if constexpr (V == S32_F16) c = __builtin_amdgcn_smfmac_f32_32x32x32_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, b), c, idx, 0, 0);
    if constexpr (V == S32_BF16) c = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(__builtin_bit_cast(b8, a), __builtin_bit_cast(b16, b), c, idx, 0, 0);
    if constexpr (V == S32_I8) c = __builtin_amdgcn_smfmac_i32_32x32x64_i8(a, b, c, idx, 0, 0);
}

// Eight independent accumulator chains per wavefront, operands fixed in registers.  clocks[2*block], [2*block+1]:
// shader cycles and 100 MHz ticks the block's first wavefront spent in the loop.
template <int V>
__global__ __launch_bounds__(256) void k_issue(int iters, uint32_t* sink, unsigned long long* clocks, uint32_t random_operands)
{
    i4 a;
    i8v b;
    uint32_t x = threadIdx.x * 40503u + blockIdx.x * 9176u + 12345u;
    for (int i = 0; i < 4; ++i) { x = x * 1664525u + 1013904223u; a[i] = random_operands ? (int)((x >> 1) ^ (x << 13)) : i; }
    for (int i = 0; i < 8; ++i) { x = x * 1664525u + 1013904223u; b[i] = random_operands ? (int)((x >> 1) ^ (x << 11)) : i; }
    if (random_operands && (V % 3) != 2) {   // keep 16-bit floats finite: clear the top exponent bit of every half
        for (int i = 0; i < 4; ++i) a[i] &= 0xbfffbfff;
        for (int i = 0; i < 8; ++i) b[i] &= 0xbfffbfff;
    }
    const int idx = 0x4444 * 0x10001;   // code 0x4 (positions 0 and 1) in every group
    constexpr bool is32 = (V % 6) >= 3, isint = (V % 3) == 2;
    using acc_t = typename std::conditional<is32, typename std::conditional<isint, i16v, f16v>::type,
                                            typename std::conditional<isint, i4, f4>::type>::type;
    acc_t c0 = {}, c1 = {}, c2 = {}, c3 = {}, c4 = {}, c5 = {}, c6 = {}, c7 = {};
    const unsigned long long t0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
        issue<V>(c0, a, b, idx); issue<V>(c1, a, b, idx); issue<V>(c2, a, b, idx); issue<V>(c3, a, b, idx);
        issue<V>(c4, a, b, idx); issue<V>(c5, a, b, idx); issue<V>(c6, a, b, idx); issue<V>(c7, a, b, idx);
    }
    const unsigned long long t1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
    c0 += c1; c2 += c3; c4 += c5; c6 += c7; c0 += c2; c4 += c6; c0 += c4;
    auto s = c0[0];
    for (int r = 1; r < (int)(sizeof(acc_t) / 4); ++r) s += c0[r];
    if (s == (decltype(s))12345.5f) sink[0] = (uint32_t)s;   // practically never: keeps the chains alive
    if (threadIdx.x == 0) { clocks[2 * blockIdx.x] = t1 - t0; clocks[2 * blockIdx.x + 1] = r1 - r0; }
}

template <int V>
static void issue_rate(int cus, uint32_t random_operands)
{
    uint32_t* sink;
    unsigned long long* clocks;
    const int blocks = cus * 2;          // 256 threads = one wavefront per SIMD; two blocks per compute unit
    const int iters = 60000 * (((V % 6) >= 3) ? 1 : 2);
    CK(hipMalloc(&sink, 4));
    CK(hipMalloc(&clocks, sizeof(unsigned long long) * 2 * blocks));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    k_issue<V><<<blocks, 256>>>(200, sink, clocks, 0u);
    CK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int rep = 0; rep < 3; ++rep) {
        CK(hipEventRecord(e0));
        k_issue<V><<<blocks, 256>>>(iters, sink, clocks, random_operands);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best) best = ms;
    }
    std::vector<unsigned long long> h(2 * blocks);
    CK(hipMemcpy(h.data(), clocks, sizeof(unsigned long long) * 2 * blocks, hipMemcpyDeviceToHost));
    double mhz = 0;
    for (int i = 0; i < blocks; ++i) mhz += (double)h[2 * i] / ((double)h[2 * i + 1] / 100.0);
    mhz /= blocks;
    const double total = (double)blocks * 4 * iters * 8 * kOps[V];
    printf("issue  %-28s %-7s operands: %8.1f Tops/s dense-equivalent, %7.2f ms, shader clock %5.0f MHz\n", kNames[V],
           random_operands ? "random" : "trivial", total / (best * 1e-3) / 1e12, best, mhz);
    CK(hipFree(sink));
    CK(hipFree(clocks));
}

__global__ void k_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}
__global__ void k_read(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint4 acc = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint4 v = src[i];
        acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345679u) dst[0] = acc;
}
__global__ void k_write(uint4* __restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const uint4 v = {1, 2, 3, 4};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = v;
}

static void bandwidth(int cus)
{
    const size_t bytes = (size_t)2 << 30, n = bytes / 16;   // 2 GiB each: far beyond the 256 MB last-level cache
    uint4 *src, *dst;
    CK(hipMalloc(&src, bytes));
    CK(hipMalloc(&dst, bytes));
    CK(hipMemset(src, 1, bytes));
    CK(hipMemset(dst, 2, bytes));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    const int blocks = cus * 16;
    const char* names[3] = {"copy ", "read ", "write"};
    for (int mode = 0; mode < 3; ++mode) {
        float best = 1e30f;
        for (int rep = 0; rep < 4; ++rep) {
            CK(hipEventRecord(e0));
            if (mode == 0) k_copy<<<blocks, 256>>>(src, dst, n);
            if (mode == 1) k_read<<<blocks, 256>>>(src, dst, n);
            if (mode == 2) k_write<<<blocks, 256>>>(dst, n);
            CK(hipEventRecord(e1));
            CK(hipEventSynchronize(e1));
            float ms;
            CK(hipEventElapsedTime(&ms, e0, e1));
            if (rep && ms < best) best = ms;
        }
        printf("stream %s 2 GiB: %7.3f ms  %7.1f GB/s\n", names[mode], best, (mode == 0 ? 2.0 : 1.0) * bytes / (best * 1e-3) / 1e9);
    }
    CK(hipFree(src));
    CK(hipFree(dst));
}

int main()
{
    setvbuf(stdout, nullptr, _IOLBF, 0);
    hipDeviceProp_t p;
    CK(hipGetDeviceProperties(&p, 0));
    const int cus = p.multiProcessorCount;
    printf("device %s (%s): %d compute units, nominal clock %.0f MHz\n", p.name, p.gcnArchName, cus, p.clockRate / 1e3);
    for (uint32_t rnd = 0; rnd < 2; ++rnd) {
        issue_rate<D32_F16>(cus, rnd);  issue_rate<D32_BF16>(cus, rnd);  issue_rate<D32_I8>(cus, rnd);
        issue_rate<D16_F16>(cus, rnd);  issue_rate<D16_BF16>(cus, rnd);  issue_rate<D16_I8>(cus, rnd);
        issue_rate<S32_F16>(cus, rnd);  issue_rate<S32_BF16>(cus, rnd);  issue_rate<S32_I8>(cus, rnd);
        issue_rate<S16_F16>(cus, rnd);  issue_rate<S16_BF16>(cus, rnd);  issue_rate<S16_I8>(cus, rnd);
    }
    bandwidth(cus);
    return 0;
}
