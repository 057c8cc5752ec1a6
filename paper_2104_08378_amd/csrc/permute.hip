// Channel permutations (Sec. 4.1, Step 2; Fig. 6): a weight matrix with its columns taken in another order, and
// the figure of merit of such an order -- the total magnitude that 2:4 pruning keeps when the groups of four are
// formed from the reordered columns.
//
// Both kernels are bound by reading A once (the gather's result is written once; the figure of merit writes one
// number).  A wavefront stages one row of A in its own LDS region with 16-byte loads and gathers from there: a
// gather of 2-byte elements straight from memory would turn every element into a request of its own.  The order
// itself is staged once per workgroup, as 16-bit column numbers, so that a lane fetches the eight entries of a
// 16-byte piece with one LDS read.  LDS is sized to the row at launch (many workgroups per compute unit for short
// rows: the passes are latency-bound).  Rows too long for a region (more than 16 KiB) are gathered from memory
// directly, entry by entry.
#include "common.hpp"
#include "launch.hpp"

namespace sp24 {

constexpr int kPermWaves = 4;         // rows per workgroup and pass
constexpr int kPermRowBytes = 16384;  // LDS region of one wavefront

// column of A that position k of the new order takes; entries outside 0 .. K-1 read column 0 (never out of bounds)
__device__ __forceinline__ int64_t source_column(const int32_t* perm, int64_t k, int64_t K)
{
    if (perm == nullptr) return k;
    const uint32_t p = (uint32_t)perm[k];
    return p < (uint64_t)K ? (int64_t)p : 0;
}

// The order as the staged path keeps it: K 16-bit column numbers in LDS (a staged row has at most 16384 columns),
// already made safe.
typedef __attribute__((address_space(3))) uint16_t* lds_order;
__device__ __forceinline__ void stage_order(const int32_t* perm, int64_t K, lds_order order)
{
    // eight loads in flight per thread (one per trip would cost a memory latency each)
    for (int64_t k0 = 0; k0 < K; k0 += 8 * blockDim.x) {
        int64_t col[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t k = k0 + j * blockDim.x + threadIdx.x;
            if (k < K) col[j] = source_column(perm, k, K);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t k = k0 + j * blockDim.x + threadIdx.x;
            if (k < K) order[k] = (uint16_t)col[j];
        }
    }
}
struct StagedOrder {
    lds_order order;
    __device__ __forceinline__ int64_t operator()(int64_t k) const { return order[k]; }
};
struct PlainOrder {
    const int32_t* perm;
    int64_t K;
    __device__ __forceinline__ int64_t operator()(int64_t k) const { return source_column(perm, k, K); }
};

// A row as the gathers see it: staged in this wavefront's LDS region, or (too long for it) where it lies in memory.
// The two cases are separate types so that every access is an LDS or a global instruction, never a generic one.
typedef __attribute__((address_space(3))) uint8_t* lds_row;
template <int ES>
__device__ __forceinline__ uint32_t element_bits(lds_row row, int64_t k)
{
    if constexpr (ES == 2) return reinterpret_cast<__attribute__((address_space(3))) const uint16_t*>(row)[k];
    else return row[k];
}
template <int ES>
__device__ __forceinline__ uint32_t element_bits(const uint8_t* row, int64_t k)
{
    if constexpr (ES == 2) return reinterpret_cast<const uint16_t*>(row)[k];
    else return row[k];
}

// A row on its way into a wavefront's LDS region: up to 16 KiB = 16 pieces of 16 bytes per lane, held in registers
// between the loads and the LDS writes, so that the loads of the next row are in flight while the current row is
// gathered.  (bytes: K * ES, a multiple of 32.)
struct RowInFlight {
    uint4v part[kPermRowBytes / 1024];
    __device__ __forceinline__ void load(const uint8_t* src, int64_t bytes, int lane)
    {
#pragma unroll
        for (int j = 0; j < kPermRowBytes / 1024; ++j) {
            const int64_t c = 64 * j + lane;
            if (c < bytes / 16) part[j] = reinterpret_cast<const uint4v*>(src)[c];
        }
    }
    __device__ __forceinline__ void store(lds_row region, int64_t bytes, int lane) const
    {
#pragma unroll
        for (int j = 0; j < kPermRowBytes / 1024; ++j) {
            const int64_t c = 64 * j + lane;
            if (c < bytes / 16) reinterpret_cast<__attribute__((address_space(3))) uint4v*>(region)[c] = part[j];
        }
    }
};

// Between a wavefront's LDS writes of a row and its own reads of it (and back): the LDS serves one wavefront's
// operations in order, so no workgroup barrier is needed -- only the compiler must keep the order.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// 16 bytes of the reordered row: elements c * EPC .. of the new order
template <int ES, typename ROW, typename ORDER>
__device__ __forceinline__ uint4v gather_chunk(ROW row, const ORDER& col, int64_t c)
{
    constexpr int EPC = 16 / ES;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
        const uint32_t v = element_bits<ES>(row, col(c * EPC + e));
        w[e * ES / 4] |= v << (8 * ((e * ES) % 4));
    }
    const uint4v out = {w[0], w[1], w[2], w[3]};
    return out;
}

// P[m][k] = A[m][perm[k]]: a lane writes 16 bytes of P (8 or 16 elements) gathered one by one
template <int ES>
__global__ __launch_bounds__(64 * kPermWaves) void k_permute_columns(const uint8_t* A, const int32_t* perm, uint8_t* P, int64_t M, int64_t K,
                                                                     int64_t lda, int64_t ldp)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];   // staged: the order (2 K bytes), then kPermWaves rows
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int EPC = 16 / ES;                       // elements per 16-byte chunk
    const bool staged = K * ES <= kPermRowBytes;       // the same for every wavefront
    const StagedOrder in_lds = {(lds_order)lds};
    const PlainOrder in_memory = {perm, K};
    const lds_row region = (lds_row)lds + (2 * K + wave * K * ES);
    // a wavefront takes rows first, first + stride, ... on its own: no barrier after the one that publishes the order
    const int64_t first = (int64_t)blockIdx.x * kPermWaves + wave, stride = (int64_t)gridDim.x * kPermWaves;
    if (staged) {
        RowInFlight next;
        if (first < M) next.load(A + first * lda * ES, K * ES, lane);
        stage_order(perm, K, in_lds.order);
        __syncthreads();
        for (int64_t row = first; row < M; row += stride) {
            next.store(region, K * ES, lane);           // (after this wavefront's reads of the previous row: in order)
            if (row + stride < M) next.load(A + (row + stride) * lda * ES, K * ES, lane);
            wave_lds_fence();
            uint8_t* dst = P + row * ldp * ES;
            for (int64_t c = lane; c < K / EPC; c += 64) *reinterpret_cast<uint4v*>(dst + c * 16) = gather_chunk<ES>(region, in_lds, c);
            wave_lds_fence();
        }
    } else {
        for (int64_t row = first; row < M; row += stride) {
            const uint8_t* src = A + row * lda * ES;
            uint8_t* dst = P + row * ldp * ES;
            for (int64_t c = lane; c < K / EPC; c += 64) *reinterpret_cast<uint4v*>(dst + c * 16) = gather_chunk<ES>(src, in_memory, c);
        }
    }
}

// The two largest magnitudes among the four columns of group g in the new order, summed.  Which of several equal
// magnitudes the selection rule of sp24_prune keeps does not change the sum, so the two largest keys (the
// magnitudes as unsigned integers, every NaN one key above infinity) are found with a min/max network and turned
// into exact doubles; a NaN among them makes the sum NaN.
template <int DT>
__device__ __forceinline__ double kept_of_keys(const uint32_t (&key)[4])
{
    const uint32_t hi01 = max(key[0], key[1]), lo01 = min(key[0], key[1]);
    const uint32_t hi23 = max(key[2], key[3]), lo23 = min(key[2], key[3]);
    const uint32_t first = max(hi01, hi23), second = max(min(hi01, hi23), max(lo01, lo23));
    if constexpr (DT == SP24_I8) return (double)(first + second);
    else if constexpr (DT == SP24_F8) {
        // the keys are the bit patterns without their sign; the NaN pattern is the largest and makes the sum NaN
        const double nan = (double)__builtin_nanf("");
        return (first == 0x7Fu ? nan : (double)magnitude_f8(first)) + (second == 0x7Fu ? nan : (double)magnitude_f8(second));
    } else if constexpr (DT == SP24_F16)
        return (double)(float)__builtin_bit_cast(_Float16, (uint16_t)first) + (double)(float)__builtin_bit_cast(_Float16, (uint16_t)second);
    else return (double)__uint_as_float(first << 16) + (double)__uint_as_float(second << 16);
}
template <int DT, typename ROW, typename ORDER>
__device__ __forceinline__ double kept_of_group(ROW row, const ORDER& col, int64_t g)
{
    constexpr int ES = is8<DT> ? 1 : 2;
    uint32_t key[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t bits = element_bits<ES>(row, col(4 * g + i));
        if constexpr (DT == SP24_I8) key[i] = mag_key8(bits);
        else if constexpr (DT == SP24_F8) key[i] = mag_key_f8(bits);
        else key[i] = mag_key16<DT>(bits);
    }
    return kept_of_keys<DT>(key);
}
// The same for the groups of 16 bytes of a row in its given order: four groups of 8-bit, two of 16-bit elements.
template <int DT>
__device__ __forceinline__ double kept_of_chunk(const uint4v& w)
{
    double sum = 0.0;
    if constexpr (DT == SP24_I8) {
        uint32_t total = 0;                                 // integers: one conversion per chunk
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint32_t k0 = mag_key8(w[g] & 0xFFu), k1 = mag_key8((w[g] >> 8) & 0xFFu), k2 = mag_key8((w[g] >> 16) & 0xFFu), k3 = mag_key8(w[g] >> 24);
            const uint32_t hi01 = max(k0, k1), lo01 = min(k0, k1), hi23 = max(k2, k3), lo23 = min(k2, k3);
            total += max(hi01, hi23) + max(min(hi01, hi23), max(lo01, lo23));
        }
        sum = (double)total;
    } else if constexpr (DT == SP24_F8) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint32_t key[4] = {mag_key_f8(w[g]), mag_key_f8(w[g] >> 8), mag_key_f8(w[g] >> 16), mag_key_f8(w[g] >> 24)};
            sum += kept_of_keys<DT>(key);
        }
    } else {
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            const uint32_t key[4] = {mag_key16<DT>(w[2 * g] & 0xFFFFu), mag_key16<DT>(w[2 * g] >> 16), mag_key16<DT>(w[2 * g + 1] & 0xFFFFu),
                                     mag_key16<DT>(w[2 * g + 1] >> 16)};
            sum += kept_of_keys<DT>(key);
        }
    }
    return sum;
}

__global__ void k_zero_double(double* out) { *out = 0.0; }

// out += sum over this workgroup's rows and all groups g of the two largest magnitudes among columns
// perm[4g] .. perm[4g+3] (the selection rule of sp24_prune: ties to the lower position, NaN highest).
template <int DT>
__global__ __launch_bounds__(64 * kPermWaves) void k_retained_magnitude(const uint8_t* A, const int32_t* perm, double* out, int64_t M, int64_t K,
                                                                        int64_t lda)
{
    constexpr int ES = is8<DT> ? 1 : 2;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];   // staged: the order (2 K bytes), then kPermWaves rows
    __shared__ double partial[kPermWaves];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool staged = K * ES <= kPermRowBytes;
    const StagedOrder in_lds = {(lds_order)lds};
    const PlainOrder in_memory = {perm, K};
    const lds_row region = (lds_row)lds + (2 * K + wave * K * ES);
    double sum = 0.0;
    const int64_t first = (int64_t)blockIdx.x * kPermWaves + wave, stride = (int64_t)gridDim.x * kPermWaves;
    if (perm == nullptr) {
        // the given order: every group lies in place, nothing to stage or gather; eight loads in flight per lane
        const int64_t chunks = K * ES / 16;
        for (int64_t row = first; row < M; row += stride) {
            const uint4v* src = reinterpret_cast<const uint4v*>(A + row * lda * ES);
            for (int64_t c0 = 0; c0 < chunks; c0 += 8 * 64) {
                uint4v part[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int64_t c = c0 + 64 * j + lane;
                    if (c < chunks) part[j] = src[c];
                }
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (c0 + 64 * j + lane < chunks) sum += kept_of_chunk<DT>(part[j]);
            }
        }
    } else if (staged) {
        RowInFlight next;
        if (first < M) next.load(A + first * lda * ES, K * ES, lane);
        stage_order(perm, K, in_lds.order);
        __syncthreads();
        for (int64_t row = first; row < M; row += stride) {
            next.store(region, K * ES, lane);
            if (row + stride < M) next.load(A + (row + stride) * lda * ES, K * ES, lane);
            wave_lds_fence();
            for (int64_t g = lane; g < K / 4; g += 64) sum += kept_of_group<DT>(region, in_lds, g);
            wave_lds_fence();
        }
    } else {
        for (int64_t row = first; row < M; row += stride) {
            const uint8_t* src = A + row * lda * ES;
            for (int64_t g = lane; g < K / 4; g += 64) sum += kept_of_group<DT>(src, in_memory, g);
        }
    }
    // wavefront, then workgroup, then one atomic per workgroup
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
    if (lane == 0) partial[wave] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
        for (int w = 0; w < kPermWaves; ++w) s += partial[w];
        atomicAdd(out, s);
    }
}

// P[m][:] = A[perm[m]][:]: whole rows, 16 bytes per lane, one row per wavefront and pass.  An entry outside
// 0 .. M-1 reads row 0.
__global__ __launch_bounds__(64 * kPermWaves) void k_permute_rows(const uint8_t* A, const int32_t* perm, uint8_t* P, int64_t M, int64_t row_bytes,
                                                                  int64_t lda_bytes, int64_t ldp_bytes)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int64_t row = (int64_t)blockIdx.x * kPermWaves + wave; row < M; row += (int64_t)gridDim.x * kPermWaves) {
        const uint32_t p = (uint32_t)perm[row];
        const uint8_t* src = A + (p < (uint64_t)M ? (int64_t)p : 0) * lda_bytes;
        uint8_t* dst = P + row * ldp_bytes;
        for (int64_t c0 = 0; c0 < row_bytes / 16; c0 += 8 * 64) {     // eight loads in flight per lane
            uint4v part[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int64_t c = c0 + 64 * j + lane;
                if (c < row_bytes / 16) part[j] = reinterpret_cast<const uint4v*>(src)[c];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int64_t c = c0 + 64 * j + lane;
                if (c < row_bytes / 16) reinterpret_cast<uint4v*>(dst)[c] = part[j];
            }
        }
    }
}

static sp24_status launch_result() { return hipGetLastError() == hipSuccess ? SP24_OK : SP24_ERR_LAUNCH; }

static unsigned grid_for_rows(int64_t M)
{
    const int64_t passes = (M + kPermWaves - 1) / kPermWaves;
    return (unsigned)(passes < 512 ? passes : 512);   // few enough that staging the order pays, enough to fill the chip
}

// dynamic LDS of the staged path: the order as 16-bit entries and one row per wavefront (0 when rows are not staged)
static size_t staged_lds_bytes(int64_t K, int es)
{
    return K * es <= kPermRowBytes ? (size_t)(2 * K + kPermWaves * K * es) : 0;
}
constexpr int kPermMaxLds = 2 * kPermRowBytes + kPermWaves * kPermRowBytes;   // int8 rows of 16384 columns

template <typename KERNEL>
static bool allow_lds(KERNEL kernel)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kPermMaxLds) == hipSuccess;
}

sp24_status launch_permute_columns(const void* A, const void* perm, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, sp24_dtype t,
                                   hipStream_t st)
{
    if (M * K == 0) return SP24_OK;
    const dim3 grid(grid_for_rows(M)), block(64 * kPermWaves);
    const uint8_t* a = static_cast<const uint8_t*>(A);
    const int32_t* p = static_cast<const int32_t*>(perm);
    uint8_t* o = static_cast<uint8_t*>(P);
    static const bool ready = allow_lds(k_permute_columns<1>) && allow_lds(k_permute_columns<2>);
    if (!ready) return SP24_ERR_LAUNCH;
    const size_t lds = staged_lds_bytes(K, esize_of(t));
    if (esize_of(t) == 1) k_permute_columns<1><<<grid, block, lds, st>>>(a, p, o, M, K, lda, ldp);
    else k_permute_columns<2><<<grid, block, lds, st>>>(a, p, o, M, K, lda, ldp);
    return launch_result();
}

sp24_status launch_permute_rows(const void* A, const void* perm, void* P, int64_t M, int64_t K, int64_t lda, int64_t ldp, sp24_dtype t,
                                hipStream_t st)
{
    if (M * K == 0) return SP24_OK;
    const int es = esize_of(t);
    const int64_t passes = (M + kPermWaves - 1) / kPermWaves;
    const dim3 grid((unsigned)(passes < 4096 ? passes : 4096)), block(64 * kPermWaves);
    k_permute_rows<<<grid, block, 0, st>>>(static_cast<const uint8_t*>(A), static_cast<const int32_t*>(perm), static_cast<uint8_t*>(P), M,
                                           K * es, lda * es, ldp * es);
    return launch_result();
}

sp24_status launch_retained_magnitude(const void* A, const void* perm, double* out, int64_t M, int64_t K, int64_t lda, sp24_dtype t,
                                      hipStream_t st)
{
    static const bool ready = allow_lds(k_retained_magnitude<SP24_F16>) && allow_lds(k_retained_magnitude<SP24_BF16>) &&
                              allow_lds(k_retained_magnitude<SP24_I8>) && allow_lds(k_retained_magnitude<SP24_F8>);
    if (!ready) return SP24_ERR_LAUNCH;
    k_zero_double<<<1, 1, 0, st>>>(out);
    if (M * K != 0) {
        const dim3 grid(grid_for_rows(M)), block(64 * kPermWaves);
        const uint8_t* a = static_cast<const uint8_t*>(A);
        const int32_t* p = static_cast<const int32_t*>(perm);
        const size_t lds = p ? staged_lds_bytes(K, esize_of(t)) : 0;   // the given order needs no staging
        if (t == SP24_F16) k_retained_magnitude<SP24_F16><<<grid, block, lds, st>>>(a, p, out, M, K, lda);
        else if (t == SP24_BF16) k_retained_magnitude<SP24_BF16><<<grid, block, lds, st>>>(a, p, out, M, K, lda);
        else if (t == SP24_F8) k_retained_magnitude<SP24_F8><<<grid, block, lds, st>>>(a, p, out, M, K, lda);
        else k_retained_magnitude<SP24_I8><<<grid, block, lds, st>>>(a, p, out, M, K, lda);
    }
    return launch_result();
}

} // namespace sp24
