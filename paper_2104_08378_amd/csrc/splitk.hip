// Second pass of a product whose inner dimension was split across workgroups: the partial products, one image per
// slice in the accumulator type, are added in slice order (so the result does not depend on which workgroup
// finished first) and converted to the output type.  Bound by reading the images once.
#include "common.hpp"
#include "launch.hpp"

namespace sp24 {

// One thread per four consecutive columns of a row (ldw is a multiple of 4 and the images are 16-byte aligned).
template <typename ACC, int OUT>
__global__ __launch_bounds__(256) void k_splitk_reduce(const ACC* partial, int slices, int64_t M, int64_t N, int64_t ldw, void* D, int64_t ldd)
{
    typedef ACC vec4 __attribute__((ext_vector_type(4)));
    const int64_t quads = ldw / 4;
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= M * quads) return;
    const int64_t row = id / quads, col = (id % quads) * 4;
    const int64_t image = M * ldw;
    const ACC* src = partial + row * ldw + col;
    vec4 sum = *reinterpret_cast<const vec4*>(src);
    for (int s = 1; s < slices; ++s) sum += *reinterpret_cast<const vec4*>(src + (int64_t)s * image);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (col + e < N) {
            if constexpr (std::is_same<ACC, int>::value) reinterpret_cast<int*>(D)[row * ldd + col + e] = sum[e];
            else store_out<OUT>(D, row * ldd + col + e, sum[e]);
        }
    }
}

sp24_status launch_splitk_reduce(const void* partial, int slices, int64_t M, int64_t N, int64_t ldw, void* D, int64_t ldd, bool integer,
                                 sp24_dtype out, hipStream_t st)
{
    const int64_t threads = M * (ldw / 4);
    if (threads == 0) return SP24_OK;
    const dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    if (integer) k_splitk_reduce<int, SP24_I32><<<grid, block, 0, st>>>(static_cast<const int*>(partial), slices, M, N, ldw, D, ldd);
    else if (out == SP24_F32) k_splitk_reduce<float, SP24_F32><<<grid, block, 0, st>>>(static_cast<const float*>(partial), slices, M, N, ldw, D, ldd);
    else if (out == SP24_F16) k_splitk_reduce<float, SP24_F16><<<grid, block, 0, st>>>(static_cast<const float*>(partial), slices, M, N, ldw, D, ldd);
    else k_splitk_reduce<float, SP24_BF16><<<grid, block, 0, st>>>(static_cast<const float*>(partial), slices, M, N, ldw, D, ldd);
    return hipGetLastError() == hipSuccess ? SP24_OK : SP24_ERR_LAUNCH;
}

} // namespace sp24
