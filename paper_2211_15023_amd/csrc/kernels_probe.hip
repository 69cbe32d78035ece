// Measurement aids, not part of the method: register-resident MFMA loops that give the matrix-core rate
// this machine sustains (the ceiling the int8 / bf16 layers are compared with), and a streaming copy.
#include "accerl_internal.h"

namespace accerl {

template <int EL>
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, int* __restrict__ sink) {
    const int lane = threadIdx.x & 63;
    v4i a = {lane, lane + 1, lane + 2, lane + 3}, b = {lane ^ 5, lane ^ 9, lane ^ 17, lane ^ 33};
    v4i ci[8];
    v4f cf[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) { ci[k] = (v4i){k, 0, 0, 0}; cf[k] = (v4f){(float)k, 0.f, 0.f, 0.f}; }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {     // eight independent accumulators: no dependency stalls
            if constexpr (EL == EL_I8) ci[k] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, ci[k], 0, 0, 0);
            else cf[k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), cf[k], 0, 0, 0);
        }
    }
    int acc = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) acc += (EL == EL_I8) ? ci[k][0] : (int)cf[k][0];
    if (acc == 0x7fffffff) sink[0] = acc;     // keeps the loop alive, never true in practice
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const v4i* __restrict__ src, v4i* __restrict__ dst, int64_t n16) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

// nothing at all: what one launch costs on this machine
__global__ void empty_kernel() {}

}  // namespace accerl

using namespace accerl;

extern "C" int accerl_probe_empty(void* hip_stream) {
    empty_kernel<<<dim3(1), dim3(64), 0, (hipStream_t)hip_stream>>>();
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? ACCERL_OK : set_error(ACCERL_EHIP, hipGetErrorString(e));
}

extern "C" int accerl_probe_mfma(int32_t bf16, int32_t iters, int32_t* sink, void* hip_stream) {
    if (iters < 1 || !sink) return set_error(ACCERL_EINVAL, "probe: iters >= 1 and a device sink word are needed");
    dim3 grid(256 * 8), block(256);          // eight workgroups of four wavefronts per compute unit
    if (bf16) mfma_loop_kernel<EL_BF16><<<grid, block, 0, (hipStream_t)hip_stream>>>(iters, sink);
    else mfma_loop_kernel<EL_I8><<<grid, block, 0, (hipStream_t)hip_stream>>>(iters, sink);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? ACCERL_OK : set_error(ACCERL_EHIP, hipGetErrorString(e));
}

extern "C" int accerl_probe_copy(const void* src, void* dst, int64_t bytes, void* hip_stream) {
    if (!src || !dst || bytes < 16 || (bytes & 15) || (((uintptr_t)src | (uintptr_t)dst) & 15))
        return set_error(ACCERL_EINVAL, "probe: 16-byte aligned buffers of a multiple of 16 bytes are needed");
    stream_copy_kernel<<<dim3(256 * 16), dim3(256), 0, (hipStream_t)hip_stream>>>((const v4i*)src, (v4i*)dst, bytes / 16);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? ACCERL_OK : set_error(ACCERL_EHIP, hipGetErrorString(e));
}
