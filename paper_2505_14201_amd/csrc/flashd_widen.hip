// fp8 (e4m3) -> f16 / bf16, exact, for the kernels that read K and V through the direct
// global->LDS copies (which cannot convert on the way): flashd_attn_fwd_kv8 on shapes the
// decode kernel does not serve first widens K and V into scratch memory.  16 elements per
// thread: one 16-byte load, two 16-byte stores.
#include "flashd_common.h"
#include "flashd_kernels.h"
#include "flashd_mma.h"

namespace flashd {

template <typename T>
__global__ __launch_bounds__(256)
void widen_fp8_kernel(const uint8_t* __restrict__ k8, const uint8_t* __restrict__ v8,
                      uint16_t* __restrict__ k, uint16_t* __restrict__ v, size_t chunks) {
    for (size_t c = (size_t)blockIdx.x * blockDim.x + threadIdx.x; c < chunks;
         c += (size_t)gridDim.x * blockDim.x) {
        const u32x4 rk = *reinterpret_cast<const u32x4*>(k8 + 16 * c);
        const u32x4 rv = *reinterpret_cast<const u32x4*>(v8 + 16 * c);
        u32x4 w[4];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const u32x4 raw = i == 0 ? rk : rv;
            w[2 * i] = u32x4{Mma<T>::from_fp8_lo(raw[0]), Mma<T>::from_fp8_hi(raw[0]),
                             Mma<T>::from_fp8_lo(raw[1]), Mma<T>::from_fp8_hi(raw[1])};
            w[2 * i + 1] = u32x4{Mma<T>::from_fp8_lo(raw[2]), Mma<T>::from_fp8_hi(raw[2]),
                                 Mma<T>::from_fp8_lo(raw[3]), Mma<T>::from_fp8_hi(raw[3])};
        }
        *reinterpret_cast<u32x4*>(k + 16 * c) = w[0];
        *reinterpret_cast<u32x4*>(k + 16 * c + 8) = w[1];
        *reinterpret_cast<u32x4*>(v + 16 * c) = w[2];
        *reinterpret_cast<u32x4*>(v + 16 * c + 8) = w[3];
    }
}

hipError_t launch_widen_fp8(const void* k8, const void* v8, void* k, void* v, size_t elements,
                            int dtype, hipStream_t st) {
    const size_t chunks = elements / 16;          // d is a multiple of 64
    const size_t want = (chunks + 255) / 256;
    const unsigned grid = (unsigned)(want < 16384 ? (want ? want : 1) : 16384);
    if (dtype == 1)
        hipLaunchKernelGGL(widen_fp8_kernel<F16>, dim3(grid), dim3(256), 0, st,
                           static_cast<const uint8_t*>(k8), static_cast<const uint8_t*>(v8),
                           static_cast<uint16_t*>(k), static_cast<uint16_t*>(v), chunks);
    else if (dtype == 2)
        hipLaunchKernelGGL(widen_fp8_kernel<BF16>, dim3(grid), dim3(256), 0, st,
                           static_cast<const uint8_t*>(k8), static_cast<const uint8_t*>(v8),
                           static_cast<uint16_t*>(k), static_cast<uint16_t*>(v), chunks);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace flashd
