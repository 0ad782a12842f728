// Device-side writer of the synthetic feature table: the same recipe as fg_inputs/features.py
// (SplitMix64 word per element, four 16-bit fields summed, centred, one fp32 multiply), so that a table
// too large to build on the host can be filled where it lives (HBM, or pinned host memory through its
// device mapping). Input generation only: no step of the method under test is in this file.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint64_t mix64(uint64_t x) {
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

__device__ __forceinline__ float feature_value(uint64_t key, uint64_t ctr) {
    const uint64_t w = mix64(key + (ctr + 1ull) * 0x9E3779B97F4A7C15ull);
    const int s = (int)(w & 0xFFFF) + (int)((w >> 16) & 0xFFFF) + (int)((w >> 32) & 0xFFFF) + (int)(w >> 48);
    return (float)(s - 131070) * __uint_as_float(0x37DDB3D7u);
}

template <typename T>
__global__ void fill_features_kernel(T* out, uint64_t key, int64_t first_row, int64_t rows, int dim) {
    const int64_t total = rows * dim;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const uint64_t base = (uint64_t)first_row * (uint64_t)dim;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        float v = feature_value(key, base + (uint64_t)i);
        if constexpr (sizeof(T) == 4) {
            out[i] = v;
        } else {
            // The fp16 value is the fp32 product rounded once more. Left to itself the compiler may merge multiply and
            // conversion into one mixed-precision instruction that rounds the exact product straight to fp16, which
            // differs where the fp32 product lands on an fp16 tie; the empty statement keeps the two roundings apart.
            asm volatile("" : "+v"(v));
            out[i] = __float2half_rn(v);
        }
    }
}

}  // namespace

// Fills rows [first_row, first_row + rows) of a [*, dim] table whose storage for those rows starts at `out`
// (device pointer, or mapped host pointer). elem_bytes = 4 (fp32) or 2 (fp16). Returns 0 on success.
extern "C" int fgin_fill_features(void* out, uint64_t key, int64_t first_row, int64_t rows, int dim, int elem_bytes,
                                  void* stream) {
    if (!out || rows < 0 || dim <= 0 || (elem_bytes != 4 && elem_bytes != 2)) return 1;
    if (rows == 0) return 0;
    const int64_t total = rows * dim;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (elem_bytes == 4)
        hipLaunchKernelGGL(fill_features_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           (float*)out, key, first_row, rows, dim);
    else
        hipLaunchKernelGGL(fill_features_kernel<__half>, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                           (__half*)out, key, first_row, rows, dim);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
