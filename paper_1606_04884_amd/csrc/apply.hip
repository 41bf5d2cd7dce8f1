// Per-element ("Apply") kernel of the paper's Sec. 3.3 experiment: bandwidth of a
// per-element operation as a function of the number of floats per launch.  The
// paper does not name the operation it timed; this one is a scalar multiply
// followed by a scalar add, y[i] = fl(fl(a * x[i]) + b), with the two operations
// rounded separately as two Torch calls (mul, add) fused into one pass would be.
// Memory-bound: 8 bytes per element.

#include "conv_internal.h"

namespace mi355conv {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// fl(fl(a * v) + b): contraction into a fused multiply-add switched off for this
// expression (the definition has two roundings)
__device__ __forceinline__ float mul_then_add(float a, float v, float b)
{
#pragma clang fp contract(off)
    const float t = a * v;
    return t + b;
}

// Vector body: 16-byte loads and stores, grid-stride; needs x and y 16-byte aligned.
__global__ __launch_bounds__(256) void apply_mul_add_vec_kernel(const floatx4 *__restrict__ x,
                                                                floatx4 *__restrict__ y, int64_t nvec,
                                                                float a, float b)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += stride) {
        const floatx4 v = x[i];
        floatx4 r;
        r[0] = mul_then_add(a, v[0], b);
        r[1] = mul_then_add(a, v[1], b);
        r[2] = mul_then_add(a, v[2], b);
        r[3] = mul_then_add(a, v[3], b);
        y[i] = r;
    }
}

// Scalar body: the tail of the vector kernel, or everything when a pointer is not
// 16-byte aligned.
__global__ __launch_bounds__(256) void apply_mul_add_scalar_kernel(const float *__restrict__ x,
                                                                   float *__restrict__ y, int64_t first,
                                                                   int64_t n, float a, float b)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = first + (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride)
        y[i] = mul_then_add(a, x[i], b);
}

hipError_t launch_apply_mul_add(const float *x, float *y, int64_t n, float a, float b, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const bool aligned = (((uintptr_t)x | (uintptr_t)y) & 15) == 0;
    const int64_t nvec = aligned ? n / 4 : 0;
    if (nvec > 0) {
        // 8 vectors in flight per thread at most: enough workgroups to fill the chip
        // for large tensors, one pass for small ones
        int64_t blocks = (nvec + 255) / 256;
        if (blocks > 256 * 16) blocks = 256 * 16;
        hipLaunchKernelGGL(apply_mul_add_vec_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                           reinterpret_cast<const floatx4 *>(x), reinterpret_cast<floatx4 *>(y), nvec, a, b);
    }
    const int64_t first = nvec * 4;
    if (first < n) {
        int64_t blocks = (n - first + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(apply_mul_add_scalar_kernel, dim3((unsigned)blocks), dim3(256), 0, s, x, y,
                           first, n, a, b);
    }
    return hipGetLastError();
}

}  // namespace mi355conv
