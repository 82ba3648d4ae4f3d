// Diagnostic kernels: what the machine sustains, measured beside the real kernels.
//   probe_mfma   register-only MFMA loop on caller-supplied operand bits (random data makes the
//                part run at the clocks it holds under load; zeros show the unthrottled rate)
//   probe_read   pure streaming read of a buffer
//   probe_copy   plain copy of known size (calibrates the HBM byte counters of the profiler)
#include "common.h"

namespace maxsim {

constexpr int PROBE_BLOCKS = 512; // two workgroups of four wavefronts per CU on a 256-CU part

template <int KIND>
__global__ void __launch_bounds__(256) probe_mfma_kernel(const uint4 *in, int iters, float *sink)
{
    const int t = threadIdx.x + blockIdx.x * 256;
    uint4 a = in[t & 0xffff], b0 = in[(t * 3 + 1) & 0xffff], b1 = in[(t * 5 + 2) & 0xffff], b2 = in[(t * 7 + 3) & 0xffff],
          b3 = in[(t * 11 + 4) & 0xffff];
    float s = 0.0f;
    if (KIND == 2) {
        i32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
        for (int it = 0; it < iters; ++it) {
            c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b0), c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b1), c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b2), c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(i32x4, a), __builtin_bit_cast(i32x4, b3), c3, 0, 0, 0);
        }
        for (int i = 0; i < 16; ++i)
            s += (float)(c0[i] + c1[i] + c2[i] + c3[i]);
    } else {
        f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
        for (int it = 0; it < iters; ++it) {
            if (KIND == 3) { // one dependent chain: every MFMA needs the result of the one before
                Traits<MAXSIM_F16>::mma(a, b0, c0);
                Traits<MAXSIM_F16>::mma(a, b1, c0);
                Traits<MAXSIM_F16>::mma(a, b2, c0);
                Traits<MAXSIM_F16>::mma(a, b3, c0);
            } else if (KIND == 0) {
                Traits<MAXSIM_F16>::mma(a, b0, c0);
                Traits<MAXSIM_F16>::mma(a, b1, c1);
                Traits<MAXSIM_F16>::mma(a, b2, c2);
                Traits<MAXSIM_F16>::mma(a, b3, c3);
            } else {
                Traits<MAXSIM_BF16>::mma(a, b0, c0);
                Traits<MAXSIM_BF16>::mma(a, b1, c1);
                Traits<MAXSIM_BF16>::mma(a, b2, c2);
                Traits<MAXSIM_BF16>::mma(a, b3, c3);
            }
        }
        for (int i = 0; i < 16; ++i)
            s += c0[i] + c1[i] + c2[i] + c3[i];
    }
    if (s == 123.456f) // never true for real data; keeps the loop alive
        sink[0] = s;
}

__global__ void __launch_bounds__(256) probe_read_kernel(const uint4 *p, int64_t n_vec, float *sink)
{
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * 256;
    uint32_t acc = 0;
    for (; i + 3 * stride < n_vec; i += 4 * stride) {
        uint4 v0 = p[i], v1 = p[i + stride], v2 = p[i + 2 * stride], v3 = p[i + 3 * stride];
        acc ^= v0.x ^ v0.y ^ v0.z ^ v0.w ^ v1.x ^ v1.y ^ v1.z ^ v1.w ^ v2.x ^ v2.y ^ v2.z ^ v2.w ^ v3.x ^ v3.y ^ v3.z ^ v3.w;
    }
    for (; i < n_vec; i += stride) {
        uint4 v = p[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x12345678u)
        sink[0] = 1.0f;
}

__global__ void __launch_bounds__(256) probe_copy_kernel(const uint4 *src, uint4 *dst, int64_t n_vec)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride)
        dst[i] = src[i];
}

hipError_t probe_mfma_launch(int kind, const void *operands, int iters, float *sink, hipStream_t stream)
{
    const uint4 *in = static_cast<const uint4 *>(operands);
    switch (kind) {
    case 0: hipLaunchKernelGGL((probe_mfma_kernel<0>), dim3(PROBE_BLOCKS), dim3(256), 0, stream, in, iters, sink); break;
    case 1: hipLaunchKernelGGL((probe_mfma_kernel<1>), dim3(PROBE_BLOCKS), dim3(256), 0, stream, in, iters, sink); break;
    case 3: hipLaunchKernelGGL((probe_mfma_kernel<3>), dim3(PROBE_BLOCKS), dim3(256), 0, stream, in, iters, sink); break;
    default: hipLaunchKernelGGL((probe_mfma_kernel<2>), dim3(PROBE_BLOCKS), dim3(256), 0, stream, in, iters, sink); break;
    }
    return hipGetLastError();
}

hipError_t probe_read_launch(const void *buf, int64_t bytes, float *sink, int num_cu, hipStream_t stream)
{
    hipLaunchKernelGGL(probe_read_kernel, dim3(num_cu * 8), dim3(256), 0, stream, static_cast<const uint4 *>(buf),
                       bytes / 16, sink);
    return hipGetLastError();
}

hipError_t probe_copy_launch(const void *src, void *dst, int64_t bytes, int num_cu, hipStream_t stream)
{
    hipLaunchKernelGGL(probe_copy_kernel, dim3(num_cu * 8), dim3(256), 0, stream, static_cast<const uint4 *>(src),
                       static_cast<uint4 *>(dst), bytes / 16);
    return hipGetLastError();
}

} // namespace maxsim
