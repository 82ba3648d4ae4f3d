// Diagnostic kernels for the benchmark (libmaxsim_probe.so, declared in include/maxsim_probe.h; not part of the
// operator's library): what the machine sustains, measured beside the real kernels.
//   probe_mfma   register-only MFMA loop on caller-supplied operand bits (random data makes the
//                part run at the clocks it holds under load; zeros show the unthrottled rate)
//   probe_read   pure streaming read of a buffer, with plain loads or with the non-temporal hint
//   probe_copy   plain copy of known size (calibrates the HBM byte counters of the profiler)
//   probe_gather random gathers of whole 256-byte rows from a table (what the caches deliver to the access
//                pattern of the backward: a row per edge)
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
            if (KIND == 0) {
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

// NT = false: grid-stride loop, plain loads.  NT = true: every wavefront reads a contiguous run of its own (the way
// the streaming kernels walk a corpus) with loads that carry the non-temporal hint: the fastest read stream found
// on this part.
template <bool NT> __global__ void __launch_bounds__(256) probe_read_kernel(const uint4 *p, int64_t n_vec, float *sink)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    uint32_t acc = 0;
    if (NT) {
        const int64_t waves = (int64_t)gridDim.x * 4;
        const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
        const int64_t per = (n_vec / 64 + waves - 1) / waves * 64; // 16-byte pieces per run, whole KB
        int64_t i = wave * per + (threadIdx.x & 63);
        const int64_t end = (wave + 1) * per < n_vec ? (wave + 1) * per : n_vec;
        for (; i + 7 * 64 < end; i += 8 * 64) { // eight loads of 1 KB in flight per wavefront
            u32x4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k)
                v[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p + i + k * 64));
#pragma unroll
            for (int k = 0; k < 8; ++k)
                acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
        }
        for (; i < end; i += 64) {
            uint4 v = p[i];
            acc ^= v.x ^ v.y ^ v.z ^ v.w;
        }
    } else {
        int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
        const int64_t stride = (int64_t)gridDim.x * 256;
        for (; i + 7 * stride < n_vec; i += 8 * stride) { // eight 16-byte loads in flight per lane
            uint4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k)
                v[k] = p[i + k * stride];
#pragma unroll
            for (int k = 0; k < 8; ++k)
                acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
        }
        for (; i < n_vec; i += stride) {
            uint4 v = p[i];
            acc ^= v.x ^ v.y ^ v.z ^ v.w;
        }
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

// Every wavefront gathers iters x 16 pseudo-random 256-byte rows of a table of `rows` rows (a power of two), sixteen
// loads in flight.  KIND 0: one row per load instruction (a dword per lane), KIND 1: four rows per load instruction
// (sixteen lanes x 16 bytes per row).
template <int KIND>
__global__ void __launch_bounds__(256) probe_gather_kernel(const char *table, uint32_t rows, int iters, float *sink)
{
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane((blockIdx.x * 256 + threadIdx.x) >> 6);
    const uint32_t seed = KIND == 0 ? wave : wave * 4 + (lane >> 4);
    const uint32_t lane_off = KIND == 0 ? lane * 4 : (lane & 15) * 16;
    uint32_t acc = 0;
    for (int it = 0; it < iters; ++it) {
        uint32_t v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            uint32_t h = (seed * 0x9E3779B1u + (uint32_t)(it * 16 + u)) * 0x85EBCA6Bu;
            h ^= h >> 15;
            const char *at = table + (uint64_t)(h & (rows - 1)) * 256 + lane_off;
            if (KIND == 0) {
                v[u] = *reinterpret_cast<const uint32_t *>(at);
            } else {
                const uint4 x = *reinterpret_cast<const uint4 *>(at);
                v[u] = x.x ^ x.y ^ x.z ^ x.w;
            }
        }
#pragma unroll
        for (int u = 0; u < 16; ++u)
            acc ^= v[u];
    }
    if (acc == 0x12345678u && iters < 0)
        sink[0] = 1.0f;
}

static hipError_t probe_gather_launch(int kind, const void *table, uint32_t rows, int iters, float *sink, int num_cu,
                                      hipStream_t stream)
{
    const char *t = static_cast<const char *>(table);
    if (kind == 0)
        hipLaunchKernelGGL((probe_gather_kernel<0>), dim3(num_cu * 4), dim3(256), 0, stream, t, rows, iters, sink);
    else
        hipLaunchKernelGGL((probe_gather_kernel<1>), dim3(num_cu * 4), dim3(256), 0, stream, t, rows, iters, sink);
    return hipGetLastError();
}

static hipError_t probe_mfma_launch(int kind, const void *operands, int iters, float *sink, hipStream_t stream)
{
    const uint4 *in = static_cast<const uint4 *>(operands);
    switch (kind) {
    case 0: hipLaunchKernelGGL((probe_mfma_kernel<0>), dim3(PROBE_BLOCKS), dim3(256), 0, stream, in, iters, sink); break;
    case 1: hipLaunchKernelGGL((probe_mfma_kernel<1>), dim3(PROBE_BLOCKS), dim3(256), 0, stream, in, iters, sink); break;
    default: hipLaunchKernelGGL((probe_mfma_kernel<2>), dim3(PROBE_BLOCKS), dim3(256), 0, stream, in, iters, sink); break;
    }
    return hipGetLastError();
}

static hipError_t probe_read_launch(const void *buf, int64_t bytes, float *sink, bool streaming, int num_cu, hipStream_t stream)
{
    if (streaming) // sixteen long runs per CU (more and shorter runs read 3 % slower)
        hipLaunchKernelGGL(probe_read_kernel<true>, dim3(num_cu * 4), dim3(256), 0, stream, static_cast<const uint4 *>(buf),
                           bytes / 16, sink);
    else
        hipLaunchKernelGGL(probe_read_kernel<false>, dim3(num_cu * 8), dim3(256), 0, stream, static_cast<const uint4 *>(buf),
                           bytes / 16, sink);
    return hipGetLastError();
}

static hipError_t probe_copy_launch(const void *src, void *dst, int64_t bytes, int num_cu, hipStream_t stream)
{
    hipLaunchKernelGGL(probe_copy_kernel, dim3(num_cu * 8), dim3(256), 0, stream, static_cast<const uint4 *>(src),
                       static_cast<uint4 *>(dst), bytes / 16);
    return hipGetLastError();
}

} // namespace maxsim

#include "../../include/maxsim_probe.h"

namespace {
int probe_num_cu()
{
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
        return 256;
    return n;
}
bool probe_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
} // namespace

extern "C" {

int maxsim_probe_mfma(int kind, const void *operands, int iters, float *sink, void *stream)
{
    if (!operands || !sink || iters < 1 || kind < 0 || kind > 2 || !probe_aligned16(operands))
        return MAXSIM_ERR_INVALID;
    return maxsim::probe_mfma_launch(kind, operands, iters, sink, static_cast<hipStream_t>(stream)) == hipSuccess ? MAXSIM_OK
                                                                                                         : MAXSIM_ERR_LAUNCH;
}

int maxsim_probe_read(const void *buf, int64_t bytes, float *sink, void *stream)
{
    if (!buf || !sink || bytes < 16 || !probe_aligned16(buf))
        return MAXSIM_ERR_INVALID;
    return maxsim::probe_read_launch(buf, bytes, sink, false, probe_num_cu(), static_cast<hipStream_t>(stream)) == hipSuccess
               ? MAXSIM_OK
               : MAXSIM_ERR_LAUNCH;
}

int maxsim_probe_read_streaming(const void *buf, int64_t bytes, float *sink, void *stream)
{
    if (!buf || !sink || bytes < 16 || !probe_aligned16(buf))
        return MAXSIM_ERR_INVALID;
    return maxsim::probe_read_launch(buf, bytes, sink, true, probe_num_cu(), static_cast<hipStream_t>(stream)) == hipSuccess
               ? MAXSIM_OK
               : MAXSIM_ERR_LAUNCH;
}

int maxsim_probe_copy(const void *src, void *dst, int64_t bytes, void *stream)
{
    if (!src || !dst || bytes < 16 || !probe_aligned16(src) || !probe_aligned16(dst))
        return MAXSIM_ERR_INVALID;
    return maxsim::probe_copy_launch(src, dst, bytes, probe_num_cu(), static_cast<hipStream_t>(stream)) == hipSuccess
               ? MAXSIM_OK
               : MAXSIM_ERR_LAUNCH;
}

int64_t maxsim_probe_gather(int kind, const void *table, int64_t rows, int iters, float *sink, void *stream)
{
    if (!table || !sink || iters < 1 || kind < 0 || kind > 1 || rows < 1 || rows > (int64_t(1) << 30) || (rows & (rows - 1)) ||
        !probe_aligned16(table))
        return MAXSIM_ERR_INVALID;
    const int cus = probe_num_cu();
    if (maxsim::probe_gather_launch(kind, table, (uint32_t)rows, iters, sink, cus, static_cast<hipStream_t>(stream)) != hipSuccess)
        return MAXSIM_ERR_LAUNCH;
    return (int64_t)cus * 16 * iters * 16 * (kind == 0 ? 1 : 4); // rows gathered by this launch
}

} // extern "C"
