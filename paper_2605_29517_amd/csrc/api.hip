// C ABI of the library: argument checks, device query, kernel selection.  See include/maxsim.h.
#include <hip/hip_runtime.h>

#include <mutex>

#include "common.h"

namespace maxsim {
hipError_t forward_launch(FwdParams p, int dtype, int d, int num_cu, hipStream_t stream);
bool forward_width_supported(int dtype, int d);
hipError_t backward_launch(const void *Q, int n_q, int l_q, const void *D, const int32_t *offsets, int64_t b, int l_d,
                           int64_t total_tokens, int d, int dtype, const int32_t *argmax, const float *dscore, float *dQ,
                           float *dD, int num_cu, hipStream_t stream);
hipError_t csr_build_launch(const int32_t *argmax, int n_q, int64_t b, int l_q, int l_d, int32_t *row_ptr,
                            int32_t *col_idx, int num_cu, hipStream_t stream);
hipError_t backward_csr_launch(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d, int dtype,
                               const int32_t *argmax, const float *dscore, int32_t *row_ptr, int32_t *col_idx, float *dQ,
                               float *dD, int num_cu, hipStream_t stream);
bool csr_static_fits(int n_q, int64_t b, int l_q, int l_d);
hipError_t backward_csr_static_launch(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d, int dtype,
                                      const int32_t *argmax, const float *dscore, float *dQ, float *dD, int num_cu,
                                      hipStream_t stream);
hipError_t quantize_launch(const void *X, int64_t rows, int dtype, int8_t *X_i8, float *scale, hipStream_t stream);
bool i8_wide_width_ok(int d);
hipError_t forward_i8_wide_launch(const int8_t *Q, const float *qs, int n_q, int l_q, const int8_t *D, const float *ds,
                                  const int32_t *offsets, int64_t b, int l_d, int64_t total_tokens, int d, float *scores,
                                  int64_t ld, int num_cu, hipStream_t stream);
hipError_t quantize_wide_launch(const void *X, int64_t rows, int d, int dtype, int8_t *X_i8, float *scale, hipStream_t stream);
hipError_t forward_i8_launch(const int8_t *Q, const float *qs, int n_q, int l_q, const int8_t *D, const float *ds,
                             const int32_t *offsets, int64_t b, int l_d, int64_t total_tokens, float *scores,
                             int64_t ld, int num_cu, hipStream_t stream);
hipError_t ce_grad_launch(const float *scores, int n, int b, float tau, float *g, float *loss, hipStream_t stream);
hipError_t forward_splitd_init_device();
hipError_t forward_i8_init_device();
hipError_t backward_init_device();
} // namespace maxsim

namespace {

bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

bool dtype_ok(int dt) { return dt == MAXSIM_F32 || dt == MAXSIM_F16 || dt == MAXSIM_BF16; }

// Compute-unit count of the current device, queried once per device.
int num_cu()
{
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

// int8 scoring: the kernels built around 128-byte rows, or (other widths) the slab kernel / the plain inner loop over d
static hipError_t i8_launch_any(const int8_t *Q, const float *qs, int n_q, int l_q, const int8_t *D, const float *ds,
                                const int32_t *offsets, int64_t b, int l_d, int64_t total_tokens, int d, float *scores,
                                int64_t ld, int cus, hipStream_t stream)
{
    if (d == maxsim::D_MODEL)
        return maxsim::forward_i8_launch(Q, qs, n_q, l_q, D, ds, offsets, b, l_d, total_tokens, scores, ld, cus, stream);
    return maxsim::forward_i8_wide_launch(Q, qs, n_q, l_q, D, ds, offsets, b, l_d, total_tokens, d, scores, ld, cus, stream);
}
static bool i8_width_ok(int d) { return d == maxsim::D_MODEL || maxsim::i8_wide_width_ok(d); }

// embedding widths of the backward entry points: whole 16-byte chunks of 8 elements, up to 64 slabs of 128 columns
bool backward_width_ok(int d) { return d >= 8 && d <= 8192 && d % 8 == 0; }
// the dD kernels address Q rows through 32-bit byte offsets: Q must stay below 4 GiB
// and the dQ kernel addresses D rows through 32-bit offsets in units of 16 bytes: D must stay below 64 GiB
bool backward_q_ok(int n_q, int l_q, int d, int dtype, int64_t total_tokens)
{
    const int64_t row_bytes = (int64_t)d * (dtype == MAXSIM_F32 ? 4 : 2);
    return (int64_t)n_q * l_q * row_bytes < (int64_t(1) << 32) && total_tokens <= ((int64_t(1) << 36) - 1) / row_bytes;
}

// Per-device set-up, done once per device under a lock (two host threads may make their first call at once):
// the kernels that use more than 64 KB of LDS are allowed to (every instantiation), and the static scratch
// array's device address is looked up.  maxsim_init runs it for the current device; every entry point runs it
// after its argument checks, so that callers who never call maxsim_init lose nothing but the freedom to make
// their first call on a device under stream capture.
int ensure_init()
{
    static bool done[64] = {};
    static std::mutex guard;
    std::lock_guard<std::mutex> lock(guard);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return MAXSIM_ERR_LAUNCH;
    if (done[dev])
        return MAXSIM_OK;
    if (maxsim::forward_splitd_init_device() != hipSuccess || maxsim::forward_i8_init_device() != hipSuccess ||
        maxsim::backward_init_device() != hipSuccess)
        return MAXSIM_ERR_LAUNCH;
    done[dev] = true;
    return MAXSIM_OK;
}

int finish(hipError_t e) { return e == hipSuccess ? MAXSIM_OK : MAXSIM_ERR_LAUNCH; }

// One copy stream per device for the out-of-core path, created on first use at the default
// priority and kept until the process ends.
hipStream_t copy_stream()
{
    static hipStream_t cached[64] = {nullptr};
    static std::mutex guard; // two host threads may make their first streamed call at once
    std::lock_guard<std::mutex> lock(guard);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return nullptr;
    if (!cached[dev]) {
        hipStream_t st = nullptr;
        if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess)
            return nullptr;
        cached[dev] = st;
    }
    return cached[dev];
}

int forward_common(const void *Q, int n_q, int l_q, const void *D, const int32_t *offsets, int64_t b, int l_d,
                   int64_t total_tokens, int d, int dtype, float *scores, int32_t *argmax, void *stream)
{
    if (!Q || !D || !scores || n_q < 1 || l_q < 1 || b < 1 || !dtype_ok(dtype))
        return MAXSIM_ERR_INVALID;
    if (!aligned(Q, 16) || !aligned(D, 16) || !aligned(scores, 4) || !aligned(argmax, 4) || !aligned(offsets, 4))
        return MAXSIM_ERR_INVALID;
    if (!maxsim::forward_width_supported(dtype, d))
        return MAXSIM_ERR_UNSUPPORTED;
    // index ranges the kernels rely on: token counts and block ids fit in int32
    if (total_tokens >= (int64_t(1) << 31) || (int64_t)n_q * ((l_q + 31) / 32) >= (int64_t(1) << 24) ||
        b >= (int64_t(1) << 31))
        return MAXSIM_ERR_UNSUPPORTED;
    maxsim::FwdParams p = {};
    p.Q = static_cast<const char *>(Q);
    p.D = static_cast<const char *>(D);
    p.offsets = offsets;
    p.scores = scores;
    p.argmax = argmax;
    p.b = b;
    p.total_tokens = total_tokens;
    p.n_q = n_q;
    p.l_q = l_q;
    p.l_d = l_d;
    if (int rc = ensure_init())
        return rc;
    return finish(maxsim::forward_launch(p, dtype, d, num_cu(), static_cast<hipStream_t>(stream)));
}

// Out-of-core driver shared by the streamed entry points: block k + 1 is copied on the copy stream while
// block k is scored on the caller's stream; two staging halves, events in both directions.
// copy(half, first, docs, copy_stream) enqueues the host-to-device copies of a block,
// launch(half, first, docs) enqueues its kernel on the caller's stream.
template <typename Copy, typename Launch>
int stream_blocks(hipStream_t compute, int64_t b, int64_t block_docs, Copy copy_block, Launch launch_block)
{
    hipStream_t copy = copy_stream();
    if (!copy)
        return MAXSIM_ERR_LAUNCH;
    // events: block k copied (per staging half), staging half free again (its kernel has run)
    hipEvent_t copied[2] = {nullptr, nullptr}, freed[2] = {nullptr, nullptr}, entry = nullptr;
    bool ok = hipEventCreateWithFlags(&entry, hipEventDisableTiming) == hipSuccess;
    for (int i = 0; i < 2 && ok; ++i)
        ok = hipEventCreateWithFlags(&copied[i], hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&freed[i], hipEventDisableTiming) == hipSuccess;
    int rc = ok ? MAXSIM_OK : MAXSIM_ERR_LAUNCH;
    // the staging buffer may still be in use by work already enqueued on the caller's stream
    if (rc == MAXSIM_OK && (hipEventRecord(entry, compute) != hipSuccess || hipStreamWaitEvent(copy, entry, 0) != hipSuccess))
        rc = MAXSIM_ERR_LAUNCH;
    const int64_t n_blocks = (b + block_docs - 1) / block_docs;
    for (int64_t k = 0; k < n_blocks && rc == MAXSIM_OK; ++k) {
        const int half = (int)(k & 1);
        const int64_t first = k * block_docs;
        const int64_t docs = (b - first < block_docs) ? b - first : block_docs;
        hipError_t e = hipSuccess;
        if (k >= 2)
            e = hipStreamWaitEvent(copy, freed[half], 0); // the kernel that read this half two blocks ago
        if (e == hipSuccess)
            e = copy_block(half, first, docs, copy);
        if (e == hipSuccess)
            e = hipEventRecord(copied[half], copy);
        if (e == hipSuccess)
            e = hipStreamWaitEvent(compute, copied[half], 0);
        if (e == hipSuccess)
            e = launch_block(half, first, docs);
        if (e == hipSuccess)
            e = hipEventRecord(freed[half], compute);
        if (e != hipSuccess)
            rc = MAXSIM_ERR_LAUNCH;
    }
    // destroying an event that is still pending only releases it once it has completed
    if (entry)
        (void)hipEventDestroy(entry);
    for (int i = 0; i < 2; ++i) {
        if (copied[i])
            (void)hipEventDestroy(copied[i]);
        if (freed[i])
            (void)hipEventDestroy(freed[i]);
    }
    return rc;
}

} // namespace

extern "C" {

int maxsim_init(void) { return ensure_init(); }

const char *maxsim_strerror(int code)
{
    switch (code) {
    case MAXSIM_OK: return "ok";
    case MAXSIM_ERR_INVALID: return "invalid argument (null or misaligned pointer, non-positive size, bad dtype)";
    case MAXSIM_ERR_UNSUPPORTED: return "unsupported shape (an embedding width or a size outside what this entry point is built for)";
    case MAXSIM_ERR_LAUNCH: return "HIP reported an error at kernel launch";
    case MAXSIM_ERR_SCRATCH: return "sizes exceed the library's static scratch buffer (use the entry point that takes caller buffers)";
    default: return "unknown maxsim error code";
    }
}

int maxsim_forward(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d, maxsim_dtype dtype,
                   float *scores, int32_t *argmax, void *stream)
{
    if (l_d < 1)
        return MAXSIM_ERR_INVALID;
    if (b > 0 && (int64_t)l_d > ((int64_t(1) << 31) - 1) / b)
        return (Q && D && scores) ? MAXSIM_ERR_UNSUPPORTED : MAXSIM_ERR_INVALID;
    return forward_common(Q, n_q, l_q, D, nullptr, b, l_d, b * (int64_t)l_d, d, (int)dtype, scores, argmax, stream);
}

int maxsim_forward_streamed(const void *Q, int n_q, int l_q, const void *D_host, int64_t b, int l_d, int d,
                            maxsim_dtype dtype, int64_t block_docs, void *staging, float *scores, void *stream)
{
    if (!Q || !D_host || !staging || !scores || n_q < 1 || l_q < 1 || b < 1 || l_d < 1 || block_docs < 1 ||
        !dtype_ok((int)dtype))
        return MAXSIM_ERR_INVALID;
    if (!aligned(Q, 16) || !aligned(D_host, 16) || !aligned(staging, 16) || !aligned(scores, 4))
        return MAXSIM_ERR_INVALID;
    if (!maxsim::forward_width_supported((int)dtype, d))
        return MAXSIM_ERR_UNSUPPORTED;
    if (block_docs > b)
        block_docs = b;
    if (block_docs > ((int64_t(1) << 31) - 1) / l_d || (int64_t)n_q * ((l_q + 31) / 32) >= (int64_t(1) << 24))
        return MAXSIM_ERR_UNSUPPORTED;
    const int64_t doc_bytes = (int64_t)l_d * d * ((int)dtype == MAXSIM_F32 ? 4 : 2);
    if (int rc = ensure_init())
        return rc;
    hipStream_t compute = static_cast<hipStream_t>(stream);
    const int cus = num_cu();
    return stream_blocks(
        compute, b, block_docs,
        [&](int half, int64_t first, int64_t docs, hipStream_t copy) {
            return hipMemcpyAsync(static_cast<char *>(staging) + half * block_docs * doc_bytes,
                                  static_cast<const char *>(D_host) + first * doc_bytes, (size_t)(docs * doc_bytes),
                                  hipMemcpyHostToDevice, copy);
        },
        [&](int half, int64_t first, int64_t docs) {
            maxsim::FwdParams p = {};
            p.Q = static_cast<const char *>(Q);
            p.D = static_cast<const char *>(staging) + half * block_docs * doc_bytes;
            p.scores = scores + first;
            p.b = docs;
            p.ld = b;
            p.total_tokens = docs * (int64_t)l_d;
            p.n_q = n_q;
            p.l_q = l_q;
            p.l_d = l_d;
            return maxsim::forward_launch(p, (int)dtype, d, cus, compute);
        });
}

int maxsim_forward_i8_streamed(const int8_t *Q_i8, const float *q_scale, int n_q, int l_q, const int8_t *D_i8_host,
                               const float *d_scale_host, int64_t b, int l_d, int d, int64_t block_docs,
                               int8_t *staging_codes, float *staging_scales, float *scores, void *stream)
{
    if (!Q_i8 || !q_scale || !D_i8_host || !d_scale_host || !staging_codes || !staging_scales || !scores || n_q < 1 ||
        l_q < 1 || b < 1 || l_d < 1 || block_docs < 1)
        return MAXSIM_ERR_INVALID;
    if (!aligned(Q_i8, 16) || !aligned(D_i8_host, 16) || !aligned(staging_codes, 16) || !aligned(q_scale, 4) ||
        !aligned(d_scale_host, 4) || !aligned(staging_scales, 4) || !aligned(scores, 4))
        return MAXSIM_ERR_INVALID;
    if (!i8_width_ok(d))
        return MAXSIM_ERR_UNSUPPORTED;
    if (block_docs > b)
        block_docs = b;
    if (block_docs > ((int64_t(1) << 31) - 1) / l_d || (int64_t)n_q * ((l_q + 31) / 32) >= (int64_t(1) << 24) || l_q > 1024)
        return MAXSIM_ERR_UNSUPPORTED;
    const int64_t doc_bytes = (int64_t)l_d * d;
    if (int rc = ensure_init())
        return rc;
    hipStream_t compute = static_cast<hipStream_t>(stream);
    const int cus = num_cu();
    return stream_blocks(
        compute, b, block_docs,
        [&](int half, int64_t first, int64_t docs, hipStream_t copy) {
            hipError_t e = hipMemcpyAsync(staging_codes + half * block_docs * doc_bytes, D_i8_host + first * doc_bytes,
                                          (size_t)(docs * doc_bytes), hipMemcpyHostToDevice, copy);
            if (e != hipSuccess)
                return e;
            return hipMemcpyAsync(staging_scales + half * block_docs * l_d, d_scale_host + first * l_d,
                                  (size_t)(docs * l_d) * sizeof(float), hipMemcpyHostToDevice, copy);
        },
        [&](int half, int64_t first, int64_t docs) {
            return i8_launch_any(Q_i8, q_scale, n_q, l_q, staging_codes + half * block_docs * doc_bytes,
                                 staging_scales + half * block_docs * l_d, nullptr, docs, l_d, docs * (int64_t)l_d, d,
                                 scores + first, b, cus, compute);
        });
}

int maxsim_forward_ragged(const void *Q, int n_q, int l_q, const void *D_packed, const int32_t *doc_offsets, int64_t b,
                          int64_t total_tokens, int d, maxsim_dtype dtype, float *scores, int32_t *argmax, void *stream)
{
    if (!doc_offsets || total_tokens < 1)
        return MAXSIM_ERR_INVALID;
    return forward_common(Q, n_q, l_q, D_packed, doc_offsets, b, 0, total_tokens, d, (int)dtype, scores, argmax, stream);
}

int maxsim_backward(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d, maxsim_dtype dtype,
                    const int32_t *argmax, const float *dscore, float *dQ, float *dD, void *stream)
{
    if (!Q || !D || !argmax || !dscore || !dQ || !dD || n_q < 1 || l_q < 1 || b < 1 || l_d < 1 || !dtype_ok((int)dtype))
        return MAXSIM_ERR_INVALID;
    if (!aligned(Q, 16) || !aligned(D, 16) || !aligned(argmax, 4) || !aligned(dscore, 4) || !aligned(dQ, 16) ||
        !aligned(dD, 16))
        return MAXSIM_ERR_INVALID;
    if (b > ((int64_t(1) << 31) - 1) / l_d || (int64_t)n_q * l_q >= (int64_t(1) << 31) ||
        (int64_t)n_q * b >= (int64_t(1) << 40))
        return MAXSIM_ERR_UNSUPPORTED;
    if (!backward_width_ok(d) || !backward_q_ok(n_q, l_q, d, (int)dtype, b * (int64_t)l_d))
        return MAXSIM_ERR_UNSUPPORTED;
    if (int rc = ensure_init())
        return rc;
    return finish(maxsim::backward_launch(Q, n_q, l_q, D, nullptr, b, l_d, b * (int64_t)l_d, d, (int)dtype, argmax, dscore,
                                          dQ, dD, num_cu(), static_cast<hipStream_t>(stream)));
}

int maxsim_backward_ragged(const void *Q, int n_q, int l_q, const void *D_packed, const int32_t *doc_offsets, int64_t b,
                           int64_t total_tokens, int d, maxsim_dtype dtype, const int32_t *argmax, const float *dscore,
                           float *dQ, float *dD_packed, void *stream)
{
    if (!Q || !D_packed || !doc_offsets || !argmax || !dscore || !dQ || !dD_packed || n_q < 1 || l_q < 1 || b < 1 ||
        total_tokens < 1 || !dtype_ok((int)dtype))
        return MAXSIM_ERR_INVALID;
    if (!aligned(Q, 16) || !aligned(D_packed, 16) || !aligned(doc_offsets, 4) || !aligned(argmax, 4) ||
        !aligned(dscore, 4) || !aligned(dQ, 16) || !aligned(dD_packed, 16))
        return MAXSIM_ERR_INVALID;
    if (!backward_width_ok(d) || !backward_q_ok(n_q, l_q, d, (int)dtype, total_tokens))
        return MAXSIM_ERR_UNSUPPORTED;
    if (total_tokens >= (int64_t(1) << 31) || b >= (int64_t(1) << 31) || (int64_t)n_q * l_q >= (int64_t(1) << 31) ||
        (int64_t)n_q * b >= (int64_t(1) << 40))
        return MAXSIM_ERR_UNSUPPORTED;
    if (int rc = ensure_init())
        return rc;
    return finish(maxsim::backward_launch(Q, n_q, l_q, D_packed, doc_offsets, b, 0, total_tokens, d, (int)dtype, argmax,
                                          dscore, dQ, dD_packed, num_cu(), static_cast<hipStream_t>(stream)));
}

static bool csr_shape_ok(int n_q, int64_t b, int l_q, int l_d)
{
    return l_d <= 4096 && b * (int64_t)l_d < (int64_t(1) << 31) - 1 && b < (int64_t(1) << 31) &&
           (int64_t)n_q * l_q < (int64_t(1) << 31) && (int64_t)n_q * l_q * b < (int64_t(1) << 31);
}

int maxsim_csr_build(const int32_t *argmax, int n_q, int64_t b, int l_q, int l_d, int32_t *row_ptr, int32_t *col_idx,
                     void *stream)
{
    if (!argmax || !row_ptr || !col_idx || n_q < 1 || l_q < 1 || b < 1 || l_d < 1)
        return MAXSIM_ERR_INVALID;
    if (!aligned(argmax, 4) || !aligned(row_ptr, 4) || !aligned(col_idx, 4))
        return MAXSIM_ERR_INVALID;
    if (!csr_shape_ok(n_q, b, l_q, l_d))
        return MAXSIM_ERR_UNSUPPORTED;
    if (int rc = ensure_init())
        return rc;
    return finish(maxsim::csr_build_launch(argmax, n_q, b, l_q, l_d, row_ptr, col_idx, num_cu(),
                                           static_cast<hipStream_t>(stream)));
}

int maxsim_backward_csr(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d, maxsim_dtype dtype,
                        const int32_t *argmax, const float *dscore, int32_t *row_ptr, int32_t *col_idx, float *dQ,
                        float *dD, void *stream)
{
    if (!Q || !D || !argmax || !dscore || !row_ptr || !col_idx || !dQ || !dD || n_q < 1 || l_q < 1 || b < 1 || l_d < 1 ||
        !dtype_ok((int)dtype))
        return MAXSIM_ERR_INVALID;
    if (!aligned(Q, 16) || !aligned(D, 16) || !aligned(argmax, 4) || !aligned(dscore, 4) || !aligned(row_ptr, 4) ||
        !aligned(col_idx, 4) || !aligned(dQ, 16) || !aligned(dD, 16))
        return MAXSIM_ERR_INVALID;
    if (!csr_shape_ok(n_q, b, l_q, l_d))
        return MAXSIM_ERR_UNSUPPORTED;
    if (!backward_width_ok(d) || !backward_q_ok(n_q, l_q, d, (int)dtype, b * (int64_t)l_d))
        return MAXSIM_ERR_UNSUPPORTED;
    if (int rc = ensure_init())
        return rc;
    return finish(maxsim::backward_csr_launch(Q, n_q, l_q, D, b, l_d, d, (int)dtype, argmax, dscore, row_ptr, col_idx, dQ,
                                              dD, num_cu(), static_cast<hipStream_t>(stream)));
}

int maxsim_backward_csr_static(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d,
                               maxsim_dtype dtype, const int32_t *argmax, const float *dscore, float *dQ, float *dD,
                               void *stream)
{
    if (!Q || !D || !argmax || !dscore || !dQ || !dD || n_q < 1 || l_q < 1 || b < 1 || l_d < 1 || !dtype_ok((int)dtype))
        return MAXSIM_ERR_INVALID;
    if (!aligned(Q, 16) || !aligned(D, 16) || !aligned(argmax, 4) || !aligned(dscore, 4) || !aligned(dQ, 16) ||
        !aligned(dD, 16))
        return MAXSIM_ERR_INVALID;
    if (!csr_shape_ok(n_q, b, l_q, l_d))
        return MAXSIM_ERR_UNSUPPORTED;
    if (!backward_width_ok(d) || !backward_q_ok(n_q, l_q, d, (int)dtype, b * (int64_t)l_d))
        return MAXSIM_ERR_UNSUPPORTED;
    if (!maxsim::csr_static_fits(n_q, b, l_q, l_d))
        return MAXSIM_ERR_SCRATCH;
    if (int rc = ensure_init())
        return rc;
    return finish(maxsim::backward_csr_static_launch(Q, n_q, l_q, D, b, l_d, d, (int)dtype, argmax, dscore, dQ, dD, num_cu(),
                                                     static_cast<hipStream_t>(stream)));
}

int maxsim_quantize_rows_i8(const void *X, int64_t rows, int d, maxsim_dtype dtype, int8_t *X_i8, float *scale,
                            void *stream)
{
    if (!X || !X_i8 || !scale || rows < 1 || !dtype_ok((int)dtype))
        return MAXSIM_ERR_INVALID;
    if (!aligned(X, 16) || !aligned(X_i8, 16) || !aligned(scale, 4))
        return MAXSIM_ERR_INVALID;
    if (!i8_width_ok(d))
        return MAXSIM_ERR_UNSUPPORTED;
    if (rows >= (int64_t(1) << 40))
        return MAXSIM_ERR_UNSUPPORTED;
    if (int rc = ensure_init())
        return rc;
    if (d != maxsim::D_MODEL)
        return finish(maxsim::quantize_wide_launch(X, rows, d, (int)dtype, X_i8, scale, static_cast<hipStream_t>(stream)));
    return finish(maxsim::quantize_launch(X, rows, (int)dtype, X_i8, scale, static_cast<hipStream_t>(stream)));
}

int maxsim_forward_i8(const int8_t *Q_i8, const float *q_scale, int n_q, int l_q, const int8_t *D_i8,
                      const float *d_scale, int64_t b, int l_d, int d, float *scores, void *stream)
{
    if (!Q_i8 || !q_scale || !D_i8 || !d_scale || !scores || n_q < 1 || l_q < 1 || b < 1 || l_d < 1)
        return MAXSIM_ERR_INVALID;
    if (!aligned(Q_i8, 16) || !aligned(D_i8, 16) || !aligned(q_scale, 4) || !aligned(d_scale, 4) || !aligned(scores, 4))
        return MAXSIM_ERR_INVALID;
    if (!i8_width_ok(d))
        return MAXSIM_ERR_UNSUPPORTED;
    if (b >= (int64_t(1) << 31) || (int64_t)n_q * ((l_q + 31) / 32) >= (int64_t(1) << 24) ||
        l_q > 1024 || b * (int64_t)l_d >= (int64_t(1) << 31))
        return MAXSIM_ERR_UNSUPPORTED;
    if (int rc = ensure_init())
        return rc;
    return finish(i8_launch_any(Q_i8, q_scale, n_q, l_q, D_i8, d_scale, nullptr, b, l_d, b * (int64_t)l_d, d, scores, b,
                                num_cu(), static_cast<hipStream_t>(stream)));
}

int maxsim_forward_i8_ragged(const int8_t *Q_i8, const float *q_scale, int n_q, int l_q, const int8_t *D_i8_packed,
                             const float *d_scale_packed, const int32_t *doc_offsets, int64_t b, int64_t total_tokens,
                             int d, float *scores, void *stream)
{
    if (!Q_i8 || !q_scale || !D_i8_packed || !d_scale_packed || !doc_offsets || !scores || n_q < 1 || l_q < 1 || b < 1 ||
        total_tokens < 1)
        return MAXSIM_ERR_INVALID;
    if (!aligned(Q_i8, 16) || !aligned(D_i8_packed, 16) || !aligned(q_scale, 4) || !aligned(d_scale_packed, 4) ||
        !aligned(doc_offsets, 4) || !aligned(scores, 4))
        return MAXSIM_ERR_INVALID;
    if (!i8_width_ok(d))
        return MAXSIM_ERR_UNSUPPORTED;
    if (b >= (int64_t(1) << 31) || total_tokens >= (int64_t(1) << 31) ||
        (int64_t)n_q * ((l_q + 31) / 32) >= (int64_t(1) << 24) || l_q > 1024)
        return MAXSIM_ERR_UNSUPPORTED;
    if (int rc = ensure_init())
        return rc;
    return finish(i8_launch_any(Q_i8, q_scale, n_q, l_q, D_i8_packed, d_scale_packed, doc_offsets, b, 0, total_tokens, d,
                                scores, b, num_cu(), static_cast<hipStream_t>(stream)));
}

int maxsim_ce_grad(const float *scores, int n, int b, float tau, float *g, float *loss, void *stream)
{
    if (!scores || !g || n < 1 || b < n || !(tau > 0.0f))
        return MAXSIM_ERR_INVALID;
    if (int rc = ensure_init())
        return rc;
    return finish(maxsim::ce_grad_launch(scores, n, b, tau, g, loss, static_cast<hipStream_t>(stream)));
}

} // extern "C"
