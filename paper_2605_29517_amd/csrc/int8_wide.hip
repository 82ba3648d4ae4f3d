// int8 scoring (Alg. 4 of the paper) and the per-token quantiser (Sec. "Quantised Scoring") for embedding widths
// other than 128: every d that is a multiple of 32 up to 8192.  The tuned kernels of int8.hip are built around
// 128-byte rows (the whole query group lives in LDS or in registers); here neither operand is resident, the
// contraction walks d in steps of 32 bytes -- the inner loop over d of App. "split-d" with an exact int32
// accumulator -- and the arithmetic after it is the same: v = fl32(n * d_scale[j]) per cell, the maximum over the
// document's tokens, r_i = fl32(q_scale[i] * max), the sum over the query's tokens carried in fp64 and rounded
// once.  The same bits as the oracle's definition.  Widths that are a multiple of 64 are scored by the slab kernel
// of forward_splitd.hip (both operands through LDS, the same arithmetic after the contraction); the kernel below
// serves the other multiples of 32 and is not tuned: every wavefront re-reads its query blocks' bytes from the
// caches for every step of 32 or 64 document tokens, which holds long queries at about 9 % of the int8 MFMA peak.
#include "common.h"

namespace maxsim {

struct I8WideParams {
    const char *Q;   // [n_q, l_q, d] int8
    const float *qs; // [n_q, l_q]
    const char *D;   // [b, l_d, d] or packed [T, d] int8
    const float *ds; // [b, l_d] or [T]
    FwdParams f;     // sizes, optional offsets, the work split (qpg whole queries per workgroup) and `scores`
    int d;
};

constexpr int I8W_NB = 4;   // column blocks (32 query tokens each) per wavefront

// n * s rounded once to fp32: the product of an int32 below 2^29 in magnitude and an fp32 is exact in fp64
// (|n| <= 127^2 * 8192 < 2^27 here, so 27 + 24 bits)
__device__ __forceinline__ float scaled_once(int n, float s) { return (float)((double)n * (double)s); }

// W wavefronts x 4 column blocks per workgroup (W = 8: 1024 query tokens, the longest query; fewer wavefronts for
// fewer query tokens, so that no wavefront is idle and more workgroups share the corpus).  All wavefronts of a
// workgroup walk the same documents, T tiles of 32 tokens per step; a wavefront loads 32 bytes of the step's document
// rows and of its 128 query tokens per 4 T MFMAs.
template <int W, int T> __global__ void __launch_bounds__(W * 64) fwd_i8_wide_kernel(I8WideParams P, OffsetsPtr off)
{
    constexpr int I8W_ROWS = 32 * T;
    const FwdParams &p = P.f;
    constexpr int BLOCKS = W * I8W_NB;
    __shared__ double lds_part[2][BLOCKS]; // per column block: the sum over its query tokens, for two documents in turn
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int rho = lane & 31, h = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int group = (int)(blockIdx.x % (unsigned)p.n_groups);
    const int64_t chunk = blockIdx.x / (unsigned)p.n_groups;
    int64_t doc0_, doc1_;
    chunk_doc_range(p, chunk, doc0_, doc1_);
    if (doc0_ >= doc1_)
        return;
    const int doc0 = (int)doc0_, doc1 = (int)doc1_;

    // the group's queries [q_first, q_first + nq) and their nb = nq * bpq column blocks (at most BLOCKS)
    const int q_first = group * p.qpg;
    const int nq = min(p.qpg, p.n_q - q_first);
    const int nb = nq * p.bpq;
    const int64_t d = P.d;
    const int n_k = P.d / 32; // steps of the contraction: 32 bytes of every row each

    if (p.offsets) { // empty documents: score -inf for every query of the group
        for (int64_t x = tid; x < (int64_t)(doc1 - doc0) * nq; x += W * 64) {
            const int64_t doc = doc0 + x / nq;
            if (p.offsets[doc + 1] == p.offsets[doc])
                p.scores[(int64_t)(q_first + (int)(x % nq)) * p.ld + doc] = neg_inf();
        }
    }

    // this wavefront's column blocks: block lb = w * NB + cb of the group -> query, first token, this lane's token
    const char *q_ptr[I8W_NB]; // this lane's 16 bytes of the first step of its query token's row
    float q_scale[I8W_NB];
    bool col_ok[I8W_NB];
#pragma unroll
    for (int cb = 0; cb < I8W_NB; ++cb) {
        const int lb = w * I8W_NB + cb;
        const int lbc = lb < nb ? lb : nb - 1; // a block past the group's last repeats it (never read back)
        const int qq = lbc / p.bpq;
        const int tok = (lbc - qq * p.bpq) * BLOCK_COLS + rho;
        col_ok[cb] = lb < nb && tok < p.l_q;
        const int64_t qrow = (int64_t)(q_first + qq) * p.l_q + (tok < p.l_q ? tok : p.l_q - 1);
        q_ptr[cb] = P.Q + qrow * d + h * 16;
        q_scale[cb] = P.qs[qrow];
    }

    TileIter it;
    it_init(it, p, off, doc0, doc1);
    float m[I8W_NB];
#pragma unroll
    for (int cb = 0; cb < I8W_NB; ++cb)
        m[cb] = neg_inf();
    int par = 0;
    while (it_valid(it)) {
        // rows past the document's end repeat its last token: a duplicate changes no maximum
        const int last = it.len - it.t0 - 1;
        const char *a_ptr[T];
        float sc[T][16]; // the scales of the rows this lane's accumulator registers hold
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int row = 32 * t + rho;
            a_ptr[t] = P.D + ((int64_t)it.row0 + (row < last ? row : last)) * d + h * 16;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rr = 32 * t + acc_row(r, h);
                sc[t][r] = P.ds[(int64_t)it.row0 + (rr < last ? rr : last)];
            }
        }
        i32x16 acc[T][I8W_NB];
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int cb = 0; cb < I8W_NB; ++cb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc[t][cb][r] = 0;
        // the loads of a step are issued before the MFMAs of the step before (two register sets)
        i32x4 a[2][T], b[2][I8W_NB];
        auto load_step = [&](int k, int set) {
            const int64_t at = (int64_t)(k < n_k ? k : n_k - 1) * 32; // past the last step: the last once more, unused
#pragma unroll
            for (int t = 0; t < T; ++t)
                a[set][t] = *reinterpret_cast<const i32x4 *>(a_ptr[t] + at);
#pragma unroll
            for (int cb = 0; cb < I8W_NB; ++cb)
                b[set][cb] = *reinterpret_cast<const i32x4 *>(q_ptr[cb] + at);
        };
        auto mma_step = [&](int set) {
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int cb = 0; cb < I8W_NB; ++cb)
                    acc[t][cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[set][t], b[set][cb], acc[t][cb], 0, 0, 0);
        };
        load_step(0, 0);
        for (int k = 0; k < n_k; k += 2) {
            load_step(k + 1, 1);
            mma_step(0);
            if (k + 1 >= n_k)
                break;
            load_step(k + 2, 0);
            mma_step(1);
        }
        // deferred dequantisation: one rounding per cell, then the running maximum per query token
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int cb = 0; cb < I8W_NB; ++cb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    m[cb] = fmaxf(m[cb], scaled_once(acc[t][cb][r], sc[t][r]));

        const bool fin = it.t0 + I8W_ROWS >= it.len; // last step of its document?
        const int fin_doc = it.doc;
        it_next(it, p, off, I8W_ROWS);
        if (fin) {
#pragma unroll
            for (int cb = 0; cb < I8W_NB; ++cb) {
                // the two halves of the wavefront hold different rows of the same query token
                const float mm = fmaxf(m[cb], __shfl_xor(m[cb], 32));
                double s = col_ok[cb] ? (double)(q_scale[cb] * mm) : 0.0; // one IEEE fp32 multiply per query token
#pragma unroll
                for (int o = 16; o > 0; o >>= 1)
                    s += __shfl_xor(s, o);
                if (lane == 0)
                    lds_part[par][w * I8W_NB + cb] = s;
                m[cb] = neg_inf();
            }
            __syncthreads(); // one barrier per document: the two halves of lds_part take turns
            if (tid < nq) {   // thread t adds up the blocks of its query in block order
                double s = 0.0;
                for (int i = 0; i < p.bpq; ++i)
                    s += lds_part[par][tid * p.bpq + i];
                p.scores[(int64_t)(q_first + tid) * p.ld + fin_doc] = (float)s;
            }
            par ^= 1;
        }
    }
}

// Per-token absmax quantiser for rows of any width that is a multiple of 8: one wavefront per row, eight
// elements per lane and step; the row is read twice (maximum, then codes; the second read comes from the caches).
// Same arithmetic as the 128-wide kernel: scale = absmax / 127 by IEEE division, code = round_half_even(x / scale)
// by IEEE division, clamped to [-127, 127]; an all-zero row gets scale 0 and codes 0.
template <int DT>
__global__ void __launch_bounds__(256) quantize_rows_wide_kernel(const char *X, int64_t rows, int d, int8_t *out, float *scale)
{
    constexpr int EB = DT == MAXSIM_F32 ? 4 : 2;
    const int lane = threadIdx.x & 63;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    auto load8 = [&](const char *p, float(&v)[8]) {
        if constexpr (DT == MAXSIM_F32) {
            const float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 16);
            v[0] = a.x, v[1] = a.y, v[2] = a.z, v[3] = a.w, v[4] = b.x, v[5] = b.y, v[6] = b.z, v[7] = b.w;
        } else {
            const uint4 raw = *reinterpret_cast<const uint4 *>(p);
            const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (DT == MAXSIM_F16) {
                    v[2 * i] = (float)__builtin_bit_cast(_Float16, (uint16_t)(u[i] & 0xffffu));
                    v[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(u[i] >> 16));
                } else {
                    v[2 * i] = __uint_as_float(u[i] << 16);
                    v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
                }
            }
        }
    };
    for (int64_t row = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; row < rows; row += n_waves) {
        const char *src = X + row * (int64_t)d * EB;
        float a = 0.0f;
        for (int e = lane * 8; e < d; e += 512) {
            float x[8];
            load8(src + (int64_t)e * EB, x);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                a = fmaxf(a, fabsf(x[i]));
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1)
            a = fmaxf(a, __shfl_xor(a, o));
        const float s = a / 127.0f;
        for (int e = lane * 8; e < d; e += 512) {
            float x[8];
            load8(src + (int64_t)e * EB, x);
            uint32_t lo = 0, hi = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int code = 0;
                if (s != 0.0f) {
                    float r = rintf(x[i] / s);
                    r = fminf(fmaxf(r, -127.0f), 127.0f);
                    code = (int)r;
                }
                if (i < 4)
                    lo |= (uint32_t)(code & 0xff) << (8 * i);
                else
                    hi |= (uint32_t)(code & 0xff) << (8 * (i - 4));
            }
            *reinterpret_cast<uint2 *>(out + row * (int64_t)d + e) = make_uint2(lo, hi);
        }
        if (lane == 0)
            scale[row] = s;
    }
}

bool i8_wide_width_ok(int d) { return d >= 32 && d <= 8192 && d % 32 == 0; }

bool forward_splitd_i8_ok(int l_q, int d);
hipError_t forward_splitd_i8_launch(FwdParams p, const float *q_scale, const float *d_scale, int d, int num_cu, hipStream_t stream);

hipError_t forward_i8_wide_launch(const int8_t *Q, const float *qs, int n_q, int l_q, const int8_t *D, const float *ds,
                                  const int32_t *offsets, int64_t b, int l_d, int64_t total_tokens, int d, float *scores,
                                  int64_t ld, int num_cu, hipStream_t stream)
{
    // widths that are a multiple of 64: the slab kernel through LDS (3 x this one on long queries; up to four column
    // blocks of rows of up to 256 bytes are faster here: 0.14 against 0.20 ms for 32 tokens on 1000 pages at d = 256)
    const bool few_narrow = d <= 256 && (int64_t)n_q * ((l_q + BLOCK_COLS - 1) / BLOCK_COLS) <= I8W_NB;
    if (forward_splitd_i8_ok(l_q, d) && !few_narrow) {
        FwdParams f{};
        f.Q = reinterpret_cast<const char *>(Q);
        f.D = reinterpret_cast<const char *>(D);
        f.offsets = offsets;
        f.scores = scores;
        f.b = b;
        f.ld = ld;
        f.total_tokens = total_tokens;
        f.n_q = n_q;
        f.l_q = l_q;
        f.l_d = l_d;
        return forward_splitd_i8_launch(f, qs, ds, d, num_cu, stream);
    }
    I8WideParams P;
    P.Q = reinterpret_cast<const char *>(Q);
    P.qs = qs;
    P.D = reinterpret_cast<const char *>(D);
    P.ds = ds;
    P.d = d;
    FwdParams &p = P.f;
    p = FwdParams{};
    p.offsets = offsets;
    p.scores = scores;
    p.b = b;
    p.ld = ld;
    p.total_tokens = total_tokens;
    p.n_q = n_q;
    p.l_q = l_q;
    p.l_d = l_d;
    p.bpq = (l_q + BLOCK_COLS - 1) / BLOCK_COLS; // <= 32 (l_q <= 1024, checked by the caller)
    // wavefronts per workgroup: as many as the queries' column blocks need, at most 8 (which hold the longest query)
    const int64_t total_blocks = (int64_t)n_q * p.bpq;
    const int want = (int)(total_blocks < 8 * I8W_NB ? total_blocks : 8 * I8W_NB);
    int w = 1;
    while (w * I8W_NB < want)
        w *= 2;
    p.qpg = w * I8W_NB / p.bpq; // whole queries per workgroup (>= 1)
    if (p.qpg > n_q)
        p.qpg = n_q;
    p.n_groups = (n_q + p.qpg - 1) / p.qpg;
    p.n_pass = 1;
    // document chunks: about sixteen wavefronts per CU in all, never more chunks than documents
    const int64_t units = offsets ? total_tokens : b;
    int64_t n_chunks = ((int64_t)num_cu * 16 / w + p.n_groups - 1) / p.n_groups;
    if (n_chunks > b)
        n_chunks = b;
    if (n_chunks < 1)
        n_chunks = 1;
    p.unit_per_chunk = (units + n_chunks - 1) / n_chunks;
    if (p.unit_per_chunk < 1)
        p.unit_per_chunk = 1;
    if (!offsets)
        n_chunks = (units + p.unit_per_chunk - 1) / p.unit_per_chunk;
    p.n_chunks = (int)n_chunks;
    const int64_t grid = n_chunks * p.n_groups;
    if (grid >= (int64_t(1) << 31))
        return hipErrorInvalidValue;
    // two document tiles per step where the registers allow it (up to four wavefronts: 0.14 against 0.20 ms for one
    // block of 32 query tokens on 1000 pages at d = 256); with eight wavefronts the 128 accumulator registers of two
    // tiles no longer fit beside the operands
    switch (w) {
    case 1: hipLaunchKernelGGL((fwd_i8_wide_kernel<1, 2>), dim3((unsigned)grid), dim3(64), 0, stream, P, offsets); break;
    case 2: hipLaunchKernelGGL((fwd_i8_wide_kernel<2, 2>), dim3((unsigned)grid), dim3(128), 0, stream, P, offsets); break;
    case 4: hipLaunchKernelGGL((fwd_i8_wide_kernel<4, 2>), dim3((unsigned)grid), dim3(256), 0, stream, P, offsets); break;
    default: hipLaunchKernelGGL((fwd_i8_wide_kernel<8, 1>), dim3((unsigned)grid), dim3(512), 0, stream, P, offsets); break;
    }
    return hipGetLastError();
}

hipError_t quantize_wide_launch(const void *X, int64_t rows, int d, int dtype, int8_t *X_i8, float *scale, hipStream_t stream)
{
    int64_t blocks = (rows + 3) / 4; // 4 wavefronts per workgroup, a row per wavefront and step
    if (blocks > 65536 * 4)
        blocks = 65536 * 4;
    const char *x = static_cast<const char *>(X);
    switch (dtype) {
    case MAXSIM_F32:
        hipLaunchKernelGGL((quantize_rows_wide_kernel<MAXSIM_F32>), dim3((unsigned)blocks), dim3(256), 0, stream, x, rows, d, X_i8, scale);
        break;
    case MAXSIM_F16:
        hipLaunchKernelGGL((quantize_rows_wide_kernel<MAXSIM_F16>), dim3((unsigned)blocks), dim3(256), 0, stream, x, rows, d, X_i8, scale);
        break;
    default:
        hipLaunchKernelGGL((quantize_rows_wide_kernel<MAXSIM_BF16>), dim3((unsigned)blocks), dim3(256), 0, stream, x, rows, d, X_i8, scale);
        break;
    }
    return hipGetLastError();
}

} // namespace maxsim
