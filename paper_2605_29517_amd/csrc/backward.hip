// MaxSim backward through the stored argmax (Eqs. 2-3 of the paper) for gfx950, plus the
// in-batch-negatives cross-entropy gradient helper.
//
// dQ (Eq. 2) is a collision-free gather: one wavefront per query token (q, i) walks the
// documents, four document rows per load instruction (16 lanes x 16 bytes cover a row).
//
// dD (Eq. 3) is the contended side.  The paper resolves it either with atomics or with an
// inverse-grid CSR built by bincount / cumsum / argsort.  Here every dD row has exactly one
// owner instead: a workgroup owns a block of consecutive tokens of one document and keeps
// their fp32 gradient rows in LDS; wavefront w of the workgroup owns the rows t with
// t % W == w.  Every wavefront scans the document's argmax column [n_q * l_q entries],
// picks out the edges that land on its rows and accumulates them in scan order.  No atomics,
// no sort, no zero-fill pass over dD, and the summation order is fixed, so the result is
// bitwise reproducible.
#include "common.h"

namespace maxsim {

template <int DT> struct Elem;
template <> struct Elem<MAXSIM_F32> {
    static constexpr int BYTES = 4;
    static __device__ __forceinline__ float get(const char *row, int k) { return reinterpret_cast<const float *>(row)[k]; }
};
template <> struct Elem<MAXSIM_F16> {
    static constexpr int BYTES = 2;
    static __device__ __forceinline__ float get(const char *row, int k)
    {
        return (float)reinterpret_cast<const _Float16 *>(row)[k];
    }
};
template <> struct Elem<MAXSIM_BF16> {
    static constexpr int BYTES = 2;
    static __device__ __forceinline__ float get(const char *row, int k)
    {
        uint32_t bits = (uint32_t)reinterpret_cast<const uint16_t *>(row)[k] << 16;
        return __uint_as_float(bits);
    }
};

// 8 consecutive elements of a row, decoded to fp32
template <int DT> __device__ __forceinline__ void load8(const char *p, float (&v)[8])
{
    if (DT == MAXSIM_F32) {
        float4 a = *reinterpret_cast<const float4 *>(p);
        float4 b = *reinterpret_cast<const float4 *>(p + 16);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
        uint4 raw = *reinterpret_cast<const uint4 *>(p);
        uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (DT == MAXSIM_F16) {
                v[2 * i] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] & 0xffffu));
                v[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] >> 16));
            } else {
                v[2 * i] = __uint_as_float(w[i] << 16);
                v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
            }
        }
    }
}

struct BwdParams {
    const char *Q;
    const char *D;
    const int32_t *A;
    const float *g;
    float *dQ;
    float *dD;
    int64_t b;
    int n_q, l_q, l_d;
};

// ---------------------------------------------------------------------------------------
// dQ[q,i,:] = sum_j g[q,j] * D[j, A[q,j,i], :]
// ---------------------------------------------------------------------------------------
template <int DT>
__global__ void __launch_bounds__(256) bwd_dq_kernel(BwdParams p)
{
    constexpr int ROWB = D_MODEL * Elem<DT>::BYTES;
    const int lane = threadIdx.x & 63;
    const int grp = lane >> 4; // which of 4 documents per step
    const int c = lane & 15;   // which 8 columns of the row
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    if (wave >= (int64_t)p.n_q * p.l_q)
        return;
    const int q = (int)(wave / p.l_q);
    const int i = (int)(wave % p.l_q);
    const int32_t *Aq = p.A + (int64_t)q * p.b * p.l_q + i;
    const float *gq = p.g + (int64_t)q * p.b;

    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    constexpr int UNROLL = 4;
    for (int64_t j0 = 0; j0 < p.b; j0 += 4 * UNROLL) {
        int t[UNROLL];
        float gg[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            int64_t j = j0 + u * 4 + grp;
            bool ok = j < p.b;
            int tt = ok ? Aq[j * p.l_q] : -1;
            ok = ok && tt >= 0 && tt < p.l_d;
            t[u] = ok ? tt : 0;
            gg[u] = ok ? gq[j] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            int64_t j = j0 + u * 4 + grp;
            if (j >= p.b)
                j = p.b - 1; // contributes with weight 0
            float v[8];
            load8<DT>(p.D + (j * p.l_d + t[u]) * ROWB + c * 8 * Elem<DT>::BYTES, v);
#pragma unroll
            for (int k = 0; k < 8; ++k)
                acc[k] = fmaf(gg[u], v[k], acc[k]);
        }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        acc[k] += __shfl_xor(acc[k], 16);
        acc[k] += __shfl_xor(acc[k], 32);
    }
    if (grp == 0) {
        float4 *dst = reinterpret_cast<float4 *>(p.dQ + wave * D_MODEL + c * 8);
        dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
}

// ---------------------------------------------------------------------------------------
// dD[j,t,:] = sum over edges (q,i) with A[q,j,i] = t of g[q,j] * Q[q,i,:]
// ---------------------------------------------------------------------------------------
constexpr int DD_TOKENS = 128; // token rows per workgroup: 128 x 128 fp32 = 64 KB of LDS
constexpr int DD_WAVES = 8;

template <int DT>
__global__ void __launch_bounds__(DD_WAVES * 64) bwd_dd_kernel(BwdParams p, int blocks_per_doc)
{
    constexpr int ROWB = D_MODEL * Elem<DT>::BYTES;
    __shared__ __attribute__((aligned(16))) float tile[DD_TOKENS * D_MODEL];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t j = blockIdx.x / blocks_per_doc;
    const int t_base = (int)(blockIdx.x % blocks_per_doc) * DD_TOKENS;

    for (int x = tid; x < DD_TOKENS * D_MODEL / 4; x += DD_WAVES * 64)
        reinterpret_cast<float4 *>(tile)[x] = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();

    // every wavefront walks all n_q * l_q entries of column j, 64 per step, in entry order
    const int64_t n_entries = (int64_t)p.n_q * p.l_q;
    const int dq = 64 / p.l_q, di = 64 % p.l_q; // advance of (q, i) per step
    int q = lane / p.l_q, i = lane % p.l_q;
    for (int64_t n0 = 0; n0 < n_entries; n0 += 64) {
        int64_t n = n0 + lane;
        int t = -1;
        if (n < n_entries)
            t = p.A[((int64_t)q * p.b + j) * p.l_q + i];
        int rel = t - t_base;
        bool mine = rel >= 0 && rel < DD_TOKENS && t < p.l_d && (rel & (DD_WAVES - 1)) == w;
        unsigned long long mask = __ballot(mine);
        while (mask) {
            int e = __builtin_ctzll(mask);
            mask &= mask - 1;
            int eq = __builtin_amdgcn_readlane(q, e);
            int ei = __builtin_amdgcn_readlane(i, e);
            int er = __builtin_amdgcn_readlane(rel, e);
            float gg = p.g[(int64_t)eq * p.b + j];
            const char *qrow = p.Q + ((int64_t)eq * p.l_q + ei) * ROWB;
            float x0 = Elem<DT>::get(qrow, 2 * lane);
            float x1 = Elem<DT>::get(qrow, 2 * lane + 1);
            float2 *cell = reinterpret_cast<float2 *>(tile + er * D_MODEL) + lane;
            float2 cur = *cell;
            cur.x = fmaf(gg, x0, cur.x);
            cur.y = fmaf(gg, x1, cur.y);
            *cell = cur;
        }
        q += dq;
        i += di;
        if (i >= p.l_q) {
            i -= p.l_q;
            q += 1;
        }
    }
    __syncthreads();

    int rows = p.l_d - t_base;
    if (rows > DD_TOKENS)
        rows = DD_TOKENS;
    float4 *dst = reinterpret_cast<float4 *>(p.dD + (j * p.l_d + t_base) * D_MODEL);
    for (int x = tid; x < rows * (D_MODEL / 4); x += DD_WAVES * 64)
        dst[x] = reinterpret_cast<const float4 *>(tile)[x];
}

template <int DT> static hipError_t launch_bwd(const BwdParams &p, hipStream_t stream)
{
    int64_t waves = (int64_t)p.n_q * p.l_q;
    int grid_q = (int)((waves + 3) / 4);
    hipLaunchKernelGGL((bwd_dq_kernel<DT>), dim3(grid_q), dim3(256), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    int blocks_per_doc = (p.l_d + DD_TOKENS - 1) / DD_TOKENS;
    int64_t grid_d = p.b * blocks_per_doc;
    hipLaunchKernelGGL((bwd_dd_kernel<DT>), dim3((unsigned)grid_d), dim3(DD_WAVES * 64), 0, stream, p, blocks_per_doc);
    return hipGetLastError();
}

hipError_t backward_launch(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int dtype,
                           const int32_t *argmax, const float *dscore, float *dQ, float *dD, int /*num_cu*/,
                           hipStream_t stream)
{
    BwdParams p;
    p.Q = static_cast<const char *>(Q);
    p.D = static_cast<const char *>(D);
    p.A = argmax;
    p.g = dscore;
    p.dQ = dQ;
    p.dD = dD;
    p.b = b;
    p.n_q = n_q;
    p.l_q = l_q;
    p.l_d = l_d;
    switch (dtype) {
    case MAXSIM_F32: return launch_bwd<MAXSIM_F32>(p, stream);
    case MAXSIM_F16: return launch_bwd<MAXSIM_F16>(p, stream);
    default: return launch_bwd<MAXSIM_BF16>(p, stream);
    }
}

// ---------------------------------------------------------------------------------------
// cross-entropy gradient on the [n, b] score matrix (labels on the diagonal)
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_xor(v, o);
    return v;
}

// One wavefront per row, rows dealt round-robin to the wavefronts of the grid.  The loss is
// summed by the last block alone, again one wavefront per row, in a fixed order.
__global__ void __launch_bounds__(256) ce_grad_kernel(const float *s, int n, int b, float inv_tau, float *g,
                                                      float *loss, int row_blocks)
{
    __shared__ float part[4];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const bool loss_block = (int)blockIdx.x == row_blocks;
    if (loss_block && !loss)
        return;
    float local = 0.0f;
    int first = loss_block ? w : (int)blockIdx.x * 4 + w;
    int step = loss_block ? 4 : row_blocks * 4;
    for (int i = first; i < n; i += step) {
        const float *row = s + (int64_t)i * b;
        float mx = neg_inf();
        for (int j = lane; j < b; j += 64)
            mx = fmaxf(mx, row[j] * inv_tau);
        mx = wave_max(mx);
        float z = 0.0f;
        for (int j = lane; j < b; j += 64)
            z += expf(row[j] * inv_tau - mx);
        z = wave_sum(z);
        if (loss_block) {
            local += logf(z) + mx - row[i] * inv_tau;
        } else {
            float scale = inv_tau / (float)n;
            for (int j = lane; j < b; j += 64) {
                float pj = expf(row[j] * inv_tau - mx) / z;
                g[(int64_t)i * b + j] = (pj - (j == i ? 1.0f : 0.0f)) * scale;
            }
        }
    }
    if (loss_block) {
        if (lane == 0)
            part[w] = local;
        __syncthreads();
        if (threadIdx.x == 0)
            *loss = (part[0] + part[1] + part[2] + part[3]) / (float)n;
    }
}

hipError_t ce_grad_launch(const float *scores, int n, int b, float tau, float *g, float *loss, hipStream_t stream)
{
    int row_blocks = (n + 3) / 4;
    hipLaunchKernelGGL(ce_grad_kernel, dim3(row_blocks + 1), dim3(256), 0, stream, scores, n, b, 1.0f / tau, g, loss,
                       row_blocks);
    return hipGetLastError();
}

} // namespace maxsim
