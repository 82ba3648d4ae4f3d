// MaxSim backward through the stored argmax (Eqs. 2-3 of the paper) for gfx950, plus the
// in-batch-negatives cross-entropy gradient helper.
//
// dQ (Eq. 2) is a collision-free gather: one wavefront per query token (q, i) walks the
// documents, four document rows per load instruction (16 lanes x 16 bytes cover a row).
//
// dD (Eq. 3) is the contended side.  The paper resolves it either with atomics or with an
// inverse-grid CSR built by bincount / cumsum / argsort.  Here every dD row has exactly one
// owner instead: a workgroup owns a block of consecutive rows of the (packed) corpus; wavefront w
// of the workgroup owns the rows with row % W == w and keeps their fp32 gradient in registers.
// Every wavefront scans the argmax column [n_q * l_q entries] of each document with rows in the
// block, picks out the edges that land on its rows and accumulates them in scan order.  No atomics, no sort, no zero-fill
// pass over dD, and the summation order is fixed, so the result is bitwise reproducible.  With many edges per row
// (short documents, many queries) a second kernel takes over that sorts the block's edges by row inside the
// workgroup (a stable counting sort in LDS) and lets sixteen lanes walk each row's list: same order, same bits.
// The explicit CSR of the paper (built in global memory, then walked by row owners) is there as an opt-in.
#include <mutex>

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
    const char *D;          // [b, l_d, d] or packed [total_tokens, d]
    const int32_t *offsets; // [b + 1] for a packed corpus, nullptr for a uniform one
    const int32_t *A;
    const float *g;
    float *dQ;
    float *dD;              // laid out like D
    int64_t b;
    int64_t total_tokens;   // b * l_d for a uniform corpus
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
        int64_t row[UNROLL]; // packed row of the winning token (row 0 with weight 0 if there is none)
        float gg[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            int64_t j = j0 + u * 4 + grp;
            bool ok = j < p.b;
            int tt = ok ? Aq[j * p.l_q] : -1;
            int64_t first = 0;
            int len = p.l_d;
            if (ok) {
                if (p.offsets) {
                    first = p.offsets[j];
                    len = p.offsets[j + 1] - (int)first;
                } else {
                    first = j * p.l_d;
                }
            }
            ok = ok && tt >= 0 && tt < len && first >= 0 && first + tt < p.total_tokens; // also guards bad offsets
            row[u] = ok ? first + tt : 0;
            gg[u] = ok ? gq[j] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float v[8];
            load8<DT>(p.D + row[u] * ROWB + c * 8 * Elem<DT>::BYTES, v);
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
constexpr int DD_WAVES = 8;
// gradient rows a wavefront keeps in registers: RPW = 16 (a workgroup owns 128 consecutive rows), or 8 / 4 when the
// corpus is too small to fill the chip with blocks of 128 rows
constexpr int DD_COL = 8192;    // argmax entries of a document's column handled per round
constexpr int DD_SEG = DD_COL / DD_WAVES; // entries each wavefront filters per round
constexpr int DD_QUEUE = 128;   // edges a wavefront collects before it applies them
constexpr int DD_BATCH = 16;    // Q rows in flight while edges are applied

// two consecutive elements (2 * lane, 2 * lane + 1) of a row, decoded to fp32
template <int DT> __device__ __forceinline__ void load_pair(const char *row, int lane, float &x0, float &x1)
{
    if (DT == MAXSIM_F32) {
        float2 v = reinterpret_cast<const float2 *>(row)[lane];
        x0 = v.x;
        x1 = v.y;
    } else {
        uint32_t wv = reinterpret_cast<const uint32_t *>(row)[lane];
        if (DT == MAXSIM_F16) {
            x0 = (float)__builtin_bit_cast(_Float16, (uint16_t)(wv & 0xffffu));
            x1 = (float)__builtin_bit_cast(_Float16, (uint16_t)(wv >> 16));
        } else {
            x0 = __uint_as_float(wv << 16);
            x1 = __uint_as_float(wv & 0xffff0000u);
        }
    }
}

// A workgroup owns 128 consecutive rows of the (packed) corpus, whichever documents they belong
// to.  Wavefront w owns the rows row0 + 8 * r + w (r = 0..15) and keeps them in registers: lane
// l holds columns 2l, 2l+1 of each.  For every document that has rows in the block, per round:
// (1) each wavefront reads an eighth of DD_COL entries of that document's argmax column and
// writes those that land in this block, compacted by ballot and in entry order, to its list in
// LDS; (2) every wavefront walks the eight lists in order and queues the edges that land on its
// rows; (3) when a queue holds 64 edges, the 64 lanes look up
// q, i, g and the Q row address of one edge each, and the edges are then applied in order, 16
// Q-row loads in flight, the target row picked by a wavefront-uniform register index
// (s_set_gpr_idx).  Every row has one owner and a fixed order of accumulation (entry order), so
// the result is bitwise reproducible; there are no atomics, no sort and no zero-fill pass.
template <int DT, int RPW>
__global__ void __launch_bounds__(DD_WAVES * 64) bwd_dd_kernel(BwdParams p)
{
    constexpr int DD_ROWS_PER_WAVE = RPW;
    constexpr int DD_TOKENS = DD_WAVES * RPW;
    constexpr int ROWB = D_MODEL * Elem<DT>::BYTES;
    __shared__ int seg[DD_WAVES][DD_SEG]; // per filtering wavefront: the round's edges into this block, in entry order
    __shared__ int seg_len[DD_WAVES];
    __shared__ int queue[DD_WAVES][DD_QUEUE];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t row0 = (int64_t)blockIdx.x * DD_TOKENS;
    const int64_t row_end = min(row0 + DD_TOKENS, p.total_tokens);

    // documents with rows in [row0, row_end): the last document that starts at or before a row owns it
    int64_t j_first, j_last;
    if (p.offsets) {
        j_first = lower_bound_offsets(p.offsets, p.b, row0 + 1) - 1;
        j_last = lower_bound_offsets(p.offsets, p.b, row_end) - 1;
        j_first = j_first < 0 ? 0 : j_first; // only offsets that break their contract get here
        j_last = j_last > p.b - 1 ? p.b - 1 : j_last;
    } else {
        j_first = row0 / p.l_d;
        j_last = (row_end - 1) / p.l_d;
    }

    typedef float rowvec __attribute__((ext_vector_type(DD_ROWS_PER_WAVE)));
    rowvec ax, ay; // ax[r], ay[r]: columns 2 * lane, 2 * lane + 1 of owned row r
#pragma unroll
    for (int r = 0; r < DD_ROWS_PER_WAVE; ++r) {
        ax[r] = 0.0f;
        ay[r] = 0.0f;
    }

    const int n_entries = p.n_q * p.l_q; // < 2^31 (checked by the caller)
    for (int64_t j = j_first; j <= j_last; ++j) {
        int64_t first;
        int len;
        if (p.offsets) {
            first = p.offsets[j];
            len = p.offsets[j + 1] - (int)first;
        } else {
            first = j * p.l_d;
            len = p.l_d;
        }
        if (len == 0)
            continue;
        const int t_base = (int)(row0 - first); // document-local index of the block's first row (may be negative)

        // apply the first `cnt` (<= 64) queued edges of this wavefront
        auto process = [&](int cnt, int c0) {
            int packed = lane < cnt ? queue[w][lane] : 0;
            int n = c0 + (packed & 0xffff);
            int rel = packed >> 16;
            int q = n / p.l_q;
            int i = n - q * p.l_q;
            float gv = lane < cnt ? p.g[(int64_t)q * p.b + j] : 0.0f;
            int64_t roff = ((int64_t)q * p.l_q + i) * ROWB;
            int rlo = (int)(roff & 0xffffffff), rhi = (int)(roff >> 32);
            for (int e0 = 0; e0 < cnt; e0 += DD_BATCH) {
                float x0[DD_BATCH], x1[DD_BATCH];
#pragma unroll
                for (int k = 0; k < DD_BATCH; ++k) {
                    int e = e0 + k < cnt ? e0 + k : cnt - 1; // past the end: a harmless re-read of the last row
                    int64_t off = ((int64_t)__builtin_amdgcn_readlane(rhi, e) << 32) |
                                  (uint32_t)__builtin_amdgcn_readlane(rlo, e);
                    load_pair<DT>(p.Q + off, lane, x0[k], x1[k]);
                }
#pragma unroll
                for (int k = 0; k < DD_BATCH; ++k) {
                    if (e0 + k < cnt) {
                        float gg = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(gv), e0 + k));
                        int r = __builtin_amdgcn_readlane(rel, e0 + k) >> 3; // rel = 8 * r + w
                        ax[r] = fmaf(gg, x0[k], ax[r]); // r is uniform: indexed register access, no branch
                        ay[r] = fmaf(gg, x1[k], ay[r]);
                    }
                }
            }
        };

        for (int64_t c64 = 0; c64 < n_entries; c64 += DD_COL) { // 64-bit: n_entries may be within DD_COL of 2^31
            const int c0 = (int)c64;
            const int cn = min(DD_COL, n_entries - c0);
            __syncthreads(); // the previous round's lists have been consumed
            {
                // (1) wavefront w filters entries [w * DD_SEG, (w + 1) * DD_SEG) of the round: entry
                // n = c0 + x -> (q, i); all loads are issued before the first result is used
                constexpr int PER = DD_SEG / 64;
                int x = w * DD_SEG + lane;
                int n = (int)((unsigned)c0 + (unsigned)x); // entries past the end of the column are masked below
                int q = n / p.l_q, i = n - q * p.l_q;
                const int dq = 64 / p.l_q, di = 64 % p.l_q;
                int t[PER];
#pragma unroll
                for (int k = 0; k < PER; ++k) {
                    t[k] = (x + k * 64) < cn ? p.A[((int64_t)q * p.b + j) * p.l_q + i] : -1;
                    q += dq;
                    i += di;
                    if (i >= p.l_q) {
                        i -= p.l_q;
                        q += 1;
                    }
                }
                int kept = 0;
#pragma unroll
                for (int k = 0; k < PER; ++k) {
                    int rel = t[k] - t_base;
                    bool in = t[k] >= 0 && t[k] < len && rel >= 0 && rel < DD_TOKENS;
                    unsigned long long mask = __ballot(in);
                    int before =
                        __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0));
                    if (in)
                        seg[w][kept + before] = (x + k * 64) | (rel << 16);
                    kept += __builtin_popcountll(mask);
                }
                if (lane == 0)
                    seg_len[w] = kept;
            }
            __syncthreads();
            // (2) every wavefront walks the eight lists in order and queues the edges on its rows
            int qlen = 0;
            for (int sw = 0; sw < DD_WAVES; ++sw) {
                const int sn = __builtin_amdgcn_readfirstlane(seg_len[sw]);
                for (int e0 = 0; e0 < sn; e0 += 64) {
                    int ent = e0 + lane < sn ? seg[sw][e0 + lane] : -1;
                    bool mine = ent >= 0 && ((ent >> 16) & (DD_WAVES - 1)) == w;
                    unsigned long long mask = __ballot(mine);
                    if (mask == 0)
                        continue;
                    int before =
                        __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0));
                    if (mine)
                        queue[w][qlen + before] = ent;
                    qlen += __builtin_popcountll(mask);
                    if (qlen >= 64) {
                        process(64, c0);
                        int rest = qlen - 64; // at most 63 edges move to the front
                        int moved = lane < rest ? queue[w][64 + lane] : 0;
                        if (lane < rest)
                            queue[w][lane] = moved;
                        qlen = rest;
                    }
                }
            }
            if (qlen > 0)
                process(qlen, c0);
        }
    }

#pragma unroll
    for (int r = 0; r < DD_ROWS_PER_WAVE; ++r) {
        int64_t row = row0 + r * DD_WAVES + w;
        if (row < row_end)
            reinterpret_cast<float2 *>(p.dD + row * D_MODEL)[lane] = make_float2(ax[r], ay[r]);
    }
}

// Which of the four row lists of a wavefront (lengths len[0..3], one per group of 16 lanes) the whole wavefront
// should walk: with the lists sorted by length, L1 >= L2 >= L3 >= L4, walking the k longest one after the other with
// 16 rows in flight and the rest side by side with 4 in flight each costs about (L1 + .. + Lk) / 16 + L(k+1) / 4 load
// round trips; the k that minimises this is returned (only lists of at least DS_LONG count), order[0..k) are their
// groups.  All values are wavefront-uniform.
constexpr int DS_LONG = 32;
__device__ __forceinline__ int pick_long_lists(const int (&len)[4], int (&order)[4])
{
    int sorted[5] = {0, 0, 0, 0, 0};
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
        int rank = 0;
#pragma unroll
        for (int gj = 0; gj < 4; ++gj)
            rank += (len[gj] > len[gi] || (len[gj] == len[gi] && gj < gi)) ? 1 : 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (rank == t) {
                order[t] = gi;
                sorted[t] = len[gi];
            }
        }
    }
    int best_k = 0, best = 4 * sorted[0], sum = 0;
#pragma unroll
    for (int k = 1; k <= 4; ++k) {
        sum += sorted[k - 1];
        const int cost = sum + 4 * sorted[k];
        if (sorted[k - 1] >= DS_LONG && cost < best) {
            best = cost;
            best_k = k;
        }
    }
    return best_k;
}

// inclusive wave scan
__device__ __forceinline__ int wave_scan_incl(int v, int lane)
{
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int u = __shfl_up(v, o);
        if (lane >= o)
            v += u;
    }
    return v;
}

// ---------------------------------------------------------------------------------------
// dD by sorting inside the workgroup.  A workgroup owns R = 32 * PASSES consecutive rows of the (packed) corpus
// and, for every document with rows in the block and every round of DS_COL argmax entries of that document's
// column: (A) each wavefront reads a contiguous eighth of the round, notes for every entry the row of the block it
// lands on (or none) in LDS and counts it into its own histogram over the block's rows; (B) one wavefront turns the
// histograms into list starts and per-wavefront write cursors; (C) each wavefront walks its eighth again, 64 entries at
// a time, ranks equal rows inside the 64 by ballots and writes the entry numbers to the row lists: a stable counting
// sort, so every list is in entry order; (D) sixteen lanes per row (8 columns each), four rows per wavefront, walk
// the lists with four Q rows in flight each; lists much longer than the others of their wavefront (hot tokens) are
// walked by the whole wavefront, one after the other.  The gradient of a row stays in registers until all its
// document's rounds are done and is written once.  Same edges in the same order with the same fused multiply-add as
// bwd_dd_kernel, hence the same bits; the difference is parallelism: every edge is touched by one wavefront
// (bwd_dd_kernel lets all eight walk all lists) and four rows advance per load instruction.
// ---------------------------------------------------------------------------------------
constexpr int DS_COL = 8192;               // entries per round: an entry's number within the round fits 16 bits
constexpr int DS_SEG = DS_COL / DD_WAVES;  // entries each wavefront sorts per round
constexpr int DS_NONE = 0xffff;
#ifndef DD_SORT_MIN_EDGES
#define DD_SORT_MIN_EDGES 20 // average edges per dD row from which the sorting kernel is used
#endif

template <int DT, int PASSES>
__global__ void __launch_bounds__(DD_WAVES * 64) bwd_dd_sort_kernel(BwdParams p, uint32_t lq_magic, int lq_shift)
{
    constexpr int R = 32 * PASSES;
    constexpr int RBITS = PASSES == 1 ? 5 : PASSES == 2 ? 6 : 7;
    constexpr int EB = Elem<DT>::BYTES;
    constexpr int ROWB = D_MODEL * EB;
    __shared__ uint16_t ent[DS_COL];   // per entry of the round: row of the block it lands on, or DS_NONE
    __shared__ uint16_t list[DS_COL];  // entry numbers (within the round) by row, in entry order
    __shared__ int hist[DD_WAVES][R];  // per wavefront: entries per row, then write cursors
    __shared__ int start[R + 1];       // list of row r: list[start[r] .. start[r + 1])
    __shared__ float xfer[DD_WAVES][D_MODEL]; // one gradient row per wavefront on its way between register layouts
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int grp = lane >> 4, c = lane & 15;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t row0 = (int64_t)blockIdx.x * R;
    const int64_t row_end = min(row0 + R, p.total_tokens);

    int64_t j_first, j_last;
    if (p.offsets) {
        j_first = lower_bound_offsets(p.offsets, p.b, row0 + 1) - 1;
        j_last = lower_bound_offsets(p.offsets, p.b, row_end) - 1;
        j_first = j_first < 0 ? 0 : j_first; // only offsets that break their contract get here
        j_last = j_last > p.b - 1 ? p.b - 1 : j_last;
    } else {
        j_first = row0 / p.l_d;
        j_last = (row_end - 1) / p.l_d;
    }

    float acc[PASSES][8];
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps)
#pragma unroll
        for (int x = 0; x < 8; ++x)
            acc[ps][x] = 0.0f;

    const int n_entries = p.n_q * p.l_q; // < 2^31 (checked by the caller)
    for (int64_t j = j_first; j <= j_last; ++j) {
        int64_t first;
        int len;
        if (p.offsets) {
            first = p.offsets[j];
            len = p.offsets[j + 1] - (int)first;
        } else {
            first = j * p.l_d;
            len = p.l_d;
        }
        if (len <= 0)
            continue;
        const int t_base = (int)(row0 - first); // document-local index of the block's first row (may be negative)

        for (int64_t c64 = 0; c64 < n_entries; c64 += DS_COL) { // 64-bit: n_entries may be within DS_COL of 2^31
            const int c0 = (int)c64;
            const int cn = min(DS_COL, n_entries - c0);
            __syncthreads(); // the previous round's lists have been walked
            for (int x = tid; x < DD_WAVES * R; x += DD_WAVES * 64)
                (&hist[0][0])[x] = 0;
            __syncthreads();
            {
                // (A) entry n = c0 + x -> (q, i); all loads are issued before the first result is used
                constexpr int PER = DS_SEG / 64;
                int x = w * DS_SEG + lane;
                int n = (int)((unsigned)c0 + (unsigned)x); // entries past the end of the column are masked below
                int q = n / p.l_q, i = n - q * p.l_q;
                const int dq = 64 / p.l_q, di = 64 % p.l_q;
                int t[PER];
#pragma unroll
                for (int k = 0; k < PER; ++k) {
                    t[k] = (x + k * 64) < cn ? p.A[((int64_t)q * p.b + j) * p.l_q + i] : -1;
                    q += dq;
                    i += di;
                    if (i >= p.l_q) {
                        i -= p.l_q;
                        q += 1;
                    }
                }
#pragma unroll
                for (int k = 0; k < PER; ++k) {
                    int rel = t[k] - t_base;
                    bool in = t[k] >= 0 && t[k] < len && rel >= 0 && rel < R;
                    ent[x + k * 64] = (uint16_t)(in ? rel : DS_NONE);
                    if (in)
                        atomicAdd(&hist[w][rel], 1);
                }
            }
            __syncthreads();
            if (w == 0) {
                // (B) rows lane and lane + 64: list starts, then each wavefront's cursor within the list
                int tot[2], cur[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int r = lane + 64 * u;
                    tot[u] = 0;
                    if (r < R)
                        for (int sw = 0; sw < DD_WAVES; ++sw)
                            tot[u] += hist[sw][r];
                }
                const int inc0 = wave_scan_incl(tot[0], lane);
                const int all0 = __builtin_amdgcn_readlane(inc0, 63);
                const int inc1 = wave_scan_incl(tot[1], lane);
                cur[0] = inc0 - tot[0];
                cur[1] = all0 + inc1 - tot[1];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int r = lane + 64 * u;
                    if (r < R) {
                        start[r] = cur[u];
                        int run = cur[u];
                        for (int sw = 0; sw < DD_WAVES; ++sw) {
                            int cnt = hist[sw][r];
                            hist[sw][r] = run;
                            run += cnt;
                        }
                        if (r == R - 1)
                            start[R] = run;
                    }
                }
            }
            __syncthreads();
            {
                // (C) stable placement: entries in order, equal rows ranked by lane
                volatile int *cursor = &hist[w][0];
                for (int k = 0; k < DS_SEG / 64; ++k) {
                    const int x = w * DS_SEG + k * 64 + lane;
                    const int rel = ent[x];
                    const bool valid = rel != DS_NONE;
                    uint64_t same = __ballot(valid);
                    if (same == 0)
                        continue;
#pragma unroll
                    for (int bit = 0; bit < RBITS; ++bit) {
                        const bool one = (rel >> bit) & 1;
                        const uint64_t bm = __ballot(one);
                        same &= one ? bm : ~bm;
                    }
                    if (valid) {
                        const int rank = __popcll(same & ((uint64_t(1) << lane) - 1));
                        const int pos = cursor[rel] + rank;
                        list[pos] = (uint16_t)x;
                        if (rank == 0)
                            cursor[rel] = pos + __popcll(same);
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            }
            __syncthreads();
            // (D) walk the lists
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                const int r = ps * 32 + grp * DD_WAVES + w; // neighbouring rows (hot tokens often are) go to different wavefronts
                int beg = start[r], end = start[r + 1];
                // A list much longer than the others of the wavefront (a hot token) would leave 48 lanes idle for
                // most of its length: the whole wavefront walks such lists instead, one after the other, one Q row per
                // load instruction and 16 in flight, in the same order and with the same arithmetic.  The row's gradient moves between the two
                // register layouts (8 columns per lane of its group <-> 2 columns per lane of the wavefront) through LDS.
                {
                    int len_g[4], order[4];
#pragma unroll
                    for (int gi = 0; gi < 4; ++gi)
                        len_g[gi] = __builtin_amdgcn_readlane(end - beg, 16 * gi);
                    const int n_long = pick_long_lists(len_g, order);
                    for (int t = 0; t < n_long; ++t) {
                        const int who = t == 0 ? order[0] : t == 1 ? order[1] : t == 2 ? order[2] : order[3];
                        const int lb = __builtin_amdgcn_readlane(beg, 16 * who);
                        const int le = __builtin_amdgcn_readlane(end, 16 * who);
                        float *xf = &xfer[w][0];
                        if (grp == who) {
#pragma unroll
                            for (int x = 0; x < 8; ++x)
                                xf[c * 8 + x] = acc[ps][x];
                        }
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        float ax = xf[2 * lane], ay = xf[2 * lane + 1];
                        for (int k = lb; k < le; k += DD_BATCH) {
                            // lanes 0 .. 15 look up one edge each
                            const int kk = k + (lane & (DD_BATCH - 1));
                            const uint32_t n = (uint32_t)c0 + (kk < le ? (uint32_t)list[kk] : 0u);
                            const uint32_t q = (uint32_t)(((uint64_t)n * lq_magic) >> lq_shift);
                            const bool ok = kk < le && q < (uint32_t)p.n_q;
                            const float gv = ok ? p.g[(int64_t)q * p.b + j] : 0.0f;
                            const int64_t roff = (int64_t)(ok ? n : 0u) * ROWB;
                            const int rlo = (int)(roff & 0xffffffff), rhi = (int)(roff >> 32);
                            const int okv = ok ? 1 : 0;
                            float x0[DD_BATCH], x1[DD_BATCH];
#pragma unroll
                            for (int u = 0; u < DD_BATCH; ++u) {
                                const int64_t off = ((int64_t)__builtin_amdgcn_readlane(rhi, u) << 32) |
                                                    (uint32_t)__builtin_amdgcn_readlane(rlo, u);
                                load_pair<DT>(p.Q + off, lane, x0[u], x1[u]);
                            }
#pragma unroll
                            for (int u = 0; u < DD_BATCH; ++u) {
                                if (__builtin_amdgcn_readlane(okv, u)) {
                                    const float gg = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(gv), u));
                                    ax = fmaf(gg, x0[u], ax);
                                    ay = fmaf(gg, x1[u], ay);
                                }
                            }
                        }
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        xf[2 * lane] = ax;
                        xf[2 * lane + 1] = ay;
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        if (grp == who) {
#pragma unroll
                            for (int x = 0; x < 8; ++x)
                                acc[ps][x] = xf[c * 8 + x];
                            end = beg; // done
                        }
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); // xfer is written again by the next list
                        __builtin_amdgcn_wave_barrier();
                    }
                }
                constexpr int UNROLL = 4;
                for (int k = beg; k < end; k += UNROLL) {
                    int64_t qrow[UNROLL];
                    float gg[UNROLL];
                    bool on[UNROLL];
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u) {
                        on[u] = k + u < end;
                        const uint32_t n = (uint32_t)c0 + (on[u] ? (uint32_t)list[k + u] : 0u); // = q * l_q + i: the Q row
                        const uint32_t q = (uint32_t)(((uint64_t)n * lq_magic) >> lq_shift);
                        on[u] = on[u] && q < (uint32_t)p.n_q;
                        qrow[u] = on[u] ? (int64_t)n : 0;
                        gg[u] = on[u] ? p.g[(int64_t)q * p.b + j] : 0.0f;
                    }
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u) {
                        float v[8];
                        load8<DT>(p.Q + qrow[u] * ROWB + c * 8 * EB, v);
#pragma unroll
                        for (int x = 0; x < 8; ++x)
                            acc[ps][x] = on[u] ? fmaf(gg[u], v[x], acc[ps][x]) : acc[ps][x];
                    }
                }
            }
        }
    }

#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
        const int64_t row = row0 + ps * 32 + grp * DD_WAVES + w;
        if (row < row_end) {
            float4 *dst = reinterpret_cast<float4 *>(p.dD + row * D_MODEL + c * 8);
            dst[0] = make_float4(acc[ps][0], acc[ps][1], acc[ps][2], acc[ps][3]);
            dst[1] = make_float4(acc[ps][4], acc[ps][5], acc[ps][6], acc[ps][7]);
        }
    }
}

template <int DT> static hipError_t launch_bwd(const BwdParams &p, int num_cu, hipStream_t stream)
{
    int64_t waves = (int64_t)p.n_q * p.l_q;
    int grid_q = (int)((waves + 3) / 4);
    hipLaunchKernelGGL((bwd_dq_kernel<DT>), dim3(grid_q), dim3(256), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    // blocks of 128 rows unless that leaves the chip short of workgroups (about 4 per CU wanted)
    const int64_t want = (int64_t)num_cu * 4;
    // Many edges per dD row (short documents, many queries) or a corpus of fewer than 128 rows per wanted workgroup:
    // the kernel that sorts inside the workgroup; few edges per row on a large corpus: the kernel whose wavefronts
    // filter the lists.  Same bits either way.  Measured (L_q = 32, fp16, whole backward, sort / filter):
    // 512 x 128 tokens 0.40 / 0.90 ms, 256 x 300 0.17 / 0.27, 256 x 64 0.13 / 0.19, 192 x 256 0.10 / 0.12,
    // 128 x 512 0.072 / 0.097, 256 x 512 0.157 / 0.166, 128 x 300 0.082 / 0.080, 64 x 180 0.050 / 0.044,
    // 512 x 1024 0.74 / 0.66, 256 x 1024 0.206 / 0.188.  With a quarter or more of a document's edges on a few hot
    // tokens the sorting kernel is ahead everywhere except 256 x 1024 (0.30 / 0.28 ms).
    const int64_t avg_len = p.total_tokens / p.b > 0 ? p.total_tokens / p.b : 1;
    const int64_t edges = (int64_t)p.n_q * p.l_q; // per document
    if (edges >= (int64_t)DD_SORT_MIN_EDGES * avg_len || (edges >= 8 * avg_len && p.total_tokens / 128 < want)) {
        // q = n / l_q for n < 2^31 as (n * magic) >> shift
        int lg = 0;
        while ((1 << lg) < p.l_q)
            ++lg;
        const int shift = 31 + lg;
        const uint32_t magic = (uint32_t)((((uint64_t)1 << shift) + (uint64_t)p.l_q - 1) / (uint64_t)p.l_q);
        if (p.total_tokens / 128 >= want) {
            int64_t grid_d = (p.total_tokens + 127) / 128;
            hipLaunchKernelGGL((bwd_dd_sort_kernel<DT, 4>), dim3((unsigned)grid_d), dim3(DD_WAVES * 64), 0, stream, p, magic, shift);
        } else if (p.total_tokens / 64 >= want) {
            int64_t grid_d = (p.total_tokens + 63) / 64;
            hipLaunchKernelGGL((bwd_dd_sort_kernel<DT, 2>), dim3((unsigned)grid_d), dim3(DD_WAVES * 64), 0, stream, p, magic, shift);
        } else {
            int64_t grid_d = (p.total_tokens + 31) / 32;
            hipLaunchKernelGGL((bwd_dd_sort_kernel<DT, 1>), dim3((unsigned)grid_d), dim3(DD_WAVES * 64), 0, stream, p, magic, shift);
        }
        return hipGetLastError();
    }
    if (p.total_tokens / (DD_WAVES * 16) >= want) {
        int64_t grid_d = (p.total_tokens + DD_WAVES * 16 - 1) / (DD_WAVES * 16);
        hipLaunchKernelGGL((bwd_dd_kernel<DT, 16>), dim3((unsigned)grid_d), dim3(DD_WAVES * 64), 0, stream, p);
    } else if (p.total_tokens / (DD_WAVES * 8) >= want) {
        int64_t grid_d = (p.total_tokens + DD_WAVES * 8 - 1) / (DD_WAVES * 8);
        hipLaunchKernelGGL((bwd_dd_kernel<DT, 8>), dim3((unsigned)grid_d), dim3(DD_WAVES * 64), 0, stream, p);
    } else {
        int64_t grid_d = (p.total_tokens + DD_WAVES * 4 - 1) / (DD_WAVES * 4);
        hipLaunchKernelGGL((bwd_dd_kernel<DT, 4>), dim3((unsigned)grid_d), dim3(DD_WAVES * 64), 0, stream, p);
    }
    return hipGetLastError();
}

hipError_t backward_launch(const void *Q, int n_q, int l_q, const void *D, const int32_t *offsets, int64_t b, int l_d,
                           int64_t total_tokens, int dtype, const int32_t *argmax, const float *dscore, float *dQ,
                           float *dD, int num_cu, hipStream_t stream)
{
    BwdParams p;
    p.Q = static_cast<const char *>(Q);
    p.D = static_cast<const char *>(D);
    p.offsets = offsets;
    p.total_tokens = total_tokens;
    p.A = argmax;
    p.g = dscore;
    p.dQ = dQ;
    p.dD = dD;
    p.b = b;
    p.n_q = n_q;
    p.l_q = l_q;
    p.l_d = l_d;
    switch (dtype) {
    case MAXSIM_F32: return launch_bwd<MAXSIM_F32>(p, num_cu, stream);
    case MAXSIM_F16: return launch_bwd<MAXSIM_F16>(p, num_cu, stream);
    default: return launch_bwd<MAXSIM_BF16>(p, num_cu, stream);
    }
}

// ---------------------------------------------------------------------------------------
// Explicit inverse-grid CSR (Alg. 2): destination row j * l_d + t -> the edges that land on it.
//
// An edge is an argmax entry A[i, j, s] = t with 0 <= t < l_d; its id is the flat index
// e = (i * b + j) * l_q + s.  row_ptr [b * l_d + 1] and col_idx [number of edges] are what
// bincount + cumsum + a stable argsort by destination give: the edges of a row are listed by
// increasing id.  Because all rows of document j are consecutive, the build is a counting sort
// per document:
//   csr_count_kernel   edges of document j            -> row_ptr[(j + 1) * l_d]
//   csr_scan_kernel    running sum over the documents  (in place, stride l_d; row_ptr[0] = 0)
//   csr_place_kernel   one workgroup per document: each of its 8 wavefronts takes a contiguous
//                      eighth of the document's n_q * l_q entries and counts it into its own
//                      histogram over t; a scan over (t, wavefront) turns the histograms into
//                      write cursors and gives row_ptr; each wavefront then walks its entries
//                      again, 64 at a time, ranks equal t within the 64 by ballots and writes
//                      the edge ids.  No atomics decide an order, so the CSR is the same on
//                      every run.
//   csr_apply_kernel   sixteen lanes per dD row walk the row's list in order (Eq. 3).
// ---------------------------------------------------------------------------------------
constexpr int CSR_WAVES = 8;
constexpr int CSR_MAX_LD = 4096;
constexpr int CSR_LOADS = 8;      // argmax entries a lane fetches before it uses the first
#ifndef CSR_APPLY_WAVES
#define CSR_APPLY_WAVES 8 // wavefronts per workgroup of csr_apply_kernel (4 rows each)
#endif
constexpr int CSR_LDS_EXTRA = 16; // ints after the histograms: one sum per wavefront for the block scan

struct CsrParams {
    const int32_t *A;
    int32_t *row_ptr;
    int32_t *col_idx;
    int64_t b;
    int n_q, l_q, l_d;
};

__global__ void __launch_bounds__(1024) csr_count_kernel(CsrParams p)
{
    __shared__ int part[16];
    const int tid = threadIdx.x;
    const int n = p.n_q * p.l_q;
    for (int64_t j = blockIdx.x; j < p.b; j += gridDim.x) {
        int cnt = 0;
        for (int64_t kb = tid; kb < n; kb += 1024 * CSR_LOADS) { // CSR_LOADS entries in flight per lane
            int t[CSR_LOADS];
#pragma unroll
            for (int u = 0; u < CSR_LOADS; ++u) {
                const int64_t k = kb + u * 1024;
                const int i = (int)(k / p.l_q);
                const int s = (int)(k - (int64_t)i * p.l_q);
                t[u] = k < n ? p.A[((int64_t)i * p.b + j) * p.l_q + s] : -1;
            }
#pragma unroll
            for (int u = 0; u < CSR_LOADS; ++u)
                cnt += (unsigned)t[u] < (unsigned)p.l_d ? 1 : 0;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1)
            cnt += __shfl_xor(cnt, o);
        if ((tid & 63) == 0)
            part[tid >> 6] = cnt;
        __syncthreads();
        if (tid == 0) {
            int total = 0;
#pragma unroll
            for (int x = 0; x < 16; ++x)
                total += part[x];
            p.row_ptr[(j + 1) * p.l_d] = total;
        }
        __syncthreads();
    }
}

__global__ void __launch_bounds__(1024) csr_scan_kernel(CsrParams p)
{
    __shared__ int wsum[16];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    int carry = 0;
    for (int64_t c0 = 0; c0 < p.b; c0 += 1024) {
        int64_t j = c0 + tid;
        int v = j < p.b ? p.row_ptr[(j + 1) * p.l_d] : 0;
        int incl = wave_scan_incl(v, lane);
        if (lane == 63)
            wsum[w] = incl;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int x = 0; x < 16; ++x) {
            int sx = wsum[x];
            before += x < w ? sx : 0;
            total += sx;
        }
        if (j < p.b)
            p.row_ptr[(j + 1) * p.l_d] = carry + before + incl;
        carry += total;
        __syncthreads();
    }
    if (tid == 0)
        p.row_ptr[0] = 0;
}

__global__ void __launch_bounds__(CSR_WAVES * 64) csr_place_kernel(CsrParams p)
{
    extern __shared__ int csr_lds[]; // [CSR_WAVES][l_d] histograms, then cursors; CSR_LDS_EXTRA ints of scan space
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int l_d = p.l_d;
    int *wsum = csr_lds + CSR_WAVES * l_d;
    volatile int *H = csr_lds + w * l_d;
    const int n = p.n_q * p.l_q;
    const int chunk = (int)((((int64_t)n + CSR_WAVES * 64 - 1) / (CSR_WAVES * 64)) * 64);
    const int64_t k0 = (int64_t)w * chunk;
    const int64_t k1 = k0 + chunk < n ? k0 + chunk : n;
    const int tpt = (l_d + CSR_WAVES * 64 - 1) / (CSR_WAVES * 64); // tokens per thread in the scan
    int nbits = 0;
    while ((1 << nbits) < l_d)
        ++nbits;

    for (int64_t j = blockIdx.x; j < p.b; j += gridDim.x) {
        for (int x = tid; x < CSR_WAVES * l_d; x += CSR_WAVES * 64)
            csr_lds[x] = 0;
        __syncthreads();
        for (int64_t kb = k0 + lane; kb < k1; kb += 64 * CSR_LOADS) {
            int t[CSR_LOADS];
#pragma unroll
            for (int u = 0; u < CSR_LOADS; ++u) {
                const int64_t k = kb + u * 64;
                const int i = (int)(k / p.l_q);
                const int s = (int)(k - (int64_t)i * p.l_q);
                t[u] = k < k1 ? p.A[((int64_t)i * p.b + j) * p.l_q + s] : -1;
            }
#pragma unroll
            for (int u = 0; u < CSR_LOADS; ++u)
                if ((unsigned)t[u] < (unsigned)l_d)
                    atomicAdd(csr_lds + w * l_d + t[u], 1);
        }
        __syncthreads();
        // exclusive scan over (t major, wavefront minor), starting at the document's first edge
        const int t_lo = tid * tpt;
        const int t_hi = t_lo + tpt < l_d ? t_lo + tpt : l_d;
        int local = 0;
        for (int t = t_lo; t < t_hi; ++t)
            for (int x = 0; x < CSR_WAVES; ++x)
                local += csr_lds[x * l_d + t];
        int incl = wave_scan_incl(local, lane);
        if (lane == 63)
            wsum[w] = incl;
        __syncthreads();
        int run = p.row_ptr[j * l_d] + incl - local;
        for (int x = 0; x < w; ++x)
            run += wsum[x];
        for (int t = t_lo; t < t_hi; ++t) {
            p.row_ptr[j * l_d + t] = run;
            for (int x = 0; x < CSR_WAVES; ++x) {
                int c = csr_lds[x * l_d + t];
                csr_lds[x * l_d + t] = run;
                run += c;
            }
        }
        __syncthreads();
        // placement: entries in order, equal t ranked by lane
        for (int64_t kb0 = k0; kb0 < k1; kb0 += 64 * CSR_LOADS) {
            int tt[CSR_LOADS], ee[CSR_LOADS];
#pragma unroll
            for (int u = 0; u < CSR_LOADS; ++u) { // all loads of the batch before the first is used
                const int64_t k = kb0 + u * 64 + lane;
                const int i = (int)(k / p.l_q);
                const int s = (int)(k - (int64_t)i * p.l_q);
                const int64_t e64 = ((int64_t)i * p.b + j) * p.l_q + s;
                tt[u] = k < k1 ? p.A[e64] : -1;
                ee[u] = (int)e64;
            }
#pragma unroll
            for (int u = 0; u < CSR_LOADS; ++u) {
                if (kb0 + u * 64 >= k1)
                    break;
                const int t = tt[u];
                const bool valid = (unsigned)t < (unsigned)l_d;
                uint64_t same = __ballot(valid);
                for (int bit = 0; bit < nbits; ++bit) {
                    bool one = (t >> bit) & 1;
                    uint64_t bm = __ballot(one);
                    same &= one ? bm : ~bm;
                }
                if (valid) {
                    uint64_t below = same & ((uint64_t(1) << lane) - 1);
                    int rank = __popcll(below);
                    int pos = H[t] + rank;
                    if ((int64_t)pos < (int64_t)n * p.b) // holds unless argmax changed since it was counted
                        p.col_idx[pos] = ee[u];
                    if (rank == 0)
                        H[t] = pos + __popcll(same);
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
        __syncthreads();
    }
}

// dD[r, :] = sum over the edges of row r, in list order, of g[i, j] * Q[i, s, :].  Sixteen lanes per row; lists
// much longer than the others of their wavefront are walked by the whole wavefront (as in bwd_dd_sort_kernel:
// same order, same arithmetic).
template <int DT>
__global__ void __launch_bounds__(CSR_APPLY_WAVES * 64) csr_apply_kernel(BwdParams p, const int32_t *__restrict__ row_ptr,
                                                        const int32_t *__restrict__ col_idx)
{
    constexpr int ROWB = D_MODEL * Elem<DT>::BYTES;
    __shared__ float xfer[CSR_APPLY_WAVES][D_MODEL];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int grp = lane >> 4;
    const int c = lane & 15;
    const int64_t row = (int64_t)blockIdx.x * (4 * CSR_APPLY_WAVES) + grp * CSR_APPLY_WAVES + w; // neighbouring rows go to different wavefronts
    const bool live = row < p.total_tokens;
    const int64_t rr = live ? row : p.total_tokens - 1;
    const int64_t j = rr / p.l_d;
    const int64_t n_edges = (int64_t)p.n_q * p.l_q * p.b;
    int beg = row_ptr[rr] > 0 ? row_ptr[rr] : 0;
    int end = row_ptr[rr + 1] < n_edges ? row_ptr[rr + 1] : (int)n_edges;
    if (!live || end < beg)
        end = beg;
    const uint32_t bl = (uint32_t)(p.b * p.l_q); // edge ids of one query
    const int64_t jl = j * p.l_q;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};

    // edge id -> (usable, Q row, weight) for a row of document jd
    auto decode = [&](bool want, int e, int64_t jd, int64_t jld, bool &ok, int64_t &qrow, float &gv) {
        int64_t rem = (want ? (int64_t)e : jld) - jld; // i * (b * l_q) + s
        uint32_t i = (uint32_t)rem / bl;
        uint32_t s_ = (uint32_t)rem - i * bl;
        ok = want && rem >= 0 && rem < (int64_t(1) << 31) && i < (uint32_t)p.n_q && s_ < (uint32_t)p.l_q;
        qrow = ok ? (int64_t)i * p.l_q + s_ : 0;
        gv = ok ? p.g[(int64_t)i * p.b + jd] : 0.0f;
    };

    {
        int len_g[4], order[4];
#pragma unroll
        for (int gi = 0; gi < 4; ++gi)
            len_g[gi] = __builtin_amdgcn_readlane(end - beg, 16 * gi);
        const int n_long = pick_long_lists(len_g, order);
        for (int t = 0; t < n_long; ++t) {
            const int who = t == 0 ? order[0] : t == 1 ? order[1] : t == 2 ? order[2] : order[3];
            const int lb = __builtin_amdgcn_readlane(beg, 16 * who);
            const int le = __builtin_amdgcn_readlane(end, 16 * who);
            const int64_t row_w = (int64_t)blockIdx.x * (4 * CSR_APPLY_WAVES) + who * CSR_APPLY_WAVES + w; // a live row
            const int64_t jw = row_w / p.l_d;
            const int64_t jlw = jw * p.l_q;
            float ax = 0.0f, ay = 0.0f;
            for (int k = lb; k < le; k += DD_BATCH) {
                const int kk = k + (lane & (DD_BATCH - 1));
                bool ok;
                int64_t qrow;
                float gv;
                decode(kk < le, kk < le ? col_idx[kk] : 0, jw, jlw, ok, qrow, gv);
                const int64_t roff = qrow * ROWB;
                const int rlo = (int)(roff & 0xffffffff), rhi = (int)(roff >> 32);
                const int okv = ok ? 1 : 0;
                float x0[DD_BATCH], x1[DD_BATCH];
#pragma unroll
                for (int u = 0; u < DD_BATCH; ++u) {
                    const int64_t off = ((int64_t)__builtin_amdgcn_readlane(rhi, u) << 32) |
                                        (uint32_t)__builtin_amdgcn_readlane(rlo, u);
                    load_pair<DT>(p.Q + off, lane, x0[u], x1[u]);
                }
#pragma unroll
                for (int u = 0; u < DD_BATCH; ++u) {
                    if (__builtin_amdgcn_readlane(okv, u)) {
                        const float gg = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(gv), u));
                        ax = fmaf(gg, x0[u], ax);
                        ay = fmaf(gg, x1[u], ay);
                    }
                }
            }
            float *xf = &xfer[w][0];
            xf[2 * lane] = ax;
            xf[2 * lane + 1] = ay;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (grp == who) {
#pragma unroll
                for (int x = 0; x < 8; ++x)
                    acc[x] = xf[c * 8 + x];
                end = beg; // done
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); // xfer is written again by the next list
            __builtin_amdgcn_wave_barrier();
        }
    }

    constexpr int UNROLL = 4;
    for (int k = beg; k < end; k += UNROLL) {
        int64_t qrow[UNROLL];
        float gg[UNROLL];
        bool on[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            decode(k + u < end, k + u < end ? col_idx[k + u] : 0, j, jl, on[u], qrow[u], gg[u]);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float v[8];
            load8<DT>(p.Q + qrow[u] * ROWB + c * 8 * Elem<DT>::BYTES, v);
#pragma unroll
            for (int x = 0; x < 8; ++x)
                acc[x] = on[u] ? fmaf(gg[u], v[x], acc[x]) : acc[x];
        }
    }
    if (live) {
        float4 *dst = reinterpret_cast<float4 *>(p.dD + row * D_MODEL + c * 8);
        dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
}

hipError_t csr_build_launch(const int32_t *argmax, int n_q, int64_t b, int l_q, int l_d, int32_t *row_ptr,
                            int32_t *col_idx, int num_cu, hipStream_t stream)
{
    if (l_d > CSR_MAX_LD)
        return hipErrorInvalidValue;
    CsrParams c;
    c.A = argmax;
    c.row_ptr = row_ptr;
    c.col_idx = col_idx;
    c.b = b;
    c.n_q = n_q;
    c.l_q = l_q;
    c.l_d = l_d;
    // more than 64 KB of dynamic LDS has to be allowed once per device
    static bool allowed[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return e;
    if (dev < 0 || dev >= 64)
        return hipErrorInvalidDevice;
    if (!allowed[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&csr_place_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                (CSR_WAVES * CSR_MAX_LD + CSR_LDS_EXTRA) * (int)sizeof(int));
        if (e != hipSuccess)
            return e;
        allowed[dev] = true;
    }
    const int64_t cap = (int64_t)num_cu * 64;
    const unsigned grid = (unsigned)(b < cap ? b : cap);
    hipLaunchKernelGGL(csr_count_kernel, dim3(grid), dim3(1024), 0, stream, c);
    if ((e = hipGetLastError()) != hipSuccess)
        return e;
    hipLaunchKernelGGL(csr_scan_kernel, dim3(1), dim3(1024), 0, stream, c);
    if ((e = hipGetLastError()) != hipSuccess)
        return e;
    const size_t lds = (size_t)(CSR_WAVES * l_d + CSR_LDS_EXTRA) * sizeof(int);
    hipLaunchKernelGGL(csr_place_kernel, dim3(grid), dim3(CSR_WAVES * 64), lds, stream, c);
    return hipGetLastError();
}

template <int DT> static hipError_t launch_bwd_csr(const BwdParams &p, const int32_t *row_ptr, const int32_t *col_idx,
                                                   hipStream_t stream)
{
    int64_t waves = (int64_t)p.n_q * p.l_q;
    hipLaunchKernelGGL((bwd_dq_kernel<DT>), dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return e;
    constexpr int ROWS = 4 * CSR_APPLY_WAVES; // rows per workgroup
    int64_t groups = (p.total_tokens + ROWS - 1) / ROWS;
    hipLaunchKernelGGL((csr_apply_kernel<DT>), dim3((unsigned)groups), dim3(CSR_APPLY_WAVES * 64), 0, stream, p, row_ptr, col_idx);
    return hipGetLastError();
}

hipError_t backward_csr_launch(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int dtype,
                               const int32_t *argmax, const float *dscore, int32_t *row_ptr, int32_t *col_idx, float *dQ,
                               float *dD, int num_cu, hipStream_t stream)
{
    hipError_t e = csr_build_launch(argmax, n_q, b, l_q, l_d, row_ptr, col_idx, num_cu, stream);
    if (e != hipSuccess)
        return e;
    BwdParams p;
    p.Q = static_cast<const char *>(Q);
    p.D = static_cast<const char *>(D);
    p.offsets = nullptr;
    p.total_tokens = b * (int64_t)l_d;
    p.A = argmax;
    p.g = dscore;
    p.dQ = dQ;
    p.dD = dD;
    p.b = b;
    p.n_q = n_q;
    p.l_q = l_q;
    p.l_d = l_d;
    switch (dtype) {
    case MAXSIM_F32: return launch_bwd_csr<MAXSIM_F32>(p, row_ptr, col_idx, stream);
    case MAXSIM_F16: return launch_bwd_csr<MAXSIM_F16>(p, row_ptr, col_idx, stream);
    default: return launch_bwd_csr<MAXSIM_BF16>(p, row_ptr, col_idx, stream);
    }
}

// ---------------------------------------------------------------------------------------
// The CSR backward for callers that cannot allocate (code under graph capture, serving loops): row_ptr and
// col_idx live in a device array that is part of the library's image, one copy per GPU, held until the process
// ends.  Every call on a GPU uses that GPU's copy: calls that overlap on one GPU race.  Nothing in it has to
// start at zero: the build writes every row_ptr entry and every col_idx entry that the walk reads.
// ---------------------------------------------------------------------------------------
constexpr int64_t CSR_STATIC_MAX_ROWS = int64_t(1) << 18;  // b * l_d
constexpr int64_t CSR_STATIC_MAX_EDGES = int64_t(1) << 21; // n_q * b * l_q
constexpr int64_t CSR_STATIC_COL_AT = CSR_STATIC_MAX_ROWS + 64; // col_idx starts here (ints; keeps 256-byte alignment)
static __device__ __align__(256) int32_t scratch[CSR_STATIC_COL_AT + CSR_STATIC_MAX_EDGES];

namespace {
int32_t *scratch_ptr[64] = {nullptr}; // device address of `scratch` on each GPU (the array's name is no address on the host)
std::mutex scratch_guard;
} // namespace

// Once per device, with that device current: the address of the device's copy of `scratch`.
static hipError_t csr_static_buffer(int32_t **out)
{
    std::lock_guard<std::mutex> lock(scratch_guard);
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return e;
    if (dev < 0 || dev >= 64)
        return hipErrorInvalidDevice;
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess)
            return e;
        if (!ptr)
            return hipErrorInvalidSymbol;
        scratch_ptr[dev] = static_cast<int32_t *>(ptr);
    }
    *out = scratch_ptr[dev];
    return hipSuccess;
}

bool csr_static_fits(int n_q, int64_t b, int l_q, int l_d)
{
    return b * (int64_t)l_d <= CSR_STATIC_MAX_ROWS && (int64_t)n_q * l_q * b <= CSR_STATIC_MAX_EDGES;
}

hipError_t backward_csr_static_launch(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int dtype,
                                      const int32_t *argmax, const float *dscore, float *dQ, float *dD, int num_cu,
                                      hipStream_t stream)
{
    if (!csr_static_fits(n_q, b, l_q, l_d))
        return hipErrorInvalidValue;
    int32_t *buf = nullptr;
    hipError_t e = csr_static_buffer(&buf);
    if (e != hipSuccess)
        return e;
    return backward_csr_launch(Q, n_q, l_q, D, b, l_d, dtype, argmax, dscore, buf, buf + CSR_STATIC_COL_AT, dQ, dD, num_cu,
                               stream);
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

// s / tau as one rounded multiply that may not be contracted into a fused multiply-add
__device__ __forceinline__ float scaled(float s, float inv_tau)
{
#pragma clang fp contract(off)
    return s * inv_tau;
}

// s / tau is formed with an explicitly rounded multiply everywhere, so that the same value
// enters the max, the exponent and the label term (no fused multiply-add may split them).
// Gradient: one wavefront per row, rows dealt round-robin to the wavefronts of the grid.
__global__ void __launch_bounds__(256) ce_grad_kernel(const float *s, int n, int b, float inv_tau, float *g)
{
    const int lane = threadIdx.x & 63;
    const int n_waves = (int)gridDim.x * 4;
    for (int i = (int)blockIdx.x * 4 + (threadIdx.x >> 6); i < n; i += n_waves) {
        const float *row = s + (int64_t)i * b;
        float mx = neg_inf();
        for (int j = lane; j < b; j += 64)
            mx = fmaxf(mx, scaled(row[j], inv_tau));
        mx = wave_max(mx);
        float z = 0.0f;
        for (int j = lane; j < b; j += 64)
            z += expf(scaled(row[j], inv_tau) - mx);
        z = wave_sum(z);
        float scale = inv_tau / (float)n;
        for (int j = lane; j < b; j += 64) {
            float pj = expf(scaled(row[j], inv_tau) - mx) / z;
            g[(int64_t)i * b + j] = (pj - (j == i ? 1.0f : 0.0f)) * scale;
        }
    }
}

// Loss: a single block (fixed summation order); 16 lanes per row, 64 rows at a time.  When a row has at most
// 16 * KEEP columns (KEEP = 16 or 32) the scaled scores of a lane live in registers, and the loads of two to four
// rows are issued together before any of them is reduced: the kernel is a chain of memory latencies, not
// of arithmetic.  Wider rows (KEEP = 0) are re-read from memory for each of the sweeps.
template <int KEEP>
__global__ void __launch_bounds__(1024) ce_loss_kernel(const float *s, int n, int b, float inv_tau, float *loss)
{
    __shared__ float part[64];
    const int sub = threadIdx.x & 15;
    const int slot = threadIdx.x >> 4;
    float local = 0.0f;
    if constexpr (KEEP > 0) {
        constexpr int ROWS = 64 / KEEP; // rows of a slot in flight together (64 registers)
        for (int i0 = slot; i0 < n; i0 += 64 * ROWS) {
            float v[ROWS][KEEP];
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                const int i = i0 + 64 * r;
                const float *row = s + (int64_t)(i < n ? i : i0) * b;
#pragma unroll
                for (int k = 0; k < KEEP; ++k) {
                    const int j = sub + 16 * k;
                    v[r][k] = j < b ? scaled(row[j], inv_tau) : neg_inf();
                }
            }
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                const int i = i0 + 64 * r;
                float mx = neg_inf();
#pragma unroll
                for (int k = 0; k < KEEP; ++k)
                    mx = fmaxf(mx, v[r][k]);
#pragma unroll
                for (int o = 8; o > 0; o >>= 1)
                    mx = fmaxf(mx, __shfl_xor(mx, o));
                float z = 0.0f;
#pragma unroll
                for (int k = 0; k < KEEP; ++k)
                    z += (sub + 16 * k < b) ? expf(v[r][k] - mx) : 0.0f; // same order as the sweep over memory
#pragma unroll
                for (int o = 8; o > 0; o >>= 1)
                    z += __shfl_xor(z, o);
                if (i < n)
                    local += logf(z) + mx - scaled(s[(int64_t)i * b + i], inv_tau);
            }
        }
    } else {
        for (int i = slot; i < n; i += 64) {
            const float *row = s + (int64_t)i * b;
            float mx = neg_inf();
            for (int j = sub; j < b; j += 16)
                mx = fmaxf(mx, scaled(row[j], inv_tau));
#pragma unroll
            for (int o = 8; o > 0; o >>= 1)
                mx = fmaxf(mx, __shfl_xor(mx, o));
            float z = 0.0f;
            for (int j = sub; j < b; j += 16)
                z += expf(scaled(row[j], inv_tau) - mx);
#pragma unroll
            for (int o = 8; o > 0; o >>= 1)
                z += __shfl_xor(z, o);
            local += logf(z) + mx - scaled(row[i], inv_tau);
        }
    }
    if (sub == 0)
        part[slot] = local;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.0f;
        for (int k = 0; k < 64; ++k)
            t += part[k];
        *loss = t / (float)n;
    }
}

hipError_t ce_grad_launch(const float *scores, int n, int b, float tau, float *g, float *loss, hipStream_t stream)
{
    int row_blocks = (n + 3) / 4;
    hipLaunchKernelGGL(ce_grad_kernel, dim3(row_blocks), dim3(256), 0, stream, scores, n, b, 1.0f / tau, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !loss)
        return e;
    if (b <= 256)
        hipLaunchKernelGGL(ce_loss_kernel<16>, dim3(1), dim3(1024), 0, stream, scores, n, b, 1.0f / tau, loss);
    else if (b <= 512)
        hipLaunchKernelGGL(ce_loss_kernel<32>, dim3(1), dim3(1024), 0, stream, scores, n, b, 1.0f / tau, loss);
    else
        hipLaunchKernelGGL(ce_loss_kernel<0>, dim3(1), dim3(1024), 0, stream, scores, n, b, 1.0f / tau, loss);
    return hipGetLastError();
}

} // namespace maxsim
