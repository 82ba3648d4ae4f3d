// Fused MaxSim forward for gfx950 (Alg. 1 of the paper, re-designed around 64-wide
// wavefronts and the 32x32 MFMA result layout).
//
// Orientation.  Document tokens sit on the MFMA rows (A operand), query tokens on the
// columns (B operand).  A lane of the 32x32 result holds ONE query token (column
// lane % 32) and 16 document tokens, so the max over document tokens (line 9 of Alg. 1)
// is an in-lane chain of v_max3 over the accumulator registers and the running row-max is
// one register per lane per 32 query tokens.  The two lane halves are merged once per
// document; the sum over query tokens (line 11) is a butterfly over 32 lanes.
//
// Masking (line 8 of Alg. 1).  Rows past the end of a document are not set to -inf after
// the product; instead the loads clamp the row index to the document's last token.  A
// duplicated token cannot change a max, and it cannot win the argmax because ties go to the
// lowest index, so the result is the same and the epilogue stays mask-free.
//
// Two kernels share these pieces:
//   fwd_stream_kernel  few query tokens (<= 128 in total): the corpus read is the cost.
//                      Every wavefront works alone on its own run of documents; document
//                      tiles go HBM -> registers directly in MFMA operand layout (32 rows x
//                      32 contiguous bytes per load instruction), one tile ahead.
//   fwd_tile_kernel    many query tokens: the contraction is the cost.  A workgroup keeps up
//                      to 1024 query tokens stationary in registers (128 per wavefront) and
//                      streams document tiles through LDS, shared by all its wavefronts.
#include "common.h"

namespace maxsim {

// ---------------------------------------------------------------------------------------
// pieces shared by both kernels
// ---------------------------------------------------------------------------------------

// Query fragments of column block `gb` (global block id): column rho of the block is query
// token (gb % bpq) * 32 + rho of query gb / bpq; columns past l_q re-read the last token
// and are dropped from the sum later.
template <int DT>
__device__ __forceinline__ void load_q_block(const FwdParams &p, int gb, int rho, int h,
                                             uint4 (&qf)[Traits<DT>::NU], bool &col_valid)
{
    using TR = Traits<DT>;
    int total_blocks = p.n_q * p.bpq;
    bool active = gb < total_blocks;
    int g = active ? gb : 0;
    int q = g / p.bpq;
    int tok = (g % p.bpq) * BLOCK_COLS + rho;
    col_valid = active && tok < p.l_q;
    if (tok > p.l_q - 1)
        tok = p.l_q - 1;
    const char *row = p.Q + ((int64_t)q * p.l_q + tok) * TR::ROW_BYTES + h * 16;
#pragma unroll
    for (int u = 0; u < TR::NU; ++u)
        qf[u] = *reinterpret_cast<const uint4 *>(row + u * 32);
}

// Fold one 32x32 result tile into the running max (and argmax) of this lane's query token.
template <bool ARGMAX>
__device__ __forceinline__ void fold_tile(const f32x16 &acc, float &m, int &idx, int row_base, int h)
{
    if (ARGMAX) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            bool up = acc[r] > m; // strict: the first occurrence keeps a tie
            m = up ? acc[r] : m;
            idx = up ? row_base + acc_row(r, h) : idx;
        }
    } else {
#pragma unroll
        for (int r = 0; r < 16; r += 2)
            m = fmaxf(m, fmaxf(acc[r], acc[r + 1]));
    }
}

// End of a document for one column block: merge the lane halves, write the argmax of valid
// columns, and return the sum over the block's valid query tokens (same value in all lanes).
template <bool ARGMAX>
__device__ __forceinline__ float finish_block(const FwdParams &p, float m, int idx, bool col_valid,
                                              int gb, int64_t doc, int len, int rho, int h)
{
    float mo = __shfl_xor(m, 32);
    if (ARGMAX) {
        int io = __shfl_xor(idx, 32);
        bool take = (mo > m) || (mo == m && io < idx);
        m = take ? mo : m;
        idx = take ? io : idx;
        if (col_valid && h == 0) {
            int q = gb / p.bpq;
            int tok = (gb % p.bpq) * BLOCK_COLS + rho;
            if (idx > len - 1)
                idx = len - 1;
            p.argmax[((int64_t)q * p.b + doc) * p.l_q + tok] = idx;
        }
    } else {
        m = fmaxf(m, mo);
    }
    float v = col_valid ? m : 0.0f;
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 8);
    v += __shfl_xor(v, 4);
    v += __shfl_xor(v, 2);
    v += __shfl_xor(v, 1);
    return v;
}

// Documents of length 0 in [doc0, doc1): score -inf, argmax -1 (ragged corpora only).
__device__ __forceinline__ void write_empty_docs(const FwdParams &p, int64_t doc0, int64_t doc1,
                                                 int tid, int nthreads)
{
    if (!p.offsets)
        return;
    for (int64_t doc = doc0 + tid; doc < doc1; doc += nthreads) {
        if (p.offsets[doc + 1] != p.offsets[doc])
            continue;
        for (int q = 0; q < p.n_q; ++q) {
            p.scores[(int64_t)q * p.b + doc] = neg_inf();
            if (p.argmax)
                for (int i = 0; i < p.l_q; ++i)
                    p.argmax[((int64_t)q * p.b + doc) * p.l_q + i] = -1;
        }
    }
}

// ---------------------------------------------------------------------------------------
// streaming kernel: one wavefront per run of documents, all query blocks in registers
// ---------------------------------------------------------------------------------------

template <int DT, int NCB, bool ARGMAX> struct StreamState {
    uint4 qf[NCB][Traits<DT>::NU];
    bool col_valid[NCB];
    float m[NCB];
    int idx[NCB];
};

template <int DT>
__device__ __forceinline__ void stream_load_tile(const FwdParams &p, const Cursor &c, int rho, int h,
                                                 uint4 (&a)[Traits<DT>::NU])
{
    using TR = Traits<DT>;
    int row = c.t0 + rho;
    if (row > c.len - 1)
        row = c.len - 1;
    const char *ptr = p.D + (c.start + row) * TR::ROW_BYTES + h * 16;
#pragma unroll
    for (int u = 0; u < TR::NU; ++u)
        a[u] = *reinterpret_cast<const uint4 *>(ptr + u * 32);
}

template <int DT, int NCB, bool ARGMAX>
__device__ __forceinline__ void stream_compute(const FwdParams &p, const Cursor &c,
                                               StreamState<DT, NCB, ARGMAX> &st,
                                               const uint4 (&a)[Traits<DT>::NU], int lane, int rho, int h)
{
    using TR = Traits<DT>;
    if (c.t0 == 0) {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            st.m[cb] = neg_inf();
            st.idx[cb] = 0;
        }
    }
    f32x16 acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            acc[cb][r] = 0.0f;
#pragma unroll
    for (int u = 0; u < TR::NU; ++u)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
            TR::mma(a[u], st.qf[cb][u], acc[cb]);
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
        fold_tile<ARGMAX>(acc[cb], st.m[cb], st.idx[cb], c.t0, h);

    if (c.t0 + TILE_ROWS >= c.len) { // last tile of the document
        float part[NCB];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
            part[cb] = finish_block<ARGMAX>(p, st.m[cb], st.idx[cb], st.col_valid[cb], cb, c.doc, c.len, rho, h);
        // lane q (< n_q) adds up the blocks of query q in block order and writes its score
        float s = 0.0f;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
            if (cb / p.bpq == lane)
                s += part[cb];
        if (lane < p.n_q)
            p.scores[(int64_t)lane * p.b + c.doc] = s;
    }
}

template <int DT, int NCB, bool ARGMAX>
__global__ void __launch_bounds__(256) fwd_stream_kernel(FwdParams p)
{
    using TR = Traits<DT>;
    const int lane = threadIdx.x & 63;
    const int rho = lane & 31, h = lane >> 5;
    const int64_t wave =
        __builtin_amdgcn_readfirstlane((int)(((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6));
    int64_t doc0, doc1;
    chunk_doc_range(p, wave, doc0, doc1);
    if (doc0 >= doc1)
        return;
    write_empty_docs(p, doc0, doc1, lane, 64);

    StreamState<DT, NCB, ARGMAX> st;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
        load_q_block<DT>(p, cb, rho, h, st.qf[cb], st.col_valid[cb]);

    Cursor pc; // prefetch cursor, one tile ahead of the compute cursor
    cursor_init(pc, p, doc0, doc1);
    if (!pc.valid)
        return;
    uint4 a0[TR::NU], a1[TR::NU];
    stream_load_tile<DT>(p, pc, rho, h, a0);
    Cursor cc = pc;
    cursor_next_tile(pc, p);
    for (;;) {
        if (pc.valid)
            stream_load_tile<DT>(p, pc, rho, h, a1);
        stream_compute<DT, NCB, ARGMAX>(p, cc, st, a0, lane, rho, h);
        cc = pc;
        if (!cc.valid)
            break;
        cursor_next_tile(pc, p);
        if (pc.valid)
            stream_load_tile<DT>(p, pc, rho, h, a0);
        stream_compute<DT, NCB, ARGMAX>(p, cc, st, a1, lane, rho, h);
        cc = pc;
        if (!cc.valid)
            break;
        cursor_next_tile(pc, p);
    }
}

// ---------------------------------------------------------------------------------------
// tile kernel: query-stationary workgroup, document tiles staged through LDS
// ---------------------------------------------------------------------------------------

template <int DT> struct LdsTile {
    // rows padded by one 16-byte chunk so that the 32 rows read by one ds_read_b128 of the
    // MFMA operand layout fall into different banks
    static constexpr int ROW_STRIDE = Traits<DT>::ROW_BYTES + 16;
    static constexpr int BYTES = TILE_ROWS * ROW_STRIDE;
    static constexpr int CHUNKS = TILE_ROWS * Traits<DT>::ROW_BYTES / 16;
};

template <int DT, int W, int NCB, bool ARGMAX>
__global__ void __launch_bounds__(W * 64) fwd_tile_kernel(FwdParams p)
{
    using TR = Traits<DT>;
    using LT = LdsTile<DT>;
    constexpr int NT = W * 64;
    constexpr int CPT = LT::CHUNKS / NT; // 16-byte chunks each thread moves per tile
    static_assert(LT::CHUNKS % NT == 0, "tile must split evenly over the workgroup");
    constexpr int CPR = TR::ROW_BYTES / 16; // chunks per row
    constexpr int GROUP_BLOCKS = W * NCB;

    __shared__ __attribute__((aligned(16))) char lds_tile[2][LT::BYTES];
    __shared__ float lds_part[2][GROUP_BLOCKS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int rho = lane & 31, h = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Renumber so
    // that the column groups sharing a document chunk are neighbours on one XCD and run at
    // the same time: the chunk then comes from HBM once and from L2 for the other groups.
    const int n_wg = gridDim.x;
    int v = blockIdx.x;
    if ((n_wg & 7) == 0)
        v = (blockIdx.x & 7) * (n_wg >> 3) + (blockIdx.x >> 3);
    const int group = v % p.n_groups;
    const int chunk = v / p.n_groups;

    int64_t doc0, doc1;
    chunk_doc_range(p, chunk, doc0, doc1);
    if (doc0 >= doc1)
        return;
    if (group == 0)
        write_empty_docs(p, doc0, doc1, tid, NT);

    for (int pass = 0; pass < p.n_pass; ++pass) {
        // column blocks of this pass: [gb0, gb0 + nb); queries [q_first, q_first + nq)
        int gb0, nb, q_first, nq;
        const bool accumulate = pass > 0;
        if (p.n_pass == 1) {
            q_first = group * p.qpg;
            nq = min(p.qpg, p.n_q - q_first);
            gb0 = q_first * p.bpq;
            nb = nq * p.bpq;
        } else { // one long query per group, GROUP_BLOCKS blocks of it per pass
            q_first = group;
            nq = 1;
            gb0 = group * p.bpq + pass * GROUP_BLOCKS;
            nb = min(GROUP_BLOCKS, p.bpq - pass * GROUP_BLOCKS);
        }

        uint4 qf[NCB][TR::NU];
        bool col_valid[NCB];
        float m[NCB];
        int idx[NCB];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            int lb = w * NCB + cb;
            load_q_block<DT>(p, gb0 + lb, rho, h, qf[cb], col_valid[cb]);
            col_valid[cb] = col_valid[cb] && lb < nb;
            m[cb] = neg_inf();
            idx[cb] = 0;
        }

        Cursor lc; // load cursor: the tile whose data is in `g`
        cursor_init(lc, p, doc0, doc1);
        if (!lc.valid)
            break;
        uint4 g[CPT];
        auto gload = [&](const Cursor &c) {
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                int ch = tid + i * NT;
                int row = c.t0 + ch / CPR;
                if (row > c.len - 1)
                    row = c.len - 1;
                g[i] = *reinterpret_cast<const uint4 *>(p.D + (c.start + row) * TR::ROW_BYTES + (ch % CPR) * 16);
            }
        };
        auto lstore = [&](int buf) {
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                int ch = tid + i * NT;
                *reinterpret_cast<uint4 *>(&lds_tile[buf][(ch / CPR) * LT::ROW_STRIDE + (ch % CPR) * 16]) = g[i];
            }
        };

        gload(lc);
        lstore(0);
        Cursor cc = lc;
        cursor_next_tile(lc, p);
        if (lc.valid)
            gload(lc);
        __syncthreads();

        int cur = 0;
        int par = 0; // parity of the partial-sum buffer, flips per document
        while (cc.valid) {
            Cursor cnext = lc;
            if (lc.valid) {
                lstore(cur ^ 1);
                cursor_next_tile(lc, p);
                if (lc.valid)
                    gload(lc);
            }

            uint4 a[TR::NU];
            const char *src = &lds_tile[cur][rho * LT::ROW_STRIDE + h * 16];
#pragma unroll
            for (int u = 0; u < TR::NU; ++u)
                a[u] = *reinterpret_cast<const uint4 *>(src + u * 32);

            if (cc.t0 == 0) {
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) {
                    m[cb] = neg_inf();
                    idx[cb] = 0;
                }
            }
            // two column blocks at a time: two independent accumulator chains in flight
#pragma unroll
            for (int cb = 0; cb < NCB; cb += 2) {
                f32x16 acc0, acc1;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    acc0[r] = 0.0f;
                    acc1[r] = 0.0f;
                }
#pragma unroll
                for (int u = 0; u < TR::NU; ++u) {
                    TR::mma(a[u], qf[cb][u], acc0);
                    if (cb + 1 < NCB)
                        TR::mma(a[u], qf[cb + 1][u], acc1);
                }
                fold_tile<ARGMAX>(acc0, m[cb], idx[cb], cc.t0, h);
                if (cb + 1 < NCB)
                    fold_tile<ARGMAX>(acc1, m[cb + 1], idx[cb + 1], cc.t0, h);
            }

            const bool last_tile = cc.t0 + TILE_ROWS >= cc.len;
            if (last_tile) {
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) {
                    int lb = w * NCB + cb;
                    float s = finish_block<ARGMAX>(p, m[cb], idx[cb], col_valid[cb], gb0 + lb, cc.doc, cc.len, rho, h);
                    if (lane == 0)
                        lds_part[par][lb] = s;
                }
            }
            __syncthreads();
            if (last_tile) {
                if (tid < nq) { // thread t adds up the blocks of its query in block order
                    float s = 0.0f;
                    int first = (p.n_pass == 1) ? tid * p.bpq : 0;
                    int cnt = (p.n_pass == 1) ? p.bpq : nb;
                    for (int i = 0; i < cnt; ++i)
                        s += lds_part[par][first + i];
                    float *dst = p.scores + (int64_t)(q_first + tid) * p.b + cc.doc;
                    *dst = accumulate ? *dst + s : s;
                }
                par ^= 1;
            }
            cc = cnext;
            cur ^= 1;
        }
        __syncthreads(); // LDS tiles are reused by the next pass
    }
}

// ---------------------------------------------------------------------------------------
// host-side launchers (called from the C ABI)
// ---------------------------------------------------------------------------------------

template <int DT, int NCB, bool ARGMAX>
static hipError_t launch_stream(const FwdParams &p, int grid, hipStream_t stream)
{
    hipLaunchKernelGGL((fwd_stream_kernel<DT, NCB, ARGMAX>), dim3(grid), dim3(256), 0, stream, p);
    return hipGetLastError();
}

template <int DT, int W, int NCB, bool ARGMAX>
static hipError_t launch_tile(const FwdParams &p, int grid, hipStream_t stream)
{
    hipLaunchKernelGGL((fwd_tile_kernel<DT, W, NCB, ARGMAX>), dim3(grid), dim3(W * 64), 0, stream, p);
    return hipGetLastError();
}

template <int DT, bool ARGMAX>
static hipError_t dispatch_stream(const FwdParams &p, int ncb, int grid, hipStream_t s)
{
    switch (ncb) {
    case 1: return launch_stream<DT, 1, ARGMAX>(p, grid, s);
    case 2: return launch_stream<DT, 2, ARGMAX>(p, grid, s);
    case 3: return launch_stream<DT, 3, ARGMAX>(p, grid, s);
    default: return launch_stream<DT, 4, ARGMAX>(p, grid, s);
    }
}

template <int DT, bool ARGMAX>
static hipError_t dispatch_tile(const FwdParams &p, int w, int grid, hipStream_t s)
{
    constexpr int NCB = (DT == MAXSIM_F32) ? 2 : 4;
    switch (w) {
    case 1: return launch_tile<DT, 1, NCB, ARGMAX>(p, grid, s);
    case 2: return launch_tile<DT, 2, NCB, ARGMAX>(p, grid, s);
    case 4: return launch_tile<DT, 4, NCB, ARGMAX>(p, grid, s);
    default: return launch_tile<DT, 8, NCB, ARGMAX>(p, grid, s);
    }
}

static int round_up(int64_t x, int m) { return (int)((x + m - 1) / m * m); }

// Chooses kernel and launch shape from the problem size; `num_cu` is the device's CU count.
hipError_t forward_launch(FwdParams p, int dtype, int num_cu, hipStream_t stream)
{
    const bool ragged = p.offsets != nullptr;
    const bool am = p.argmax != nullptr;
    p.bpq = (p.l_q + BLOCK_COLS - 1) / BLOCK_COLS;
    const int64_t total_blocks = (int64_t)p.n_q * p.bpq;
    const int64_t units = ragged ? p.total_tokens : p.b; // what is split across chunks
    const int stream_max_blocks = (dtype == MAXSIM_F32) ? 2 : 4;

    if (total_blocks <= stream_max_blocks) {
        // one work chunk per wavefront; enough chunks to oversubscribe the chip a few times,
        // but no chunk smaller than about 2K tokens
        const int64_t tokens = ragged ? p.total_tokens : p.b * (int64_t)p.l_d;
        int64_t want = (int64_t)num_cu * 16 * 4;
        int64_t by_size = (tokens + 2047) / 2048;
        int64_t n_chunks = want < by_size ? want : by_size;
        if (n_chunks > p.b)
            n_chunks = p.b;
        if (n_chunks < 1)
            n_chunks = 1;
        p.unit_per_chunk = (units + n_chunks - 1) / n_chunks;
        if (p.unit_per_chunk < 1)
            p.unit_per_chunk = 1;
        if (!ragged)
            n_chunks = (units + p.unit_per_chunk - 1) / p.unit_per_chunk;
        p.n_chunks = (int)n_chunks;
        p.n_groups = 1;
        p.qpg = p.n_q;
        p.n_pass = 1;
        int grid = (int)((n_chunks + 3) / 4);
        const int ncb = (int)total_blocks;
        switch (dtype) {
        case MAXSIM_F32:
            return am ? dispatch_stream<MAXSIM_F32, true>(p, ncb, grid, stream)
                      : dispatch_stream<MAXSIM_F32, false>(p, ncb, grid, stream);
        case MAXSIM_F16:
            return am ? dispatch_stream<MAXSIM_F16, true>(p, ncb, grid, stream)
                      : dispatch_stream<MAXSIM_F16, false>(p, ncb, grid, stream);
        default:
            return am ? dispatch_stream<MAXSIM_BF16, true>(p, ncb, grid, stream)
                      : dispatch_stream<MAXSIM_BF16, false>(p, ncb, grid, stream);
        }
    }

    // tile kernel: W wavefronts x NCB blocks per group
    const int ncb = (dtype == MAXSIM_F32) ? 2 : 4;
    int w = 8;
    if (total_blocks <= 1 * ncb)
        w = 1;
    else if (total_blocks <= 2 * ncb)
        w = 2;
    else if (total_blocks <= 4 * ncb)
        w = 4;
    const int group_blocks = w * ncb;
    if (p.bpq <= group_blocks) {
        p.qpg = group_blocks / p.bpq;
        if (p.qpg > p.n_q)
            p.qpg = p.n_q;
        p.n_groups = (p.n_q + p.qpg - 1) / p.qpg;
        p.n_pass = 1;
    } else {
        p.qpg = 1;
        p.n_groups = p.n_q;
        p.n_pass = (p.bpq + group_blocks - 1) / group_blocks;
    }
    // document chunks: about two workgroups per CU and group in total, a multiple of 8 so
    // that the XCD renumbering applies, and never more chunks than documents
    int64_t wg_target = (int64_t)num_cu * 2;
    int64_t n_chunks = (wg_target + p.n_groups - 1) / p.n_groups;
    if (n_chunks < 8)
        n_chunks = 8;
    n_chunks = round_up(n_chunks, 8);
    p.unit_per_chunk = (units + n_chunks - 1) / n_chunks;
    if (p.unit_per_chunk < 1)
        p.unit_per_chunk = 1;
    p.n_chunks = (int)n_chunks;
    int grid = p.n_groups * p.n_chunks;
    switch (dtype) {
    case MAXSIM_F32:
        return am ? dispatch_tile<MAXSIM_F32, true>(p, w, grid, stream)
                  : dispatch_tile<MAXSIM_F32, false>(p, w, grid, stream);
    case MAXSIM_F16:
        return am ? dispatch_tile<MAXSIM_F16, true>(p, w, grid, stream)
                  : dispatch_tile<MAXSIM_F16, false>(p, w, grid, stream);
    default:
        return am ? dispatch_tile<MAXSIM_BF16, true>(p, w, grid, stream)
                  : dispatch_tile<MAXSIM_BF16, false>(p, w, grid, stream);
    }
}

} // namespace maxsim
