// Fused MaxSim forward for gfx950 (Alg. 1 of the paper, re-designed around 64-wide
// wavefronts and the 32x32 MFMA result layout).
//
// Orientation.  Document tokens sit on the MFMA rows (A operand), query tokens on the
// columns (B operand).  A lane of the 32x32 result holds ONE query token (column
// lane % 32) and 16 document tokens, so the max over document tokens (the running row-max step of Alg. 1)
// is an in-lane chain of v_max3 over the accumulator registers and the running row-max is
// one register per lane per 32 query tokens.  The two lane halves are merged once per
// document; the sum over query tokens (the final reduction of Alg. 1) is a butterfly over 32 lanes.
//
// Masking (the -inf step of Alg. 1).  Rows past the end of a document are not set to -inf after
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
#pragma once
#include "common.h"

#include <type_traits>

namespace maxsim {
namespace {

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
            m = fmaxf(fmaxf(m, acc[r]), acc[r + 1]); // one v_max3_f32 per pair
    }
}

// Cross-lane helpers on the VALU (no LDS traffic): v_permlane32_swap exchanges the two lane
// halves, DPP row operations add within a row of 16 lanes.
__device__ __forceinline__ void swap_halves(float x, float &lo_from_hi, float &hi_from_lo)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    hi_from_lo = __uint_as_float(r[0]); // lanes 32..63 now hold lanes 0..31 (lanes 0..31 unchanged)
    lo_from_hi = __uint_as_float(r[1]); // lanes 0..31 now hold lanes 32..63 (lanes 32..63 unchanged)
}

template <int CTRL> __device__ __forceinline__ float dpp_add(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Sum over lanes 0..31 (a fixed tree: pairs, quads, eights, sixteens, then the two rows).
__device__ __forceinline__ float sum_low32(float v)
{
    v = dpp_add<0xB1>(v);  // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);  // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v); // row_half_mirror
    v = dpp_add<0x140>(v); // row_mirror
    float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    return r0 + r1;
}

// End of a document for one column block: merge the lane halves, write the argmax of valid
// columns, and return the sum over the block's valid query tokens (same value in all lanes).
template <bool ARGMAX>
__device__ __forceinline__ float finish_block(const FwdParams &p, float m, int idx, bool col_valid,
                                              int gb, int64_t doc, int len, int rho, int h)
{
    float a, b; // a: this lane's value or its partner's, so that max(a, b) is the merged value in every lane
    swap_halves(m, a, b);
    if (ARGMAX) {
        float ia, ib;
        swap_halves(__int_as_float(idx), ia, ib);
        // lanes 0..31: (a, ia) came from the upper half, (b, ib) is the lane's own; upper lanes: the reverse
        int i0 = __float_as_int(ia), i1 = __float_as_int(ib);
        bool take = (a > b) || (a == b && i0 < i1);
        m = take ? a : b;
        idx = take ? i0 : i1;
        if (col_valid && h == 0) {
            // the address is formed here, at the end of a document, from an opaque copy of the lane's
            // column: hoisted out of the tile loop its per-lane 64-bit parts would cost registers there
            int col = rho;
            asm volatile("" : "+v"(col));
            int q = gb / p.bpq;
            int tok = (gb % p.bpq) * BLOCK_COLS + col;
            if (idx > len - 1)
                idx = len - 1;
            p.argmax[((int64_t)q * p.ld + doc) * p.l_q + tok] = idx;
        }
    } else {
        m = fmaxf(a, b);
    }
    return sum_low32(col_valid ? m : 0.0f);
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
            p.scores[(int64_t)q * p.ld + doc] = neg_inf();
            if (p.argmax)
                for (int i = 0; i < p.l_q; ++i)
                    p.argmax[((int64_t)q * p.ld + doc) * p.l_q + i] = -1;
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

// The position of a tile: first packed row of its document, the document's length, first row of the tile
struct TilePos {
    int64_t start;
    int32_t len, t0;
};

template <int DT>
__device__ __forceinline__ void stream_load_tile(const FwdParams &p, const TilePos &c, int rho, int h,
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
                                               const uint4 (&a)[Traits<DT>::NU], int gb0, int lane, int rho, int h)
{
    using TR = Traits<DT>;
    if (c.t0 == 0) {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            st.m[cb] = neg_inf();
            st.idx[cb] = 0;
        }
    }
    // two column blocks at a time (two accumulator chains in flight); the scheduling barrier keeps
    // the pairs apart so that only two accumulators are live and more wavefronts fit on a SIMD
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
            TR::mma(a[u], st.qf[cb][u], acc0);
            if (cb + 1 < NCB)
                TR::mma(a[u], st.qf[cb + 1][u], acc1);
        }
        fold_tile<ARGMAX>(acc0, st.m[cb], st.idx[cb], c.t0, h);
        if (cb + 1 < NCB)
            fold_tile<ARGMAX>(acc1, st.m[cb + 1], st.idx[cb + 1], c.t0, h);
        if (cb + 2 < NCB)
            __builtin_amdgcn_sched_barrier(0);
    }

    if (c.t0 + TILE_ROWS >= c.len) { // last tile of the document
        float part[NCB];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
            part[cb] = finish_block<ARGMAX>(p, st.m[cb], st.idx[cb], st.col_valid[cb], gb0 + cb, c.doc, c.len, rho, h);
        // this wavefront holds whole queries: lane k adds up the blocks of its k-th query in block
        // order and writes the score
        float s = 0.0f;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
            if (cb / p.bpq == lane)
                s += part[cb];
        const int q = gb0 / p.bpq + lane;
        if (lane < NCB / p.bpq && q < p.n_q)
            p.scores[(int64_t)q * p.ld + c.doc] = s;
    }
}

template <int DT, int NCB, bool ARGMAX>
__global__ void __launch_bounds__(256) fwd_stream_kernel(FwdParams p, OffsetsPtr off)
{
    using TR = Traits<DT>;
    const int lane = threadIdx.x & 63;
    const int rho = lane & 31, h = lane >> 5;
    // p.n_groups (1, 2 or 4) wavefronts of a workgroup share a run of documents, each with its own
    // NCB column blocks (whole queries); they read the same tiles at about the same time, so all
    // but the first read hit in the CU's vector cache.  No LDS and no barrier is involved.
    const int wib = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int group = wib % p.n_groups;
    const int64_t chunk = (int64_t)blockIdx.x * (4 / p.n_groups) + wib / p.n_groups;
    const int gb0 = group * NCB;
    int64_t doc0, doc1;
    chunk_doc_range(p, chunk, doc0, doc1);
    if (doc0 >= doc1)
        return;
    if (group == 0)
        write_empty_docs(p, doc0, doc1, lane, 64);

    StreamState<DT, NCB, ARGMAX> st;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
        load_q_block<DT>(p, gb0 + cb, rho, h, st.qf[cb], st.col_valid[cb]);

    Cursor pc; // prefetch cursor, one tile ahead of the compute cursor
    cursor_init(pc, p, off, doc0, doc1);
    if (!pc.valid)
        return;
    uint4 a0[TR::NU], a1[TR::NU];
    TilePos lp = {pc.start, pc.len, pc.t0}; // where the prefetch reads: pc while it is valid, else the last valid tile
    auto follow = [&]() { // (field by field: a select between whole cursors would put them into memory)
        lp.start = pc.valid ? pc.start : lp.start;
        lp.len = pc.valid ? pc.len : lp.len;
        lp.t0 = pc.valid ? pc.t0 : lp.t0;
    };
    stream_load_tile<DT>(p, lp, rho, h, a0);
    Cursor cc = pc;
    // The prefetch is issued without a condition: past the end of the run the last tile is loaded once more
    // (in bounds, never used).  With `if (pc.valid)` around the loads the compiler has to assume, where the two
    // paths meet, that no load was issued, and makes every MFMA wait for the tile that was only just requested.
    cursor_next_tile(pc, p, off);
    for (;;) {
        follow();
        stream_load_tile<DT>(p, lp, rho, h, a1);
        stream_compute<DT, NCB, ARGMAX>(p, cc, st, a0, gb0, lane, rho, h);
        cc = pc;
        if (!cc.valid)
            break;
        cursor_next_tile(pc, p, off);
        follow();
        stream_load_tile<DT>(p, lp, rho, h, a0);
        stream_compute<DT, NCB, ARGMAX>(p, cc, st, a1, gb0, lane, rho, h);
        cc = pc;
        if (!cc.valid)
            break;
        cursor_next_tile(pc, p, off);
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

// The streaming kernel with whole-line loads (one wavefront per run, rows of up to 256 bytes).  A tile of 32
// consecutive rows is one contiguous piece of memory: the wavefront reads it with NU instructions of 1 KB each
// (lane l the l-th 16 bytes: sixteen or eight lanes per row), with the non-temporal hint, parks it in its own
// piece of LDS (padded rows, no barrier: nobody else touches it) and reads it back in MFMA operand layout.  The
// direct loads of fwd_stream_kernel take 32 bytes of each of 32 lines per instruction and cannot carry the hint;
// a read stream of this shape measures 6.8 TB/s with it and 6.0 without.
template <int DT> constexpr int lin_waves() { return Traits<DT>::NU <= 8 ? 4 : 2; } // wavefronts per workgroup (LDS tiles of 4 to 17 KB)

template <int DT, int NCB, bool ARGMAX>
__global__ void __launch_bounds__(lin_waves<DT>() * 64) fwd_stream_lin_kernel(FwdParams p, OffsetsPtr off)
{
    using TR = Traits<DT>;
    using LT = LdsTile<DT>;
    constexpr int NU = TR::NU;
    constexpr int WPB = lin_waves<DT>();
    constexpr int CPR = TR::ROW_BYTES / 16; // 16-byte chunks (= lanes) per row
    constexpr int RPI = 64 / CPR;           // rows per load instruction
    static_assert(CPR <= 64 && RPI * NU == TILE_ROWS, "NU instructions of 64 lanes cover a tile");
    __shared__ __attribute__((aligned(16))) char lds_all[WPB][LT::BYTES];
    const int lane = threadIdx.x & 63;
    const int rho = lane & 31, h = lane >> 5;
    const int wib = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    char *lds = lds_all[wib];
    const int64_t chunk = (int64_t)blockIdx.x * WPB + wib;
    const int gb0 = 0;
    int64_t doc0, doc1;
    chunk_doc_range(p, chunk, doc0, doc1);
    if (doc0 >= doc1)
        return;
    write_empty_docs(p, doc0, doc1, lane, 64);

    StreamState<DT, NCB, ARGMAX> st;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
        load_q_block<DT>(p, gb0 + cb, rho, h, st.qf[cb], st.col_valid[cb]);

    Cursor pc; // prefetch cursor, one tile ahead of the compute cursor
    cursor_init(pc, p, off, doc0, doc1);
    if (!pc.valid)
        return;
    TilePos lp = {pc.start, pc.len, pc.t0}; // where the prefetch reads: pc while it is valid, else the last valid tile
    auto follow = [&]() {
        lp.start = pc.valid ? pc.start : lp.start;
        lp.len = pc.valid ? pc.len : lp.len;
        lp.t0 = pc.valid ? pc.t0 : lp.t0;
    };
    const int lrow = lane / CPR, lcol = (lane % CPR) * 16;
    const int st_off = lrow * LT::ROW_STRIDE + lcol;
    const int rd_off = rho * LT::ROW_STRIDE + h * 16;
    uint4 g[NU], a[NU];
    auto load_lin = [&]() { // rows past the document's end repeat its last token
#pragma unroll
        for (int i = 0; i < NU; ++i) {
            int row = lp.t0 + i * RPI + lrow;
            if (row > lp.len - 1)
                row = lp.len - 1;
            g[i] = load_stream16(p.D + (lp.start + row) * TR::ROW_BYTES + lcol);
        }
    };
    load_lin();
    Cursor cc = pc;
    cursor_next_tile(pc, p, off);
    for (;;) {
#pragma unroll
        for (int i = 0; i < NU; ++i)
            *reinterpret_cast<uint4 *>(&lds[st_off + i * RPI * LT::ROW_STRIDE]) = g[i];
        follow();
        load_lin(); // the next tile (past the end of the run: the last one again, in bounds, never used)
#pragma unroll
        for (int u = 0; u < NU; ++u)
            a[u] = *reinterpret_cast<const uint4 *>(&lds[rd_off + u * 32]);
        stream_compute<DT, NCB, ARGMAX>(p, cc, st, a, gb0, lane, rho, h);
        cc = pc;
        if (!cc.valid)
            break;
        cursor_next_tile(pc, p, off);
    }
}

// Part `u` (of NU) of folding a result tile into the running max.  The first LAG steps do nothing, so
// that the MFMA chain which produced the tile has left the matrix pipeline before its results are read
// (no wait states); the 16 rows are spread over the remaining steps in even-sized pieces.
template <bool ARGMAX, int NU>
__device__ __forceinline__ void fold_step(const f32x16 &acc, int u, float &m, int &idx, int row_base, int h)
{
    constexpr int LAG = NU >= 4 ? 2 : NU / 2;
    if (u < LAG)
        return;
    const int lo = 2 * (8 * (u - LAG) / (NU - LAG)), hi = 2 * (8 * (u - LAG + 1) / (NU - LAG));
    if (ARGMAX) {
#pragma unroll
        for (int r = lo; r < hi; ++r) {
            bool up = acc[r] > m; // strict: the first occurrence keeps a tie
            m = up ? acc[r] : m;
            idx = up ? row_base + acc_row(r, h) : idx;
        }
    } else {
#pragma unroll
        for (int r = lo; r < hi; r += 2)
            m = fmaxf(fmaxf(m, acc[r]), acc[r + 1]); // one v_max3_f32
    }
}

// The fold with argmax for 16-bit inputs (the running maximum is an fp32 sum of 128 products).  Compare-and-select
// per cell is three VALU operations against half an operation for the plain maximum, which makes the argmax
// variant VALU-bound.  Here every cell's low four mantissa bits are replaced by 15 - r (r = the accumulator
// register, which grows with the row), one operation per cell, and the tile's maximum is again a v_max3 chain:
// among cells that agree in the upper 28 bits the lowest row wins.  Once per tile and column block the tile's
// maximum, with those four bits cleared, is compared (strictly: an earlier tile keeps a tie) with the running one
// and the row is read back from the four bits.  Consequences: the maxima that enter the score are truncated by at
// most 2^-19 relative (the score tolerance is 2e-3); cells closer than that to each other count as tied and the
// earlier one wins (the argmax rule asks for the exact winner only where the margin exceeds 1e-3).  The ordering
// of the patched values is right among non-negative cells only, which is all that matters once the running
// maximum is non-negative (a negative cell cannot beat it); if any lane of the wavefront has a negative tile
// maximum while its running maximum is still negative, that tile is folded again, exactly, with compare-and-select
// (the first tiles of a document whose similarities with a query token are all negative).  The same exact fold
// takes every tile in which a lane's maximum reaches 512 in magnitude: above that, 2^-19 relative would no longer be
// inside the 1e-3 margin below which the argmax rule lets near-ties go either way.  The running winner is
// kept as a key, the tile's first row (a multiple of 32) | the four bits, and turned into a row at the end of the
// document.
template <int NU>
__device__ __forceinline__ void fold_step_packed(const f32x16 &acc, int u, float &tmax, float &m, int &key, int row_base)
{
    constexpr int LAG = NU >= 4 ? 2 : NU / 2;
    if (u < LAG)
        return;
    const int lo = 2 * (8 * (u - LAG) / (NU - LAG)), hi = 2 * (8 * (u - LAG + 1) / (NU - LAG));
    if (u == LAG)
        tmax = neg_inf();
#pragma unroll
    for (int r = lo; r < hi; r += 2) {
        const float p0 = __uint_as_float((__float_as_uint(acc[r]) & 0xfffffff0u) | (uint32_t)(15 - r));
        const float p1 = __uint_as_float((__float_as_uint(acc[r + 1]) & 0xfffffff0u) | (uint32_t)(14 - r));
        tmax = fmaxf(fmaxf(tmax, p0), p1); // one v_max3_f32
    }
    if (u == NU - 1) {
        const uint32_t tb = __float_as_uint(tmax);
        // one unsigned compare finds the tiles that MAY need the exact fold (a negative maximum has the sign bit set);
        // the precise condition is looked at only then
        bool exact = false;
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(tb >= 0x44000000u /* 512.0f */) != 0, 0))
            exact = __builtin_amdgcn_ballot_w64(((int)tb < 0 && m < 0.0f) || fabsf(tmax) >= 512.0f) != 0;
        if (exact) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const bool up = acc[r] > m; // strict: the first occurrence keeps a tie
                m = up ? acc[r] : m;
                key = up ? (row_base | (15 - r)) : key;
            }
        } else {
            const float ts = __uint_as_float(tb & 0xfffffff0u);
            const bool up = ts > m;
            m = up ? ts : m;
            key = up ? (int)((tb & 15u) | (uint32_t)row_base) : key;
        }
    }
}

// The document-local row behind a key of fold_step_packed in lane half h
__device__ __forceinline__ int packed_key_row(int key, int h)
{
    const int r = 15 - (key & 15);
    return (key & ~31) + h * 4 + (((r & 12) << 1) | (r & 3));
}

// The main loop is software-pipelined by hand and pinned with scheduling barriers, one MFMA
// (16-bit inputs) per step:
//   * the MFMA chain of column block cb runs while the previous block's result tile is folded
//     into the running max, one slice of the fold per step, so the VALU work sits under MFMAs
//     whose results it does not need;
//   * during the first chain of a tile the wavefront also reads the NEXT tile's A operands from
//     LDS into a second register set, writes the tile after that from registers to LDS and
//     issues the global loads of the tile after that, so no memory latency is exposed between
//     tiles: three LDS buffers rotate (being computed / prefetched into registers / being
//     written), one barrier per tile.  (The fp32 and the argmax variants have no registers
//     left for the second operand set; there each operand chunk is replaced by the next tile's
//     right after its last MFMA, during the last chain of the tile.)
//   * with one or two column blocks per wavefront a tile takes too little time for a load issued
//     one tile ahead to have arrived: PFD tiles are then in flight in a ring of registers.
template <int DT, int W, int NCB, bool ARGMAX, int PFD = 1>
__global__ void __launch_bounds__(W * 64, (Traits<DT>::NU <= 8 || W == 8) ? 2 : 1) fwd_tile_kernel(FwdParams p, OffsetsPtr off)
{
    using TR = Traits<DT>;
    using LT = LdsTile<DT>;
    constexpr int NU = TR::NU;
    constexpr int NT = W * 64;
    constexpr int CPT = (LT::CHUNKS + NT - 1) / NT; // 16-byte chunks each thread moves per tile
    static_assert(LT::CHUNKS % NT == 0 || LT::CHUNKS < NT, "tile must split evenly over the workgroup");
    const bool copies = LT::CHUNKS >= NT || (int)threadIdx.x < LT::CHUNKS; // narrow rows: fewer chunks than threads
    constexpr int CPR = TR::ROW_BYTES / 16; // chunks per row
    constexpr int GROUP_BLOCKS = W * NCB;
    constexpr bool PF = NU <= 8 && !ARGMAX && !(W <= 2 && NCB == 4); // operands of the next tile prefetched into registers (no room for them beside four chunks in flight per thread)

    __shared__ __attribute__((aligned(16))) char lds_tile[3 * LT::BYTES];
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

    int64_t doc0_, doc1_;
    chunk_doc_range(p, chunk, doc0_, doc1_);
    if (doc0_ >= doc1_)
        return;
    const int doc0 = (int)doc0_, doc1 = (int)doc1_;
    if (group == 0)
        write_empty_docs(p, doc0, doc1, tid, NT);

    // this thread's share of a tile copy: chunk ch = tid + i * NT -> (row, 16-byte column)
    int cp_row[CPT], cp_goff[CPT], cp_loff[CPT];
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        int ch = tid + i * NT;
        cp_row[i] = ch / CPR;
        cp_goff[i] = (ch % CPR) * 16;
        cp_loff[i] = (ch / CPR) * LT::ROW_STRIDE + (ch % CPR) * 16;
    }
    const int a_off = rho * LT::ROW_STRIDE + h * 16;

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
        // a query of one block needs no combination across blocks: its lane writes the score
        const bool direct = p.bpq == 1;

        uint4 qf[NCB][NU];
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

        const bool wave_active = w * NCB < nb;
        TileIter li, ci; // load iterator (three tiles ahead of the compute iterator at steady state)
        it_init(li, p, off, doc0, doc1);
        ci = li;
        if (!it_valid(ci))
            break;

        // tiles in flight from HBM: ring slot 0 is the oldest (next to be stored to LDS), bit s of g_mask says that slot s holds a tile
        constexpr bool NAMED = PFD * CPT <= 8;
        uint4 g0, g1, g2, g3, g4, g5, g6, g7;
        uint4 g_arr[NAMED ? 1 : PFD][NAMED ? 1 : CPT]; // workgroups of one wavefront and wide rows: more than eight chunks
        auto g = [&](auto slot, auto i) -> uint4 & {
            if constexpr (NAMED)
                return reg_at<decltype(slot)::value * CPT + decltype(i)::value>(g0, g1, g2, g3, g4, g5, g6, g7);
            else
                return g_arr[decltype(slot)::value][decltype(i)::value];
        };
        constexpr std::integral_constant<int, 0> OLDEST{};
        constexpr std::integral_constant<int, PFD - 1> NEWEST{};
        unsigned g_mask = 0;
        // HBM -> registers (newest ring slot) for the next tile of the stream
        auto gload = [&]() {
            g_mask &= ~(1u << (PFD - 1));
            if (!it_valid(li))
                return;
            g_mask |= 1u << (PFD - 1);
            if (!copies) {
                it_next(li, p, off);
                return;
            }
            int last_row = li.len - li.t0 - 1; // rows past the document re-read its last token
            const char *base = p.D + (int64_t)li.row0 * TR::ROW_BYTES;
            static_for<CPT>([&](auto i) {
                int row = cp_row[i] < last_row ? cp_row[i] : last_row;
                g(NEWEST, i) = *reinterpret_cast<const uint4 *>(base + row * TR::ROW_BYTES + cp_goff[i]);
            });
            it_next(li, p, off);
        };
        // oldest ring slot -> LDS
        auto lstore = [&](int buf_off) {
            if (!(g_mask & 1u) || !copies)
                return;
            static_for<CPT>([&](auto i) { *reinterpret_cast<uint4 *>(&lds_tile[buf_off + cp_loff[i]]) = g(OLDEST, i); });
        };
        auto rotate = [&]() {
            static_for<PFD - 1>([&](auto slot) {
                static_for<CPT>([&](auto i) { g(slot, i) = g(std::integral_constant<int, decltype(slot)::value + 1>{}, i); });
            });
            g_mask >>= 1;
        };

        // LDS buffers (byte offsets): o_cur holds the tile being computed (already in registers),
        // o_nxt the next one (read into registers during this tile), o_wr receives the one after
        int o_cur = 0, o_nxt = LT::BYTES, o_wr = 2 * LT::BYTES;
        // tiles 0 and 1 go straight to LDS, the next PFD tiles into the ring
#pragma unroll
        for (int s = 0; s < PFD + 2; ++s) {
            rotate();
            gload();
            if (s < 2) { // the tile just loaded sits in the newest slot: pull it to the front and store it
#pragma unroll
                for (int r = 0; r + 1 < PFD; ++r)
                    rotate();
                lstore(s == 0 ? o_cur : o_nxt);
            }
        }
        __syncthreads();
        // a wavefront with a single column block uses every operand chunk once: a ring of four
        // registers, read three steps ahead, replaces the full operand set (the argmax variant with one block of 256-byte rows per wavefront)
        constexpr bool RING = !PF && NCB == 1 && NU >= 8;
        // no registers for a second operand set (fp32, argmax): each chunk is replaced by the next tile's
        // right after its last MFMA, during the last chain
        constexpr bool INPLACE = !PF && !RING;
        uint4 a0[NU], a1[PF ? NU : 1]; // (a0 stays unused when the operand ring is in use)
        if (PF || INPLACE) {
#pragma unroll
            for (int u = 0; u < NU; ++u)
                a0[u] = *reinterpret_cast<const uint4 *>(&lds_tile[o_cur + a_off + u * 32]);
        }
        int par = 0;

        // one tile: operands in `ac`; the next tile's operands are read into `an` on the way
        auto stage = [&](uint4(&ac)[NU], uint4(&an)[PF ? NU : 1]) {
            const int fin_doc = (ci.t0 + TILE_ROWS >= ci.len) ? ci.doc : -1; // last tile of its document?
            uint4 ring[4];
            if (RING) {
#pragma unroll
                for (int u = 0; u < 3; ++u)
                    ring[u] = *reinterpret_cast<const uint4 *>(&lds_tile[o_cur + a_off + u * 32]);
            }
            __builtin_amdgcn_sched_barrier(0);
            f32x16 acc[NCB];
            float tmax[NCB]; // the tile's maximum per column block (argmax with 16-bit inputs only)
            auto fold = [&](int cbx, int u) {
                if constexpr (ARGMAX && TR::DT != MAXSIM_F32)
                    fold_step_packed<NU>(acc[cbx], u, tmax[cbx], m[cbx], idx[cbx], ci.t0);
                else
                    fold_step<ARGMAX, NU>(acc[cbx], u, m[cbx], idx[cbx], ci.t0, h);
            };
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    acc[cb][r] = 0.0f;
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    if (RING) {
                        if (u + 3 < NU)
                            ring[(u + 3) & 3] = *reinterpret_cast<const uint4 *>(&lds_tile[o_cur + a_off + (u + 3) * 32]);
                        TR::mma(ring[u & 3], qf[cb][u], acc[cb]);
                    } else {
                        TR::mma(ac[u], qf[cb][u], acc[cb]);
                        if (INPLACE && cb == NCB - 1)
                            ac[u] = *reinterpret_cast<const uint4 *>(&lds_tile[o_nxt + a_off + u * 32]);
                    }
                    if (cb == 0) {
                        if (PF)
                            an[u] = *reinterpret_cast<const uint4 *>(&lds_tile[o_nxt + a_off + u * 32]);
                        if (u == NU - 1) {
                            lstore(o_wr);
                            rotate();
                            gload();
                        }
                    } else {
                        fold(cb - 1, u);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int u = 0; u < NU; ++u)
                fold(NCB - 1, u);

            if (fin_doc >= 0) {
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) {
                    int lb = w * NCB + cb;
                    int row = idx[cb];
                    if constexpr (ARGMAX && TR::DT != MAXSIM_F32)
                        row = packed_key_row(row, h);
                    float sum = finish_block<ARGMAX>(p, m[cb], row, col_valid[cb], gb0 + lb, ci.doc, ci.len, rho, h);
                    if (lane == 0) {
                        if (direct) {
                            if (lb < nb)
                                p.scores[(int64_t)(gb0 + lb) * p.ld + ci.doc] = sum;
                        } else {
                            lds_part[par][lb] = sum;
                        }
                    }
                    m[cb] = neg_inf(); // the next document starts from nothing
                    idx[cb] = 0;
                }
            }
            it_next(ci, p, off);
            __syncthreads();
            if (fin_doc >= 0) {
                if (!direct && tid < nq) { // thread t adds up the blocks of its query in block order
                    float sum = 0.0f;
                    int first_blk = (p.n_pass == 1) ? tid * p.bpq : 0;
                    int cnt = (p.n_pass == 1) ? p.bpq : nb;
                    for (int i = 0; i < cnt; ++i)
                        sum += lds_part[par][first_blk + i];
                    float *dst = p.scores + (int64_t)(q_first + tid) * p.ld + fin_doc;
                    *dst = accumulate ? *dst + sum : sum;
                }
                par ^= 1;
            }
            int t = o_cur;
            o_cur = o_nxt;
            o_nxt = o_wr;
            o_wr = t;
        };

        if (!wave_active) {
            // no column block in this pass: the wavefront only helps moving tiles (same barriers as the others)
            while (it_valid(ci)) {
                lstore(o_wr);
                rotate();
                gload();
                it_next(ci, p, off);
                __syncthreads();
                int t = o_cur;
                o_cur = o_nxt;
                o_nxt = o_wr;
                o_wr = t;
            }
        } else if constexpr (PF) {
            for (;;) {
                stage(a0, a1);
                if (!it_valid(ci))
                    break;
                stage(a1, a0);
                if (!it_valid(ci))
                    break;
            }
        } else {
            while (it_valid(ci))
                stage(a0, a1);
        }
        __syncthreads(); // LDS is reused by the next pass
    }
}

// ---------------------------------------------------------------------------------------
// packed-window kernel: the tile kernel for ragged corpora and queries of one column block
// ---------------------------------------------------------------------------------------
//
// With documents of 64-300 tokens a sixth of the 32-row tiles is the ragged end of a document, and
// half of such a tile is padding.  Here a 32-row window may hold the last rows of document A and, from
// the next multiple of 4 rows on, the first rows of the next (non-empty) document B; it is cut short
// only where a third document would begin.  The MFMAs are the same.  The boundary sits on a multiple of
// 4 rows because a lane of the 32x32 result keeps rows 8q + 4h .. 8q + 4h + 3 (h = its lane half) in
// accumulator registers 4q .. 4q+3: a group of four registers then belongs to one document, and a window
// with a boundary folds the maximum of each group into A's or B's maximum by one compare per group (no
// per-row masks).  Such a window finishes A and carries B's maximum on.  Everything else (rotating LDS
// buffers, pinned pipeline) is fwd_tile_kernel's.  Queries have one column block here (L_q <= 32), so a
// wavefront's lane writes a score directly and no partial sums are combined.

struct WinIter {
    int doc, doc_end; // document that owns the window's first row; end of the run
    int row0;         // packed row of the window's first token
    int rem;          // tokens of `doc` from row0 on (> 0 while the iterator is valid)
    int end;          // packed row one past `doc`
    int nxt;          // offsets[doc + 2], unclamped, fetched while `doc` is walked
};

struct Window {
    int n_a;   // rows of document A = it.doc
    int pa;    // window row at which B starts: n_a rounded up to a multiple of 4 (rows n_a .. pa-1 repeat A's last)
    int n_b;   // rows of document B (0: no boundary inside the window)
    int doc_b; // next non-empty document (doc_end if there is none); only known when A ends in the window
    int len_b, end_b;
    bool fin_a, fin_b; // A / B end inside this window
};

__device__ __forceinline__ bool win_valid(const WinIter &it) { return it.doc < it.doc_end; }

// offsets[i] (i <= b), or i * l_d for a uniform corpus (UNI: a compile-time choice, so that the ragged case keeps
// its branch-free scalar loads)
template <bool UNI> __device__ __forceinline__ int win_offset(OffsetsPtr off, const FwdParams &p, int i)
{
    if constexpr (UNI)
        return (i < p.b ? i : (int)p.b) * p.l_d;
    else
        return it_offset(off, p, i);
}

// First non-empty document after it.doc within the run: d (doc_end if none) and its end e.  Offsets are
// forced into [previous end, T], so malformed offsets give wrong scores but no address outside D.
// The common case costs no memory access (it.nxt was fetched ahead); only empty documents take the loop,
// whose loads are made scalar values by hand so that the state stays in scalar registers.
template <bool UNI>
__device__ __forceinline__ void win_find_next(const WinIter &it, const FwdParams &p, OffsetsPtr off, int &d, int &e)
{
    const int t_all = (int)p.total_tokens;
    d = it.doc + 1;
    e = min(max(it.nxt, it.end), t_all); // offsets[d + 1]
    if (!UNI && d < it.doc_end && e == it.end) {
        do {
            ++d;
            if (d >= it.doc_end)
                break;
            const int raw = __builtin_amdgcn_readfirstlane(p.offsets[d + 1]);
            e = min(max(raw, it.end), t_all);
        } while (e == it.end);
    }
    if (d > it.doc_end)
        d = it.doc_end;
}

// Makes d (with end e, `used` of its rows already consumed) the current document; no branch around the
// read of the offset after next, so that it stays a scalar load
template <bool UNI>
__device__ __forceinline__ void win_enter(WinIter &it, const FwdParams &p, OffsetsPtr off, int d, int e, int used)
{
    const bool ok = d < it.doc_end;
    it.doc = d;
    it.nxt = win_offset<UNI>(off, p, d + 2);
    it.rem = ok ? e - it.end - used : 0;
    it.end = ok ? e : it.end;
}

template <bool UNI>
__device__ __forceinline__ void win_init(WinIter &it, const FwdParams &p, OffsetsPtr off, int doc0, int doc1)
{
    it.doc = doc0 - 1; // a virtual empty document before the run: its successor is the first real one
    it.doc_end = doc1;
    it.rem = 0;
    it.end = min(max(win_offset<UNI>(off, p, doc0), 0), (int)p.total_tokens);
    it.row0 = it.end;
    it.nxt = win_offset<UNI>(off, p, doc0 + 1);
    int d, e;
    win_find_next<UNI>(it, p, off, d, e);
    win_enter<UNI>(it, p, off, d, e, 0);
}

template <bool UNI>
__device__ __forceinline__ Window win_describe(const WinIter &it, const FwdParams &p, OffsetsPtr off)
{
    Window w;
    w.n_a = min(TILE_ROWS, it.rem);
    w.fin_a = w.n_a == it.rem;
    w.pa = (w.n_a + 3) & ~3;
    w.n_b = 0;
    w.doc_b = it.doc_end;
    w.len_b = 0;
    w.end_b = it.end;
    w.fin_b = false;
    if (w.fin_a) {
        win_find_next<UNI>(it, p, off, w.doc_b, w.end_b);
        if (w.doc_b < it.doc_end) {
            w.len_b = w.end_b - it.end;
            w.n_b = min(w.len_b, TILE_ROWS - w.pa);
            w.fin_b = w.n_b > 0 && w.n_b == w.len_b;
        }
    }
    return w;
}

template <bool UNI>
__device__ __forceinline__ void win_advance(WinIter &it, const Window &w, const FwdParams &p, OffsetsPtr off)
{
    it.row0 += w.n_a + w.n_b;
    if (!w.fin_a) {
        it.rem -= TILE_ROWS;
        return;
    }
    win_enter<UNI>(it, p, off, w.doc_b, w.end_b, w.n_b);
    if (win_valid(it) && it.rem == 0) { // B lay inside the window whole: on to the document after it
        int d, e;
        win_find_next<UNI>(it, p, off, d, e);
        win_enter<UNI>(it, p, off, d, e, 0);
    }
}

// NCB: column blocks (queries) per wavefront, 2 to 4; W: wavefronts per workgroup (8: 16 to 32 queries; 4 and 2 give
//      fewer queries the same 3 or 4 blocks per wavefront, i.e. as many MFMAs per window and barrier)
// UNI: uniform corpus (documents of l_d tokens, no offsets array)
template <int DT, int NCB, bool UNI, int W = 8>
__global__ void __launch_bounds__(W * 64, 2) fwd_pack_kernel(FwdParams p, OffsetsPtr off)
{
    using TR = Traits<DT>;
    using LT = LdsTile<DT>;
    constexpr int NU = TR::NU;
    constexpr int NT = W * 64;
    static_assert(NU <= 8, "the operand prefetch needs rows of at most 256 bytes");
    constexpr int CPT = (LT::CHUNKS + NT - 1) / NT;
    static_assert(LT::CHUNKS % NT == 0 || LT::CHUNKS < NT, "tile must split evenly over the workgroup");
    const bool copies = LT::CHUNKS >= NT || (int)threadIdx.x < LT::CHUNKS;
    constexpr int CPR = TR::ROW_BYTES / 16;
    constexpr int GROUP_BLOCKS = W * NCB;

    __shared__ __attribute__((aligned(16))) char lds_tile[3 * LT::BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int rho = lane & 31, h = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int n_wg = gridDim.x;
    int v = blockIdx.x;
    if ((n_wg & 7) == 0)
        v = (blockIdx.x & 7) * (n_wg >> 3) + (blockIdx.x >> 3);
    const int group = v % p.n_groups;
    const int chunk = v / p.n_groups;

    int64_t doc0_, doc1_;
    chunk_doc_range(p, chunk, doc0_, doc1_);
    if (doc0_ >= doc1_)
        return;
    const int doc0 = (int)doc0_, doc1 = (int)doc1_;
    if (group == 0)
        write_empty_docs(p, doc0, doc1, tid, NT);

    // this thread's share of a tile copy: chunk ch = tid + i * NT -> (row, 16-byte column); recomputed where it
    // is used (a handful of shifts) rather than kept in registers, which are all taken
    auto cp_row = [&](int i) { return (tid + i * NT) / CPR; };
    auto cp_goff = [&](int i) { return ((tid + i * NT) % CPR) * 16; };
    auto cp_loff = [&](int i) { return ((tid + i * NT) / CPR) * LT::ROW_STRIDE + ((tid + i * NT) % CPR) * 16; };
    const int a_off = rho * LT::ROW_STRIDE + h * 16;

    // one column block = one query: blocks [gb0, gb0 + nb) of this group
    const int gb0 = group * GROUP_BLOCKS;
    const int nb = min(GROUP_BLOCKS, p.n_q - gb0);
    uint4 qf[NCB][NU];
    bool col_valid[NCB];
    float m[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
        int lb = w * NCB + cb;
        load_q_block<DT>(p, gb0 + lb, rho, h, qf[cb], col_valid[cb]);
        col_valid[cb] = col_valid[cb] && lb < nb;
        m[cb] = neg_inf();
    }
    const bool wave_active = w * NCB < nb;

    // One iterator walks the windows, three ahead of the MFMAs (at load time).  What the stage needs of a window
    // later -- is there one, does it hold a boundary and where, which documents end in it -- travels in three scalar
    // words through a ring of three descriptors, instead of a second iterator that would derive it all again.
    struct WinDesc {
        int flags; // bit 0: the window exists; 1: it holds a boundary; 2: A ends in it; 3: B ends in it; bits 8..: pa
        int doc_a, doc_b;
    };
    WinIter li;
    win_init<UNI>(li, p, off, doc0, doc1);
    if (!win_valid(li))
        return;

    static_assert(CPT <= 4, "a thread moves at most four chunks per window");
    uint4 g0, g1, g2, g3, g4, g5, g6, g7; // the window on its way from HBM (see reg_at); four at most are used
    auto g = [&](auto i) -> uint4 & { return reg_at<decltype(i)::value>(g0, g1, g2, g3, g4, g5, g6, g7); };
    auto gload = [&]() -> WinDesc { // the next window of the stream -> registers; returns its descriptor
        WinDesc d = {0, 0, 0};
        if (!win_valid(li))
            return d;
        const Window lw = win_describe<UNI>(li, p, off);
        d.flags = 1 | (lw.n_b > 0 ? 2 : 0) | (lw.fin_a ? 4 : 0) | (lw.fin_b ? 8 : 0) | (lw.pa << 8);
        d.doc_a = li.doc;
        d.doc_b = lw.doc_b;
        if (copies) {
            // window row i holds A's row min(i, n_a - 1) below pa and B's row min(i - pa, n_b - 1) from pa on
            // (without a B that is A's last row again); A and B are neighbours in the packed corpus
            const char *base = p.D + (int64_t)li.row0 * TR::ROW_BYTES;
            static_for<CPT>([&](auto i) {
                const int wr = cp_row(i);
                const int row = wr < lw.pa ? min(wr, lw.n_a - 1) : lw.n_a + min(wr - lw.pa, lw.n_b - 1);
                g(i) = *reinterpret_cast<const uint4 *>(base + row * TR::ROW_BYTES + cp_goff(i));
            });
        }
        win_advance<UNI>(li, lw, p, off);
        return d;
    };
    WinDesc d_cur, d_n1, d_n2; // the windows being computed, read from LDS next, and on their way from HBM
    auto lstore = [&](int buf_off) { // the window in the registers (d_n2) -> LDS
        if (!(d_n2.flags & 1) || !copies)
            return;
        static_for<CPT>([&](auto i) { *reinterpret_cast<uint4 *>(&lds_tile[buf_off + cp_loff(i)]) = g(i); });
    };

    int o_cur = 0, o_nxt = LT::BYTES, o_wr = 2 * LT::BYTES;
    d_n2 = gload();
    lstore(o_cur);
    d_cur = d_n2;
    d_n2 = gload();
    lstore(o_nxt);
    d_n1 = d_n2;
    d_n2 = gload();
    __syncthreads();
    // One operand set: during the LAST chain of a window every operand chunk is replaced, right after the
    // MFMA that used it last, by the next window's (the second set of fwd_tile_kernel would not fit beside
    // the two maxima of a boundary window).
    uint4 ac[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u)
        ac[u] = *reinterpret_cast<const uint4 *>(&lds_tile[o_cur + a_off + u * 32]);

    // BND: the window holds rows of two documents
    auto stage = [&](auto bnd_tag) {
        constexpr bool BND = decltype(bnd_tag)::value;
        const int cw_pa = d_cur.flags >> 8;
        const bool cw_fin_a = (d_cur.flags & 4) != 0, cw_fin_b = (d_cur.flags & 8) != 0;
        WinDesc d_new = {0, 0, 0};
        constexpr int LAG = NU >= 4 ? 2 : NU / 2;
        float mb[NCB];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
            mb[cb] = neg_inf();
        // part u (of NU) of folding a result tile; nothing in the first LAG steps (see fold_step)
        auto fold = [&](const f32x16 &acc, int u, float &ma, float &mbv) {
            if (u < LAG)
                return;
            if (BND) { // register groups 4q .. 4q+3 (rows 8q + 4h .. 8q + 4h + 3) go to A below the boundary, to B from it on
                const int q0 = 4 * (u - LAG) / (NU - LAG), q1 = 4 * (u - LAG + 1) / (NU - LAG);
#pragma unroll
                for (int q = q0; q < q1; ++q) {
                    const float qm = fmaxf(fmaxf(fmaxf(acc[4 * q], acc[4 * q + 1]), acc[4 * q + 2]), acc[4 * q + 3]);
                    const bool in_a = 8 * q + 4 * h < cw_pa;
                    ma = fmaxf(ma, in_a ? qm : neg_inf());
                    mbv = fmaxf(mbv, in_a ? neg_inf() : qm);
                }
            } else {
                const int lo = 2 * (8 * (u - LAG) / (NU - LAG)), hi = 2 * (8 * (u - LAG + 1) / (NU - LAG));
#pragma unroll
                for (int r = lo; r < hi; r += 2)
                    ma = fmaxf(fmaxf(ma, acc[r]), acc[r + 1]);
            }
        };
        __builtin_amdgcn_sched_barrier(0);
        f32x16 acc[NCB];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[cb][r] = 0.0f;
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                TR::mma(ac[u], qf[cb][u], acc[cb]);
                if (cb == NCB - 1)
                    ac[u] = *reinterpret_cast<const uint4 *>(&lds_tile[o_nxt + a_off + u * 32]);
                if (cb == 0) {
                    if (u == NU - 1) {
                        lstore(o_wr);
                        d_new = gload();
                    }
                } else {
                    fold(acc[cb - 1], u, m[cb - 1], mb[cb - 1]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int u = 0; u < NU; ++u)
            fold(acc[NCB - 1], u, m[NCB - 1], mb[NCB - 1]);

        if (cw_fin_a) {
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                int lb = w * NCB + cb;
                float sum = finish_block<false>(p, m[cb], 0, col_valid[cb], gb0 + lb, d_cur.doc_a, 0, rho, h);
                if (lane == 0 && lb < nb)
                    p.scores[(int64_t)(gb0 + lb) * p.ld + d_cur.doc_a] = sum;
                m[cb] = BND ? mb[cb] : neg_inf();
            }
            if (BND && cw_fin_b) {
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) {
                    int lb = w * NCB + cb;
                    float sum = finish_block<false>(p, m[cb], 0, col_valid[cb], gb0 + lb, d_cur.doc_b, 0, rho, h);
                    if (lane == 0 && lb < nb)
                        p.scores[(int64_t)(gb0 + lb) * p.ld + d_cur.doc_b] = sum;
                    m[cb] = neg_inf();
                }
            }
        }
        __syncthreads();
        int t = o_cur;
        o_cur = o_nxt;
        o_nxt = o_wr;
        o_wr = t;
        d_cur = d_n1;
        d_n1 = d_n2;
        d_n2 = d_new;
    };

    if (!wave_active) {
        // fewer than 32 queries in this group: the wavefront only helps moving tiles (same barriers as the others)
        while (d_cur.flags & 1) {
            lstore(o_wr);
            const WinDesc d_new = gload();
            __syncthreads();
            int t = o_cur;
            o_cur = o_nxt;
            o_nxt = o_wr;
            o_wr = t;
            d_cur = d_n1;
            d_n1 = d_n2;
            d_n2 = d_new;
        }
    } else {
        // runs of plain windows, each ended by one boundary window
        for (;;) {
            while (!(d_cur.flags & 2)) {
                stage(std::false_type{});
                if (!(d_cur.flags & 1))
                    return;
            }
            stage(std::true_type{});
            if (!(d_cur.flags & 1))
                return;
        }
    }
}

// ---------------------------------------------------------------------------------------
// host-side launchers (called from the C ABI)
// ---------------------------------------------------------------------------------------

template <int DT, int NCB, bool ARGMAX>
static hipError_t launch_stream(const FwdParams &p, int grid, hipStream_t stream)
{
    if (p.n_groups == 1) { // one wavefront per run: whole-line loads through LDS
        constexpr int WPB = lin_waves<DT>();
        const int grid_lin = (p.n_chunks + WPB - 1) / WPB;
        hipLaunchKernelGGL((fwd_stream_lin_kernel<DT, NCB, ARGMAX>), dim3(grid_lin), dim3(WPB * 64), 0, stream, p, p.offsets);
        return hipGetLastError();
    }
    if constexpr (Traits<DT>::NU <= 8) { // narrow rows: more than four column blocks go to the tile kernel
        return hipErrorInvalidValue;
    } else {
        hipLaunchKernelGGL((fwd_stream_kernel<DT, NCB, ARGMAX>), dim3(grid), dim3(256), 0, stream, p, p.offsets);
        return hipGetLastError();
    }
}

template <int DT, int W, int NCB, bool ARGMAX, int PFD = 1>
static hipError_t launch_tile(const FwdParams &p, int grid, hipStream_t stream)
{
    hipLaunchKernelGGL((fwd_tile_kernel<DT, W, NCB, ARGMAX, PFD>), dim3(grid), dim3(W * 64), 0, stream, p, p.offsets);
    return hipGetLastError();
}

template <int DT, int NCB, int W = 8>
static hipError_t launch_pack(const FwdParams &p, int grid, hipStream_t stream)
{
    if (p.offsets)
        hipLaunchKernelGGL((fwd_pack_kernel<DT, NCB, false, W>), dim3(grid), dim3(W * 64), 0, stream, p, p.offsets);
    else
        hipLaunchKernelGGL((fwd_pack_kernel<DT, NCB, true, W>), dim3(grid), dim3(W * 64), 0, stream, p, p.offsets);
    return hipGetLastError();
}

template <int DT, bool ARGMAX>
static hipError_t dispatch_stream(const FwdParams &p, int ncb, int grid, hipStream_t s)
{
    constexpr int NU = Traits<DT>::NU;
    if constexpr (NU <= 8) {
        switch (ncb) {
        case 1: return launch_stream<DT, 1, ARGMAX>(p, grid, s);
        case 2: return launch_stream<DT, 2, ARGMAX>(p, grid, s);
        case 3: return launch_stream<DT, 3, ARGMAX>(p, grid, s);
        default: return launch_stream<DT, 4, ARGMAX>(p, grid, s);
        }
    } else {
        return ncb == 1 ? launch_stream<DT, 1, ARGMAX>(p, grid, s) : launch_stream<DT, 2, ARGMAX>(p, grid, s);
    }
}

template <int DT, bool ARGMAX>
static hipError_t dispatch_tile(const FwdParams &p, int w, int grid, hipStream_t s)
{
    constexpr int NU = Traits<DT>::NU;
    constexpr int NCB = NU <= 8 ? 4 : 32 / NU; // query fragments fill 128 registers
    if constexpr (NCB == 4) { // few column blocks: eight wavefronts with one or two blocks each
        if (w == 81)
            return launch_tile<DT, 8, 1, ARGMAX, 6>(p, grid, s);
        if (w == 82)
            return launch_tile<DT, 8, 2, ARGMAX, 3>(p, grid, s);
        if (w == 42)
            return launch_tile<DT, 4, 2, ARGMAX, 4>(p, grid, s);
        if constexpr (!ARGMAX) {
            if (w == 93) // ragged corpus, queries of one block: windows over the packed rows; 24 or 32 queries per workgroup
                return launch_pack<DT, 3>(p, grid, s);
            if (w == 94)
                return launch_pack<DT, 4>(p, grid, s);
            if (w == 943)
                return launch_pack<DT, 3, 4>(p, grid, s);
            if (w == 944)
                return launch_pack<DT, 4, 4>(p, grid, s);
            if (w == 923)
                return launch_pack<DT, 3, 2>(p, grid, s);
            if (w == 924)
                return launch_pack<DT, 4, 2>(p, grid, s);
        }
    }
    switch (w) {
    case 1: return launch_tile<DT, 1, NCB, ARGMAX>(p, grid, s);
    case 2: return launch_tile<DT, 2, NCB, ARGMAX>(p, grid, s);
    case 4: return launch_tile<DT, 4, NCB, ARGMAX>(p, grid, s);
    default: return launch_tile<DT, 8, NCB, ARGMAX>(p, grid, s);
    }
}


template <int F>
static hipError_t run_format(const FwdParams &p, bool argmax, bool tile, int x, int grid, hipStream_t s)
{
    if (tile)
        return argmax ? dispatch_tile<F, true>(p, x, grid, s) : dispatch_tile<F, false>(p, x, grid, s);
    return argmax ? dispatch_stream<F, true>(p, x, grid, s) : dispatch_stream<F, false>(p, x, grid, s);
}

// All widths of one element type: nu = row bytes / 32.  `tile` picks the kernel, x is its shape
// parameter (wavefronts per workgroup for the tile kernel, column blocks per wavefront for the
// streaming kernel).
template <int DTYPE>
static hipError_t run_dtype(const FwdParams &p, int nu, bool argmax, bool tile, int x, int grid, hipStream_t s)
{
    switch (nu) {
    case 4: return run_format<fmt(DTYPE, 4)>(p, argmax, tile, x, grid, s);
    case 8: return run_format<fmt(DTYPE, 8)>(p, argmax, tile, x, grid, s);
    case 16: return run_format<fmt(DTYPE, 16)>(p, argmax, tile, x, grid, s);
    default: return hipErrorNotSupported;
    }
}

} // namespace
} // namespace maxsim
