// Fused MaxSim forward for any embedding width (the "split-d" forward of the paper's appendix on fat
// embeddings: an inner loop over slabs of the embedding dimension, accumulated in fp32, with the
// reduction of Alg. 1 unchanged), for gfx950.
//
// The register-stationary kernels of forward_impl.h hold a query block's fragments for the whole
// embedding width, which pays up to rows of 512 bytes.  Here neither operand is stationary: a workgroup
// of eight wavefronts (two per SIMD) computes the similarities of a MACRO TILE of 128 document tokens x
// 512 query tokens, every wavefront a 128 x 64 piece of it in eight 32x32 accumulators (128 registers),
// while both operands stream through LDS in slabs of 64 bytes per row:
//
//   HBM/L2 -> registers (two slabs in flight) -> LDS (three rotating slabs, XOR-swizzled 64-byte rows,
//   no padding) -> MFMA operand registers (read one half slab ahead of the MFMAs that use them).
//
// One barrier per slab; per slab a wavefront issues 16 MFMAs (16-bit inputs), 12 LDS reads, 5 LDS
// writes and 5 global loads, all placed between the MFMAs by hand.  When the last slab of a macro tile
// is done the eight tiles are folded into the running max (and argmax) of the wavefront's 64 query
// tokens exactly as in the other kernels (documents on the MFMA rows, so the max is in-lane), and at the
// end of a document the block sums are combined in block order.  A macro tile never spans two documents
// (rows past the end re-read the document's last token).
//
// The same kernel scores int8 codes (Alg. 4 at embedding widths other than 128): element "type" SD_I8 runs the
// contraction with v_mfma_i32_32x32x32_i8 on the same 16-byte chunks into exact int32 accumulators (kept in the
// float accumulator registers bit for bit), and the fold after the last slab applies the document token's scale
// with a single rounding, v = fl32(n * d_scale[j]); at the end of a document r_i = fl32(q_scale[i] * max) and the
// sum over the query's tokens is carried in fp64 and rounded once: the oracle's bits.
#include "forward_impl.h"

#include <type_traits>

namespace maxsim {
namespace {

constexpr int SD_W = 8;                                  // wavefronts per workgroup
constexpr int SD_NCB = 2;                                // column blocks per wavefront
constexpr int SD_MT = 4;                                 // 32-token document tiles per macro tile
constexpr int SD_ROWS_A = SD_MT * TILE_ROWS;             // document tokens per macro tile
constexpr int SD_GROUP_BLOCKS = SD_W * SD_NCB;           // column blocks per workgroup
constexpr int SD_ROWS_B = SD_GROUP_BLOCKS * BLOCK_COLS;  // query tokens per workgroup
constexpr int SD_SLAB = 64;                              // bytes of every row in one slab (4 chunks of 16)
constexpr int SD_BUF = (SD_ROWS_A + SD_ROWS_B) * SD_SLAB; // one slab of both operands in LDS
constexpr int SD_CP_ROWS = SD_W * 64 / 4;                // rows covered by one copy instruction of the workgroup (4 chunks per row)
constexpr int SD_NG = (SD_ROWS_A + SD_ROWS_B) / SD_CP_ROWS; // 16-byte chunks a thread moves per slab
constexpr int SD_NGA = SD_ROWS_A / SD_CP_ROWS;            // ... of which document rows
constexpr int SD_LDS = 3 * SD_BUF + 2 * SD_GROUP_BLOCKS * (int)sizeof(double); // + per-block sums of two documents in turn
constexpr int SD_I8 = 3;                                 // element type code of int8 codes (beside maxsim_dtype's 0, 1, 2)
// int8 queries of 17-32 blocks take two passes over a chunk; the fp64 sum of a document's first pass waits in LDS
// for the second (a float in `scores` would round twice): one slot per non-empty document of the chunk
constexpr int SD_I8_CARRY_DOCS = 4096;
// the scales of a macro tile's 128 document tokens travel with its first slab into one of four LDS buffers (a tile's
// slab is stored up to two tiles before the tile is folded)
constexpr int SD_I8_SC_BUFS = 4;
constexpr int SD_LDS_I8 = SD_LDS + SD_I8_CARRY_DOCS * (int)sizeof(double) + SD_I8_SC_BUFS * SD_ROWS_A * (int)sizeof(float);

// One MFMA step (k = 16 for 16-bit inputs; a 16-byte chunk of fp32 is four steps of k = 2).
template <int DT> __device__ __forceinline__ void sd_mma(const i32x4 &a, const i32x4 &b, f32x16 &c)
{
    if constexpr (DT == MAXSIM_F16) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    } else if constexpr (DT == MAXSIM_BF16) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    } else if constexpr (DT == SD_I8) { // 16 bytes = 16 codes per lane: k = 32 with both lane halves; int32 sums in c's bits
        c = __builtin_bit_cast(f32x16, __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, __builtin_bit_cast(i32x16, c), 0, 0, 0));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            c = __builtin_amdgcn_mfma_f32_32x32x2f32(__int_as_float(a[e]), __int_as_float(b[e]), c, 0, 0, 0);
    }
}

// n * s rounded once to fp32: the product of an int32 below 2^29 in magnitude and an fp32 is exact in fp64
// (|n| <= 127^2 * 8192 < 2^27 here, so 27 + 24 bits)
__device__ __forceinline__ float sd_scaled_once(int n, float s) { return (float)((double)n * (double)s); }

// q_scale [n_q, l_q] and d_scale [b, l_d] or [T]: the per-token scales of int8 codes (DT == SD_I8), else unused
template <int DT, bool ARGMAX>
__global__ void __launch_bounds__(SD_W * 64) fwd_splitd_kernel(FwdParams p, OffsetsPtr off, int row_bytes, const float *q_scale, const float *d_scale)
{
    static_assert(!(DT == SD_I8 && ARGMAX), "int8 scoring has no argmax output");
    extern __shared__ __attribute__((aligned(16))) char lds[];
    float *lds_part = reinterpret_cast<float *>(lds + 3 * SD_BUF);    // [2][SD_GROUP_BLOCKS]
    double *lds_part_d = reinterpret_cast<double *>(lds + 3 * SD_BUF); // the same for int8: sums in fp64
    double *lds_carry = reinterpret_cast<double *>(lds + SD_LDS);      // int8 only: [SD_I8_CARRY_DOCS]
    float *lds_sc = reinterpret_cast<float *>(lds + SD_LDS + SD_I8_CARRY_DOCS * sizeof(double)); // int8 only: [SD_I8_SC_BUFS][SD_ROWS_A]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int rho = lane & 31, h = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_slabs = row_bytes / SD_SLAB;

    // column groups sharing a document chunk are neighbours on one XCD (see fwd_tile_kernel)
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
        write_empty_docs(p, doc0, doc1, tid, SD_W * 64);

    // copy role of this thread: chunk cc of rows r0 + SD_CP_ROWS i.  A row's chunk c sits at position
    // c ^ ((row >> 2) & 3) of its 64 bytes, which makes both the 16-row x 16-byte operand reads and
    // these 4-row x 64-byte writes hit all banks once.
    const int cc = tid & 3, r0 = tid >> 2;
    const int w_off = r0 * SD_SLAB + ((cc ^ ((r0 >> 2) & 3)) << 4);
    // operand reads: lane (rho, h) takes chunk 2u + h of row rho of a 32-row tile, u = 0, 1
    const int rd0 = rho * SD_SLAB + ((h ^ ((rho >> 2) & 3)) << 4);
    const int rd1 = rd0 ^ 32;
    const int b_base = SD_ROWS_A * SD_SLAB + w * (SD_NCB * BLOCK_COLS * SD_SLAB);
    constexpr int TILE_BYTES = TILE_ROWS * SD_SLAB;

    const int total_blocks = p.n_q * p.bpq;

    for (int pass = 0; pass < p.n_pass; ++pass) {
        int gb0, nb, q_first, nq;
        const bool accumulate = pass > 0;
        if (p.n_pass == 1) {
            q_first = group * p.qpg;
            nq = min(p.qpg, p.n_q - q_first);
            gb0 = q_first * p.bpq;
            nb = nq * p.bpq;
        } else { // one long query per group, SD_GROUP_BLOCKS blocks of it per pass
            q_first = group;
            nq = 1;
            gb0 = group * p.bpq + pass * SD_GROUP_BLOCKS;
            nb = min(SD_GROUP_BLOCKS, p.bpq - pass * SD_GROUP_BLOCKS);
        }
        const bool direct = p.bpq == 1;

        // byte offsets of the query rows this thread copies (row r0 + SD_CP_ROWS j of the group's 512 columns);
        // columns past the query or past the group's blocks re-read a valid row and are never summed
        int64_t qoff[SD_NG - SD_NGA];
#pragma unroll
        for (int j = 0; j < SD_NG - SD_NGA; ++j) {
            int r = r0 + SD_CP_ROWS * j;
            int lb = r >> 5;
            int gb = gb0 + lb;
            bool active = lb < nb && gb < total_blocks;
            int g = active ? gb : 0;
            int q = g / p.bpq;
            int tok = (g % p.bpq) * BLOCK_COLS + (r & 31);
            if (tok > p.l_q - 1)
                tok = p.l_q - 1;
            qoff[j] = ((int64_t)q * p.l_q + tok) * row_bytes + cc * 16;
        }

        bool col_valid[SD_NCB];
        float m[SD_NCB];
        int idx[SD_NCB];
        float qsc[SD_NCB]; // int8: the scale of this lane's query token
#pragma unroll
        for (int cb = 0; cb < SD_NCB; ++cb) {
            int lb = w * SD_NCB + cb;
            int gb = gb0 + lb;
            int tok = (gb % p.bpq) * BLOCK_COLS + rho;
            col_valid[cb] = lb < nb && gb < total_blocks && tok < p.l_q;
            m[cb] = neg_inf();
            idx[cb] = 0;
            qsc[cb] = 0.0f;
            if constexpr (DT == SD_I8)
                if (col_valid[cb])
                    qsc[cb] = q_scale[(int64_t)(gb / p.bpq) * p.l_q + tok];
        }
        const bool wave_active = w * SD_NCB < nb;
        int fin_count = 0; // documents finished in this pass (the same sequence in every pass)

        TileIter li, ci; // loader (four slabs ahead at steady state) and compute position
        int lks = 0, cks = 0;
        it_init(li, p, off, doc0, doc1);
        ci = li;
        if (!it_valid(ci))
            break;

        // Addresses of the loader's slab.  When the stream has ended the last slab is loaded again
        // (in bounds, never used), so that the loads need no predicate.
        int s_last = 0, s_ks = 0;
        int64_t s_row0 = 0;
        const char *a_base = nullptr;
        int64_t q_add = 0;
        bool s_new_tile = false; // the loader's slab is the first of a macro tile
        int l_tile = 0, c_tile = 0; // macro tiles begun by the loader / folded, modulo SD_I8_SC_BUFS
        auto gaddr = [&]() {
            s_new_tile = false;
            if (it_valid(li)) {
                s_row0 = li.row0;
                s_last = li.len - li.t0 - 1;
                s_ks = lks;
                s_new_tile = lks == 0;
                if (++lks == n_slabs) {
                    lks = 0;
                    it_next(li, p, off, SD_ROWS_A);
                }
            }
            a_base = p.D + s_row0 * row_bytes + s_ks * SD_SLAB + cc * 16;
            q_add = (int64_t)s_ks * SD_SLAB;
        };
        // two register sets of staged slabs; which one is a compile-time choice (the two copies of the loop body
        // must not be merged into one that selects a set through a pointer)
        i32x4 g[2][SD_NG];
        float g_sc[2] = {0.0f, 0.0f}; // int8: the scale of document row r0 of a macro tile, in flight with its first slab
        int g_sc_buf[2] = {-1, -1};   // ... and the LDS buffer it goes to (-1: this set carries none)
        constexpr std::integral_constant<int, 0> g0{};
        constexpr std::integral_constant<int, 1> g1{};
        static_assert(DT != SD_I8 || SD_NGA == 1, "one copy instruction of the workgroup covers a macro tile's rows");
        auto gload1 = [&](auto set, int k) {
            i32x4(&gs)[SD_NG] = g[decltype(set)::value];
            if (k < SD_NGA) {
                int row = min(r0 + SD_CP_ROWS * k, s_last);
                gs[k] = *reinterpret_cast<const i32x4 *>(a_base + (int64_t)row * row_bytes);
                if constexpr (DT == SD_I8) {
                    g_sc_buf[decltype(set)::value] = -1;
                    if (s_new_tile) {
                        g_sc_buf[decltype(set)::value] = l_tile;
                        l_tile = (l_tile + 1) & (SD_I8_SC_BUFS - 1);
                        if (cc == 0)
                            g_sc[decltype(set)::value] = d_scale[s_row0 + row];
                    }
                }
            } else {
                gs[k] = *reinterpret_cast<const i32x4 *>(p.Q + qoff[k - SD_NGA] + q_add);
            }
        };
        auto lstore1 = [&](auto set, int k, int buf_off) {
            const i32x4(&gs)[SD_NG] = g[decltype(set)::value];
            *reinterpret_cast<i32x4 *>(&lds[buf_off + w_off + k * (SD_CP_ROWS * SD_SLAB)]) = gs[k];
            if constexpr (DT == SD_I8) {
                if (k == 0 && g_sc_buf[decltype(set)::value] >= 0 && cc == 0)
                    lds_sc[g_sc_buf[decltype(set)::value] * SD_ROWS_A + r0] = g_sc[decltype(set)::value];
            }
        };

        int o_cur = 0, o_nxt = SD_BUF, o_wr = 2 * SD_BUF;
        // slabs 0 and 1 go to LDS, slabs 2 and 3 stay in flight.  The order of the loads is pinned: the wait
        // counts of the main loop are derived from the order in which the loop is entered, and if the compiler
        // moves the last two groups of loads the loop waits for loads it has only just issued.
        gaddr();
#pragma unroll
        for (int k = 0; k < SD_NG; ++k)
            gload1(g0, k);
        __builtin_amdgcn_sched_barrier(0);
        gaddr();
#pragma unroll
        for (int k = 0; k < SD_NG; ++k)
            gload1(g1, k);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < SD_NG; ++k)
            lstore1(g0, k, o_cur);
        gaddr();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < SD_NG; ++k)
            gload1(g0, k);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < SD_NG; ++k)
            lstore1(g1, k, o_nxt);
        gaddr();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < SD_NG; ++k)
            gload1(g1, k);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();

        int par = 0;
        auto rotate_buffers = [&]() {
            int t = o_cur;
            o_cur = o_nxt;
            o_nxt = o_wr;
            o_wr = t;
        };
        auto advance_compute = [&]() -> bool { // true when the slab just done was the last of its macro tile
            if (++cks == n_slabs) {
                cks = 0;
                return true;
            }
            return false;
        };

        if (!wave_active) {
            // no column block of this pass: the wavefront only moves slabs (same barriers as the others)
            auto idle = [&](auto gs) {
                gaddr();
#pragma unroll
                for (int k = 0; k < SD_NG; ++k) {
                    lstore1(gs, k, o_wr);
                    gload1(gs, k);
                }
                if (advance_compute())
                    it_next(ci, p, off, SD_ROWS_A);
                __syncthreads();
                rotate_buffers();
            };
            for (;;) {
                idle(g0);
                if (!it_valid(ci))
                    break;
                idle(g1);
                if (!it_valid(ci))
                    break;
            }
        } else {
            f32x16 acc[SD_MT][SD_NCB];
#pragma unroll
            for (int t = 0; t < SD_MT; ++t)
#pragma unroll
                for (int c = 0; c < SD_NCB; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        acc[t][c][r] = 0.0f;

            i32x4 fa0[SD_MT], fb0[SD_NCB], fa1[SD_MT], fb1[SD_NCB];
#pragma unroll
            for (int t = 0; t < SD_MT; ++t)
                fa0[t] = *reinterpret_cast<const i32x4 *>(&lds[o_cur + rd0 + t * TILE_BYTES]);
#pragma unroll
            for (int c = 0; c < SD_NCB; ++c)
                fb0[c] = *reinterpret_cast<const i32x4 *>(&lds[o_cur + b_base + rd0 + c * TILE_BYTES]);

            // one slab: `gs` holds the slab two ahead (to be stored), and is refilled with the slab four ahead
            constexpr int COPIES0 = SD_MT * SD_NCB - (SD_MT + SD_NCB); // copies placed in the first half of a slab
            auto iter = [&](auto gs) {
                // first half of the slab (chunks h): meanwhile read the second half's operands, then store and reload
#pragma unroll
                for (int i = 0; i < SD_MT * SD_NCB; ++i) {
                    const int t = i / SD_NCB, c = i % SD_NCB;
                    sd_mma<DT>(fa0[t], fb0[c], acc[t][c]);
                    if (i == 0)
                        gaddr(); // scalar work for this slab's loads, under the first MFMA
                    if (i < SD_MT)
                        fa1[i] = *reinterpret_cast<const i32x4 *>(&lds[o_cur + rd1 + i * TILE_BYTES]);
                    else if (i < SD_MT + SD_NCB)
                        fb1[i - SD_MT] = *reinterpret_cast<const i32x4 *>(&lds[o_cur + b_base + rd1 + (i - SD_MT) * TILE_BYTES]);
                    // the slots without an operand read take the copies (one LDS instruction per slot)
                    if (i >= SD_MT + SD_NCB) {
                        lstore1(gs, i - (SD_MT + SD_NCB), o_wr);
                        gload1(gs, i - (SD_MT + SD_NCB));
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                // second half (chunks 2 + h): meanwhile read the next slab's first-half operands
#pragma unroll
                for (int i = 0; i < SD_MT * SD_NCB; ++i) {
                    const int t = i / SD_NCB, c = i % SD_NCB;
                    sd_mma<DT>(fa1[t], fb1[c], acc[t][c]);
                    const int k = i;
                    if (k >= 0 && k < SD_MT)
                        fa0[k] = *reinterpret_cast<const i32x4 *>(&lds[o_nxt + rd0 + k * TILE_BYTES]);
                    else if (k >= SD_MT && k < SD_MT + SD_NCB)
                        fb0[k - SD_MT] = *reinterpret_cast<const i32x4 *>(&lds[o_nxt + b_base + rd0 + (k - SD_MT) * TILE_BYTES]);
                    constexpr int FIRST1 = SD_MT * SD_NCB - (SD_NG - COPIES0); // the remaining copies end with the slab
                    if (i >= FIRST1) {
                        lstore1(gs, COPIES0 + i - FIRST1, o_wr);
                        gload1(gs, COPIES0 + i - FIRST1);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }

                int fin_doc = -1;
                if (advance_compute()) {
                    // macro tile complete: fold its eight result tiles, rows ascending (first occurrence wins)
                    if constexpr (DT == SD_I8) {
                        // v = fl32(n * d_scale[row]) per cell; rows past the document's end hold its last token again
                        // (an fp32 product would do up to d = 1024, where |n| < 2^24; as a second variant of this fold it
                        // cost registers in the slab loop and was slower).  The scales came into LDS with the tile's first slab.
                        const float *sc_tile = lds_sc + c_tile * SD_ROWS_A;
                        c_tile = (c_tile + 1) & (SD_I8_SC_BUFS - 1);
#pragma unroll
                        for (int t = 0; t < SD_MT; ++t) {
#pragma unroll
                            for (int q4 = 0; q4 < 4; ++q4) { // accumulator registers 4 q4 .. 4 q4 + 3 hold rows 8 q4 + 4 h .. + 3
                                const float4 sc = *reinterpret_cast<const float4 *>(sc_tile + t * TILE_ROWS + q4 * 8 + h * 4);
#pragma unroll
                                for (int c = 0; c < SD_NCB; ++c) {
                                    float v = m[c];
                                    v = fmaxf(v, sd_scaled_once(__float_as_int(acc[t][c][4 * q4 + 0]), sc.x));
                                    v = fmaxf(v, sd_scaled_once(__float_as_int(acc[t][c][4 * q4 + 1]), sc.y));
                                    v = fmaxf(v, sd_scaled_once(__float_as_int(acc[t][c][4 * q4 + 2]), sc.z));
                                    v = fmaxf(v, sd_scaled_once(__float_as_int(acc[t][c][4 * q4 + 3]), sc.w));
                                    m[c] = v;
#pragma unroll
                                    for (int j = 0; j < 4; ++j)
                                        acc[t][c][4 * q4 + j] = 0.0f;
                                }
                            }
                        }
                    } else {
#pragma unroll
                        for (int c = 0; c < SD_NCB; ++c) {
#pragma unroll
                            for (int t = 0; t < SD_MT; ++t) {
                                fold_tile<ARGMAX>(acc[t][c], m[c], idx[c], ci.t0 + t * TILE_ROWS, h);
#pragma unroll
                                for (int r = 0; r < 16; ++r)
                                    acc[t][c][r] = 0.0f;
                            }
                        }
                    }
                    if (ci.t0 + SD_ROWS_A >= ci.len) { // last macro tile of its document
                        fin_doc = ci.doc;
#pragma unroll
                        for (int cb = 0; cb < SD_NCB; ++cb) {
                            int lb = w * SD_NCB + cb;
                            if constexpr (DT == SD_I8) {
                                // the two lane halves hold the same column: merge, one IEEE fp32 multiply by the
                                // query token's scale, the 32 columns added up in fp64
                                const float mm = fmaxf(m[cb], __shfl_xor(m[cb], 32));
                                double dv = col_valid[cb] ? (double)(qsc[cb] * mm) : 0.0;
#pragma unroll
                                for (int o = 16; o > 0; o >>= 1)
                                    dv += __shfl_xor(dv, o);
                                if (lane == 0) {
                                    if (direct) {
                                        if (lb < nb)
                                            p.scores[(int64_t)(gb0 + lb) * p.ld + ci.doc] = (float)dv;
                                    } else {
                                        lds_part_d[par * SD_GROUP_BLOCKS + lb] = dv;
                                    }
                                }
                            } else {
                                float sum = finish_block<ARGMAX>(p, m[cb], idx[cb], col_valid[cb], gb0 + lb, ci.doc, ci.len, rho, h);
                                if (lane == 0) {
                                    if (direct) {
                                        if (lb < nb)
                                            p.scores[(int64_t)(gb0 + lb) * p.ld + ci.doc] = sum;
                                    } else {
                                        lds_part[par * SD_GROUP_BLOCKS + lb] = sum;
                                    }
                                }
                            }
                            m[cb] = neg_inf();
                            idx[cb] = 0;
                        }
                    }
                    it_next(ci, p, off, SD_ROWS_A);
                }
                __syncthreads();
                if (fin_doc >= 0) {
                    if (!direct && tid < nq) { // thread t adds up the blocks of its query in block order
                        int first_blk = (p.n_pass == 1) ? tid * p.bpq : 0;
                        int cnt = (p.n_pass == 1) ? p.bpq : nb;
                        float *dst = p.scores + (int64_t)(q_first + tid) * p.ld + fin_doc;
                        if constexpr (DT == SD_I8) { // fp64 sum over all tokens of the query, rounded once
                            double sum = 0.0;
                            for (int i = 0; i < cnt; ++i)
                                sum += lds_part_d[par * SD_GROUP_BLOCKS + first_blk + i];
                            if (p.n_pass > 1 && fin_count < SD_I8_CARRY_DOCS) { // (the host sizes chunks to that many documents)
                                if (accumulate)
                                    sum += lds_carry[fin_count];
                                lds_carry[fin_count] = sum;
                            }
                            if (pass == p.n_pass - 1)
                                *dst = (float)sum;
                        } else {
                            float sum = 0.0f;
                            for (int i = 0; i < cnt; ++i)
                                sum += lds_part[par * SD_GROUP_BLOCKS + first_blk + i];
                            *dst = accumulate ? *dst + sum : sum;
                        }
                    }
                    par ^= 1;
                    ++fin_count;
                }
                rotate_buffers();
            };
            for (;;) {
                iter(g0);
                if (!it_valid(ci))
                    break;
                iter(g1);
                if (!it_valid(ci))
                    break;
            }
        }
        __syncthreads(); // LDS is reused by the next pass
    }
}

template <int DT, bool ARGMAX>
hipError_t launch_splitd(const FwdParams &p, int row_bytes, int grid, hipStream_t stream)
{
    hipLaunchKernelGGL((fwd_splitd_kernel<DT, ARGMAX>), dim3(grid), dim3(SD_W * 64), SD_LDS, stream, p, p.offsets, row_bytes,
                       static_cast<const float *>(nullptr), static_cast<const float *>(nullptr));
    return hipGetLastError();
}

template <int DT, bool ARGMAX> hipError_t allow_splitd_lds()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&fwd_splitd_kernel<DT, ARGMAX>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, DT == SD_I8 ? SD_LDS_I8 : SD_LDS);
}

} // namespace

// More than 64 KB of dynamic LDS has to be allowed per kernel and device: every instantiation, for the current
// device (called once per device by the library's set-up).
hipError_t forward_splitd_init_device()
{
    hipError_t e = hipSuccess;
    if ((e = allow_splitd_lds<MAXSIM_F32, false>()) != hipSuccess || (e = allow_splitd_lds<MAXSIM_F32, true>()) != hipSuccess ||
        (e = allow_splitd_lds<MAXSIM_F16, false>()) != hipSuccess || (e = allow_splitd_lds<MAXSIM_F16, true>()) != hipSuccess ||
        (e = allow_splitd_lds<MAXSIM_BF16, false>()) != hipSuccess || (e = allow_splitd_lds<MAXSIM_BF16, true>()) != hipSuccess ||
        (e = allow_splitd_lds<SD_I8, false>()) != hipSuccess)
        return e;
    return hipSuccess;
}

// The work split of the slab kernel: column groups of up to 16 blocks, document chunks.  Returns the grid size.
// max_chunk_docs > 0: no chunk may hold more non-empty documents than that.
static int64_t splitd_plan(FwdParams &p, int num_cu, int max_chunk_docs = 0)
{
    const bool ragged = p.offsets != nullptr;
    p.bpq = (p.l_q + BLOCK_COLS - 1) / BLOCK_COLS;
    if (p.ld == 0)
        p.ld = p.b;
    if (p.bpq <= SD_GROUP_BLOCKS) {
        p.qpg = SD_GROUP_BLOCKS / p.bpq;
        if (p.qpg > p.n_q)
            p.qpg = p.n_q;
        p.n_groups = (p.n_q + p.qpg - 1) / p.qpg;
        p.n_pass = 1;
    } else {
        p.qpg = 1;
        p.n_groups = p.n_q;
        p.n_pass = (p.bpq + SD_GROUP_BLOCKS - 1) / SD_GROUP_BLOCKS;
    }
    // one workgroup per CU at a time; about four chunks per CU so that the tail is short, a multiple of 8
    // for the XCD renumbering, never more chunks than documents
    const int64_t units = ragged ? p.total_tokens : p.b;
    int64_t n_chunks = ((int64_t)num_cu * 4 + p.n_groups - 1) / p.n_groups;
    if (n_chunks > p.b)
        n_chunks = p.b;
    if (max_chunk_docs > 0) { // a chunk of u tokens (ragged) or u documents holds at most u non-empty documents
        const int64_t need = (units + max_chunk_docs - 1) / max_chunk_docs;
        if (n_chunks < need)
            n_chunks = need;
    }
    n_chunks = (n_chunks + 7) / 8 * 8;
    p.unit_per_chunk = (units + n_chunks - 1) / n_chunks;
    if (p.unit_per_chunk < 1)
        p.unit_per_chunk = 1;
    p.n_chunks = (int)n_chunks;
    return (int64_t)p.n_groups * n_chunks;
}

// Any row width that is a multiple of 64 bytes.  `num_cu` is the device's CU count.
hipError_t forward_splitd_launch(FwdParams p, int dtype, int row_bytes, int num_cu, hipStream_t stream)
{
    if (row_bytes < SD_SLAB || row_bytes % SD_SLAB != 0)
        return hipErrorNotSupported;
    const bool am = p.argmax != nullptr;
    const int grid = (int)splitd_plan(p, num_cu);
    switch (dtype) {
    case MAXSIM_F32:
        return am ? launch_splitd<MAXSIM_F32, true>(p, row_bytes, grid, stream) : launch_splitd<MAXSIM_F32, false>(p, row_bytes, grid, stream);
    case MAXSIM_F16:
        return am ? launch_splitd<MAXSIM_F16, true>(p, row_bytes, grid, stream) : launch_splitd<MAXSIM_F16, false>(p, row_bytes, grid, stream);
    default:
        return am ? launch_splitd<MAXSIM_BF16, true>(p, row_bytes, grid, stream) : launch_splitd<MAXSIM_BF16, false>(p, row_bytes, grid, stream);
    }
}

// int8 codes with per-token scales through the slab kernel: widths that are a multiple of 64 and queries of up to
// 1024 tokens (up to 512: whole queries per workgroup; beyond: two passes with the fp64 carry in LDS)
bool forward_splitd_i8_ok(int l_q, int d) { return d >= SD_SLAB && d % SD_SLAB == 0 && (l_q + BLOCK_COLS - 1) / BLOCK_COLS <= 2 * SD_GROUP_BLOCKS; }

hipError_t forward_splitd_i8_launch(FwdParams p, const float *q_scale, const float *d_scale, int d, int num_cu, hipStream_t stream)
{
    if (!forward_splitd_i8_ok(p.l_q, d) || p.argmax != nullptr)
        return hipErrorNotSupported;
    const bool two_pass = (p.l_q + BLOCK_COLS - 1) / BLOCK_COLS > SD_GROUP_BLOCKS;
    const int64_t grid = splitd_plan(p, num_cu, two_pass ? SD_I8_CARRY_DOCS : 0);
    if (grid >= (int64_t(1) << 31))
        return hipErrorInvalidValue;
    hipLaunchKernelGGL((fwd_splitd_kernel<SD_I8, false>), dim3((unsigned)grid), dim3(SD_W * 64), SD_LDS_I8, stream, p, p.offsets, d, q_scale,
                       d_scale);
    return hipGetLastError();
}

} // namespace maxsim
