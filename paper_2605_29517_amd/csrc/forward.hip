// Fused MaxSim forward for gfx950: choice of kernel and launch shape (the kernels themselves are
// in forward_impl.h, compiled once per element type in forward_{f16,bf16,f32}.hip).
#include "common.h"

namespace maxsim {

hipError_t forward_run_f16(const FwdParams &p, int nu, bool argmax, bool tile, int x, int grid, hipStream_t s);
hipError_t forward_run_bf16(const FwdParams &p, int nu, bool argmax, bool tile, int x, int grid, hipStream_t s);
hipError_t forward_run_f32(const FwdParams &p, int nu, bool argmax, bool tile, int x, int grid, hipStream_t s);

static int round_up(int64_t x, int m) { return (int)((x + m - 1) / m * m); }

hipError_t forward_splitd_launch(FwdParams p, int dtype, int row_bytes, int num_cu, hipStream_t stream);

constexpr int MAX_ROW_BYTES = 16384; // d = 8192 (16-bit) or 4096 (fp32)

// Rows of 128, 256 or 512 bytes have kernels that keep the queries in registers.  (Such kernels for rows of
// 1024 bytes were measured slower than the slab-streaming kernel at every shape: one column block per
// wavefront leaves one MFMA per LDS operand read.)
static bool register_stationary_width(int row_bytes)
{
    return row_bytes == 128 || row_bytes == 256 || row_bytes == 512;
}

// Embedding widths the float forward takes: rows that are a multiple of 64 bytes (d a multiple of 32 for
// 16-bit inputs, of 16 for fp32), from d = 32 up to MAX_ROW_BYTES.
bool forward_width_supported(int dtype, int d)
{
    const int64_t row_bytes = (int64_t)d * (dtype == MAXSIM_F32 ? 4 : 2);
    return d >= 32 && row_bytes % 64 == 0 && row_bytes <= MAX_ROW_BYTES;
}

// Chooses kernel and launch shape from the problem size; `num_cu` is the device's CU count.
hipError_t forward_launch(FwdParams p, int dtype, int d, int num_cu, hipStream_t stream)
{
    if (!forward_width_supported(dtype, d))
        return hipErrorNotSupported;
    const int row_bytes = d * (dtype == MAXSIM_F32 ? 4 : 2);
    // any other width: both operands stream through LDS in slabs of the width; so do rows of 512 bytes from 8 column
    // blocks on (two blocks per wavefront in the register-stationary kernel: measured 3-11 % slower there)
    const int64_t all_blocks = (int64_t)p.n_q * ((p.l_q + BLOCK_COLS - 1) / BLOCK_COLS);
    if (!register_stationary_width(row_bytes) || (row_bytes == 512 && all_blocks >= 8))
        return forward_splitd_launch(p, dtype, row_bytes, num_cu, stream);
    const int nu = row_bytes / 32; // 16-byte chunk pairs per row
    const bool ragged = p.offsets != nullptr;
    const bool am = p.argmax != nullptr;
    p.bpq = (p.l_q + BLOCK_COLS - 1) / BLOCK_COLS;
    if (p.ld == 0)
        p.ld = p.b;
    const int64_t total_blocks = (int64_t)p.n_q * p.bpq;
    const int64_t units = ragged ? p.total_tokens : p.b; // what is split across chunks
    auto run = [&](bool tile, int x, int grid) {
        switch (dtype) {
        case MAXSIM_F32: return forward_run_f32(p, nu, am, tile, x, grid, stream);
        case MAXSIM_F16: return forward_run_f16(p, nu, am, tile, x, grid, stream);
        default: return forward_run_bf16(p, nu, am, tile, x, grid, stream);
        }
    };

    // Streaming kernel: every wavefront holds whole queries in as many column blocks as fit beside two
    // document tiles in registers (4 for rows of up to 256 bytes, 2 for 512 bytes), and up
    // to 4 wavefronts share a run of documents.  That covers up to 16 blocks of short queries.
    const int stream_max_blocks = nu <= 8 ? 4 : 2;
    int s_ncb = 0, s_groups = 0;
    if (total_blocks <= stream_max_blocks) {
        s_ncb = (int)total_blocks;
        s_groups = 1;
    } else if (p.bpq <= stream_max_blocks) {
        int qpw = stream_max_blocks / p.bpq; // whole queries per wavefront
        int groups = (p.n_q + qpw - 1) / qpw;
        if (groups <= 4) {
            s_ncb = qpw * p.bpq;
            s_groups = groups == 3 ? 4 : groups;
        }
    }

    // five to sixteen blocks of narrow rows: the tile kernel with two blocks per wavefront is faster than two to
    // four streaming wavefronts per run (measured on the ragged 100K corpus: 1.37 against 1.60 ms at 5 blocks,
    // 2.1-2.6 against 2.7 ms at 9-16; uniform corpora of 50K documents: 10-22 % at 5-8 blocks)
    if (nu <= 8 && total_blocks > 4)
        s_groups = 0;

    if (s_groups > 0) {
        // one work chunk per group of wavefronts; enough chunks to oversubscribe the chip a few times, but no
        // chunk smaller than about 2K tokens -- unless that leaves wavefront slots empty (a small corpus is a chain
        // of memory latencies per wavefront): then chunks go down to 128 tokens until every slot has one
        const int64_t tokens = ragged ? p.total_tokens : p.b * (int64_t)p.l_d;
        int64_t want = (int64_t)num_cu * 16 * 4 / s_groups;
        int64_t by_size = (tokens + 2047) / 2048;
        const int64_t slots = (int64_t)num_cu * 16 / s_groups;
        if (by_size < slots) {
            by_size = (tokens + 127) / 128;
            if (by_size > slots)
                by_size = slots;
        } else if (s_groups == 1) {
            // a large corpus, one wavefront per run: eight long runs per CU, all resident at once, stream 2-5 % faster
            // than more and shorter ones (0.679 against 0.694 ms on the ragged 100K corpus; a read probe shows the same,
            // 7.0 against 6.8 TB/s)
            want = (int64_t)num_cu * 8;
        }
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
        p.n_groups = s_groups;
        p.qpg = p.n_q;
        p.n_pass = 1;
        const int chunks_per_block = 4 / s_groups;
        int grid = (int)((n_chunks + chunks_per_block - 1) / chunks_per_block);
        return run(false, s_ncb, grid);
    }

    // tile kernel: W wavefronts x NCB blocks per group (the query fragments of a wavefront fill 128 registers)
    const int ncb = nu <= 8 ? 4 : 32 / nu;
    int w = 8;
    if (total_blocks <= 1 * ncb)
        w = 1;
    else if (total_blocks <= 2 * ncb)
        w = 2;
    else if (total_blocks <= 4 * ncb)
        w = 4;
    int shape = w, wave_blocks = ncb;
    // Five to sixteen blocks of narrow rows.  What a wavefront spends per tile beside its MFMAs (iterator, copies,
    // barrier) does not depend on how many blocks it holds, so workgroups of two (up to 8 blocks) or four wavefronts
    // with four blocks each beat eight wavefronts with one or two blocks by 6-15 % -- as long as there are documents
    // enough for their many workgroups (at least two per workgroup; a small corpus is a chain of memory latencies
    // per workgroup, and the shapes below keep several tiles in flight for that).
    const int narrow_w = total_blocks <= 8 ? 2 : 4;
    // (fp32 rows carry four times the MFMAs per block: there two wavefronts are 3 % behind four with two blocks each)
    const bool narrow = ncb == 4 && total_blocks > 4 && total_blocks <= 16 && p.b >= 2 * ((int64_t)num_cu * 16 / narrow_w) &&
                        !(dtype == MAXSIM_F32 && narrow_w == 2);
    if (narrow) {
        w = narrow_w;
        shape = w;
    } else if (ncb == 4 && total_blocks <= 16) {
        if (total_blocks <= 8 && !(am && p.bpq > 4)) {
            // four wavefronts with two column blocks each (shape code 42), two workgroups per CU
            wave_blocks = 2;
            w = 4;
            shape = 42;
        } else { // eight wavefronts with one or two column blocks each (shape code 81 / 82)
            wave_blocks = total_blocks <= 8 ? 1 : 2;
            w = 8;
            shape = 80 + wave_blocks;
        }
    }
    // a ragged corpus (or a uniform one whose documents are not a whole number of tiles) scored by many queries of
    // one block: 32-row windows over the packed rows (no padded tiles at the ends of documents)
    // (the windows also serve uniform corpora of whole tiles at 5-16 queries, where their narrow workgroups beat the
    // tile kernel's by 5-17 %)
    const bool rows_32bit = ragged || p.b * (int64_t)p.l_d < ((int64_t)1 << 31); // the window iterator counts packed rows in 32 bits
    const bool ragged_ends = rows_32bit && (ragged || p.l_d % TILE_ROWS != 0 || total_blocks <= 16);
    if (ragged_ends && !am && p.bpq == 1 && narrow) {
        // five to sixteen queries: the same narrow workgroups with 3 or 4 queries per wavefront (7-16 % over eight
        // wavefronts with two queries each, and over the per-document tiles, on the ragged 100K corpus)
        wave_blocks = (total_blocks + w - 1) / w <= 3 ? 3 : 4;
        shape = 900 + w * 10 + wave_blocks;
    }
    if (ragged_ends && !am && ncb == 4 && p.bpq == 1 && total_blocks > 16) {
        // as many workgroups per chunk as 32 queries each would need, then 3 or 4 queries per wavefront so that the
        // queries are spread evenly (48 queries: two workgroups of 24 rather than 32 + 16)
        const int64_t groups = (total_blocks + 31) / 32;
        const int64_t per_group = (total_blocks + groups - 1) / groups;
        wave_blocks = per_group <= 24 ? 3 : 4;
        shape = 90 + wave_blocks;
    }
    const int group_blocks = w * wave_blocks;
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
    // document chunks: about sixteen wavefronts per CU in total, i.e. twice what a CU holds at a time (256 registers
    // per wavefront: two wavefronts per SIMD; one round or two measured the same), a multiple of 8 so that the XCD
    // renumbering applies, and never more chunks than documents
    int64_t wg_target = (int64_t)num_cu * 16 / w;
    int64_t n_chunks = (wg_target + p.n_groups - 1) / p.n_groups;
    if (n_chunks < 8)
        n_chunks = 8;
    n_chunks = round_up(n_chunks, 8);
    p.unit_per_chunk = (units + n_chunks - 1) / n_chunks;
    if (p.unit_per_chunk < 1)
        p.unit_per_chunk = 1;
    p.n_chunks = (int)n_chunks;
    return run(true, shape, p.n_groups * p.n_chunks);
}

} // namespace maxsim
