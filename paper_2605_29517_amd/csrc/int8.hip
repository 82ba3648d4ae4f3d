// int8 x int8 MaxSim scoring with deferred dequantisation (Alg. 4 of the paper) and the
// per-token absmax quantiser, for gfx950.
//
// Same query-stationary structure as the 16-bit tile kernel: a workgroup keeps up to 1024
// query tokens in registers as i8 MFMA B operands and streams 64-token document tiles
// through LDS; v_mfma_i32_32x32x32_i8 produces exact int32 dot products.  The per-token
// document scale is applied once per similarity cell in the epilogue, the row max is taken
// on the scaled values, the query scale is applied once per query token after the max, and
// the sum over query tokens is carried in fp64 and rounded once, which makes the score a
// pure function of the inputs (independent of tiling and of the order of the final sum for
// any realistic range of magnitudes).
//
// Epilogue arithmetic.  The cell value is fl32(n * s) (n the integer dot product, s the
// token's scale).  Converting n to float and multiplying costs two VALU operations per cell,
// and the VALU, not the matrix core, is what binds this kernel.  Instead the accumulators
// start at the integer 0x4B000000, the bit pattern of the float 2^23: for 0 <= n < 2^23 the
// accumulator's bits then ARE the float x = 2^23 + n, and one fused multiply-add
// fma(x, s, -2^23 * s) forms x*s - 2^23*s = n*s exactly and rounds it once, i.e. returns
// fl32(n * s) bit for bit (2^23 * s is a pure exponent shift, hence exact).  For -2^23 < n < 0
// the bits are the float 2^23 + n/2 (the spacing below 2^23 is one half), so the same
// instruction returns fl32(n*s/2) = fl32(n*s)/2 (exact halving; the only exception would be a
// product in the subnormal range, |n*s| < 2^-125, which needs a scale below 2^-100).  Halving
// keeps the order among negative values and any non-negative value still beats them, so
// the running max stays correct and a negative final max is doubled once per query token
// at the end of the document.  |n| <= 128 * 127^2 < 2^21.
#include "common.h"

namespace maxsim {

constexpr int I8_ROW_BYTES = 128;
constexpr int I8_NU = 4;          // 16-byte chunks per lane per row (chunks 2u + h)
constexpr int I8_TILE_ROWS = 64;  // document tokens staged per barrier (two MFMA row tiles)
constexpr int I8_ROW_STRIDE = I8_ROW_BYTES + 16;
constexpr int I8_NCB = 4;
constexpr int I8_PIPE = 1; // result blocks between a block's MFMAs and its epilogue (2 needs more registers than there are)

struct I8Params {
    const char *Q;      // [n_q, l_q, 128] int8
    const float *qs;    // [n_q, l_q]
    const char *D;      // [b, l_d, 128] int8
    const float *ds;    // [b, l_d]
    float *scores;      // [n_q, b]
    FwdParams f;        // sizes, optional offsets and the work split
};

// (four wavefronts: asked to fit two per SIMD, which they do without spilling; one or two run faster unconstrained)
template <int W>
__global__ void __launch_bounds__(W * 64, W >= 4 ? 2 : 1) fwd_i8_kernel(I8Params P, OffsetsPtr off)
{
    const FwdParams &p = P.f;
    constexpr int NT = W * 64;
    constexpr int CHUNKS = I8_TILE_ROWS * I8_ROW_BYTES / 16; // 512
    constexpr int CPT = CHUNKS / NT;
    static_assert(CHUNKS % NT == 0, "tile must split evenly over the workgroup");
    constexpr int CPR = I8_ROW_BYTES / 16;
    constexpr int GROUP_BLOCKS = W * I8_NCB;

    __shared__ __attribute__((aligned(16))) char lds_tile[2][I8_TILE_ROWS * I8_ROW_STRIDE];
    __shared__ __attribute__((aligned(16))) float lds_scale[2][I8_TILE_ROWS];
    __shared__ __attribute__((aligned(16))) float lds_bias[2][I8_TILE_ROWS]; // -2^23 * scale
    __shared__ double lds_part[2][GROUP_BLOCKS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int rho = lane & 31, h = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int n_wg = gridDim.x;
    int v = blockIdx.x;
    if ((n_wg & 7) == 0) // keep the column groups of one document chunk on one XCD
        v = (blockIdx.x & 7) * (n_wg >> 3) + (blockIdx.x >> 3);
    const int group = v % p.n_groups;
    const int chunk = v / p.n_groups;
    int64_t doc0, doc1;
    chunk_doc_range(p, chunk, doc0, doc1);
    if (doc0 >= doc1)
        return;
    if (group == 0 && p.offsets) { // empty documents: score -inf
        for (int64_t doc = doc0 + tid; doc < doc1; doc += NT)
            if (p.offsets[doc + 1] == p.offsets[doc])
                for (int q = 0; q < p.n_q; ++q)
                    P.scores[(int64_t)q * p.ld + doc] = neg_inf();
    }

    const int q_first = group * p.qpg;
    const int nq = min(p.qpg, p.n_q - q_first);
    const int gb0 = q_first * p.bpq;
    const int nb = nq * p.bpq;

    i32x4 qf[I8_NCB][I8_NU];
    float qscale[I8_NCB];
    bool col_valid[I8_NCB];
    float m[I8_NCB];
#pragma unroll
    for (int cb = 0; cb < I8_NCB; ++cb) {
        int lb = w * I8_NCB + cb;
        bool active = lb < nb;
        int gb = active ? gb0 + lb : 0;
        int q = gb / p.bpq;
        int tok = (gb % p.bpq) * BLOCK_COLS + rho;
        col_valid[cb] = active && tok < p.l_q;
        if (tok > p.l_q - 1)
            tok = p.l_q - 1;
        const char *row = P.Q + ((int64_t)q * p.l_q + tok) * I8_ROW_BYTES + h * 16;
#pragma unroll
        for (int u = 0; u < I8_NU; ++u)
            qf[cb][u] = *reinterpret_cast<const i32x4 *>(row + u * 32);
        qscale[cb] = P.qs[(int64_t)q * p.l_q + tok];
        m[cb] = neg_inf();
    }

    Cursor lc;
    cursor_init(lc, p, off, doc0, doc1);
    static_assert(CPT <= 8, "eight named registers hold a thread's share of a tile");
    uint4 g0, g1, g2, g3, g4, g5, g6, g7; // (named: see reg_at)
    auto g = [&](auto i) -> uint4 & { return reg_at<decltype(i)::value>(g0, g1, g2, g3, g4, g5, g6, g7); };
    float gs = 0.0f;
    auto gload = [&](const Cursor &c) {
        static_for<CPT>([&](auto i) {
            int ch = tid + i * NT;
            int row = c.t0 + ch / CPR;
            if (row > c.len - 1)
                row = c.len - 1;
            g(i) = *reinterpret_cast<const uint4 *>(P.D + (c.start + row) * I8_ROW_BYTES + (ch % CPR) * 16);
        });
        if (tid < I8_TILE_ROWS) {
            int row = c.t0 + tid;
            if (row > c.len - 1)
                row = c.len - 1;
            gs = P.ds[c.start + row];
        }
    };
    auto lstore = [&](int buf) {
        static_for<CPT>([&](auto i) {
            int ch = tid + i * NT;
            *reinterpret_cast<uint4 *>(&lds_tile[buf][(ch / CPR) * I8_ROW_STRIDE + (ch % CPR) * 16]) = g(i);
        });
        if (tid < I8_TILE_ROWS) {
            lds_scale[buf][tid] = gs;
            lds_bias[buf][tid] = gs * -8388608.0f;
        }
    };

    gload(lc);
    lstore(0);
    Cursor cc = lc;
    cursor_next_tile(lc, p, off, I8_TILE_ROWS);
    if (lc.valid)
        gload(lc);
    __syncthreads();

    // accumulator start value (see the header); made opaque so that it stays in 16 registers
    // for the whole kernel instead of being rebuilt with 16 moves per result block
    i32x16 seed;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        int v = 0x4B000000;
        asm volatile("" : "+v"(v));
        seed[r] = v;
    }

    int cur = 0, par = 0;
    while (cc.valid) {
        Cursor cnext = lc;
        if (lc.valid) {
            lstore(cur ^ 1);
            cursor_next_tile(lc, p, off, I8_TILE_ROWS);
            if (lc.valid)
                gload(lc);
        }
        if (cc.t0 == 0) {
#pragma unroll
            for (int cb = 0; cb < I8_NCB; ++cb)
                m[cb] = neg_inf();
        }
        {
            constexpr int NSUB = I8_TILE_ROWS / TILE_ROWS;
            i32x4 a[NSUB][I8_NU];
            // scale and bias of this lane's 16 result rows: four runs of four consecutive rows
            float sc[NSUB][16], bi[NSUB][16];
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub) {
                const char *src = &lds_tile[cur][(sub * TILE_ROWS + rho) * I8_ROW_STRIDE + h * 16];
#pragma unroll
                for (int u = 0; u < I8_NU; ++u)
                    a[sub][u] = *reinterpret_cast<const i32x4 *>(src + u * 32);
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    float4 s4 = *reinterpret_cast<const float4 *>(&lds_scale[cur][sub * TILE_ROWS + r4 * 8 + h * 4]);
                    float4 b4 = *reinterpret_cast<const float4 *>(&lds_bias[cur][sub * TILE_ROWS + r4 * 8 + h * 4]);
                    sc[sub][r4 * 4 + 0] = s4.x;
                    sc[sub][r4 * 4 + 1] = s4.y;
                    sc[sub][r4 * 4 + 2] = s4.z;
                    sc[sub][r4 * 4 + 3] = s4.w;
                    bi[sub][r4 * 4 + 0] = b4.x;
                    bi[sub][r4 * 4 + 1] = b4.y;
                    bi[sub][r4 * 4 + 2] = b4.z;
                    bi[sub][r4 * 4 + 3] = b4.w;
                }
            }
            // Software pipeline over the NSUB x NCB result blocks of the stage.  One step = one MFMA of
            // block k plus a quarter (4 of 16 rows: four multiply-adds, two max3) of the epilogue of
            // block k - I8_PIPE, whose MFMAs have long retired; scheduling barriers keep the steps
            // apart, so the VALU work (1.5 operations per cell) always runs under an MFMA in flight.
            constexpr int NBLK = NSUB * I8_NCB;
            i32x16 acc[NBLK];
#pragma unroll
            for (int blk = 0; blk < NBLK + I8_PIPE; ++blk) {
#pragma unroll
                for (int u = 0; u < I8_NU; ++u) {
                    if (blk < NBLK) {
                        const int sub = blk / I8_NCB, cb = blk % I8_NCB;
                        acc[blk] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[sub][u], qf[cb][u], u == 0 ? seed : acc[blk], 0, 0, 0);
                    }
                    if (blk >= I8_PIPE) {
                        const int e = blk - I8_PIPE, es = e / I8_NCB, ec = e % I8_NCB;
                        const int r = 4 * u;
                        float v0 = __builtin_fmaf(__int_as_float(acc[e][r + 0]), sc[es][r + 0], bi[es][r + 0]);
                        float v1 = __builtin_fmaf(__int_as_float(acc[e][r + 1]), sc[es][r + 1], bi[es][r + 1]);
                        float v2 = __builtin_fmaf(__int_as_float(acc[e][r + 2]), sc[es][r + 2], bi[es][r + 2]);
                        float v3 = __builtin_fmaf(__int_as_float(acc[e][r + 3]), sc[es][r + 3], bi[es][r + 3]);
                        m[ec] = fmaxf(fmaxf(m[ec], v0), v1);
                        m[ec] = fmaxf(fmaxf(m[ec], v2), v3);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }

        const bool last_tile = cc.t0 + I8_TILE_ROWS >= cc.len;
        if (last_tile) {
#pragma unroll
            for (int cb = 0; cb < I8_NCB; ++cb) {
                float mm = fmaxf(m[cb], __shfl_xor(m[cb], 32));
                mm = mm < 0.0f ? mm + mm : mm; // negative maxima were carried halved
                float r = qscale[cb] * mm;     // one IEEE fp32 multiply per query token
                double dv = col_valid[cb] ? (double)r : 0.0;
#pragma unroll
                for (int o = 16; o > 0; o >>= 1)
                    dv += __shfl_xor(dv, o);
                if (lane == 0)
                    lds_part[par][w * I8_NCB + cb] = dv;
            }
        }
        __syncthreads();
        if (last_tile) {
            if (tid < nq) {
                double s = 0.0;
                for (int i = 0; i < p.bpq; ++i)
                    s += lds_part[par][tid * p.bpq + i];
                P.scores[(int64_t)(q_first + tid) * p.ld + cc.doc] = (float)s;
            }
            par ^= 1;
        }
        cc = cnext;
        cur ^= 1;
    }
}

// ---------------------------------------------------------------------------------------
// document-stationary kernel for large corpora
// ---------------------------------------------------------------------------------------
// The roles are turned around: the query tokens of a group (up to 1024, padded rows, plus
// their scales) are copied into LDS once per workgroup, and every wavefront works alone on
// its own run of documents.  A 32-token document tile goes from HBM straight into registers
// in MFMA operand layout, one tile ahead, and stays there while the wavefront walks over all
// column blocks of the group, reading the B operands of block k + 1 from LDS during the
// MFMAs of block k and folding block k - 1 under them.  There is no barrier, no LDS write
// and no staging copy in the main loop, the per-tile work (scales, loads, iterator) is
// spread over up to 128 MFMAs instead of 32, and the wavefronts of a SIMD drift apart so
// that one computes while the other waits.  The token scales of a tile take a detour through
// 512 bytes of LDS private to the wavefront to get from "one per lane" to "the 16 rows of
// this lane's accumulator registers".
constexpr int I8D_WAVES = 8;
constexpr int I8D_LIN_BLOCKS = 2;                        // up to this many column blocks the tiles are read as whole lines (no gain from 4 on)
constexpr int I8D_MAX_BLOCKS = 32;                       // column blocks per group (1024 query tokens)
constexpr int I8D_QSTRIDE = I8_ROW_BYTES + 16;           // padded LDS row of a query token

// The token scales of a tile, from "one per lane" (lane rho holds row rho's scale) to the 16 rows of this
// lane's accumulator registers, through 512 bytes of LDS private to the wavefront.
__device__ __forceinline__ void i8d_tile_scales(float *w_scale, float *w_bias, float s_n, int rho, int h,
                                                float (&sc)[16], float (&bi)[16])
{
    if (h == 0) {
        w_scale[rho] = s_n;
        w_bias[rho] = s_n * -8388608.0f;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
        float4 s4 = *reinterpret_cast<const float4 *>(&w_scale[r4 * 8 + h * 4]);
        float4 b4 = *reinterpret_cast<const float4 *>(&w_bias[r4 * 8 + h * 4]);
        sc[r4 * 4 + 0] = s4.x;
        sc[r4 * 4 + 1] = s4.y;
        sc[r4 * 4 + 2] = s4.z;
        sc[r4 * 4 + 3] = s4.w;
        bi[r4 * 4 + 0] = b4.x;
        bi[r4 * 4 + 1] = b4.y;
        bi[r4 * 4 + 2] = b4.z;
        bi[r4 * 4 + 3] = b4.w;
    }
}

// dynamic LDS of the document-stationary kernels for NB column blocks (queries, their scales, per wavefront 32 token
// scales and biases); the whole-line variant adds a document tile per wavefront
constexpr size_t i8_doc_lds(int nb) { return (size_t)nb * BLOCK_COLS * (I8D_QSTRIDE + 4) + I8D_WAVES * 64 * sizeof(float); }
constexpr size_t i8_doc_lin_lds(int nb) { return i8_doc_lds(nb) + (size_t)I8D_WAVES * TILE_ROWS * I8D_QSTRIDE; }
constexpr size_t i8_split_lds(int nb) { return i8_doc_lds(nb) + (size_t)2 * I8D_WAVES * nb * BLOCK_COLS * sizeof(float); }

constexpr int I8D_LAG_STEPS = 2; // steps between a block's MFMAs and its epilogue in the document-stationary kernels

// One document tile (operands `a`, row scales sc / biases bi) against the NB column blocks in LDS, folded into
// the running maxima m.  Step t: MFMA (t % 4) of block t / 4, the LDS read of the same chunk of the next block,
// and a quarter of the epilogue of the block whose chain ended I8D_LAG steps ago (so that its results have long
// left the matrix pipeline); three accumulators rotate.
template <int NB>
__device__ __forceinline__ void i8d_tile_blocks(const i32x4 (&a)[I8_NU], const float (&sc)[16], const float (&bi)[16],
                                                const char *q_tile, int b_off, const i32x16 &seed, float (&m)[NB])
{
    i32x4 qb[2][I8_NU];
#pragma unroll
    for (int u = 0; u < I8_NU; ++u)
        qb[0][u] = *reinterpret_cast<const i32x4 *>(q_tile + b_off + u * 32);
    i32x16 acc[3];
    __builtin_amdgcn_sched_barrier(0);
    constexpr int I8D_LAG = I8D_LAG_STEPS;
#pragma unroll
    for (int t = 0; t < NB * I8_NU + I8_NU + I8D_LAG; ++t) {
        const int blk = t / I8_NU, u = t % I8_NU;
        if (blk < NB) {
            acc[blk % 3] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[u], qb[blk & 1][u], u == 0 ? seed : acc[blk % 3], 0, 0, 0);
            if (blk + 1 < NB)
                qb[(blk + 1) & 1][u] = *reinterpret_cast<const i32x4 *>(
                    q_tile + (blk + 1) * (BLOCK_COLS * I8D_QSTRIDE) + b_off + u * 32);
        }
        const int te = t - I8_NU - I8D_LAG; // epilogue step
        if (te >= 0) {
            const int eb = te / I8_NU, r = 4 * (te % I8_NU);
            const i32x16 &e = acc[eb % 3];
            float v0 = __builtin_fmaf(__int_as_float(e[r + 0]), sc[r + 0], bi[r + 0]);
            float v1 = __builtin_fmaf(__int_as_float(e[r + 1]), sc[r + 1], bi[r + 1]);
            float v2 = __builtin_fmaf(__int_as_float(e[r + 2]), sc[r + 2], bi[r + 2]);
            float v3 = __builtin_fmaf(__int_as_float(e[r + 3]), sc[r + 3], bi[r + 3]);
            float mm = m[eb];
            mm = fmaxf(fmaxf(mm, v0), v1);
            mm = fmaxf(fmaxf(mm, v2), v3);
            m[eb] = mm;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// End of a document: mm[blk] is the maximum per query token (column rho of block blk; in lanes 0..31 and again
// in lanes 32..63) in the halved-negatives form of the seeded accumulator.  Per query: one IEEE fp32 multiply
// by the query scale per token, a lane-local fp64 sum over the query's blocks, one butterfly over the 32
// columns, one rounding.
template <int NB>
__device__ __forceinline__ void i8d_finish(const I8Params &P, const float (&mmv)[NB], const float *q_scale, int nb,
                                           int q_first, int doc, int lane, int rho)
{
    const FwdParams &p = P.f;
    double dv = 0.0;
    int iq = 0, j = 0; // block inside the query, query inside the group
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
        if (blk >= nb)
            continue;
        float mm = mmv[blk];
        mm = mm < 0.0f ? mm + mm : mm;                     // negative maxima were carried halved
        float r = q_scale[blk * BLOCK_COLS + rho] * mm;    // one IEEE fp32 multiply per query token
        dv += (iq * BLOCK_COLS + rho < p.l_q) ? (double)r : 0.0;
        if (++iq == p.bpq) {
#pragma unroll
            for (int o = 16; o > 0; o >>= 1)
                dv += __shfl_xor(dv, o);
            if (lane == 0)
                P.scores[(int64_t)(q_first + j) * p.ld + doc] = (float)dv;
            dv = 0.0;
            iq = 0;
            ++j;
        }
    }
}

// Copies the group's query rows (padded) and scales (0 for padding columns) into LDS.
template <int NB>
__device__ __forceinline__ void i8d_load_queries(const I8Params &P, char *q_tile, float *q_scale, int gb0, int nb, int tid)
{
    const FwdParams &p = P.f;
    for (int c = tid; c < NB * BLOCK_COLS * 8; c += I8D_WAVES * 64) { // 16-byte chunks of the group's query rows
        int col = c >> 3, part = c & 7;
        uint4 chunk = make_uint4(0, 0, 0, 0);
        float qsv = 0.0f;
        if (col < nb * BLOCK_COLS) {
            int gb = gb0 + col / BLOCK_COLS;
            int q = gb / p.bpq;
            int tok = (gb % p.bpq) * BLOCK_COLS + col % BLOCK_COLS;
            bool valid = tok < p.l_q;
            if (!valid)
                tok = p.l_q - 1;
            const int64_t qrow = (int64_t)q * p.l_q + tok;
            chunk = *reinterpret_cast<const uint4 *>(P.Q + qrow * I8_ROW_BYTES + part * 16);
            qsv = valid ? P.qs[qrow] : 0.0f;
        }
        *reinterpret_cast<uint4 *>(q_tile + col * I8D_QSTRIDE + part * 16) = chunk;
        if (part == 0)
            q_scale[col] = qsv;
    }
}

// NB: column blocks the tile loop walks over (the group's block count rounded up; the surplus
// blocks multiply zero rows and are never looked at).
//
// LIN (few column blocks, where the corpus read is the cost): a tile of 32 rows is 4 KB of contiguous memory and
// is read as such, with four non-temporal loads of 1 KB (eight lanes per row), parked in a piece of LDS of the
// wavefront's own and read back in operand layout; the direct loads take 32 bytes of each of 32 lines per
// instruction and cannot carry the hint (see load_stream16).
template <int NB, bool LIN>
__global__ void __launch_bounds__(I8D_WAVES * 64) fwd_i8_doc_kernel(I8Params P, OffsetsPtr off)
{
    const FwdParams &p = P.f;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int rho = lane & 31, h = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int group = blockIdx.x % p.n_groups;
    const int wg_chunk = blockIdx.x / p.n_groups;
    const int q_first = group * p.qpg;
    const int nq = min(p.qpg, p.n_q - q_first);
    const int gb0 = q_first * p.bpq;
    const int nb = nq * p.bpq; // column blocks of this group, <= I8D_MAX_BLOCKS

    // LDS: query rows [NB * 32][144 B], query scales [NB * 32] (0 for padding columns), then
    // per wavefront 32 token scales and 32 biases
    char *q_tile = smem;
    float *q_scale = reinterpret_cast<float *>(smem + NB * BLOCK_COLS * I8D_QSTRIDE);
    float *w_scale = q_scale + NB * BLOCK_COLS + w * 64;
    float *w_bias = w_scale + 32;
    char *w_tile = smem + i8_doc_lds(NB) + w * (TILE_ROWS * I8D_QSTRIDE); // LIN only: this wavefront's document tile

    i8d_load_queries<NB>(P, q_tile, q_scale, gb0, nb, tid);
    __syncthreads(); // the only barrier: from here on every wavefront is on its own

    int64_t doc0_, doc1_;
    chunk_doc_range(p, (int64_t)wg_chunk * I8D_WAVES + w, doc0_, doc1_);
    if (doc0_ >= doc1_)
        return;
    const int doc0 = (int)doc0_, doc1 = (int)doc1_;
    if (group == 0 && p.offsets) { // empty documents of this wavefront's run: score -inf
        for (int doc = doc0 + lane; doc < doc1; doc += 64)
            if (p.offsets[doc + 1] == p.offsets[doc])
                for (int q = 0; q < p.n_q; ++q)
                    P.scores[(int64_t)q * p.ld + doc] = neg_inf();
    }

    TileIter li, ci; // load iterator: one tile ahead of the compute iterator
    it_init(li, p, off, doc0, doc1);
    ci = li;
    if (!it_valid(ci))
        return;

    i32x4 a_n[I8_NU]; // LIN: piece i holds 16 bytes of row 8 i + lane / 8, else chunk 2 u + h of row rho
    float s_n = 0.0f;
    auto gload = [&]() {
        if (!it_valid(li))
            return;
        const int last = li.len - li.t0 - 1; // rows past the document re-read its last token
        const int row = rho < last ? rho : last;
        const int64_t grow = (int64_t)li.row0 + row;
        if constexpr (LIN) {
#pragma unroll
            for (int i = 0; i < I8_NU; ++i) {
                int r = i * 8 + (lane >> 3);
                r = r < last ? r : last;
                const uint4 t = load_stream16(P.D + ((int64_t)li.row0 + r) * I8_ROW_BYTES + (lane & 7) * 16);
                a_n[i] = i32x4{(int)t.x, (int)t.y, (int)t.z, (int)t.w};
            }
        } else {
            const char *src = P.D + grow * I8_ROW_BYTES + h * 16;
#pragma unroll
            for (int u = 0; u < I8_NU; ++u)
                a_n[u] = *reinterpret_cast<const i32x4 *>(src + u * 32);
        }
        s_n = P.ds[grow];
        it_next(li, p, off);
    };
    gload();

    i32x16 seed;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        int v = 0x4B000000;
        asm volatile("" : "+v"(v));
        seed[r] = v;
    }

    float m[NB];
    const int b_off = rho * I8D_QSTRIDE + h * 16; // this lane's B operand chunk 0 inside a block

    while (it_valid(ci)) {
        // the prefetched tile becomes the current one; its scales go through the wavefront's LDS area
        i32x4 a[I8_NU];
        if constexpr (LIN) {
#pragma unroll
            for (int i = 0; i < I8_NU; ++i)
                *reinterpret_cast<i32x4 *>(w_tile + (i * 8 + (lane >> 3)) * I8D_QSTRIDE + (lane & 7) * 16) = a_n[i];
        } else {
#pragma unroll
            for (int u = 0; u < I8_NU; ++u)
                a[u] = a_n[u];
        }
        const float s_cur = s_n;
        gload(); // next tile, in flight during this one
        if constexpr (LIN) {
#pragma unroll
            for (int u = 0; u < I8_NU; ++u)
                a[u] = *reinterpret_cast<const i32x4 *>(w_tile + b_off + u * 32);
        }
        float sc[16], bi[16];
        i8d_tile_scales(w_scale, w_bias, s_cur, rho, h, sc, bi);
        if (ci.t0 == 0) {
#pragma unroll
            for (int blk = 0; blk < NB; ++blk)
                m[blk] = neg_inf();
        }

        i8d_tile_blocks<NB>(a, sc, bi, q_tile, b_off, seed, m);

        if (ci.t0 + TILE_ROWS >= ci.len) { // last tile of the document
            float mm[NB];
#pragma unroll
            for (int blk = 0; blk < NB; ++blk)
                mm[blk] = fmaxf(m[blk], __shfl_xor(m[blk], 32));
            i8d_finish<NB>(P, mm, q_scale, nb, q_first, ci.doc, lane, rho);
        }
        it_next(ci, p, off);
    }
}

// ---------------------------------------------------------------------------------------
// the same for uniform corpora too small to give every wavefront documents of its own
// ---------------------------------------------------------------------------------------
// With a thousand long documents and a short query the corpus read is the cost, and a wavefront per document
// would leave most of the chip idle.  Here a workgroup takes documents one after the other and its eight
// wavefronts share each document's tiles (wavefront w the w-th eighth); the query tokens sit in LDS as above and
// every wavefront still streams its tiles HBM -> registers, one tile ahead, across document borders.  At the end
// of a document the eight partial maxima per query token meet in LDS (double-buffered, one barrier per
// document) and one wavefront, a different one each time, finishes the score.  Built for up to 16 column
// blocks (512 query tokens): beyond that the maxima of eight wavefronts no longer fit beside the queries in LDS.
template <int NB>
__global__ void __launch_bounds__(I8D_WAVES * 64) fwd_i8_split_kernel(I8Params P)
{
    const FwdParams &p = P.f;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int rho = lane & 31, h = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int group = blockIdx.x % p.n_groups;
    const int chunk = blockIdx.x / p.n_groups;
    const int q_first = group * p.qpg;
    const int nq = min(p.qpg, p.n_q - q_first);
    const int gb0 = q_first * p.bpq;
    const int nb = nq * p.bpq;

    // LDS: query rows and scales, per wavefront 32 token scales and 32 biases, then the partial maxima
    // comb[2][8 wavefronts][NB][32 columns]
    char *q_tile = smem;
    float *q_scale = reinterpret_cast<float *>(smem + NB * BLOCK_COLS * I8D_QSTRIDE);
    float *w_scale = q_scale + NB * BLOCK_COLS + w * 64;
    float *w_bias = w_scale + 32;
    float *comb = q_scale + NB * BLOCK_COLS + I8D_WAVES * 64;
    i8d_load_queries<NB>(P, q_tile, q_scale, gb0, nb, tid);
    __syncthreads();

    int64_t doc0_, doc1_;
    chunk_doc_range(p, chunk, doc0_, doc1_);
    if (doc0_ >= doc1_)
        return;
    const int doc0 = (int)doc0_, n_docs = (int)(doc1_ - doc0_);

    // this wavefront's tiles of every document: [t_lo, t_lo + cnt)
    const int n_tiles = (p.l_d + TILE_ROWS - 1) / TILE_ROWS;
    const int t_lo = w * (n_tiles / I8D_WAVES) + min(w, n_tiles % I8D_WAVES);
    const int cnt = n_tiles / I8D_WAVES + (w < n_tiles % I8D_WAVES ? 1 : 0);

    // the loader walks (document, tile) pairs in order; past the end it stays on the last pair
    i32x4 a_n[I8_NU];
    float s_n = 0.0f;
    int ld_doc = 0, ld_t = 0; // document (relative to doc0) and tile (relative to t_lo) of the next load
    auto gload = [&]() {
        if (cnt == 0)
            return;
        const int t0 = (t_lo + ld_t) * TILE_ROWS;
        int row = p.l_d - t0 - 1; // rows past the document re-read its last token
        row = rho < row ? rho : row;
        const int64_t grow = (int64_t)(doc0 + ld_doc) * p.l_d + t0 + row;
        const char *src = P.D + grow * I8_ROW_BYTES + h * 16;
#pragma unroll
        for (int u = 0; u < I8_NU; ++u)
            a_n[u] = *reinterpret_cast<const i32x4 *>(src + u * 32);
        s_n = P.ds[grow];
        if (ld_t + 1 < cnt) {
            ld_t += 1;
        } else if (ld_doc + 1 < n_docs) {
            ld_doc += 1;
            ld_t = 0;
        }
    };
    gload();

    i32x16 seed;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        int v = 0x4B000000;
        asm volatile("" : "+v"(v));
        seed[r] = v;
    }
    const int b_off = rho * I8D_QSTRIDE + h * 16;

    int par = 0;
    for (int d = 0; d < n_docs; ++d) {
        float m[NB];
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
            m[blk] = neg_inf();
        for (int t = 0; t < cnt; ++t) {
            i32x4 a[I8_NU];
#pragma unroll
            for (int u = 0; u < I8_NU; ++u)
                a[u] = a_n[u];
            const float s_cur = s_n;
            gload();
            float sc[16], bi[16];
            i8d_tile_scales(w_scale, w_bias, s_cur, rho, h, sc, bi);
            i8d_tile_blocks<NB>(a, sc, bi, q_tile, b_off, seed, m);
        }
        // partial maxima of this wavefront (the halved-negatives form keeps the order, so they can be compared
        // as they are)
        float *mine = comb + ((par * I8D_WAVES + w) * NB) * BLOCK_COLS;
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            float mm = fmaxf(m[blk], __shfl_xor(m[blk], 32));
            if (h == 0)
                mine[blk * BLOCK_COLS + rho] = mm;
        }
        __syncthreads();
        if (w == (d & (I8D_WAVES - 1))) {
            float mm[NB];
#pragma unroll
            for (int blk = 0; blk < NB; ++blk) {
                float x = neg_inf();
#pragma unroll
                for (int ww = 0; ww < I8D_WAVES; ++ww)
                    x = fmaxf(x, comb[((par * I8D_WAVES + ww) * NB + blk) * BLOCK_COLS + rho]);
                mm[blk] = x;
            }
            i8d_finish<NB>(P, mm, q_scale, nb, q_first, doc0 + d, lane, rho);
        }
        par ^= 1;
    }
}


template <int NB> static hipError_t launch_i8_split(const I8Params &P, int grid, hipStream_t s)
{
    hipLaunchKernelGGL((fwd_i8_split_kernel<NB>), dim3(grid), dim3(I8D_WAVES * 64), i8_split_lds(NB), s, P);
    return hipGetLastError();
}

template <int W> static hipError_t launch_i8(const I8Params &P, int grid, hipStream_t s)
{
    hipLaunchKernelGGL((fwd_i8_kernel<W>), dim3(grid), dim3(W * 64), 0, s, P, P.f.offsets);
    return hipGetLastError();
}

template <int NB> static hipError_t launch_i8_doc(const I8Params &P, int grid, hipStream_t s)
{
    if constexpr (NB <= I8D_LIN_BLOCKS)
        hipLaunchKernelGGL((fwd_i8_doc_kernel<NB, true>), dim3(grid), dim3(I8D_WAVES * 64), i8_doc_lin_lds(NB), s, P, P.f.offsets);
    else
        hipLaunchKernelGGL((fwd_i8_doc_kernel<NB, false>), dim3(grid), dim3(I8D_WAVES * 64), i8_doc_lds(NB), s, P, P.f.offsets);
    return hipGetLastError();
}

// More than 64 KB of dynamic LDS has to be allowed per kernel and device: every instantiation that needs it, for
// the current device (called once per device by the library's set-up).
template <int NB> static hipError_t allow_i8_lds()
{
    if (i8_doc_lds(NB) > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fwd_i8_doc_kernel<NB, false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)i8_doc_lds(NB));
        if (e != hipSuccess)
            return e;
    }
    if (NB <= 16 && i8_split_lds(NB) > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fwd_i8_split_kernel<(NB <= 16 ? NB : 16)>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)i8_split_lds(NB <= 16 ? NB : 16));
        if (e != hipSuccess)
            return e;
    }
    return hipSuccess;
}

hipError_t forward_i8_init_device()
{
    hipError_t e = hipSuccess;
    if ((e = allow_i8_lds<1>()) != hipSuccess || (e = allow_i8_lds<2>()) != hipSuccess || (e = allow_i8_lds<4>()) != hipSuccess ||
        (e = allow_i8_lds<8>()) != hipSuccess || (e = allow_i8_lds<16>()) != hipSuccess || (e = allow_i8_lds<24>()) != hipSuccess ||
        (e = allow_i8_lds<32>()) != hipSuccess)
        return e;
    return hipSuccess;
}

// offsets == nullptr: uniform corpus [b, l_d, 128]; otherwise packed [total_tokens, 128] with int32 offsets [b + 1]
hipError_t forward_i8_launch(const int8_t *Q, const float *qs, int n_q, int l_q, const int8_t *D, const float *ds,
                             const int32_t *offsets, int64_t b, int l_d, int64_t total_tokens, float *scores,
                             int64_t ld, int num_cu, hipStream_t stream)
{
    I8Params P;
    P.Q = reinterpret_cast<const char *>(Q);
    P.qs = qs;
    P.D = reinterpret_cast<const char *>(D);
    P.ds = ds;
    P.scores = scores;
    FwdParams &p = P.f;
    p = FwdParams{};
    p.offsets = offsets;
    p.scores = scores;
    p.b = b;
    p.ld = ld; // documents per row of `scores` (the whole corpus when b is a block of it)
    p.total_tokens = total_tokens;
    p.n_q = n_q;
    p.l_q = l_q;
    p.l_d = l_d;
    p.bpq = (l_q + BLOCK_COLS - 1) / BLOCK_COLS;
    p.n_pass = 1;
    const int64_t total_blocks = (int64_t)n_q * p.bpq;
    const int64_t units = offsets ? total_tokens : b; // what is split across chunks
    if (p.bpq > I8D_MAX_BLOCKS)
        return hipErrorNotSupported; // l_q > 1024: would need a second pass with an fp64 carry

    // Large corpora: document-stationary kernel, one run of documents per wavefront.
    if (b >= (int64_t)num_cu * I8D_WAVES * 2) {
        p.qpg = I8D_MAX_BLOCKS / p.bpq;
        if (p.qpg > n_q)
            p.qpg = n_q;
        p.n_groups = (n_q + p.qpg - 1) / p.qpg;
        int wgs = num_cu / p.n_groups; // per group; the query copy in LDS allows one workgroup per CU
        if (wgs < 1)
            wgs = 1;
        int64_t n_chunks = (int64_t)wgs * I8D_WAVES;
        p.unit_per_chunk = (units + n_chunks - 1) / n_chunks;
        if (!offsets)
            n_chunks = (units + p.unit_per_chunk - 1) / p.unit_per_chunk;
        p.n_chunks = (int)n_chunks;
        wgs = (int)((n_chunks + I8D_WAVES - 1) / I8D_WAVES);
        const int nb = p.qpg * p.bpq;
        const int grid = wgs * p.n_groups;
        if (nb <= 1) return launch_i8_doc<1>(P, grid, stream);
        if (nb <= 2) return launch_i8_doc<2>(P, grid, stream);
        if (nb <= 4) return launch_i8_doc<4>(P, grid, stream);
        if (nb <= 8) return launch_i8_doc<8>(P, grid, stream);
        if (nb <= 16) return launch_i8_doc<16>(P, grid, stream);
        if (nb <= 24) return launch_i8_doc<24>(P, grid, stream);
        return launch_i8_doc<32>(P, grid, stream);
    }

    // Uniform corpora of long documents, up to 16 column blocks per query and one or two groups of 16: the
    // wavefronts of a workgroup share each document (document-stationary like the kernel above, at any number
    // of documents)
    constexpr int SPLIT_BLOCKS = 16;
    if (!offsets && p.bpq <= SPLIT_BLOCKS && total_blocks <= 2 * SPLIT_BLOCKS && l_d >= I8D_WAVES * TILE_ROWS) {
        p.qpg = SPLIT_BLOCKS / p.bpq;
        if (p.qpg > n_q)
            p.qpg = n_q;
        p.n_groups = (n_q + p.qpg - 1) / p.qpg;
        const int nb = p.qpg * p.bpq;
        // about four workgroups per CU while the queries are small, one when their LDS copy is large
        int64_t n_chunks = ((int64_t)num_cu * (nb <= 4 ? 4 : 1) + p.n_groups - 1) / p.n_groups;
        if (n_chunks > b)
            n_chunks = b;
        p.unit_per_chunk = (b + n_chunks - 1) / n_chunks;
        n_chunks = (b + p.unit_per_chunk - 1) / p.unit_per_chunk;
        p.n_chunks = (int)n_chunks;
        const int grid = p.n_chunks * p.n_groups;
        if (nb <= 1) return launch_i8_split<1>(P, grid, stream);
        if (nb <= 2) return launch_i8_split<2>(P, grid, stream);
        if (nb <= 4) return launch_i8_split<4>(P, grid, stream);
        if (nb <= 8) return launch_i8_split<8>(P, grid, stream);
        return launch_i8_split<16>(P, grid, stream);
    }

    int w = 8;
    if (total_blocks <= 1 * I8_NCB)
        w = 1;
    else if (total_blocks <= 2 * I8_NCB)
        w = 2;
    else if (total_blocks <= 4 * I8_NCB)
        w = 4;
    const int group_blocks = w * I8_NCB;
    p.qpg = group_blocks / p.bpq;
    if (p.qpg > n_q)
        p.qpg = n_q;
    p.n_groups = (n_q + p.qpg - 1) / p.qpg;
    int64_t n_chunks = ((int64_t)num_cu * 2 + p.n_groups - 1) / p.n_groups;
    if (n_chunks < 8)
        n_chunks = 8;
    n_chunks = (n_chunks + 7) / 8 * 8;
    p.unit_per_chunk = (units + n_chunks - 1) / n_chunks;
    if (p.unit_per_chunk < 1)
        p.unit_per_chunk = 1;
    p.n_chunks = (int)n_chunks;
    int grid = p.n_groups * p.n_chunks;
    switch (w) {
    case 1: return launch_i8<1>(P, grid, stream);
    case 2: return launch_i8<2>(P, grid, stream);
    case 4: return launch_i8<4>(P, grid, stream);
    default: return launch_i8<8>(P, grid, stream);
    }
}

// ---------------------------------------------------------------------------------------
// per-token symmetric absmax quantiser: sixteen lanes per row, eight elements per lane
template <int CTRL> __device__ __forceinline__ float dpp_max(float v)
{
    return fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true)));
}

// round_half_even(x / s) clamped to [-127, 127], with the IEEE quotient
__device__ __forceinline__ int quant_code(float x, float s)
{
    float r = rintf(x / s);
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

// Sixteen lanes per row (8 elements each), four rows per wavefront and step.  The code of an element is
// round_half_even(fl32(x / s)).  One IEEE division per element would make the kernel VALU-bound (about twelve
// instructions each), so the quotient is formed from the row's correctly rounded reciprocal r = fl32(1 / s):
// q0 = fl32(x * r), e = x - q0 * s (exact in one fused multiply-add), q = fl32(q0 + e * r), which is the correctly
// rounded x / s (Markstein's division step: r is correctly rounded and q0 is within one ulp).  Rows whose scale has
// an all-ones significand (the one case the theorem leaves out) or lies outside [2^-60, 2^60] (where e could
// underflow), and all-zero rows, take the per-element division instead.
template <int DT>
__global__ void __launch_bounds__(256) quantize_rows_kernel(const char *X, int64_t rows, int8_t *out, float *scale)
{
    constexpr int EB = DT == MAXSIM_F32 ? 4 : 2;
    constexpr int ROWB = D_MODEL * EB;
    static_assert(D_MODEL == 128, "sixteen lanes x eight elements cover a row");
    const int lane = threadIdx.x & 63;
    const int grp = lane >> 4, c = lane & 15;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t r0 = (((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6) * 4; r0 < rows; r0 += n_waves * 4) {
        const int64_t row = r0 + grp;
        const bool live = row < rows;
        const int64_t rr = live ? row : rows - 1;
        // Rows are read once: non-temporal loads, each instruction taking whole lines (a lane of an fp32 row holds
        // elements 4c .. 4c+3 and 64+4c .. 64+4c+3, so that the sixteen lanes of a row read 256 contiguous bytes twice);
        // with the streaming stores of the codes 12 % over plain loads and stores (6.3 TB/s)
        float x[8];
        if constexpr (DT == MAXSIM_F32) {
            typedef float f32x4 __attribute__((ext_vector_type(4)));
            const f32x4 u = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(X + rr * ROWB + c * 16));
            const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(X + rr * ROWB + 256 + c * 16));
            x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w; x[4] = v.x; x[5] = v.y; x[6] = v.z; x[7] = v.w;
        } else {
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(X + rr * ROWB + c * 16));
            const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (DT == MAXSIM_F16) {
                    x[2 * i] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] & 0xffffu));
                    x[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] >> 16));
                } else {
                    x[2 * i] = __uint_as_float(w[i] << 16);
                    x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
                }
            }
        }
        float a = fmaxf(fmaxf(fabsf(x[0]), fabsf(x[1])), fabsf(x[2]));
        a = fmaxf(fmaxf(a, fabsf(x[3])), fabsf(x[4]));
        a = fmaxf(fmaxf(a, fabsf(x[5])), fabsf(x[6]));
        a = fmaxf(a, fabsf(x[7]));
        a = dpp_max<0xB1>(a);  // quad_perm [1,0,3,2]
        a = dpp_max<0x4E>(a);  // quad_perm [2,3,0,1]
        a = dpp_max<0x141>(a); // row_half_mirror
        a = dpp_max<0x140>(a); // row_mirror: all sixteen lanes of the row hold its absmax
        const float s = a / 127.0f;
        const uint32_t sb = __float_as_uint(s);
        const bool fast = s >= 0x1p-60f && s <= 0x1p60f && (sb & 0x7fffffu) != 0x7fffffu;
        int code[8];
        if (fast) {
#pragma clang fp contract(off)
            const float r = 1.0f / s;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float q0 = x[i] * r;
                float e = fmaf(-q0, s, x[i]);
                float q = rintf(fmaf(e, r, q0));
                code[i] = (int)fminf(fmaxf(q, -127.0f), 127.0f);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                code[i] = s == 0.0f ? 0 : quant_code(x[i], s);
        }
        uint2 packed;
        packed.x = (uint32_t)(code[0] & 0xff) | ((uint32_t)(code[1] & 0xff) << 8) | ((uint32_t)(code[2] & 0xff) << 16) |
                   ((uint32_t)code[3] << 24);
        packed.y = (uint32_t)(code[4] & 0xff) | ((uint32_t)(code[5] & 0xff) << 8) | ((uint32_t)(code[6] & 0xff) << 16) |
                   ((uint32_t)code[7] << 24);
        if (live) {
            // the codes are written once and not read by this kernel: streaming stores
            if constexpr (DT == MAXSIM_F32) {
                __builtin_nontemporal_store(packed.x, reinterpret_cast<uint32_t *>(out + row * D_MODEL + c * 4));
                __builtin_nontemporal_store(packed.y, reinterpret_cast<uint32_t *>(out + row * D_MODEL + 64 + c * 4));
            } else {
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 pv = {packed.x, packed.y};
                __builtin_nontemporal_store(pv, reinterpret_cast<u32x2 *>(out + row * D_MODEL + c * 8));
            }
            if (c == 0)
                scale[row] = s;
        }
    }
}

hipError_t quantize_launch(const void *X, int64_t rows, int dtype, int8_t *X_i8, float *scale, hipStream_t stream)
{
    int64_t blocks = (rows + 15) / 16; // 4 wavefronts x 4 rows per step
    if (blocks > 65536 * 4)
        blocks = 65536 * 4;
    const char *x = static_cast<const char *>(X);
    switch (dtype) {
    case MAXSIM_F32:
        hipLaunchKernelGGL((quantize_rows_kernel<MAXSIM_F32>), dim3((unsigned)blocks), dim3(256), 0, stream, x, rows, X_i8, scale);
        break;
    case MAXSIM_F16:
        hipLaunchKernelGGL((quantize_rows_kernel<MAXSIM_F16>), dim3((unsigned)blocks), dim3(256), 0, stream, x, rows, X_i8, scale);
        break;
    default:
        hipLaunchKernelGGL((quantize_rows_kernel<MAXSIM_BF16>), dim3((unsigned)blocks), dim3(256), 0, stream, x, rows, X_i8, scale);
        break;
    }
    return hipGetLastError();
}

} // namespace maxsim
