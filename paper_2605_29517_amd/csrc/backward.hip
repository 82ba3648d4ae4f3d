// MaxSim backward through the stored argmax (Eqs. 2-3 of the paper) for gfx950, plus the
// in-batch-negatives cross-entropy gradient helper.
//
// dQ (Eq. 2) is a collision-free gather, partitioned by documents so that every XCD's L2 serves its own
// part of the corpus; the partial sums are combined in a fixed order.
//
// dD (Eq. 3) is the contended side.  The paper resolves it either with atomics or with an
// inverse-grid CSR built by bincount / cumsum / argsort.  Here every dD row has exactly one
// owner instead: a workgroup owns a block of consecutive rows of the (packed) corpus, sorts the edges that land
// in the block by row inside LDS (filter, count, scan, stable placement) and each of its wavefronts walks
// the lists of its rows, one row after the other, all 64 lanes on one edge.  No atomics, no zero-fill
// pass over dD, and the summation order is fixed (a row's edges by increasing edge id), so the result is
// bitwise reproducible and equal to that of the explicit CSR of the paper, which is there as an opt-in
// (built in global memory, then walked the same way).
#include <type_traits>

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
    int d;                  // embedding width: a multiple of 8, columns are handled in slabs of 128
};

constexpr int SLAB = 128; // columns a wavefront handles (blockIdx.y selects the slab of wider rows)

// n / divisor for 0 <= n < 2^31 as (n * mul) >> shift (round-up method: shift = 31 + ceil(log2(divisor)))
struct Magic {
    uint32_t mul;
    int shift;
};
static Magic magic_u31(uint32_t divisor)
{
    int lg = 0;
    while (lg < 31 && (uint32_t(1) << lg) < divisor)
        ++lg;
    Magic m;
    m.shift = 31 + lg;
    m.mul = (uint32_t)((((uint64_t)1 << m.shift) + (uint64_t)divisor - 1) / (uint64_t)divisor);
    return m;
}
__device__ __forceinline__ uint32_t magic_div(uint32_t n, Magic m) { return (uint32_t)(((uint64_t)n * m.mul) >> m.shift); }

// f(integral_constant<int, I>) for I = BEGIN .. END-1, unrolled at compile time (for builtins that want constants)
// Which block of rows a workgroup takes.  Workgroup ids are dealt round-robin to the 8 XCDs and, inside an XCD, (at
// first) round-robin to its CUs.  Every XCD gets a contiguous range of blocks (the blocks of one document read the
// same argmax column: one L2), and inside the XCD consecutive ids are a CU's share apart, so that blocks that recur
// with a period -- the first rows of every document, which collect the most edges -- are spread over the CUs
// instead of meeting on one (a plain numbering sent all of them to one XCD, or to every fourth CU).
struct BlockOrder {
    int n_blocks, per_xcd, per_cu, cus;
    unsigned grid;
};
static BlockOrder block_order(int64_t n_blocks, int num_cu)
{
    BlockOrder o;
    o.n_blocks = (int)n_blocks;
    o.cus = num_cu >= 8 ? num_cu / 8 : 1;
    o.per_xcd = (int)((n_blocks + 7) / 8);
    o.per_cu = (o.per_xcd + o.cus - 1) / o.cus;
    o.grid = 8u * (unsigned)o.cus * (unsigned)o.per_cu;
    return o;
}
__device__ __forceinline__ int ordered_block(const BlockOrder &o, unsigned id) // -1: nothing to do
{
    const int i = (int)(id >> 3);
    const int r = i / o.cus, c = i - r * o.cus;
    const int y = c * o.per_cu + r;
    const int blk = (int)(id & 7) * o.per_xcd + y;
    return y < o.per_xcd && blk < o.n_blocks ? blk : -1;
}

// Gradient rows are written once and not read again by the kernel that writes them: streaming stores, so that they
// do not push the argmax columns, the document rows and the Q rows, which are read again and again, out of the L2
__device__ __forceinline__ void store_streaming2(float *dst, float x, float y)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {x, y};
    __builtin_nontemporal_store(v, reinterpret_cast<f32x2 *>(dst));
}

template <int BEGIN, int END, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (BEGIN < END) {
        f(std::integral_constant<int, BEGIN>());
        static_for<BEGIN + 1, END>(f);
    }
}

// 8 consecutive elements of a row: the raw load and its decoding to fp32, apart, so that several loads can be in flight
struct Raw8 {
    uint4 a, b;
};
template <int DT> __device__ __forceinline__ void load_raw8(const char *p, Raw8 &r)
{
    r.a = *reinterpret_cast<const uint4 *>(p);
    if (DT == MAXSIM_F32)
        r.b = *reinterpret_cast<const uint4 *>(p + 16);
}
template <int DT> __device__ __forceinline__ void decode8(const Raw8 &r, float (&v)[8])
{
    if (DT == MAXSIM_F32) {
        v[0] = __uint_as_float(r.a.x); v[1] = __uint_as_float(r.a.y); v[2] = __uint_as_float(r.a.z); v[3] = __uint_as_float(r.a.w);
        v[4] = __uint_as_float(r.b.x); v[5] = __uint_as_float(r.b.y); v[6] = __uint_as_float(r.b.z); v[7] = __uint_as_float(r.b.w);
    } else {
        const uint32_t w[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
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

// ---------------------------------------------------------------------------------------
// dQ[q,i,:] = sum_j g[q,j] * D[j, A[q,j,i], :]                                      (Eq. 2)
//
// The documents are cut into n_part contiguous partitions and workgroup k works on partition k % n_part.
// Workgroup ids are dealt round-robin to the 8 XCDs, so with n_part = 8 every XCD gathers rows from its own
// eighth of the corpus only and its L2 fetches each document row once (a wavefront per query token over the whole
// corpus makes every XCD pull most of D: 6.6 times the corpus at 256 x 256 x 1024).  A wavefront owns four
// query tokens (one per group of sixteen lanes, 8 columns per lane) and adds its partition's documents in
// order; the n_part partial sums of a query token are then added in partition order by bwd_dq_combine_kernel
// (fixed order: bitwise reproducible).  n_part = 1 writes dQ directly.
// ---------------------------------------------------------------------------------------
constexpr int DQ_SB = 16;   // documents per index fetch: one per lane of a group of sixteen
constexpr int DQ_AHEAD = 4; // documents between the rows being gathered and the rows being read ahead in order

// TPG = query tokens per group of sixteen lanes: 1, or 4 consecutive tokens of one query (l_q a multiple of 4: their
// argmax entries are one 16-byte load and they share the weight).  With 4 the whole grid is resident at once at
// 8192 query tokens, so the wavefronts of an XCD sweep the partition's documents side by side and a document row
// that one group brought into the L2 is found there by the others.
template <int DT, int TPG>
__global__ void __launch_bounds__(256) bwd_dq_kernel(BwdParams p, float *out, int n_part, int64_t docs_per_part)
{
    constexpr int EB = Elem<DT>::BYTES;
    constexpr int U = DT == MAXSIM_F32 ? 4 : 8; // document rows per batch of loads (two batches in flight)
    constexpr int DPB = U / TPG > 0 ? U / TPG : 1; // documents per batch
    static_assert(TPG == 1 || TPG == 4, "tokens per group");
    static_assert(DPB * TPG == U, "a batch holds whole documents");
    const int lane = threadIdx.x & 63;
    const int grp = lane >> 4; // which of the wavefront's four groups
    const int c = lane & 15;   // which 8 columns of the slab
    const int part = (int)(blockIdx.x % (unsigned)n_part);
    const int64_t wave = (int64_t)(blockIdx.x / (unsigned)n_part) * 4 + (threadIdx.x >> 6);
    const int64_t nql = (int64_t)p.n_q * p.l_q;
    if (wave * 4 * TPG >= nql)
        return;
    const int64_t n0 = (wave * 4 + grp) * TPG; // the group's first query token
    const int col = (int)blockIdx.y * SLAB + c * 8;
    const bool col_ok = col < p.d;
    const int64_t row_bytes = (int64_t)p.d * EB;
    const char *Dcol = p.D + (int64_t)(col_ok ? col : 0) * EB; // lanes past the row's end re-read its first columns
    const int64_t j0 = (int64_t)part * docs_per_part;
    const int64_t j1 = j0 + docs_per_part < p.b ? j0 + docs_per_part : p.b;
    const int64_t nn = n0 < nql ? n0 : nql - TPG; // a group past the last token repeats the last one (nothing is stored)
    const int q = (int)(nn / p.l_q);
    const int i = (int)(nn - (int64_t)q * p.l_q);
    const int32_t *Aq = p.A + (int64_t)q * p.b * p.l_q + i; // A[q, 0, i]
    const float *gq = p.g + (int64_t)q * p.b;               // g[q, 0]

    float acc[TPG][8];
#pragma unroll
    for (int t = 0; t < TPG; ++t)
#pragma unroll
        for (int k = 0; k < 8; ++k)
            acc[t][k] = 0.0f;
    if (j0 < j1) {
        // Lane c of a group fetches, for document jb + c, the winning tokens and the weight and turns them into the
        // rows' offsets in D (in units of 16 bytes: D is below 64 GiB, checked by the caller; the offset of a row that
        // is not to be added is that of row 0) and a weight that is 0 where nothing is added; the group then takes
        // them from each other's registers (a swizzle inside each half of the wavefront), so that one memory round trip
        // brings the indices of 16 documents and a row costs a lane exchange or two, one address add, its load and
        // its eight multiply-adds.
        const uint32_t row16 = (uint32_t)(row_bytes >> 4);
        uint32_t o[TPG];
        float g;
        auto fetch = [&](int64_t jb) {
            const bool in = jb + c < j1;
            const int64_t j = in ? jb + c : j1 - 1;
            int64_t first;
            int len;
            if (p.offsets) {
                first = p.offsets[j];
                len = p.offsets[j + 1] - (int)first;
            } else {
                first = j * p.l_d;
                len = p.l_d;
            }
            int tt[TPG];
            if constexpr (TPG == 4) {
                const int4 v = *reinterpret_cast<const int4 *>(Aq + j * p.l_q);
                tt[0] = v.x;
                tt[1] = v.y;
                tt[2] = v.z;
                tt[3] = v.w;
            } else {
                tt[0] = Aq[j * p.l_q];
            }
            const float gv = gq[j];
            g = in ? gv : 0.0f;
#pragma unroll
            for (int t = 0; t < TPG; ++t) {
                // also guards bad offsets; the row's weight is the document's unless the row is row 0 by default
                const bool ok = tt[t] >= 0 && tt[t] < len && first >= 0 && first + tt[t] < p.total_tokens;
                o[t] = ok ? (uint32_t)(first + tt[t]) * row16 : 0xffffffffu;
            }
        };
        // With four tokens per group the whole grid is resident and the wavefronts of a partition walk its documents
        // side by side, so (uniform corpora) they also read the documents a few steps ahead in order, one kilobyte
        // per wavefront and step (wavefront k of the partition the k-th kilobyte of the step's DPB documents): most
        // rows then reach the XCD's L2 as part of a stream before they are gathered.  It changes no time that could be
        // measured (the gathers are bound by the L2's delivery rate, not by HBM) but takes a quarter off the traffic
        // between the L2s and the fabric (137 -> 106 MB at 256 x 256 x 1024).
        const bool ahead = TPG == 4 && !p.offsets;
        const int64_t step_bytes = (int64_t)DPB * p.l_d * row_bytes;
        const char *t_safe = p.D + j0 * p.l_d * row_bytes;    // a valid address of the partition
        const char *t_lim = p.D + j1 * p.l_d * row_bytes - 16; // last 16 bytes of the partition
        int64_t t_at = (wave % ((int64_t)(gridDim.x / (unsigned)n_part) * 4)) * 1024 + lane * 16;
        const char *tp = t_safe + (int64_t)DQ_AHEAD * p.l_d * row_bytes + (t_at < step_bytes - 16 ? t_at : step_bytes - 16);
        auto touch = [&]() {
            const char *at = (ahead && tp <= t_lim) ? tp : t_safe;
            tp += step_bytes;
            return *reinterpret_cast<const uint4 *>(at);
        };
        fetch(j0);
        for (int64_t jb = j0; jb < j1; jb += DQ_SB) {
            uint32_t co[TPG];
#pragma unroll
            for (int t = 0; t < TPG; ++t)
                co[t] = o[t];
            const float cg = g;
            fetch(jb + DQ_SB); // the next 16 documents' indices travel while these documents' rows do
            Raw8 raw[2][U];
            float gc[2][U];
            auto issue = [&](auto batch_tag, Raw8(&dst)[U], float(&w)[U]) {
                constexpr int m0 = decltype(batch_tag)::value * DPB;
                static_for<0, U>([&](auto u_tag) {
                    constexpr int u = decltype(u_tag)::value;
                    constexpr int t = u % TPG;
                    constexpr int m = m0 + u / TPG;
                    // ds_swizzle, bit mode (and_mask | or_mask << 5 | xor_mask << 10 on the lane id inside each half of
                    // the wavefront): keep which group of sixteen, take lane m of it
                    constexpr int pat = 0x10 | ((m & 15) << 5);
                    const uint32_t off16 = (uint32_t)__builtin_amdgcn_ds_swizzle((int)co[t], pat);
                    const float gg = __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(cg), pat));
                    w[u] = off16 == 0xffffffffu ? 0.0f : gg;
                    load_raw8<DT>(Dcol + ((uint64_t)(off16 == 0xffffffffu ? 0u : off16) << 4), dst[u]);
                });
            };
            auto consume = [&](const Raw8(&src)[U], const float(&w)[U]) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    float v[8];
                    decode8<DT>(src[u], v);
#pragma unroll
                    for (int k = 0; k < 8; ++k)
                        acc[u % TPG][k] = fmaf(w[u], v[k], acc[u % TPG][k]);
                }
            };
            // batches of DPB documents, two in flight; documents past the partition carry weight 0 (their rows are
            // the last document's)
            constexpr int NBATCH = DQ_SB / DPB;
            issue(std::integral_constant<int, 0>(), raw[0], gc[0]);
            static_for<0, NBATCH>([&](auto b_tag) {
                constexpr int bi = decltype(b_tag)::value;
                uint4 touched = make_uint4(0, 0, 0, 0);
                if constexpr (TPG == 4)
                    touched = touch();
                if constexpr (bi + 1 < NBATCH)
                    issue(std::integral_constant<int, bi + 1>(), raw[(bi + 1) & 1], gc[(bi + 1) & 1]);
                consume(raw[bi & 1], gc[bi & 1]);
                if constexpr (TPG == 4)
                    asm volatile("" ::"v"(touched.x), "v"(touched.y), "v"(touched.z), "v"(touched.w)); // the load is the point
            });
        }
    }
    if (col_ok) {
#pragma unroll
        for (int t = 0; t < TPG; ++t) {
            if (n0 + t < nql) {
                float *dst = out + ((int64_t)part * nql + n0 + t) * p.d + col;
                // (ordinary stores: the combine kernel reads these back; streaming stores cost 5 us at 256 x 256 x 1024)
                reinterpret_cast<float4 *>(dst)[0] = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
                reinterpret_cast<float4 *>(dst)[1] = make_float4(acc[t][4], acc[t][5], acc[t][6], acc[t][7]);
            }
        }
    }
}

// dQ = part[0] + part[1] + ... + part[n_part - 1], in that order; n4 = float4s per partial = n_q * l_q * d / 4
__global__ void __launch_bounds__(256) bwd_dq_combine_kernel(const float4 *part, float4 *dQ, int64_t n4, int n_part)
{
    for (int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x; x < n4; x += (int64_t)gridDim.x * 256) {
        float4 s = part[x];
        for (int k = 1; k < n_part; ++k) {
            const float4 v = part[(int64_t)k * n4 + x];
            s.x += v.x;
            s.y += v.y;
            s.z += v.z;
            s.w += v.w;
        }
        dQ[x] = s;
    }
}

// ---------------------------------------------------------------------------------------
// dD[j,t,:] = sum over edges (q,i) with A[q,j,i] = t of g[q,j] * Q[q,i,:]              (Eq. 3)
//
// A workgroup owns R = 8 * RPW consecutive rows of the (packed) corpus, whichever documents they belong to;
// wavefront w owns the rows row0 + 8 * s + w (s = 0 .. RPW-1; neighbouring rows, often hot together, go to
// different wavefronts).  For every document with rows in the block and every round of DW_COL entries of that
// document's argmax column:
//   (1) filter: each wavefront reads a contiguous eighth of the round, keeps the entries that land in the block
//       (one subtraction and one unsigned compare per entry), compacted by ballot in entry order, and counts them
//       per row into its own histogram (LDS);
//   (2) scan: the histograms become list starts per row and a write cursor per (row, filtering wavefront);
//   (3) place: each wavefront ranks its kept entries, 64 at a time, among equal rows by log2(R) ballots and
//       writes the entry numbers to the row lists -- a stable counting sort, so a row's list is in entry order and
//       the lists of a wavefront's rows are contiguous;
//   (4) walk: every wavefront walks its contiguous range of the sorted entries, ALL 64 lanes on one edge at a
//       time (two columns per lane): per 64 edges one vector step looks up (Q row, weight), then the edges are
//       applied in order with 8 to 16 Q-row loads in flight; the wavefront's rows stay in registers (two per row and
//       lane, selected by a scalar index) over all the documents and rounds of the block and are written once, at
//       the end (rows without edges as zeros).
// Every row has one owner and its edges are added in entry order with one fused multiply-add each, starting
// from zero: the same bits as the explicit CSR walk, on every run.  No atomics decide anything, no zero-fill
// pass.  Columns beyond 128 are further slabs (blockIdx.y) that repeat the integer work.
// ---------------------------------------------------------------------------------------
constexpr int DD_WAVES = 8;
constexpr int DW_COL = 8192;              // entries per round: an entry's number within the round fits 16 bits
constexpr int DD_BATCH = 8;                // Q rows per batch of loads (two batches in flight while edges are applied)

// two consecutive elements of a row as loaded (decoded when they are used, so that an edge in flight holds one
// register for 16-bit rows)
template <int DT> struct RawPair {
    typedef uint32_t type;
};
template <> struct RawPair<MAXSIM_F32> {
    typedef float type __attribute__((ext_vector_type(2)));
};
template <int DT> __device__ __forceinline__ void decode_pair(typename RawPair<DT>::type r, float &x0, float &x1)
{
    if constexpr (DT == MAXSIM_F32) {
        x0 = r.x;
        x1 = r.y;
    } else if constexpr (DT == MAXSIM_F16) {
        x0 = (float)__builtin_bit_cast(_Float16, (uint16_t)(r & 0xffffu));
        x1 = (float)__builtin_bit_cast(_Float16, (uint16_t)(r >> 16));
    } else {
        x0 = __uint_as_float(r << 16);
        x1 = __uint_as_float(r & 0xffff0000u);
    }
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

template <int N> struct RowVec {
    typedef float type __attribute__((ext_vector_type(N)));
};

// Raw buffer descriptor over the Q tensor (base, size in bytes; untyped dwords): loads take a per-lane byte
// offset from a vector register plus a per-edge byte offset from a scalar register, so an edge's row costs one
// lane read and one load instruction; offsets past the size read as zero instead of faulting.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t q_resource(const char *Q, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(Q), 0, (int)bytes, 0x00020000);
}
template <int DT> __device__ __forceinline__ typename RawPair<DT>::type load_raw_pair(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_off, uint32_t row_off)
{
    if constexpr (DT == MAXSIM_F32) {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(typename RawPair<DT>::type,
                                  (u32x2)__builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)lane_off, (int)row_off, 0));
    } else {
        return __builtin_amdgcn_raw_buffer_load_b32(rsrc, (int)lane_off, (int)row_off, 0);
    }
}

// The walk shared by bwd_dd_kernel and csr_apply_kernel.  Edges k_lo .. k_hi of an array sorted by row belong to
// NROWS consecutive lists; lane s of `boundv` holds where the list of row slot s starts (s = 0 .. NROWS, the last
// one = k_hi).  rx[s], ry[s] are the lane's two columns of row slot s.  Per 64 edges (one per lane) a vector step
// finds the edge's row slot by a binary search over boundv and looks up the Q row and the weight
// (`lookup(k, valid, slot, n, gv)`; the array may be a virtual one that the lookup maps onto the real lists); the edges are then applied one after the other by all 64 lanes, 8 Q-row loads in flight while the
// 8 before them are added (two register sets; batches of 16 cost 15 more registers and, at seven wavefronts per SIMD
// in csr_apply_kernel, were 20 % slower); the row's byte offset reaches the load through a scalar register, the
// weights come four at a time from the wavefront's LDS words.  The running row lives in two fixed registers and moves to / from its slot (register
// index from a scalar) at the edges where a ballot says the row changes, so the per-edge work is a compare, one
// lane read, a load, a quarter of an LDS read and two fused multiply-adds, and the chain holds no global memory
// operation besides the loads.
// Edges past the last one (the rest of the last batch) carry weight 0; their Q rows are rows of other lists, or,
// past the end of the edge array, whatever offset the lookup makes of it: the buffer descriptor turns a read
// outside Q into zeros.
template <int DT, int NROWS, typename Lookup>
__device__ __forceinline__ void walk_rows(__amdgpu_buffer_rsrc_t rsrc, uint32_t row_bytes, int lane, uint32_t lane_off, int k_lo,
                                          int k_hi, int boundv, float *gstage, Lookup lookup, typename RowVec<NROWS>::type &rx,
                                          typename RowVec<NROWS>::type &ry)
{
    typedef typename RawPair<DT>::type raw_t;
    static_assert(DD_BATCH == 8, "eight batches per vector step");
    constexpr int NB = 64 / DD_BATCH;
    if (k_lo >= k_hi)
        return;
    auto look = [&](int k0, uint32_t &off, float &gv, int &sv) {
        const int kk = k0 + lane;
        int s = 0; // the largest slot whose list starts at or before kk
#pragma unroll
        for (int step = NROWS / 2; step > 0; step >>= 1) {
            const int bnd = __shfl(boundv, s + step);
            s = bnd <= kk ? s + step : s;
        }
        sv = s;
        uint32_t n;
        lookup(kk, kk < k_hi, s, n, gv);
        off = n * row_bytes; // < 2^32 (checked by the caller)
    };
    auto issue = [&](raw_t(&dst)[DD_BATCH], uint32_t offv, int e0) {
#pragma unroll
        for (int u = 0; u < DD_BATCH; ++u)
            dst[u] = load_raw_pair<DT>(rsrc, lane_off, (uint32_t)__builtin_amdgcn_readlane((int)offv, e0 + u));
    };
    uint32_t o_cur, o_nxt;
    float g_nxt;
    int sv_cur, sv_nxt;
    raw_t xb[2][DD_BATCH];
    // the weights of a step's 64 edges go through this wavefront's own LDS words (two sets of 64), from where four at a
    // time are read back into all lanes: a broadcast read instead of a lane read per edge
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    int gpar = 0;
    look(k_lo, o_cur, g_nxt, sv_cur);
    gstage[lane] = g_nxt;
    issue(xb[0], o_cur, 0);
    int s_now = __builtin_amdgcn_readlane(sv_cur, 0);
    int s_carry = s_now;
    float ax = rx[s_now], ay = ry[s_now];
    // One batch of edges: the lane reads use compile-time lanes; edges past k_hi have weight 0.
    auto consume = [&](const raw_t(&src)[DD_BATCH], int e0, uint64_t &bmask, int &next_b) {
        f32x4 g4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int u = 0; u < DD_BATCH; ++u) {
            const int e = e0 + u;
            if (e == next_b) {
                const int s_new = __builtin_amdgcn_readlane(sv_cur, e);
                rx[s_now] = ax;
                ry[s_now] = ay;
                ax = rx[s_new];
                ay = ry[s_new];
                s_now = s_new;
                bmask &= bmask - 1;
                next_b = bmask ? (int)__builtin_ctzll(bmask) : 64;
            }
            if ((u & 3) == 0)
                g4 = *reinterpret_cast<const f32x4 *>(gstage + gpar * 64 + e);
            const float gg = g4[u & 3];
            float x0, x1;
            decode_pair<DT>(src[u], x0, x1);
            ax = fmaf(gg, x0, ax);
            ay = fmaf(gg, x1, ay);
        }
    };
    // Every step issues the loads of the next batch, then adds the current one; the loop is left (never
    // rejoined) once the batch that holds the last edge has been added, so the only loads wasted are one batch.
    for (int k0 = k_lo;; k0 += 64) {
        look(k0 + 64, o_nxt, g_nxt, sv_nxt);
        gstage[(gpar ^ 1) * 64 + lane] = g_nxt;
        int prev = __shfl_up(sv_cur, 1);
        prev = lane == 0 ? s_carry : prev;
        uint64_t bmask = __ballot(sv_cur != prev); // edges that begin another row's list
        int next_b = bmask ? (int)__builtin_ctzll(bmask) : 64;
#define WALK_STEP(bi)                                                                                                  \
    issue(xb[((bi) + 1) & 1], (bi) + 1 < NB ? o_cur : o_nxt, (((bi) + 1) % NB) * DD_BATCH);                           \
    consume(xb[(bi)&1], (bi)*DD_BATCH, bmask, next_b);                                                                \
    if (k0 + ((bi) + 1) * DD_BATCH >= k_hi)                                                                           \
        break;
        WALK_STEP(0)
        WALK_STEP(1)
        WALK_STEP(2)
        WALK_STEP(3)
        WALK_STEP(4)
        WALK_STEP(5)
        WALK_STEP(6)
        WALK_STEP(7)
#undef WALK_STEP
        s_carry = __builtin_amdgcn_readlane(sv_cur, 63);
        o_cur = o_nxt;
        gpar ^= 1;
        sv_cur = sv_nxt;
    }
    rx[s_now] = ax;
    ry[s_now] = ay;
}

template <int DT, int RPW, int W>
__global__ void __launch_bounds__(W * 64) bwd_dd_kernel(BwdParams p, OffsetsPtr off, Magic lq_magic, Magic ld_magic, int dq64,
                                                        int di64, BlockOrder order)
{
    constexpr int R = W * RPW;          // rows of the block
    constexpr int WBITS = W == 16 ? 4 : 3;
    constexpr int RBITS = WBITS + (RPW == 16 ? 4 : RPW == 8 ? 3 : 2);
    constexpr int SEG = DW_COL / W;     // entries each wavefront filters per round
    constexpr int KPL = (R + 63) / 64;  // keys per lane in the scan
    static_assert(RPW == 16 || RPW == 8 || RPW == 4, "rows per wavefront");
    static_assert(W == 8 || W == 16, "wavefronts per workgroup");
    constexpr int EB = Elem<DT>::BYTES;
    // seg and hist live from the filter to the placement, list and start from the placement to the end of the walk;
    // the weights staged during the walk reuse the first words of the wavefront's own seg row (dead by then).
    static_assert(SEG >= 128, "a wavefront's staged weights fit in its seg row");
    __shared__ __attribute__((aligned(16))) uint32_t seg[W][SEG]; // per filtering wavefront: kept entries, (number in round) | row << 16
    __shared__ uint16_t list[DW_COL];          // entry numbers by key (= owner wavefront * RPW + slot), in entry order
    __shared__ int hist[W][R];          // per filtering wavefront: entries per block row, then write cursors
    __shared__ int start[R + 1];               // list of key k: list[start[k] .. start[k + 1])
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int blk = ordered_block(order, blockIdx.x);
    if (blk < 0)
        return;
    const int64_t row0 = (int64_t)blk * R;
    const int64_t row_end = min(row0 + R, p.total_tokens);
    const int col = (int)blockIdx.y * SLAB + 2 * lane;
    const bool col_ok = col < p.d;
    // lanes past the row's end re-read its first columns and store nothing
    const uint32_t lane_off = (uint32_t)((col_ok ? 2 * lane : 0) + (int)blockIdx.y * SLAB) * EB;
    const uint32_t row_bytes = (uint32_t)p.d * EB;
    const __amdgpu_buffer_rsrc_t rsrc = q_resource(p.Q, (uint32_t)p.n_q * (uint32_t)p.l_q * row_bytes); // < 2^32 (checked by the caller)

    int64_t j_first, j_last;
    if (p.offsets) {
        j_first = lower_bound_offsets(p.offsets, p.b, row0 + 1) - 1;
        j_last = lower_bound_offsets(p.offsets, p.b, row_end) - 1;
        j_first = j_first < 0 ? 0 : j_first; // only offsets that break their contract get here
        j_last = j_last > p.b - 1 ? p.b - 1 : j_last;
    } else { // rows are below 2^31 (checked by the caller)
        j_first = magic_div((uint32_t)row0, ld_magic);
        j_last = magic_div((uint32_t)(row_end - 1), ld_magic);
    }

    // the gradient rows of this wavefront (slot s = row row0 + W * s + w), two columns per lane
    typename RowVec<RPW>::type rx, ry;
#pragma unroll
    for (int s = 0; s < RPW; ++s) {
        rx[s] = 0.0f;
        ry[s] = 0.0f;
    }

    const int n_entries = p.n_q * p.l_q; // < 2^31 (checked by the caller)
    // argmax entries 64 apart in a document's column: dq64 = 64 / l_q queries and di64 = 64 % l_q tokens (one more query
    // if the token wraps)
    const int64_t inc_plain = (int64_t)dq64 * p.b * p.l_q + di64;
    const int64_t inc_wrap = inc_plain + (int64_t)p.b * p.l_q - p.l_q;
    for (int64_t j = j_first; j <= j_last; ++j) {
        int64_t first;
        int len;
        if (p.offsets) {
            first = off[j];
            len = off[j + 1] - (int)first;
        } else {
            first = j * p.l_d;
            len = p.l_d;
        }
        if (len <= 0)
            continue;
        const int t_base = (int)(row0 - first); // document-local index of the block's first row (may be negative)
        // rows of the block that belong to document j: [lo_rel, hi_rel)
        const int lo_rel = (int)max((int64_t)0, first - row0);
        const int hi_rel = (int)min(row_end - row0, first + len - row0);
        if (hi_rel <= lo_rel)
            continue; // only offsets that break their contract get here

        for (int64_t c64 = 0; c64 < n_entries; c64 += DW_COL) { // 64-bit: n_entries may be within DW_COL of 2^31
            const int c0 = (int)c64;
            const int cn = min(DW_COL, n_entries - c0);
            __syncthreads(); // the previous round's lists have been walked
            for (int x = tid; x < W * R; x += W * 64)
                (&hist[0][0])[x] = 0;
            __syncthreads();
            int kept = 0;
            {
                // (1) entry n = c0 + x -> (q, i); all loads are issued before the first result is used.  The entry 64
                // further on is dq queries and di tokens ahead: its address is one of two increments away.
                constexpr int PER = SEG / 64;
                int x = w * SEG + lane;
                // (opaque to the optimiser: it would otherwise keep x + 64 k for all k in registers across the rounds)
                asm volatile("" : "+v"(x));
                const uint32_t n = (uint32_t)c0 + (uint32_t)x; // entries past the end of the column are masked below
                const uint32_t q0 = magic_div(n < (uint32_t)n_entries ? n : 0u, lq_magic);
                int i = (int)((n < (uint32_t)n_entries ? n : 0u) - q0 * (uint32_t)p.l_q);
                const int32_t *ptr = p.A + ((int64_t)q0 * p.b + j) * p.l_q + i;
                int t[PER];
                if (cn == DW_COL && di64 == 0) { // l_q divides 64: the same increment every time
#pragma unroll
                    for (int k = 0; k < PER; ++k) {
                        t[k] = *ptr;
                        ptr += inc_plain;
                    }
                } else if (cn == DW_COL) {
#pragma unroll
                    for (int k = 0; k < PER; ++k) {
                        t[k] = *ptr;
                        i += di64;
                        const bool wrap = i >= p.l_q;
                        i -= wrap ? p.l_q : 0;
                        ptr += wrap ? inc_wrap : inc_plain;
                    }
                } else {
                    const int32_t *const ptr0 = ptr;
#pragma unroll
                    for (int k = 0; k < PER; ++k) {
                        const bool live = (x + k * 64) < cn;
                        const int v = *(live ? ptr : ptr0); // past the end of the column: a harmless re-read
                        t[k] = live ? v : -1;
                        i += di64;
                        const bool wrap = i >= p.l_q;
                        i -= wrap ? p.l_q : 0;
                        ptr += wrap ? inc_wrap : inc_plain;
                    }
                }
                // An entry lands in the block iff y = t - (t_base + lo_rel), taken modulo 2^32, is below the number of
                // the document's rows in the block (that also rules out t < 0, t >= len and the -1 of masked entries);
                // y counts rows from the document's first row in the block.
                const uint32_t y_base = (uint32_t)t_base + (uint32_t)lo_rel;
                const uint32_t n_rows = (uint32_t)(hi_rel - lo_rel);
                int *const hist_w = &hist[w][lo_rel];
#pragma unroll
                for (int k = 0; k < PER; ++k) {
                    const uint32_t y = (uint32_t)t[k] - y_base;
                    const bool in = y < n_rows;
                    const unsigned long long mask = __ballot(in);
                    const int before =
                        __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0));
                    if (in) {
                        seg[w][kept + before] = (uint32_t)(x | (k * 64)) | (y << 16);
                        atomicAdd(hist_w + y, 1);
                    }
                    kept += __builtin_popcountll(mask);
                }
            }
            __syncthreads();
            if (w == 0) {
                // (2) keys lane, lane + 64, ... (key = owner wavefront * RPW + slot, i.e. block row slot * W + owner): list
                // starts in key order, then each filtering wavefront's cursor within the list; hist is indexed by block row
                int tot[KPL], cur[KPL];
#pragma unroll
                for (int u = 0; u < KPL; ++u) {
                    const int r = lane + 64 * u;
                    const int rel = (r & (RPW - 1)) * W + r / RPW;
                    tot[u] = 0;
                    if (r < R)
                        for (int sw = 0; sw < W; ++sw)
                            tot[u] += hist[sw][rel];
                }
                int before = 0;
#pragma unroll
                for (int u = 0; u < KPL; ++u) {
                    const int inc = wave_scan_incl(tot[u], lane);
                    cur[u] = before + inc - tot[u];
                    before += __builtin_amdgcn_readlane(inc, 63);
                }
#pragma unroll
                for (int u = 0; u < KPL; ++u) {
                    const int r = lane + 64 * u;
                    const int rel = (r & (RPW - 1)) * W + r / RPW;
                    if (r < R) {
                        start[r] = cur[u];
                        int run = cur[u];
                        for (int sw = 0; sw < W; ++sw) {
                            int cnt = hist[sw][rel];
                            hist[sw][rel] = run;
                            run += cnt;
                        }
                        if (r == R - 1)
                            start[R] = run;
                    }
                }
            }
            __syncthreads();
            {
                // (3) stable placement: kept entries in order, equal keys ranked by lane
                typedef volatile __attribute__((address_space(3))) int *lds_int; // LDS, not a generic pointer
                lds_int cursor = (lds_int)&hist[w][lo_rel];
                for (int e0 = 0; e0 < kept; e0 += 64) {
                    const bool valid = e0 + lane < kept;
                    const uint32_t ent = valid ? seg[w][e0 + lane] : 0u;
                    const int key = (int)(ent >> 16); // the row, counted from the document's first row in the block
                    uint64_t same = __ballot(valid);
#pragma unroll
                    for (int bit = 0; bit < RBITS; ++bit) {
                        const bool one = (key >> bit) & 1;
                        const uint64_t bm = __ballot(one);
                        same &= one ? bm : ~bm;
                    }
                    if (valid) {
                        const int rank = __popcll(same & ((uint64_t(1) << lane) - 1));
                        const int pos = cursor[key] + rank;
                        list[pos] = (uint16_t)(ent & 0xffffu);
                        if (rank == 0)
                            cursor[key] = pos + __popcll(same);
                    }
                    __builtin_amdgcn_wave_barrier();
                }
            }
            __syncthreads();
            {
                // (4) walk this wavefront's keys w * RPW .. w * RPW + RPW - 1
                const int startv = start[w * RPW + (lane < RPW ? lane : RPW)];
                const int k_lo = __builtin_amdgcn_readlane(startv, 0);
                const int k_hi = __builtin_amdgcn_readlane(startv, RPW);
                auto lookup = [&](int kk, bool valid, int, uint32_t &n, float &gv) {
                    n = (uint32_t)c0 + (valid ? (uint32_t)list[kk] : 0u); // = q * l_q + i: the Q row
                    const uint32_t q = magic_div(n, lq_magic);
                    gv = valid ? p.g[(int64_t)q * p.b + j] : 0.0f;
                };
                walk_rows<DT, RPW>(rsrc, row_bytes, lane, lane_off, k_lo, k_hi, startv, reinterpret_cast<float *>(&seg[w][0]), lookup, rx, ry);
            }
        }
    }
    if (col_ok) {
#pragma unroll
        for (int s = 0; s < RPW; ++s) {
            const int64_t row = row0 + W * s + w;
            if (row < row_end)
                store_streaming2(p.dD + row * p.d + col, rx[s], ry[s]);
        }
    }
}

// The partial sums of dQ live in the dD buffer until the dD kernel overwrites it (dD is an output that the call
// fully overwrites, and its n_part * n_q * l_q rows of d floats are free until then), so the library needs no
// scratch memory.  n_part = the largest power of two <= 8 that fits there and leaves every partition a document.
static int dq_partitions(const BwdParams &p)
{
    int n_part = 8;
    const int64_t nql = (int64_t)p.n_q * p.l_q;
    while (n_part > 1 && ((int64_t)n_part * nql > p.total_tokens || n_part > p.b))
        n_part >>= 1;
    return n_part;
}

template <int DT> static hipError_t launch_dq(const BwdParams &p, hipStream_t stream)
{
    const int64_t nql = (int64_t)p.n_q * p.l_q;
    const int n_part = dq_partitions(p);
    const int64_t dpp = (p.b + n_part - 1) / n_part;
    const unsigned slabs = (unsigned)((p.d + SLAB - 1) / SLAB);
    float *out = n_part > 1 ? p.dD : p.dQ;
    // four query tokens per group of sixteen lanes once that still gives every SIMD a wavefront or two
    if (nql * n_part >= 16384 && p.l_q % 4 == 0 && (reinterpret_cast<uintptr_t>(p.A) & 15) == 0) {
        const int64_t groups = (nql + 63) / 64; // workgroups of four wavefronts x four groups x four query tokens
        if (groups * n_part >= (int64_t(1) << 31))
            return hipErrorInvalidValue;
        hipLaunchKernelGGL((bwd_dq_kernel<DT, 4>), dim3((unsigned)(groups * n_part), slabs), dim3(256), 0, stream, p, out, n_part, dpp);
    } else {
        const int64_t groups = (nql + 15) / 16;
        hipLaunchKernelGGL((bwd_dq_kernel<DT, 1>), dim3((unsigned)(groups * n_part), slabs), dim3(256), 0, stream, p, out, n_part, dpp);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n_part == 1)
        return e;
    const int64_t n4 = nql * p.d / 4;
    int64_t blocks = (n4 + 255) / 256;
    if (blocks > 65536)
        blocks = 65536;
    hipLaunchKernelGGL(bwd_dq_combine_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                       reinterpret_cast<const float4 *>(p.dD), reinterpret_cast<float4 *>(p.dQ), n4, n_part);
    return hipGetLastError();
}

template <int DT> static hipError_t launch_bwd(const BwdParams &p, int num_cu, hipStream_t stream)
{
    hipError_t e = launch_dq<DT>(p, stream);
    if (e != hipSuccess)
        return e;
    // blocks of 128 rows unless that leaves the chip short of workgroups (about 4 per CU wanted)
    const int64_t want = (int64_t)num_cu * 4;
    const Magic lq_magic = magic_u31((uint32_t)p.l_q);
    const unsigned slabs = (unsigned)((p.d + SLAB - 1) / SLAB);
    auto go = [&](auto rpw_tag, auto w_tag) {
        constexpr int RPW = decltype(rpw_tag)::value;
        constexpr int W = decltype(w_tag)::value;
        const BlockOrder order = block_order((p.total_tokens + W * RPW - 1) / (W * RPW), num_cu);
        hipLaunchKernelGGL((bwd_dd_kernel<DT, RPW, W>), dim3(order.grid, slabs), dim3(W * 64), 0, stream, p, p.offsets,
                           lq_magic, magic_u31((uint32_t)(p.l_d > 0 ? p.l_d : 1)), 64 / p.l_q, 64 % p.l_q, order);
    };
    if (p.total_tokens / (DD_WAVES * 16) >= want)
        go(std::integral_constant<int, 16>(), std::integral_constant<int, 8>());
    else if (p.total_tokens / (DD_WAVES * 8) >= want)
        go(std::integral_constant<int, 8>(), std::integral_constant<int, 8>());
    else
        go(std::integral_constant<int, 4>(), std::integral_constant<int, 8>());
    return hipGetLastError();
}

hipError_t backward_launch(const void *Q, int n_q, int l_q, const void *D, const int32_t *offsets, int64_t b, int l_d,
                           int64_t total_tokens, int d, int dtype, const int32_t *argmax, const float *dscore, float *dQ,
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
    p.d = d;
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
//   csr_apply_kernel   a wavefront per 8 consecutive dD rows walks their lists in order (Eq. 3).
// ---------------------------------------------------------------------------------------
constexpr int CSR_WAVES = 8;
constexpr int CSR_MAX_LD = 4096;
constexpr int CSR_LOADS = 8;      // argmax entries a lane fetches before it uses the first
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

// dD[r, :] = sum over the edges of row r, in list order, of g[i, j] * Q[i, s, :]: the walk of bwd_dd_kernel over the
// CSR in global memory.  A workgroup owns CSR_APPLY_WAVES * CSR_RPW consecutive rows and wavefront w of it the rows
// w, w + CSR_APPLY_WAVES, ... (neighbouring rows are often hot together -- the first tokens of a document -- and so
// go to different wavefronts).  The wavefront walks its rows' lists as one virtual array, list after list: slot s
// starts at the sum of the lengths before it, and the lookup adds the distance between the virtual and the real start
// of the edge's list.  Per 64 edges one vector step decodes the edge ids (e = (i * b + j) * l_q + s) into Q row and
// weight, then all 64 lanes (two columns each) apply the edges in order.  Same order and arithmetic as
// bwd_dd_kernel: same bits.
constexpr int CSR_RPW = 8;
constexpr int CSR_APPLY_WAVES = 4;

template <int DT>
__global__ void __launch_bounds__(CSR_APPLY_WAVES * 64) csr_apply_kernel(BwdParams p, const int32_t *__restrict__ row_ptr,
                                                        const int32_t *__restrict__ col_idx, Magic bl_magic, Magic lq_magic,
                                                        BlockOrder order)
{
    constexpr int EB = Elem<DT>::BYTES;
    __shared__ __attribute__((aligned(16))) float gstage[CSR_APPLY_WAVES][128]; // per wavefront: the weights of the edges being walked
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int blk = ordered_block(order, blockIdx.x);
    const int64_t rb = (int64_t)blk * (CSR_APPLY_WAVES * CSR_RPW) + w; // the wavefront's first row
    if (blk < 0 || rb >= p.total_tokens)
        return;
    const int col = (int)blockIdx.y * SLAB + 2 * lane;
    const bool col_ok = col < p.d;
    const uint32_t lane_off = (uint32_t)((col_ok ? 2 * lane : 0) + (int)blockIdx.y * SLAB) * EB;
    const uint32_t row_bytes = (uint32_t)p.d * EB;
    const __amdgpu_buffer_rsrc_t rsrc = q_resource(p.Q, (uint32_t)p.n_q * (uint32_t)p.l_q * row_bytes); // < 2^32 (checked by the caller)
    const int64_t n_edges = (int64_t)p.n_q * p.l_q * p.b; // < 2^31 (checked by the caller)
    // lane s < CSR_RPW: the list of row rb + CSR_APPLY_WAVES * s
    const int64_t my_row = rb + (int64_t)CSR_APPLY_WAVES * (lane < CSR_RPW ? lane : 0);
    const bool have = lane < CSR_RPW && my_row < p.total_tokens;
    int lo = row_ptr[have ? my_row : rb], hi = row_ptr[(have ? my_row : rb) + 1];
    lo = lo < 0 ? 0 : (lo > n_edges ? (int)n_edges : lo); // device data the host cannot check
    hi = hi < lo ? lo : (hi > n_edges ? (int)n_edges : hi);
    const int len = have ? hi - lo : 0;
    const int incl = wave_scan_incl(len, lane);
    const int vstart = incl - len; // lanes >= CSR_RPW: the total
    const int k_hi = __builtin_amdgcn_readlane(incl, 63);
    const int delta = lo - vstart;
    const uint32_t bl = (uint32_t)(p.b * p.l_q); // edge ids of one query
    typename RowVec<CSR_RPW>::type rx, ry;
#pragma unroll
    for (int s = 0; s < CSR_RPW; ++s) {
        rx[s] = 0.0f;
        ry[s] = 0.0f;
    }
    auto lookup = [&](int kk, bool valid, int slot, uint32_t &n, float &gv) {
        const int at = kk + __shfl(delta, slot);
        const int e = valid ? col_idx[at] : 0;
        const uint32_t ue = e < 0 ? 0u : (uint32_t)e;
        const uint32_t i = magic_div(ue, bl_magic);
        const uint32_t rem = ue - i * bl; // j * l_q + s
        const uint32_t jj = magic_div(rem, lq_magic);
        const uint32_t s_ = rem - jj * (uint32_t)p.l_q;
        const bool ok = valid && e >= 0 && i < (uint32_t)p.n_q;
        n = ok ? i * (uint32_t)p.l_q + s_ : 0u;
        gv = ok ? p.g[(int64_t)i * p.b + jj] : 0.0f;
    };
    walk_rows<DT, CSR_RPW>(rsrc, row_bytes, lane, lane_off, 0, k_hi, vstart, &gstage[w][0], lookup, rx, ry);
    if (col_ok) {
#pragma unroll
        for (int s = 0; s < CSR_RPW; ++s) {
            const int64_t row = rb + (int64_t)CSR_APPLY_WAVES * s;
            if (row < p.total_tokens)
                store_streaming2(p.dD + row * p.d + col, rx[s], ry[s]);
        }
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
    hipError_t e = hipSuccess;
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
                                                   int num_cu, hipStream_t stream)
{
    hipError_t e = launch_dq<DT>(p, stream);
    if (e != hipSuccess)
        return e;
    constexpr int ROWS = CSR_RPW * CSR_APPLY_WAVES; // rows per workgroup
    const BlockOrder order = block_order((p.total_tokens + ROWS - 1) / ROWS, num_cu);
    const unsigned slabs = (unsigned)((p.d + SLAB - 1) / SLAB);
    hipLaunchKernelGGL((csr_apply_kernel<DT>), dim3(order.grid, slabs), dim3(CSR_APPLY_WAVES * 64), 0, stream, p, row_ptr,
                       col_idx, magic_u31((uint32_t)(p.b * p.l_q)), magic_u31((uint32_t)p.l_q), order);
    return hipGetLastError();
}

hipError_t backward_csr_launch(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d, int dtype,
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
    p.d = d;
    switch (dtype) {
    case MAXSIM_F32: return launch_bwd_csr<MAXSIM_F32>(p, row_ptr, col_idx, num_cu, stream);
    case MAXSIM_F16: return launch_bwd_csr<MAXSIM_F16>(p, row_ptr, col_idx, num_cu, stream);
    default: return launch_bwd_csr<MAXSIM_BF16>(p, row_ptr, col_idx, num_cu, stream);
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
} // namespace

// Per-device set-up of this file (called once per device, under the library's lock, with that device current):
// the address of the device's copy of `scratch`, and the LDS limit of csr_place_kernel.
hipError_t backward_init_device()
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return e;
    if (dev < 0 || dev >= 64)
        return hipErrorInvalidDevice;
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess)
        return e;
    if (!ptr)
        return hipErrorInvalidSymbol;
    scratch_ptr[dev] = static_cast<int32_t *>(ptr);
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&csr_place_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (CSR_WAVES * CSR_MAX_LD + CSR_LDS_EXTRA) * (int)sizeof(int));
}

// The device's copy of `scratch` (set up by backward_init_device before any entry point gets here).
static hipError_t csr_static_buffer(int32_t **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return e;
    if (dev < 0 || dev >= 64 || !scratch_ptr[dev])
        return hipErrorInvalidDevice;
    *out = scratch_ptr[dev];
    return hipSuccess;
}

bool csr_static_fits(int n_q, int64_t b, int l_q, int l_d)
{
    return b * (int64_t)l_d <= CSR_STATIC_MAX_ROWS && (int64_t)n_q * l_q * b <= CSR_STATIC_MAX_EDGES;
}

hipError_t backward_csr_static_launch(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d, int dtype,
                                      const int32_t *argmax, const float *dscore, float *dQ, float *dD, int num_cu,
                                      hipStream_t stream)
{
    if (!csr_static_fits(n_q, b, l_q, l_d))
        return hipErrorInvalidValue;
    int32_t *buf = nullptr;
    hipError_t e = csr_static_buffer(&buf);
    if (e != hipSuccess)
        return e;
    return backward_csr_launch(Q, n_q, l_q, D, b, l_d, d, dtype, argmax, dscore, buf, buf + CSR_STATIC_COL_AT, dQ, dD, num_cu,
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
