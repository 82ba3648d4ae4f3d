// Shared device-side vocabulary of the gfx950 MaxSim kernels (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "../../include/maxsim.h"

namespace maxsim {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr int D_MODEL = 128;  // embedding width of the backward and int8 kernels (the float forward also takes 64, 256, 512)
constexpr int TILE_ROWS = 32; // document tokens per MFMA tile (rows of the 32x32 result)
constexpr int BLOCK_COLS = 32; // query tokens per column block (columns of the 32x32 result)

// A token row is handled in 16-byte chunks.  Lane (rho = lane % 32, h = lane / 32) of a
// wavefront owns chunks 2u + h (u = 0 .. NU-1) of row rho, for documents (MFMA A operand)
// and queries (MFMA B operand) alike, so both sides pair the same k indices.
//
// The float kernels are compiled per "format" F = dtype | (NU << 4): the element type and the
// embedding width (a row is NU * 32 bytes: d = 16 * NU for 16-bit inputs, 8 * NU for fp32).
constexpr int fmt(int dtype, int nu) { return dtype | (nu << 4); }

template <int F> struct Traits {
    static constexpr int DT = F & 15;
    static constexpr int NU = F >> 4;
    static constexpr int ROW_BYTES = NU * 32;
    static __device__ __forceinline__ void mma(const uint4 &a, const uint4 &b, f32x16 &c)
    {
        if constexpr (DT == MAXSIM_F16) {
            c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
        } else if constexpr (DT == MAXSIM_BF16) {
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
        } else {
            // one chunk = 4 floats = 4 rank-2 updates (k = 2 per instruction: halves h = 0, 1)
            c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
        }
    }
};

// Row of the 32x32 MFMA result held in accumulator register r of a lane in half h.
__device__ __forceinline__ int acc_row(int r, int h) { return (r >> 2) * 8 + h * 4 + (r & 3); }

__device__ __forceinline__ float neg_inf() { return -__builtin_huge_valf(); }

// 16-byte load with the non-temporal hint, for streams that are read once by instructions that take whole lines
// (sixteen lanes on 256 contiguous bytes): 6.8 against 6.0 TB/s for a wavefront-per-run read stream.  Not for
// loads that take a part of a line and leave the rest to a neighbour: the hint keeps the caches from merging them.
__device__ __forceinline__ uint4 load_stream16(const void *p)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in this order
template <int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>{});
    }
}

// One of eight named 16-byte registers by compile-time index.  The chunks of a tile on its way from HBM to LDS are
// kept this way: as an array indexed in unrolled loops inside lambdas they stayed in scratch memory whenever a
// thread moves more than one chunk per tile.
template <int I> __device__ __forceinline__ uint4 &reg_at(uint4 &r0, uint4 &r1, uint4 &r2, uint4 &r3, uint4 &r4, uint4 &r5, uint4 &r6, uint4 &r7)
{
    static_assert(I >= 0 && I < 8, "eight registers");
    if constexpr (I == 0)
        return r0;
    else if constexpr (I == 1)
        return r1;
    else if constexpr (I == 2)
        return r2;
    else if constexpr (I == 3)
        return r3;
    else if constexpr (I == 4)
        return r4;
    else if constexpr (I == 5)
        return r5;
    else if constexpr (I == 6)
        return r6;
    else
        return r7;
}

// Arguments of the forward kernels (plain data, passed by value).
struct FwdParams {
    const char *Q;          // [n_q, l_q, d]
    const char *D;          // [b, l_d, d] or packed [T, d]
    const int32_t *offsets; // [b + 1] or nullptr for a uniform corpus
    float *scores;          // [n_q, b]
    int32_t *argmax;        // [n_q, b, l_q] or nullptr
    int64_t b;
    int64_t ld;           // documents per row of scores / argmax (b, or the whole corpus when b is a slice of it)
    int64_t total_tokens; // b * l_d for a uniform corpus
    int n_q, l_q, l_d;
    int bpq;               // column blocks per query = ceil(l_q / 32)
    int n_chunks;          // document chunks (work units along the corpus)
    int64_t unit_per_chunk; // documents (uniform) or tokens (ragged) per chunk
    int n_groups;          // column groups (tile kernel only)
    int qpg;               // queries per column group (tile kernel, bpq <= group size)
    int n_pass;            // passes over the corpus per group (tile kernel, bpq > group size)
};

// Offsets come from device memory the host cannot check.  Every offset is forced into
// [lo, total_tokens] before it is used (once per document, scalar work), so that offsets which
// are not non-decreasing or run past the corpus give wrong scores but never an address outside D.
__device__ __forceinline__ int64_t clamp_offset(int64_t x, int64_t lo, int64_t hi) { return x < lo ? lo : (x > hi ? hi : x); }

// A kernel that walks a ragged corpus takes the offsets a second time, as a `const int32_t *__restrict__`
// parameter of its own: only then does the compiler know that no store of the kernel can change them and
// reads offsets[uniform index] through the scalar cache, apart from the vector loads in flight.
typedef const int32_t *__restrict__ OffsetsPtr;

// Cursor over the 32-row tiles of a run of documents, identical in every lane of a wavefront.
struct Cursor {
    int64_t doc;     // current document
    int64_t doc_end; // end of the run (exclusive)
    int64_t start;   // first packed row of the current document
    int64_t nxt_end; // offsets[doc + 2], fetched one document ahead (ragged only)
    int32_t len;     // tokens in the current document
    int32_t t0;      // first row (document-local) of the current tile
    bool valid;
};

__device__ __forceinline__ void cursor_next_doc(Cursor &c, const FwdParams &p, OffsetsPtr off)
{
    for (;;) {
        c.doc += 1;
        c.valid = c.doc < c.doc_end;
        if (!c.valid)
            return;
        c.t0 = 0;
        if (p.offsets) {
            c.start += c.len;
            int64_t e = clamp_offset(c.nxt_end, c.start, p.total_tokens);
            c.len = (int32_t)(e - c.start);
            c.nxt_end = (int64_t)off[(c.doc + 2 <= p.b) ? c.doc + 2 : p.b]; // no branch around the load: it stays a scalar load
            if (c.len > 0)
                return;
        } else {
            c.start += p.l_d;
            return;
        }
    }
}

__device__ __forceinline__ void cursor_init(Cursor &c, const FwdParams &p, OffsetsPtr off, int64_t doc0, int64_t doc1)
{
    c.doc = doc0;
    c.doc_end = doc1;
    c.t0 = 0;
    c.valid = doc0 < doc1;
    if (!c.valid)
        return;
    if (p.offsets) {
        c.start = clamp_offset(off[doc0], 0, p.total_tokens);
        int64_t e = clamp_offset(off[doc0 + 1], c.start, p.total_tokens);
        c.len = (int32_t)(e - c.start);
        c.nxt_end = (int64_t)off[(doc0 + 2 <= p.b) ? doc0 + 2 : p.b];
        if (c.len == 0)
            cursor_next_doc(c, p, off);
    } else {
        c.start = doc0 * (int64_t)p.l_d;
        c.len = p.l_d;
        c.nxt_end = 0;
    }
}

__device__ __forceinline__ void cursor_next_tile(Cursor &c, const FwdParams &p, OffsetsPtr off, int rows = TILE_ROWS)
{
    c.t0 += rows;
    if (c.t0 >= c.len)
        cursor_next_doc(c, p, off);
}

// Documents [doc0, doc1) of work chunk `chunk`.  Uniform corpus: equal document counts.
// Ragged corpus: the packed token range is cut into equal pieces and a chunk owns every
// document that starts inside its piece (binary search over the offsets).
__device__ __forceinline__ int64_t lower_bound_offsets(const int32_t *off, int64_t n, int64_t key)
{
    // smallest i in [0, n] with off[i] >= key (off has n + 1 entries, non-decreasing)
    int64_t lo = 0, hi = n + 1;
    while (lo < hi) {
        int64_t mid = (lo + hi) >> 1;
        if ((int64_t)off[mid] < key)
            lo = mid + 1;
        else
            hi = mid;
    }
    return lo;
}

__device__ __forceinline__ void chunk_doc_range(const FwdParams &p, int64_t chunk, int64_t &doc0, int64_t &doc1)
{
    if (chunk >= p.n_chunks) {
        doc0 = doc1 = 0;
        return;
    }
    if (p.offsets) {
        int64_t lo = chunk * p.unit_per_chunk;
        int64_t hi = lo + p.unit_per_chunk;
        doc0 = (chunk == 0) ? 0 : lower_bound_offsets(p.offsets, p.b, lo);
        doc1 = (chunk == p.n_chunks - 1) ? p.b : lower_bound_offsets(p.offsets, p.b, hi);
        if (doc0 > p.b)
            doc0 = p.b;
        if (doc1 > p.b)
            doc1 = p.b;
    } else {
        doc0 = chunk * p.unit_per_chunk;
        doc1 = doc0 + p.unit_per_chunk;
        if (doc0 > p.b)
            doc0 = p.b;
        if (doc1 > p.b)
            doc1 = p.b;
    }
}

// Walks the tiles (32 tokens unless told otherwise) of documents [doc, doc_end), the same in every lane.  All
// state is 32-bit and uniform (scalar registers).  For ragged corpora the end of the NEXT document is
// fetched while the current one is walked, so that stepping to the next document waits for no memory.
struct TileIter {
    int doc, doc_end;
    int row0; // packed row of the current tile's first token
    int t0;   // document-local index of that token
    int len;  // tokens in the current document
    int end;  // packed row one past the current document (ragged only)
    int nxt;  // offsets[doc + 2], unclamped, fetched one document ahead (ragged only)
};

__device__ __forceinline__ bool it_valid(const TileIter &it) { return it.doc < it.doc_end; }

__device__ __forceinline__ int it_offset(OffsetsPtr off, const FwdParams &p, int i)
{
    const int64_t j = i < p.b ? (int64_t)i : p.b;
    return off[j];
}

// Enters document it.doc (whose first row is it.end of the previous one and whose unclamped end is it.nxt),
// skipping empty documents.  Offsets are forced into [previous end, T], so that offsets which are not
// non-decreasing or run past the corpus give wrong scores but never an address outside D.
__device__ __forceinline__ void it_enter_ragged(TileIter &it, const FwdParams &p, OffsetsPtr off)
{
    const int t_all = (int)p.total_tokens; // < 2^31
    while (it.doc < it.doc_end) {
        const int s = it.end;
        const int e = min(max(it.nxt, s), t_all);
        it.nxt = it_offset(off, p, it.doc + 2);
        it.row0 = s;
        it.end = e;
        it.len = e - s;
        it.t0 = 0;
        if (it.len > 0)
            return;
        it.doc += 1;
    }
}

__device__ __forceinline__ void it_init(TileIter &it, const FwdParams &p, OffsetsPtr off, int doc0, int doc1)
{
    it.doc = doc0;
    it.doc_end = doc1;
    it.row0 = it.t0 = it.len = it.end = it.nxt = 0;
    if (doc0 >= doc1)
        return;
    if (p.offsets) {
        it.end = min(max(it_offset(off, p, doc0), 0), (int)p.total_tokens);
        it.nxt = it_offset(off, p, doc0 + 1);
        it_enter_ragged(it, p, off);
    } else {
        it.row0 = doc0 * p.l_d;
        it.len = p.l_d;
    }
}

__device__ __forceinline__ void it_next(TileIter &it, const FwdParams &p, OffsetsPtr off, int rows = TILE_ROWS)
{
    it.t0 += rows;
    it.row0 += rows;
    if (it.t0 >= it.len) {
        it.doc += 1;
        if (p.offsets) {
            it_enter_ragged(it, p, off);
        } else {
            it.row0 = it.doc * p.l_d;
            it.t0 = 0;
        }
    }
}

} // namespace maxsim
