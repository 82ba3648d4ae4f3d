/*
 * maxsim.h -- C ABI of the fused MaxSim library for AMD MI355X (gfx950).
 *
 * The operator is the late-interaction score of the "Flash-MaxSim" paper,
 *     score(Q, D) = sum_i max_j <Q_i, D_j>                      (Eq. 1),
 * computed tile by tile so that the [N_q, B, L_q, L_d] similarity tensor is
 * never written to memory (Alg. 1), its training backward through the stored
 * argmax (Eqs. 2-3, Alg. 2), and int8 scoring with per-token scales applied
 * once per similarity cell (Sec. "Quantised Scoring", Alg. 4).
 *
 * Conventions shared by every entry point
 *   - Every pointer is a DEVICE pointer owned by the caller (the one exception, the host
 *     corpus of the *_streamed entry points, is marked HOST).  The library never allocates,
 *     frees or keeps device memory.
 *   - `stream` is a hipStream_t passed as void*.  Calls only enqueue work on it
 *     and return; they never synchronise.  NULL means the default stream.
 *   - Tensors are row-major with the innermost stride 1 and no gaps.  Base
 *     pointers of Q, D and the int8 tensors must be 16-byte aligned, all other
 *     pointers 4-byte aligned.
 *   - d (embedding width).  The paper's setting is 128 (Tab. "shapes"); its "fat embedding" extension
 *     (App. "split-d") goes to 2048.  Here:
 *       float forward (maxsim_forward, _ragged, _streamed): any width whose rows are a multiple of 64 bytes, from
 *         d = 32 up to rows of 16 KB: d = 32, 64, 96, ... , 8192 for fp16/bf16 and d = 32, 48, 64, ... , 4096 for
 *         fp32.  Rows of 128, 256 and 512 bytes can keep the queries in registers; every other width streams both
 *         operands in slabs of the embedding dimension (the paper's inner loop over d).
 *       backward (maxsim_backward, _ragged, _csr, _csr_static): any multiple of 8 from 8 to 8192; Q must stay
 *         below 4 GiB and D below 64 GiB.
 *       int8 entry points and the quantiser: any multiple of 32 from 32 to 8192.  d = 128 takes the tuned kernels
 *         (queries resident in LDS or registers); other multiples of 64 stream both operands in slabs like the
 *         float forward; the remaining widths take a plain inner loop over d at a fraction of the speed.  The same
 *         arithmetic and the same bits everywhere.
 *     Other widths must be zero-padded by the caller; anything else returns MAXSIM_ERR_UNSUPPORTED.
 *   - Four kernel families use more than 64 KB of LDS, which HIP wants allowed per kernel and device before the
 *     first launch.  maxsim_init() does that (and all other per-device set-up) for the current device; an entry
 *     point whose device has not been set up does it itself first, which is not possible while `stream` is being
 *     captured into a HIP graph: call maxsim_init() once per device before capturing anything.
 *   - L_q and L_d are arbitrary positive integers (no tile multiples needed).
 *   - Inputs must be finite; the result for NaN/Inf inputs is unspecified.
 *   - Return value: MAXSIM_OK (0) or a negative error code.  MAXSIM_ERR_INVALID, _UNSUPPORTED and _SCRATCH
 *     are found before anything is enqueued.  MAXSIM_ERR_LAUNCH means the HIP runtime refused a step of the
 *     call: earlier steps of the same call (kernels, copies, waits between streams) may already be queued and the
 *     outputs are then undefined.  No exceptions, no abort, nothing printed.
 */
#ifndef MAXSIM_H
#define MAXSIM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MAXSIM_OK 0
#define MAXSIM_ERR_INVALID (-1)     /* null pointer, non-positive size, misaligned pointer, bad enum */
#define MAXSIM_ERR_UNSUPPORTED (-2) /* an embedding width or a size that the kernels are not built for */
#define MAXSIM_ERR_LAUNCH (-3)      /* the HIP runtime reported an error at launch */
#define MAXSIM_ERR_SCRATCH (-4)     /* sizes beyond the library's static scratch buffer (maxsim_backward_csr_static) */

typedef enum { MAXSIM_F32 = 0, MAXSIM_F16 = 1, MAXSIM_BF16 = 2 } maxsim_dtype;

/* Human-readable text for a return code (static storage, never NULL). */
const char *maxsim_strerror(int code);

/*
 * Per-device set-up for the CURRENT device: raises the LDS limit of the kernels that need it and looks up
 * the library's static scratch array.  Allocates nothing, enqueues nothing, may be called any number of times
 * and from several host threads.  Optional unless entry points are to be captured into HIP graphs (see above).
 * Returns MAXSIM_OK or MAXSIM_ERR_LAUNCH (the HIP runtime refused).
 */
int maxsim_init(void);

/*
 * Fused forward over a uniform corpus (Eq. 1; Alg. 1; Prop. 1).
 *   Q       [n_q, l_q, d]  dtype          query token embeddings
 *   D       [b,   l_d, d]  dtype          document token embeddings
 *   scores  [n_q, b]       float32        fully overwritten
 *   argmax  [n_q, b, l_q]  int32 or NULL  winning document-token index, local to
 *                                         the document (Sec. "Closed-Form Gradients");
 *                                         ties go to the lowest index ("Tied maxima")
 * Products are formed in the input dtype's exact values and accumulated in fp32.
 * With fp16/bf16 inputs and argmax requested, similarities below 512 in magnitude that differ by less than
 * 2^-19 relative count as tied (the lower index wins) and the maxima that enter the score may be truncated by
 * that much; without argmax, and for fp32 inputs, the maxima are the exact fp32 sums.
 */
int maxsim_forward(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d,
                   maxsim_dtype dtype, float *scores, int32_t *argmax, void *stream);

/*
 * Out-of-core forward (Sec. "Corpus-scale scoring": a corpus that does not fit in device memory is
 * streamed through a fixed buffer while the kernel runs).
 *   D_host      [b, l_d, d] dtype in HOST memory (page-locked memory makes the copies asynchronous;
 *               pageable memory works but serialises them)
 *   block_docs  documents per block (clamped to b); block_docs * l_d must be < 2^31
 *   staging     DEVICE buffer of 2 * block_docs * l_d * d * sizeof(dtype) bytes owned by the caller;
 *               its contents are overwritten
 *   scores      [n_q, b] float32 (device), fully overwritten; no argmax
 * Block k + 1 is copied (on a copy stream the library creates once per device, default priority)
 * while block k is scored on `stream`; all work is ordered after what `stream` already holds and
 * the call returns without synchronising.  D_host and staging must stay valid until `stream`
 * has run the last kernel.  Same arithmetic as maxsim_forward (identical bits).
 */
int maxsim_forward_streamed(const void *Q, int n_q, int l_q, const void *D_host, int64_t b, int l_d,
                            int d, maxsim_dtype dtype, int64_t block_docs, void *staging,
                            float *scores, void *stream);

/*
 * Fused forward over a packed ragged corpus (Sec. "Ragged corpora and kernel family";
 * the cu_seqlens variant).  No padding is read or computed.
 *   D_packed     [total_tokens, d] dtype   documents back to back
 *   doc_offsets  [b + 1] int32 (device)    non-decreasing, doc_offsets[0] = 0,
 *                                          doc_offsets[b] = total_tokens
 *   total_tokens host copy of doc_offsets[b]; must be < 2^31
 * A document of length 0 gets score -inf and argmax -1.
 * Other arguments as in maxsim_forward.
 */
int maxsim_forward_ragged(const void *Q, int n_q, int l_q, const void *D_packed,
                          const int32_t *doc_offsets, int64_t b, int64_t total_tokens, int d,
                          maxsim_dtype dtype, float *scores, int32_t *argmax, void *stream);

/*
 * Backward through the stored argmax (Eqs. 2-3; Alg. 2), uniform corpus.
 *   argmax  [n_q, b, l_q] int32   as written by maxsim_forward; negative entries are skipped,
 *                                 entries >= l_d are a caller error (skipped, never dereferenced)
 *   dscore  [n_q, b]      float32 upstream gradient of the scores
 *   dQ      [n_q, l_q, d] float32 fully overwritten:  dQ[q,i,:] = sum_b dscore[q,b] D[b, A[q,b,i], :]
 *   dD      [b,  l_d, d]  float32 fully overwritten:  dD[b,t,:] = sum_{(q,i): A[q,b,i]=t} dscore[q,b] Q[q,i,:]
 * Accumulation is fp32 in a fixed order: results are bitwise reproducible from run to run
 * (no atomics; every dD row has one owner, a wavefront, which adds the row's edges by increasing edge id
 * (q * b + j) * l_q + i: the role of the paper's inverse-grid CSR, without building it in global memory;
 * dQ adds the documents of each of up to eight contiguous partitions in order and then the partitions in order).
 * dD doubles as work space during the call: it holds partial sums of dQ until its own rows are written.
 */
int maxsim_backward(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d,
                    maxsim_dtype dtype, const int32_t *argmax, const float *dscore, float *dQ,
                    float *dD, void *stream);

/*
 * Backward over a packed ragged corpus (Eqs. 2-3 with the ragged layout of Sec. "Ragged corpora
 * and kernel family").
 *   D_packed, doc_offsets, total_tokens as in maxsim_forward_ragged
 *   argmax  [n_q, b, l_q] int32   document-local indices as written by maxsim_forward_ragged;
 *                                 negative entries (empty documents) are skipped
 *   dQ      [n_q, l_q, d] float32 fully overwritten
 *   dD_packed [total_tokens, d] float32 fully overwritten, packed like D_packed
 * Same arithmetic and reproducibility as maxsim_backward.
 */
int maxsim_backward_ragged(const void *Q, int n_q, int l_q, const void *D_packed,
                           const int32_t *doc_offsets, int64_t b, int64_t total_tokens, int d,
                           maxsim_dtype dtype, const int32_t *argmax, const float *dscore,
                           float *dQ, float *dD_packed, void *stream);

/*
 * The inverse-grid CSR of the deterministic backward, built on the device (Alg. 2; Sec.
 * "Closed-Form Gradients"): the map destination row -> source edges that bincount, cumsum and
 * a stable argsort by destination define.  Uniform corpus.
 *   argmax   [n_q, b, l_q] int32 (device)   an entry t with 0 <= t < l_d is an edge with id
 *                                           e = (i * b + j) * l_q + s and destination row
 *                                           j * l_d + t; other entries are not edges
 *   row_ptr  [b * l_d + 1] int32 (device)   output: row r's edges are col_idx[row_ptr[r] ..
 *                                           row_ptr[r + 1]); row_ptr[b * l_d] = number of edges
 *   col_idx  [n_q * b * l_q] int32 (device) output: edge ids, by destination row and by
 *                                           increasing id within a row; only the first
 *                                           row_ptr[b * l_d] entries are written
 * Limits: l_d <= 4096 and n_q * b * l_q < 2^31 (MAXSIM_ERR_UNSUPPORTED beyond).  The result is
 * the same on every run.  argmax must not change while the call is in flight.
 */
int maxsim_csr_build(const int32_t *argmax, int n_q, int64_t b, int l_q, int l_d, int32_t *row_ptr,
                     int32_t *col_idx, void *stream);

/*
 * maxsim_backward with dD taken through the explicit CSR (Alg. 2 as stated: build the CSR from
 * argmax, then one owner per dD row walks that row's edge list).  row_ptr and col_idx are
 * caller-provided device buffers of the sizes maxsim_csr_build states; they are overwritten
 * and hold the CSR afterwards.  dQ, dD, the skipping of negative entries and the fp32
 * accumulation order (a row's edges by increasing id) are those of maxsim_backward, so the two
 * give the same bits.  Limits of maxsim_csr_build and of maxsim_backward apply.
 */
int maxsim_backward_csr(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d,
                        maxsim_dtype dtype, const int32_t *argmax, const float *dscore,
                        int32_t *row_ptr, int32_t *col_idx, float *dQ, float *dD, void *stream);

/*
 * maxsim_backward_csr for callers that cannot allocate device memory at all (code that runs under HIP graph
 * capture, tight serving loops, harnesses that forbid it): the same kernels, with row_ptr and col_idx in a
 * device array that is part of the library's image (9.4 MB, one copy on every GPU the library runs on, held
 * until the process ends) instead of caller buffers.  The call allocates and frees nothing.
 *   Limits: b * l_d <= 262144 rows and n_q * b * l_q <= 2097152 argmax entries (config 4 exactly); larger
 *   sizes return MAXSIM_ERR_SCRATCH and enqueue nothing.  Other arguments, limits, arithmetic and results
 *   as maxsim_backward_csr (identical bits); the CSR itself is not returned.
 *   All calls on one GPU share that GPU's array: two calls whose work overlaps in time on one GPU (different
 *   streams, different host threads) race; calls on one stream are ordered and safe.  Nothing has to be
 *   cleared between calls.  The array's address is looked up by the per-device set-up (maxsim_init, or the first
 *   call of any entry point on the device): no allocation there either.
 */
int maxsim_backward_csr_static(const void *Q, int n_q, int l_q, const void *D, int64_t b, int l_d, int d,
                               maxsim_dtype dtype, const int32_t *argmax, const float *dscore, float *dQ,
                               float *dD, void *stream);

/*
 * Per-token symmetric absmax quantiser (Sec. "Quantised Scoring").
 *   X      [rows, d] dtype
 *   X_i8   [rows, d] int8    round_half_even(x / scale), clamped to [-127, 127]
 *   scale  [rows]    float32 absmax / 127 (IEEE fp32 division); an all-zero row gets scale 0, codes 0
 */
int maxsim_quantize_rows_i8(const void *X, int64_t rows, int d, maxsim_dtype dtype, int8_t *X_i8,
                            float *scale, void *stream);

/*
 * int8 x int8 scoring with deferred dequantisation (Alg. 4; App. "INT8 Kernel").
 *   Q_i8 [n_q, l_q, d] int8, q_scale [n_q, l_q] float32
 *   D_i8 [b,   l_d, d] int8, d_scale [b,   l_d] float32   (scales must be >= 0; a nonzero
 *        scale below 2^-100 may cost the last bit of a negative score)
 *   scores [n_q, b] float32;  l_q <= 1024, b * l_d < 2^31
 * Per cell: n = exact int32 dot product; v = fl32(n * d_scale[j]); m_i = max_j v;
 * r_i = fl32(q_scale[i] * m_i); score = sum_i r_i carried in fp64 and rounded once to fp32.
 * The result is a pure function of the inputs (bitwise reproducible).
 */
int maxsim_forward_i8(const int8_t *Q_i8, const float *q_scale, int n_q, int l_q,
                      const int8_t *D_i8, const float *d_scale, int64_t b, int l_d, int d,
                      float *scores, void *stream);

/*
 * int8 scoring of a packed ragged corpus (Sec. "Ragged corpora and kernel family" applied to Alg. 4).
 *   D_i8_packed    [total_tokens, d] int8, d_scale_packed [total_tokens] float32
 *   doc_offsets    [b + 1] int32 (device), as in maxsim_forward_ragged; total_tokens < 2^31
 * A document of length 0 gets score -inf.  Arithmetic and other arguments as in maxsim_forward_i8.
 */
int maxsim_forward_i8_ragged(const int8_t *Q_i8, const float *q_scale, int n_q, int l_q,
                             const int8_t *D_i8_packed, const float *d_scale_packed,
                             const int32_t *doc_offsets, int64_t b, int64_t total_tokens, int d,
                             float *scores, void *stream);

/*
 * Out-of-core int8 scoring: maxsim_forward_i8 with codes and scales in HOST memory, streamed like
 * maxsim_forward_streamed.
 *   D_i8_host [b, l_d, d] int8 and d_scale_host [b, l_d] float32 in HOST memory
 *   staging_codes  DEVICE, 2 * block_docs * l_d * d bytes;  staging_scales  DEVICE, 2 * block_docs * l_d floats
 * Other arguments, limits and arithmetic as in maxsim_forward_i8 (identical bits).
 */
int maxsim_forward_i8_streamed(const int8_t *Q_i8, const float *q_scale, int n_q, int l_q,
                               const int8_t *D_i8_host, const float *d_scale_host, int64_t b, int l_d,
                               int d, int64_t block_docs, int8_t *staging_codes, float *staging_scales,
                               float *scores, void *stream);

/*
 * Gradient of the in-batch-negatives cross-entropy on a score matrix (helper for the
 * contrastive training step; the paper leaves the loss open, this is softmax
 * cross-entropy with temperature tau, label of query i = document i, mean over queries).
 *   scores [n, b] float32 (b >= n);  g [n, b] float32 = (softmax_j(s_i/tau) - [i==j]) / (tau n)
 *   loss   [1] float32 or NULL
 */
int maxsim_ce_grad(const float *scores, int n, int b, float tau, float *g, float *loss,
                   void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MAXSIM_H */
