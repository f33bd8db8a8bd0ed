/*
 * svg2.h -- C ABI of the MI355X (gfx950) implementation of the per-layer
 * sparse-attention path of Sparse VideoGen2 (arXiv 2505.18875):
 *
 *   k-means of Q and K tokens per head          Section 4.1
 *   semantic-aware permutation                  Section 4.1
 *   centroid-based top-p selection              Section 4.2, Eq. 1, Eq. 2
 *   block-sparse attention, variable block size Section 4.3
 *
 * Conventions (all entry points)
 *   - Every data pointer is a DEVICE pointer owned by the caller unless the
 *     comment says HOST.  Tensors are dense, row-major, innermost dimension
 *     contiguous; a batch dimension is folded into H.  Nothing is retained
 *     after a call returns.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without synchronising.  The
 *     library allocates no device memory: scratch comes in through
 *     (ws, ws_bytes), whose required size the matching *_workspace_size
 *     function returns (0 is never returned; ws must be 256-byte aligned).
 *     A call enqueues kernel launches only (no memset or copy commands, no
 *     read-back of device values, launch sizes depend on the arguments
 *     alone), so it may be recorded into a HIP graph and replayed; stale
 *     workspace contents never matter.
 *   - Return value: SVG2_OK or an error code; svg2_last_error() (thread-local,
 *     HOST string) says why.  Arguments, workspace and kernel attributes are
 *     checked before the first launch: SVG2_INVALID_ARG, SVG2_UNSUPPORTED and
 *     SVG2_WORKSPACE_TOO_SMALL mean that nothing was enqueued and no buffer was
 *     touched.  SVG2_HIP_ERROR can also come from a launch in the middle of a
 *     call; outputs and in/out buffers are then undefined.
 *   - dtype is SVG2_F32 or SVG2_BF16 (storage type of Q, K, V, O); d is 64 or
 *     128; 1 <= C <= min(N, SVG2_MAX_CLUSTERS); 1 <= H <= 65535 (svg2_forward*:
 *     H <= 32767); N >= 1 and
 *     H*N*d < 2^40.  The attention entry points (svg2_sparse_attn*,
 *     svg2_forward*, svg2_sparse_attn_fp8) also need one head of K or V to stay
 *     below 2^31 bytes (N*d*sizeof(element) < 2^31; for svg2_sparse_attn_fp8
 *     counted at two bytes per element): their kernels address rows by 32-bit
 *     byte offsets, and a longer head is SVG2_INVALID_ARG.  Attention
 *     accumulates in fp32.
 *   - Readings of the paper where it is silent: squared Euclidean distance;
 *     one k-means iteration = assign then update; an empty cluster keeps its
 *     centroid; argmin ties go to the lowest cluster index; for bf16 input
 *     the assign step uses the centroids rounded to bf16 (returned centroids
 *     stay fp32 means: the cluster sums are formed in double precision and
 *     rounded once) and its labels are those of exact arithmetic on these
 *     operands (a token whose two best candidates are closer than the rounding
 *     error of the fp32 contraction is re-decided in double precision); for
 *     fp32 input the labels are those of fp32 arithmetic; tokens keep their
 *     original order inside a cluster;
 *     top-p keeps the cluster whose mass crosses p; equal P' goes to the lower
 *     index; empty key clusters are never selected; softmax is renormalised
 *     over the selected keys.
 */
#ifndef SVG2_H
#define SVG2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SVG2_MAX_CLUSTERS 4096

enum {
    SVG2_OK = 0,
    SVG2_INVALID_ARG = 1,          /* null pointer, size out of range, ... */
    SVG2_UNSUPPORTED = 2,          /* dtype or head dimension not built    */
    SVG2_WORKSPACE_TOO_SMALL = 3,
    SVG2_HIP_ERROR = 4             /* a HIP runtime call failed            */
};

enum { SVG2_F32 = 0, SVG2_BF16 = 1 };

/* HOST string describing the last error on the calling thread ("" if none). */
const char *svg2_last_error(void);

/* Library version, major*100 + minor. */
int svg2_version(void);

/* ---------------------------------------------------------------------------
 * svg2_kmeans -- Section 4.1: Lloyd k-means, independently for each head.
 *   X              [H,N,d] dtype          tokens (Q or K of one layer)
 *   init_centroids [H,C,d] fp32           required; pass last step's output to
 *                                         warm-start (centroid cache, Section 4.3)
 *   centroids      [H,C,d] fp32  out      means of the returned clusters; may
 *                                         alias init_centroids
 *   labels         [H,N]   int32 out      cluster of each token (last assign)
 *   counts         [H,C]   int32 out      cluster sizes |Q_i| / |K_j|
 *   objective      [H,iters] fp32 out or NULL: sum of squared distances right
 *                                         after each assign step
 *   iters >= 1 iterations of (assign, update).
 * ------------------------------------------------------------------------- */
size_t svg2_kmeans_workspace_size(int dtype, int H, int N, int d, int C);
int svg2_kmeans(const void *X, int dtype, int H, int N, int d, int C, int iters,
                const float *init_centroids, float *centroids, int32_t *labels,
                int32_t *counts, float *objective,
                void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * svg2_permute -- Section 4.1: the permutation pi that makes every cluster
 * contiguous, as an index vector, and its application to up to two tensors
 * (K and V share pi_k).
 *   labels   [H,N]   int32            values in [0,C)
 *   offsets  [H,C+1] int32 out        cluster c occupies sorted rows
 *                                     offsets[c] .. offsets[c+1]; offsets[C] = N
 *   perm     [H,N]   int32 out        sorted row r holds original token perm[r]
 *                                     (clusters ascending, stable inside)
 *   inv_perm [H,N]   int32 out or NULL  inv_perm[perm[r]] = r
 *   n_tensors in 0..2; src, dst: HOST arrays of n_tensors DEVICE pointers,
 *   each [H,N,d] dtype; dst[t][h,r,:] = src[t][h,perm[h,r],:].  dst must not
 *   overlap src.  With n_tensors = 0, src/dst/dtype/d are ignored.
 *   A label outside [0,C) is undefined behaviour (it is the output of
 *   svg2_kmeans in the intended use).
 * ------------------------------------------------------------------------- */
size_t svg2_permute_workspace_size(int H, int N, int C);
int svg2_permute(const int32_t *labels, int H, int N, int C,
                 int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                 int n_tensors, const void *const *src, void *const *dst,
                 int dtype, int d, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * svg2_permute_noalloc -- svg2_permute for callers that cannot allocate device
 * memory or size a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid the allocator.  Same arguments (minus the
 * workspace) and bit-identical results; the sort's scratch (one int32 per head,
 * chunk of 1024 tokens and cluster) lives in an array of
 * SVG2_PERMUTE_NOALLOC_SCRATCH_BYTES inside the library, which every GPU the
 * library runs on holds until the process ends.  The call allocates nothing,
 * frees nothing and only enqueues kernels on `stream`.
 *   Limit: H * ceil(N / 1024) * C * 4 <= SVG2_PERMUTE_NOALLOC_SCRATCH_BYTES,
 *   else SVG2_WORKSPACE_TOO_SMALL and nothing is launched (the Wan-like K side,
 *   H = 40, N = 75,600, C = 500, needs 5.9 MB).
 *   Every call on one GPU uses the same array: calls that overlap in time on
 *   one GPU (different streams, different threads) race and must be serialised
 *   by the caller; calls on one stream are ordered and safe.  Stale contents of
 *   the array never matter (every entry that is read is written first).
 * ------------------------------------------------------------------------- */
#define SVG2_PERMUTE_NOALLOC_SCRATCH_BYTES (16u << 20)
int svg2_permute_noalloc(const int32_t *labels, int H, int N, int C,
                         int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                         int n_tensors, const void *const *src, void *const *dst,
                         int dtype, int d, void *stream);

/* ---------------------------------------------------------------------------
 * svg2_select_topp -- Section 4.2: S_ij = cq_i . ck_j / sqrt(d) (Eq. 1),
 * P'_ij = |K_j| exp(S_ij) / sum_k |K_k| exp(S_ik) (Eq. 2); for each query
 * cluster the key clusters are taken in descending P' until the accumulated
 * P' reaches top_p (0 < top_p <= 1; top_p = 1 keeps every non-empty cluster).
 *   cq [H,Cq,d], ck [H,Ck,d] fp32     centroids
 *   counts_q [H,Cq] int32 or NULL     query clusters of size 0 get an empty row
 *   counts_k [H,Ck] int32             |K_j|
 *   row_ptr  [H,Cq+1] int32 out       CSR row pointers, relative to the head's
 *                                     segment of col_idx (row_ptr[h,0] = 0)
 *   col_idx  [H,Cq*Ck] int32 out      head h owns entries h*Cq*Ck ...; selected
 *                                     key clusters of row i, ascending
 *   p_est    [H,Cq,Ck] fp32 out or NULL   P'
 *   density  [H] fp32 out or NULL     sum over selected pairs |Q_i||K_j| /
 *                                     (N_q N_k) (Section 5.1); needs counts_q
 * ------------------------------------------------------------------------- */
size_t svg2_select_topp_workspace_size(int H, int Cq, int Ck);
int svg2_select_topp(const float *cq, const float *ck,
                     const int32_t *counts_q, const int32_t *counts_k,
                     int H, int Cq, int Ck, int d, float top_p,
                     int32_t *row_ptr, int32_t *col_idx, float *p_est, float *density,
                     void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * svg2_sparse_attn -- Section 4.3: every row of query cluster i attends, with
 * an ordinary softmax, over the keys of the key clusters selected for i.
 *   Qp, Kp, Vp [H,N,d] dtype          permuted tensors (clusters contiguous)
 *   offsets_q [H,Cq+1], offsets_k [H,Ck+1], row_ptr [H,Cq+1],
 *   col_idx [H,Cq*Ck]                 as produced by svg2_permute / svg2_select_topp
 *   perm_q [H,N] int32 or NULL        result of sorted row r is stored at row
 *                                     perm_q[r] (the inverse permutation of
 *                                     Section 4.1); NULL leaves sorted order
 *   scale <= 0 means 1/sqrt(d)
 *   O   [H,N,d] dtype out; lse [H,N] fp32 out or NULL (natural log of the
 *   softmax denominator, -inf for a row with no selected key, whose O is 0).
 *   Dense attention is the special case Cq = Ck = 1, row_ptr = {0,1},
 *   col_idx = {0}, offsets = {0,N}.
 * ------------------------------------------------------------------------- */
size_t svg2_sparse_attn_workspace_size(int dtype, int H, int N, int d, int Cq, int Ck);
int svg2_sparse_attn(const void *Qp, const void *Kp, const void *Vp, int dtype,
                     int H, int N, int d, int Cq, int Ck,
                     const int32_t *offsets_q, const int32_t *offsets_k,
                     const int32_t *row_ptr, const int32_t *col_idx,
                     const int32_t *perm_q, float scale, void *O, float *lse,
                     void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * svg2_sparse_attn_gather_free -- Section 4.3 as the paper describes its own
 * kernel: keys and values are loaded sparsely, token by token, and computed
 * densely, so no permuted copy of Q, K or V exists.  Same result as
 * svg2_sparse_attn on the permuted copies.
 *   Q, K, V [H,N,d] dtype             in ORIGINAL token order
 *   perm_q, perm_k [H,N] int32        both required (svg2_permute's perm)
 *   every other argument as in svg2_sparse_attn; O is in original token order.
 * Workspace: svg2_sparse_attn_workspace_size.
 * ------------------------------------------------------------------------- */
int svg2_sparse_attn_gather_free(const void *Q, const void *K, const void *V, int dtype,
                                 int H, int N, int d, int Cq, int Ck,
                                 const int32_t *offsets_q, const int32_t *offsets_k,
                                 const int32_t *row_ptr, const int32_t *col_idx,
                                 const int32_t *perm_q, const int32_t *perm_k,
                                 float scale, void *O, float *lse,
                                 void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * svg2_forward -- the whole layer (Section 4): k-means of Q and of K,
 * both permutations, selection, sparse attention, output in original order.
 *   Q, K, V [H,N,d] dtype; O [H,N,d] dtype out
 *   cq_inout [H,Cq,d], ck_inout [H,Ck,d] fp32: initial centroids in, final
 *   centroids out -- pass the same buffers at the next denoising step to
 *   warm-start it (centroid cache, Section 4.3).
 *   aux: HOST struct or NULL.  A non-NULL member is a DEVICE buffer that
 *   receives that intermediate result; a NULL member lives in the workspace.
 * ------------------------------------------------------------------------- */
typedef struct svg2_forward_aux {
    int32_t *labels_q;   /* [H,N]     */
    int32_t *labels_k;   /* [H,N]     */
    int32_t *counts_q;   /* [H,Cq]    */
    int32_t *counts_k;   /* [H,Ck]    */
    int32_t *offsets_q;  /* [H,Cq+1]  */
    int32_t *offsets_k;  /* [H,Ck+1]  */
    int32_t *perm_q;     /* [H,N]     */
    int32_t *perm_k;     /* [H,N]     */
    int32_t *row_ptr;    /* [H,Cq+1]  */
    int32_t *col_idx;    /* [H,Cq*Ck] */
    float *density;      /* [H]       */
    float *lse;          /* [H,N]     */
} svg2_forward_aux;

size_t svg2_forward_workspace_size(int dtype, int H, int N, int d, int Cq, int Ck);
int svg2_forward(const void *Q, const void *K, const void *V, int dtype,
                 int H, int N, int d, int Cq, int Ck, float top_p, int iters,
                 float *cq_inout, float *ck_inout, void *O,
                 const svg2_forward_aux *aux,
                 void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * svg2_forward_gather_free -- svg2_forward without the physical permutation of
 * Q, K and V (Section 4.3, sparse loading): the permutations exist as index
 * vectors only and the attention kernel fetches rows through them.  Same
 * arguments and results as svg2_forward; the workspace is smaller by three
 * [H,N,d] tensors.
 * ------------------------------------------------------------------------- */
size_t svg2_forward_gather_free_workspace_size(int dtype, int H, int N, int d, int Cq, int Ck);
int svg2_forward_gather_free(const void *Q, const void *K, const void *V, int dtype,
                             int H, int N, int d, int Cq, int Ck, float top_p, int iters,
                             float *cq_inout, float *ck_inout, void *O,
                             const svg2_forward_aux *aux,
                             void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * FP8 attention -- the "+ FP8" rows of Table 1.  The paper names the precision
 * but not the recipe; this library's reading: Q, K and V are stored as OCP
 * E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, largest value
 * 448, no infinities) with ONE scale per head and tensor; scores, softmax and
 * accumulators are fp32; the probabilities enter the second matrix product as
 * E4M3 as well.  k-means, permutation and selection are unchanged (they read
 * the bf16 tensors).  Head dimension 128 and SVG2_BF16 outputs only
 * (SVG2_UNSUPPORTED otherwise).
 *
 * svg2_quantize_fp8: per head h, amax = max |X[h]|, X8 = E4M3(X * (448 / amax))
 * (single-precision product, round to nearest even), scale[h] = amax / 448, so
 * X ~ decode(X8) * scale[h]; an all-zero head gets scale 1.
 *   X [H,N,d] dtype; X8 [H,N,d] bytes out; scale [H] fp32 out
 *
 * svg2_sparse_attn_fp8: svg2_sparse_attn on such operands.
 *   Q8, K8, V8 [H,N,d] bytes; scale_q, scale_k, scale_v [H] fp32
 *   perm_k NULL: the operands are the PERMUTED copies (perm_q optional, as in
 *   svg2_sparse_attn); perm_k given: they are in token order and rows are
 *   fetched through perm_q / perm_k (as in svg2_sparse_attn_gather_free).
 *   O [H,N,d] bf16 out, lse [H,N] fp32 out or NULL (of the scores the kernel
 *   actually used, i.e. of the quantised operands).
 *   Workspace: svg2_sparse_attn_workspace_size(SVG2_BF16, ...).
 *
 * svg2_forward_fp8: svg2_forward_gather_free with the attention step on E4M3
 * copies of Q, K, V (made in the workspace, in token order).  Arguments and
 * results as svg2_forward; dtype must be SVG2_BF16.
 * ------------------------------------------------------------------------- */
size_t svg2_quantize_fp8_workspace_size(int H);
int svg2_quantize_fp8(const void *X, int dtype, int H, int N, int d,
                      void *X8, float *scale,
                      void *ws, size_t ws_bytes, void *stream);
int svg2_sparse_attn_fp8(const void *Q8, const void *K8, const void *V8,
                         const float *scale_q, const float *scale_k, const float *scale_v,
                         int H, int N, int d, int Cq, int Ck,
                         const int32_t *offsets_q, const int32_t *offsets_k,
                         const int32_t *row_ptr, const int32_t *col_idx,
                         const int32_t *perm_q, const int32_t *perm_k,
                         float scale, void *O, float *lse,
                         void *ws, size_t ws_bytes, void *stream);
size_t svg2_forward_fp8_workspace_size(int dtype, int H, int N, int d, int Cq, int Ck);
int svg2_forward_fp8(const void *Q, const void *K, const void *V, int dtype,
                     int H, int N, int d, int Cq, int Ck, float top_p, int iters,
                     float *cq_inout, float *ck_inout, void *O,
                     const svg2_forward_aux *aux,
                     void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * svg2_attention_recall -- Section 3.1: attention recall = the share of a
 * query's true attention mass (softmax over ALL keys) that the computed keys
 * capture.  For query n, with lse_selected[n] the log-sum-exp of its scores
 * over the selected keys (svg2_sparse_attn's lse) and lse_all[n] the one over
 * all keys (svg2_sparse_attn's lse in the dense special case),
 * recall[n] = exp(lse_selected[n] - lse_all[n]) (0 when nothing is selected).
 *   lse_selected, lse_all [H,N] fp32
 *   recall      [H,N] fp32 out or NULL
 *   recall_mean [H]   fp32 out          mean over the head's queries
 * ------------------------------------------------------------------------- */
size_t svg2_attention_recall_workspace_size(int H, int N);
int svg2_attention_recall(const float *lse_selected, const float *lse_all, int H, int N,
                          float *recall, float *recall_mean,
                          void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * svg2_kmeans_pp_init -- Sections 4.3 / 5.3: k-means++ seeding, the
 * initialisation of a k-means that has no centroid cache to start from.
 * Per head: centre 0 is token floor(u[0] N); centre k >= 1 is the first token
 * whose running sum of D2 exceeds u[k] sum(D2), where D2 is the squared
 * distance of a token to the nearest centre chosen so far (so a token is
 * drawn with probability D2 / sum(D2)); if every D2 is zero, token
 * floor(u[k] N).  The random numbers are the caller's.
 *   X         [H,N,d] dtype
 *   u         [H,C]   fp64              uniform numbers in [0,1)
 *   centroids [H,C,d] fp32 out          the drawn tokens (input of svg2_kmeans)
 *   picked    [H,C]   int32 out or NULL their token indices
 * All arithmetic is fp64; C passes over X.
 * ------------------------------------------------------------------------- */
size_t svg2_kmeans_pp_init_workspace_size(int H, int N, int C);
int svg2_kmeans_pp_init(const void *X, int dtype, int H, int N, int d, int C,
                        const double *u, float *centroids, int32_t *picked,
                        void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * Timing for benchmarks (HOST-side state, one per process).
 * svg2_profile_enable(1): every later svg2_forward* call records HIP events
 * around its stages on the caller's stream (events are created on first use;
 * at most SVG2_PROFILE_MAX_CALLS calls are kept, later ones go unrecorded).
 * svg2_profile_enable(2): additionally an event pair around every kernel launch
 * of k-means and of the permutation (also inside svg2_kmeans / svg2_permute),
 * at most SVG2_PROFILE_MAX_SPANS of them; these events sit between kernels
 * that otherwise run back to back, so level 2 is for attributing time to
 * kernels, not for timing the layer.  svg2_profile_enable(0) stops recording.
 * svg2_profile_read waits for the recorded events, writes the summed
 * milliseconds per stage to stage_ms (HOST array of SVG2_N_STAGES floats, in
 * the order k-means of Q and K (both sides share their launches), permutation
 * Q+K (svg2_forward_fp8: plus the E4M3 quantisation of Q, K, V), selection,
 * attention plan, attention kernel) and the number of recorded calls to
 * n_calls (HOST), then clears the record.
 * svg2_profile_read_kernels does the same per kernel class (HOST arrays of
 * SVG2_N_KERNEL_CLASSES floats / ints: summed milliseconds, launches), in the
 * order of the SVG2_K_* constants.
 * ------------------------------------------------------------------------- */
#define SVG2_N_STAGES 5
#define SVG2_PROFILE_MAX_CALLS 256
#define SVG2_PROFILE_MAX_SPANS 16384
enum {
    SVG2_K_KMEANS_ASSIGN = 0,      /* assign step, Q and K side in one launch (Section 4.1) */
    SVG2_K_KMEANS_SETTLE = 1,      /* near-ties again in double precision                   */
    SVG2_K_KMEANS_SORT = 2,        /* counting sort of the labels (3 kernels)               */
    SVG2_K_KMEANS_SEGSUM_FULL = 3, /* segmented sum over all tokens                         */
    SVG2_K_KMEANS_SEGSUM_DELTA = 4,/* segmented sum over the tokens whose label changed     */
    SVG2_K_KMEANS_FINALIZE = 5,    /* means, bf16 copy, norms                               */
    SVG2_K_PERMUTE_SORT = 6,       /* permutation index vectors of Q and K (3 kernels)      */
    SVG2_K_PERMUTE_GATHER = 7,     /* permuted copies of Q, K, V                            */
    SVG2_N_KERNEL_CLASSES = 8
};
int svg2_profile_enable(int level);
int svg2_profile_read(float *stage_ms, int *n_calls);
int svg2_profile_read_kernels(float *kernel_ms, int *launches);

#ifdef __cplusplus
}
#endif
#endif /* SVG2_H */
