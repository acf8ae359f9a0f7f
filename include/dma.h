/*
 * dma.h -- C ABI of the MI355X (gfx950) Dynamic Mask Attention hot path.
 *
 * The operations are those of arxiv 2508.02124, Section 4 ("Method"):
 *   dma_mask_gen : content scores  z = exp(A * softplus(v . w))            (Eq. 3)
 *                  and the per-row top-k + causal kept sets                (Eq. 4, Listing 1)
 *   dma_fwd      : O = softmax(Q K^T * scale + z, over the kept set) V     (Eq. 5-6, Alg. 1)
 *   dma_bwd      : dQ, dK, dV and the gradient into z                      (Eq. 7-10, Alg. 2)
 *
 * Conventions for every entry point
 *   - All tensor arguments are DEVICE pointers, 16-byte aligned, densely packed,
 *     token-major, last dimension contiguous:
 *         Q, O, dO, dQ : [T, H_q , d]      K, V, dK, dV : [T, H_kv, d]
 *         z, dz, LSE   : [H_q, T] float    expiry       : [H_q, T] int32
 *         W : [H_q, d] float               A            : [H_q] float
 *         cu_seqlens   : [n_docs + 1] int32, cu[0] = 0, cu[n_docs] = T
 *     Q/K/V/O/dO/dQ/dK/dV are bf16 (dtype DMA_BF16) or float (DMA_F32, a slow
 *     debug path).  A fixed batch of B sequences of length L is T = B*L with
 *     cu_seqlens = {0, L, 2L, ...}.
 *   - q-head h reads kv-head h / (H_q / H_kv) (contiguous grouping).
 *   - The `dma_shape` argument is a HOST pointer, read during the call.
 *   - The caller owns every buffer.  The compute entry points allocate nothing,
 *     free nothing and keep no pointer after the call returns.  The library's only
 *     state between calls: the host array of event handles that dma_profile_events
 *     was given (per host thread, until it is called with NULL), and the address of
 *     dma_decode_static's own device scratch array (per GPU).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and the call returns without synchronising.
 *   - Return value: DMA_OK (0) or a negative dma_status.  All argument checks
 *     happen before the first launch, so a failing call enqueues nothing.
 *   - Outputs are fully overwritten; the caller need not clear them.
 */
#ifndef DMA_H_
#define DMA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DMA_OK = 0,
  DMA_EINVAL = -1,       /* null pointer, misaligned pointer, T<=0, k<=0, n_docs<=0, H_q % H_kv != 0 */
  DMA_EUNSUPPORTED = -2, /* d not in {64,128,256} (cross-head scores: {64,128}),
                            unknown dtype, more than 256 q-heads per kv-head,
                            more than 32 heads for the cross-head scores,
                            bf16 dma_fwd / dma_bwd with T >= 2^24 or Q (or K, V) larger than 4 GiB         */
  DMA_EWORKSPACE = -3,   /* ws_bytes smaller than dma_workspace_bytes() */
  DMA_EHIP = -4          /* a launch failed (hipGetLastError) */
} dma_status;

typedef enum { DMA_BF16 = 0, DMA_F32 = 1 } dma_dtype;

typedef struct {
  int32_t T;            /* total packed tokens                                        */
  int32_t n_docs;       /* number of documents (sequences) packed into T              */
  int32_t max_seqlen;   /* upper bound on the longest document (0 => T)               */
  int32_t H_q;          /* query heads                                                */
  int32_t H_kv;         /* key/value heads, divides H_q                               */
  int32_t d;            /* head dimension: 64, 128 or 256 (256: not for the cross-head
                           scores)                                                    */
  int32_t k;            /* keep-window (the paper's w): kept keys per query row;
                           k larger than a document keeps all of its causal keys      */
  int32_t causal;       /* 1: candidates of row i are the keys j <= i of its document;
                           0: all keys of its document (every row keeps the same keys)  */
  int32_t dtype;        /* dma_dtype of Q/K/V/O and their gradients                   */
  float softmax_scale;  /* 0 => d^-1/2                                                */
} dma_shape;

/* Size in bytes of the opaque mask plan written by dma_mask_gen (slot table,
 * per-block key lists and scratch of the selection), and of the scratch
 * workspace dma_fwd / dma_bwd need.  0 if the shape is invalid.
 * The plan is not linear in T: its slot table holds one int32 per (q-head, block of
 * 256 query rows, slot), slots = min(k, max_seqlen) rounded up to 128, i.e. about
 * H_q * T * min(k, max_seqlen) / 64 bytes, on top of about 40 bytes per (q-head, token)
 * (scores, expiry, key lists, scratch of the selection).  Examples with H_q = 32: 36 MiB
 * at T = 16384, k = 2048; 111 MiB at T = 65536, k = 1024; 0.58 GiB at k = 16384; 2.1 GiB
 * at T = k = 65536 (every key kept: the quadratic corner).  There is no cap: a caller
 * that sweeps k towards T pays this. */
size_t dma_mask_bytes(const dma_shape* shape);
size_t dma_workspace_bytes(const dma_shape* shape);

/*
 * Where the parts of the mask plan lie, for tools and tests that inspect what dma_mask_gen wrote
 * (the occupancy structure of Section 4.2: per block of query rows, the keys resident for the whole
 * block -- one slot column each -- and the keys that enter or expire inside it).  The attention
 * entry points need none of this.  `out` is a HOST pointer; offsets are bytes from the start of the
 * mask buffer.  Returns DMA_OK or the error of an invalid shape.
 *   blocks         int32[nblk_cap][4]: {document, first row, end row, document start}; document -1 past the end
 *   slot_table     int32[H_q][nblk_cap][kpad]: resident key of each slot column, -1 = none
 *   partial_count  int32[H_q][nblk_cap];  partial_list int32[H_q][nblk_cap][max_partial]
 *   header         int32[16], [0] = number of blocks;  zq float[H_q][T] = z / softmax_scale
 */
typedef struct {
  int32_t block_rows;   /* query rows per block                          */
  int32_t group_cols;   /* slot columns per key-stationary workgroup     */
  int32_t max_partial;  /* capacity of a block's partial list            */
  int32_t nblk_cap;     /* rows of the block table: T / block_rows + n_docs */
  int32_t kpad;         /* slot-table row length                         */
  int32_t reserved;
  uint64_t off_header, off_zq, off_blocks, off_slot_table, off_partial_count, off_partial_list, total;
} dma_mask_layout;
int dma_mask_describe(const dma_shape* shape, dma_mask_layout* out);

/*
 * Mask generation (Eq. 3, Eq. 4, Listing 1's mask block).
 *   V          in   [T, H_kv, d]
 *   W, A       in   per-q-head projection vector and gate.  W == NULL means the
 *                   caller supplies z (A is then ignored); z must be finite.
 *   z          out if W != NULL, else in.  z[h, j] = exp(A_h * softplus(w_h . v_{g(h), j}))
 *   expiry     out  e[h, j] (global row index) = first row >= j of j's document
 *                   that does NOT keep key j; e == j: never kept; e == end of the
 *                   document: kept to the end.  Row i keeps key j  <=>  j <= i < e[h, j].
 *                   The kept set of a row is its min(k, i - doc_start + 1) best causal
 *                   keys by (z descending, index ascending).  With causal == 0 every row of a
 *                   document keeps the document's min(k, n) best keys: e[h, j] = end of the
 *                   document for those keys (kept by all rows) and e[h, j] = j for the others.
 *   topk_idx   out, nullable: [H_q, T, k] int32, the kept keys of each row as global
 *                   indices in ascending order, padded with -1 (debug; O(T k) memory).
 *   mask       out  dma_mask_bytes(shape) bytes; consumed by dma_fwd / dma_bwd.  It also holds
 *                   z / softmax_scale (the attention kernels start their score accumulators
 *                   at it) and that softmax_scale itself.  The plan is the authority on both:
 *                   dma_fwd / dma_bwd read the scores and the scale from it, not from their
 *                   own z and shape->softmax_scale arguments (which therefore cannot disagree
 *                   with the stored scores); a changed z or scale needs a new dma_mask_gen.
 *                   The other fields of the shape must be the ones the plan was made with.
 */
int dma_mask_gen(const dma_shape* shape, const void* V, const float* W, const float* A,
                 const int32_t* cu_seqlens, float* z, int32_t* expiry, int32_t* topk_idx,
                 void* mask, void* stream);

/*
 * Mask generation with a further, caller-supplied attention bias (Section 1, "Kernel Design": the
 * kernel takes masks and biases with batch, head and query broadcasting).  The bias holds one value
 * per key, broadcast over the query rows; it is added to the scores of the kept pairs next to z,
 *     S_ij = scale q_i . k_j + z[h, j] + bias[h, j],
 * while the kept sets are selected on z alone (Eq. 4 ranks the content scores).  Everything else is
 * dma_mask_gen; dma_fwd / dma_bwd are called as usual with the mask written here.
 *   bias            in  float, finite (a large negative value acts as a key mask)
 *   bias_heads      H_q: one row per q-head; 1: one row shared by all heads (head broadcast)
 *   bias_per_token  != 0: bias is [bias_heads, T], packed like z;
 *                   == 0: bias is [bias_heads, shape->max_seqlen], indexed by the key's position in
 *                   its document and shared by all documents (batch broadcast); max_seqlen must be
 *                   set and no document may be longer
 * z and the bias enter the score as a sum, so the dz of dma_bwd is also the gradient with respect
 * to the bias as applied; dma_bias_bwd reduces it over the heads and documents that share an entry:
 *   dbias out [bias_heads, T] or [bias_heads, max_seqlen] float, fully overwritten (no atomics).
 * A bias per (query, key) pair has no per-key structure and is not supported.
 */
int dma_mask_gen_bias(const dma_shape* shape, const void* V, const float* W, const float* A,
                      const int32_t* cu_seqlens, const float* bias, int32_t bias_heads, int32_t bias_per_token,
                      float* z, int32_t* expiry, int32_t* topk_idx, void* mask, void* stream);
int dma_bias_bwd(const dma_shape* shape, const float* dz, const int32_t* cu_seqlens, int32_t bias_heads,
                 int32_t bias_per_token, float* dbias, void* stream);

/*
 * Forward (Eq. 5-6; online softmax as in Alg. 1, query-stationary).
 *   O   out [T, H_q, d]     LSE out [H_q, T], natural-log sum-exp of the kept scores.
 *   ws  scratch of at least dma_workspace_bytes(shape) (may be NULL if that is 0).
 */
int dma_fwd(const dma_shape* shape, const void* Q, const void* K, const void* V, const float* z,
            const int32_t* expiry, const void* mask, const int32_t* cu_seqlens,
            void* O, float* LSE, void* ws, size_t ws_bytes, void* stream);

/*
 * Backward (Eq. 7-10; Alg. 2 with D_i = rowsum(dO o O)).
 *   dQ out [T, H_q, d]; dK, dV out [T, H_kv, d], summed over the q-heads of a group;
 *   dz out [H_q, T] = sum over query rows of dS (exactly 0 for keys never kept).
 *   dV is the attention-path gradient only (not the path through z).
 *   dK, dV and dz are accumulated with floating-point atomics: results can differ
 *   in the last bits between runs.
 */
int dma_bwd(const dma_shape* shape, const void* Q, const void* K, const void* V, const void* O,
            const void* dO, const float* LSE, const float* z, const int32_t* expiry,
            const void* mask, const int32_t* cu_seqlens,
            void* dQ, void* dK, void* dV, float* dz, void* ws, size_t ws_bytes, void* stream);

/*
 * Gradient of the content scores (the chain rule of Eq. 3; Section 6: the bias is the path by
 * which gradients reach the score parameters).  With x = w_h . v_{g(h), j}, z = exp(A_h softplus(x)):
 *   dz  in  [H_q, T]        the gradient that dma_bwd returned for the bias
 *   dW  out [H_q, d] f32    dW_h = sum_j dx_{h,j} v_{g(h),j},  dx = dz z A_h sigmoid(x)
 *   dA  out [H_q]    f32    dA_h = sum_j dz z softplus(x)
 *   dV  [T, H_kv, d], dtype of V: the part of dV that flows through z,
 *       sum over the q-heads h of kv-head g of dx_{h,j} w_h; written if accumulate == 0, added
 *       to the existing contents (e.g. the dV of dma_bwd; one rounding of the sum) otherwise.
 * z is recomputed from V, W, A.  dW and dA are accumulated with floating-point atomics.  No
 * workspace; shape->k, n_docs and softmax_scale are not used.  Errors as for the other entry points.
 * Shapes whose group (H_q / H_kv q-heads per kv-head) does not fit the kernel's 64 KiB of LDS --
 * (tile * d + 2 G d + 2 G tile + G) floats with tile = 64 tokens (32 at d = 256), i.e. more than 47 / 21 / 14 q-heads per kv-head at d = 64 / 128 / 256 --
 * are refused with DMA_EUNSUPPORTED before any launch.
 */
int dma_mask_bwd(const dma_shape* shape, const void* V, const float* W, const float* A, const float* dz,
                 float* dW, float* dA, void* dV, int accumulate, void* stream);

/*
 * Content scores with the paper's full sampling tensor (Eq. 3 states Delta in R^{n_h x d_h x n_h};
 * Listing 1 flattens the values of all heads of a token before the projection): the score of q-head
 * h contracts the token's value vectors of ALL kv-heads,
 *     z[h, j] = exp(A_h * softplus(sum_{g, c} V[j, g, c] * Delta[h, g, c])).
 *   Delta in  [H_q, H_kv * d] float, row h = the [H_kv, d] weights of head h (the layout of a linear
 *             layer's weight from the flattened values to the heads)
 *   z     out [H_q, T]; pass it to dma_mask_gen with W == NULL (caller-supplied scores).
 * dma_scores_xhead_bwd is its chain rule, the counterpart of dma_mask_bwd:
 *   dz in [H_q, T];  dDelta out [H_q, H_kv * d] f32 = sum_j dx[h, j] V[j, g, c];  dA out [H_q] f32;
 *   dV [T, H_kv, d], dtype of V: sum_h dx[h, j] Delta[h, g, c], written (accumulate == 0) or added.
 * dDelta and dA are accumulated with floating-point atomics.  H_q <= 32 (DMA_EUNSUPPORTED beyond);
 * shape->k, n_docs and softmax_scale are not used.  No workspace.
 */
int dma_scores_xhead(const dma_shape* shape, const void* V, const float* Delta, const float* A, float* z,
                     void* stream);
int dma_scores_xhead_bwd(const dma_shape* shape, const void* V, const float* Delta, const float* A, const float* dz,
                         float* dDelta, float* dA, void* dV, int accumulate, void* stream);

/*
 * Decode: the newest row of every sequence against its KV cache (Eq. 4-6 for one query row; the
 * regime of the paper's largest speed-ups, Section 5).  Sequence b occupies rows
 * [cu_seqlens[b], cu_seqlens[b+1]) of K, V and z, its last row being the new token; that row's
 * candidates are all n keys of the sequence, of which it keeps the min(k, n) best by
 * (z descending, index ascending).
 *   q     in  [n_docs, H_q, d]   the query of the last row of each sequence
 *   K, V  in  [T, H_kv, d];  z in [H_q, T] (the caller appends the new token's score, e.g. with
 *             dma_mask_gen on the new row or its own Eq. 3)
 *   o     out [n_docs, H_q, d];  lse out [H_q, n_docs] (natural log; -inf and o = 0 for an empty sequence)
 *   kept  out [n_docs, H_q, min(k, T)] int32: the kept keys of each (sequence, head) as global row
 *             indices, ascending, the first min(k, n) entries valid.  The buffer also carries
 *             the kernels' scratch behind that array (per-chunk partial outputs), so it is
 *             required and must hold dma_decode_kept_bytes(shape) bytes (DMA_EWORKSPACE otherwise).
 * Stateless: the selection is redone from z on every call (z is n floats per head, the gathered
 * K/V rows are min(k, n) d-vectors; both are read once or a few times).  No mask plan is needed.
 */
size_t dma_decode_kept_bytes(const dma_shape* shape);
int dma_decode(const dma_shape* shape, const void* q, const void* K, const void* V, const float* z,
               const int32_t* cu_seqlens, void* o, float* lse, int32_t* kept, size_t kept_bytes, void* stream);

/*
 * dma_decode for callers that cannot allocate device memory or pass a scratch region: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same
 * kernels and same results as dma_decode, but the kernels' scratch (per-chunk partial outputs, the
 * selection's histograms and counts) lies in a device array owned by the library, of
 * DMA_DECODE_STATIC_SCRATCH_BYTES on every GPU the library is used on (held until the process ends;
 * its address is looked up on the first call on each device).  The call allocates and frees nothing.
 *   kept  out [n_docs, H_q, min(k, T)] int32 only (no scratch behind it)
 *   Shapes whose scratch, dma_decode_static_scratch_bytes(shape), exceeds the array are refused with
 *   DMA_EWORKSPACE before anything is enqueued (e.g. 1 sequence x 32 heads x k = 2048 x d = 128
 *   needs 0.32 MiB; about 12 such sequences fit).
 *   Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two
 *   streams, two threads) race; calls on one stream are ordered and safe.  Nothing in the array
 *   needs clearing by the caller (each call clears what it accumulates into with a fill kernel).
 */
#define DMA_DECODE_STATIC_SCRATCH_BYTES (4u << 20)
size_t dma_decode_static_scratch_bytes(const dma_shape* shape);
int dma_decode_static(const dma_shape* shape, const void* q, const void* K, const void* V, const float* z,
                      const int32_t* cu_seqlens, void* o, float* lse, int32_t* kept, void* stream);

/*
 * Decode in a loop, with the kept sets carried from step to step (Eq. 4 as a one-in / one-out update:
 * the newest key joins the kept set, or replaces its worst member if it beats it).  For callers
 * that keep every sequence in a region of fixed capacity: sequence b owns rows
 * [cu_seqlens[b], cu_seqlens[b+1]) of K, V and z and currently fills the first seq_lens[b] of them
 * (clamped to the capacity), the last of these being the new token.
 *   seq_lens in  [n_docs] int32 (device)
 *   refresh  != 0: select the kept sets from all scores, as dma_decode does (the first step, or after
 *            anything but "every non-empty sequence grew by exactly one token" happened);
 *            == 0: `kept` still holds what the previous call left for lengths seq_lens[b] - 1; it is
 *            updated in place in O(k) per (sequence, head) instead of O(n).
 *   q, o, lse, kept, kept_bytes: as for dma_decode; the entries of `kept` are global row indices.
 * The scores of earlier tokens must not change between calls (they depend on each token's own value
 * vector only).  Every other argument and error as for dma_decode.
 */
int dma_decode_step(const dma_shape* shape, const void* q, const void* K, const void* V, const float* z,
                    const int32_t* cu_seqlens, const int32_t* seq_lens, int refresh, void* o, float* lse,
                    int32_t* kept, size_t kept_bytes, void* stream);

/*
 * Per-stage timing aid.  dma_mask_gen, dma_fwd and dma_bwd each launch several kernels, so a
 * caller cannot bracket one of them with events from outside.  `events` is a HOST array of
 * 2 * DMA_N_STAGES hipEvent_t handles (as void*) owned by the caller, or NULL to switch the aid
 * off (the default).  While set -- per host thread -- every entry point records events[2*s] on its
 * stream immediately before stage s and events[2*s + 1] immediately after it.  Nothing is
 * synchronised; the caller reads the events after synchronising the stream itself.  The library
 * keeps the `events` pointer (not a copy of the array) until the next call of this function on the
 * same host thread: the array must stay valid that long.  A measurement aid: the step's results do
 * not depend on it.
 */
typedef enum {
  DMA_STAGE_Z = 0,          /* mask_gen: block table + content scores (Eq. 3)            */
  DMA_STAGE_SORT = 1,       /* mask_gen: stable sort + wavelet matrix per (document, head) */
  DMA_STAGE_EXPIRY = 2,     /* mask_gen: expiry of every key (Eq. 4)                      */
  DMA_STAGE_PLAN = 3,       /* mask_gen: slots, slot table, partial lists, topk_idx       */
  DMA_STAGE_FWD = 4,        /* fwd: the attention kernel                                  */
  DMA_STAGE_BWD_ZERO = 5,   /* bwd: (empty: the dQ stage clears the fp32 accumulators)   */
  DMA_STAGE_BWD_DQ = 6,     /* bwd: D and dQ (query-stationary)                           */
  DMA_STAGE_BWD_DKV = 7,    /* bwd: dK, dV, dz on the slot columns (key-stationary)       */
  DMA_STAGE_BWD_PART = 8,   /* bwd: dK, dV, dz of keys entering / expiring inside a block */
  DMA_STAGE_BWD_CVT = 9,    /* bwd: fp32 accumulators -> output dtype                     */
  DMA_N_STAGES = 10
} dma_stage;
void dma_profile_events(void** events);

const char* dma_strerror(int status);
int dma_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DMA_H_ */
