/*
 * rr_attn.h -- C ABI of the RRAttention prefill path for AMD MI355X (gfx950).
 *
 * Two stages, as in the paper (arxiv 2602.05853):
 *   rr_estimate     pattern estimation (Sec. 3.1-3.3): per-head round-robin query sampling,
 *                   stride-level importance, causal stride softmax, block mass, adaptive
 *                   Top-tau selection with last-query-block protection -> block mask.
 *   rr_sparse_attn  causal block-sparse attention over the selected blocks (Sec. 2.1).
 *   rr_dense_attn   the dense causal baseline (every causal block), same kernels.
 * All three also take a step of the last Lq positions of a context (chunked prefill, decode stage).
 * Around them: rr_estimate_ex (estimator variants of the ablations, packed sequences),
 * rr_dense_attn_packed, rr_mask_from_dense (caller-made masks), rr_selection_accuracy (the
 * appendix's precision / recall / F1 diagnostic), rr_sparse_attn_ws / rr_dense_attn_ws (attention with a
 * workspace, for short steps), rr_estimate_static (estimation without a workspace argument).
 *
 * Conventions common to all entry points
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library allocates
 *     nothing, frees nothing and never synchronises: work is enqueued on `hip_stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and results are valid once
 *     that stream has reached the end of the call.
 *   - Argument errors are detected on the host before any launch and reported through the
 *     return code; nothing is written in that case.  A failed launch returns RR_ERR_LAUNCH.
 *   - Indices are 0-based.  Query head h reads KV head h / (Hq / Hkv).
 *   - Tensors are addressed as base + b*stride_b + h*stride_h + l*stride_l + c with strides in
 *     ELEMENTS and the head dimension contiguous.  Rows must be 16-byte aligned (base pointer
 *     and every stride a multiple of 16 bytes).  O uses the layout of Q.
 *   - Lengths.  L need not be a multiple of B or S.  As in the paper's problem statement there are
 *     Nb = ceil(L/B) blocks, the last one possibly partial (Sec. 2.1), and floor(L/S) strides, one
 *     sampled query each (Sec. 3.1); positions after the last complete stride are in no stride --
 *     never sampled, never scored -- but are attended like any other.  A last query block without
 *     one complete stride has no estimate and keeps every causal block.  Tensors hold exactly L
 *     (or Lq) positions: nothing past them is read or written.  Below, x/B for a length x means
 *     ceil(x/B).
 *   - Steps: chunked prefill and the decode stage.  L is the number of keys (the context so far).  With
 *     0 < Lq < L the Q and O tensors hold only the LAST Lq positions of the sequence (row r of Q is token
 *     q0 + r, q0 = L - Lq) and every entry point works on those query rows against all L keys.  Any Lq >= 1
 *     and any q0 are allowed: a chunk of a long prompt, a few speculative tokens, one decoded token.  (The
 *     paper applies the method to prefill and decodes densely, Sec. 4.1; its "Future Work" names the decode
 *     stage as an extension without giving an algorithm.  What this library computes for a step is the method
 *     of Sec. 3.1-3.3 applied to the queries the step holds, as follows.)
 *     The query blocks of a step are the blocks its positions touch, floor(q0/B) .. ceil(L/B) - 1; the first
 *     one may begin in front of q0.  Mask arrays have that many rows (first row = query block floor(q0/B)) of
 *     L/B entries: dense / row_list / block_mass [batch, Hq, rows, L/B], row_count [batch, Hq, rows],
 *     row_order [batch, Hkv, G*rows] with rows encoded as hl*rows + local row; lse is [batch, Hq, Lq].
 *     A row's estimate uses those sampled positions of its block (Sec. 3.1) that lie inside the step
 *     (>= q0) and in a complete stride; a row left without any keeps every causal block -- so a one-token
 *     step attends densely unless the token is its head's sampled position of a stride it completes.
 *     The "last query block" of RR_FLAG_PROTECT_LAST is block ceil(L/B) - 1, the last row of the step: set
 *     the flag only when the context ends there (the final chunk of a prompt); a decode step that should
 *     select blocks leaves it clear.  Lq = 0 or L is ordinary prefill.  rr_selection_accuracy takes whole
 *     blocks only (B divides q0).
 *   - Supported: dtype bf16 or f32; d a multiple of 8 with 8 <= d <= 256; S | B;
 *     B <= 128 (so B/S <= 128; S = 1 yields the exact block mass of full attention);
 *     L/B <= 8192.  Attention with bf16, d = 128, B = 128 runs on the MFMA kernel; every other
 *     attention shape on a generic kernel that needs B*d <= 8192 (RR_ERR_SHAPE otherwise).  Estimation with bf16, d = 128, B/S in {4, 8, 16, 32} and
 *     (Hq/Hkv)*(B/S) <= 256 runs on the MFMA kernel, everything else on a generic one.
 */
#ifndef RR_ATTN_H
#define RR_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RR_OK = 0,
    RR_ERR_NULL = -1,      /* a required pointer is NULL                                    */
    RR_ERR_SHAPE = -2,     /* S does not divide B, more queries than keys,                    */
                           /* Hkv does not divide Hq, unsupported d / B / S, misaligned stride */
    RR_ERR_DTYPE = -3,     /* dtype is neither RR_BF16 nor RR_F32                            */
    RR_ERR_PARAM = -4,     /* tau outside (0, 1], unknown flag bits, mask geometry mismatch  */
    RR_ERR_WORKSPACE = -5, /* workspace NULL or smaller than rr_workspace_bytes()            */
    RR_ERR_LAUNCH = -6,    /* the HIP runtime refused a launch                               */
    RR_ERR_SCRATCH_LIMIT = -7 /* rr_estimate_static: the geometry needs more scratch than the library holds */
} rr_status;

typedef enum { RR_BF16 = 0, RR_F32 = 1 } rr_dtype;

/* Geometry of Q [batch, Hq, L, d] and of K, V [batch, Hkv, L, d]; strides in elements. */
typedef struct {
    int32_t batch, L, Hq, Hkv, d;
    int32_t dtype;                                   /* rr_dtype */
    int64_t q_stride_b, q_stride_h, q_stride_l;      /* also the layout of O */
    int64_t kv_stride_b, kv_stride_h, kv_stride_l;   /* K and V share one layout */
    int32_t Lq;                                      /* chunked prefill: number of queries, see below; 0 = L */
} rr_shape;

/*
 * Block selection of one call: the matrix B of Sec. 2.1 in three equivalent forms.
 * Nb = ceil(L / B).  All arrays are device memory, contiguous, row-major.
 *   dense      [batch, Hq, Nb, Nb] 0/1 bytes, entry (m, n) = query block m attends key block n;
 *              entries with n > m are always 0.  May be NULL (not written then).
 *   row_count  [batch, Hq, Nb]     number of selected key blocks of query block m.  Required.
 *   row_list   [batch, Hq, Nb, Nb] the selected n of row m in ascending order in the first
 *              row_count entries; the rest of the row is left untouched.  Required.
 *   block_mass [batch, Hq, Nb, Nb] optional diagnostic: block mass of Sec. 3.3 divided by the
 *              row total (so each row sums to 1), 0 for n > m.  NULL = not written.
 *   row_order  [batch, Hkv, G*Nb]  optional scheduling hint, G = Hq/Hkv: per KV head, the rows
 *              (hl, m) of its G query heads encoded as hl*Nb + m, in the order their workgroups
 *              should start (rows of similar row_count together, heaviest first).  rr_estimate fills it when non-NULL; rr_sparse_attn, when it is non-NULL,
 *              starts the rows in this order so that equally loaded workgroups run side by side.
 *              It must be a permutation of 0 .. G*Nb-1 per (batch, KV head): a row that is missing
 *              is not computed; out-of-range entries are ignored.  NULL = rows are started by
 *              descending m.  It never changes any result.  Not used when G*Nb > 32768.
 *   queue      [RR_QUEUE_WORDS] int32, optional: row counters for rr_sparse_attn.  With row_order and
 *              queue both non-NULL (bf16, d = 128, B = 128) the launch is one workgroup per compute unit
 *              that draws rows from these counters in the order of row_order, instead of one workgroup
 *              per row: the compute units share the rows dynamically and each fetches its next row's
 *              list while it works.  The words must be zero when a launch starts; the launch leaves them
 *              zero, and rr_estimate / rr_mask_from_dense zero them when they fill row_order.  Two
 *              launches that overlap in time must not share a queue (give each mask its own).  NULL =
 *              one workgroup per row.  It never changes any result.  (Used for contexts of up to 256
 *              blocks, where the start of a row is a visible share of it; longer ones are launched one
 *              workgroup per row either way.)
 * rr_sparse_attn reads only row_count, row_list, row_order and queue; entries of row_list must satisfy
 * 0 <= n <= m, strictly ascending (counts and entries outside these ranges are clamped into them
 * on the device, so a malformed list gives a wrong row but no stray memory access).  A row with
 * count 0 yields O = 0 and lse = -inf for its queries.
 */
typedef struct {
    uint8_t* dense;
    int32_t* row_count;
    int32_t* row_list;
    float*   block_mass;
    int32_t  Nb;
    int32_t  B;
    int32_t* row_order;
    int32_t* queue;
} rr_mask;
#define RR_QUEUE_WORDS 160

/* flags of rr_estimate */
#define RR_FLAG_PROTECT_LAST 1u   /* keep every block of the last query block (Sec. 3.3, B^static) */
#define RR_FLAG_DIAGONAL_TOKEN 2u /* alternative reading of the importance equation (Sec. 3.2) for the sampled
                                     query's own stride: only the keys up to the query's position are summed
                                     there (default: the whole stride, whatever the head's offset) */

/* Library version as major*10000 + minor*100 + patch (500 = 0.5.0). */
int rr_version(void);

/* Static text for a status code; never NULL. */
const char* rr_status_string(int status);

/*
 * Bytes of scratch rr_estimate needs for this geometry: the per-KV-head stride sums of K (inner sum
 * of the importance equation, Sec. 3.2) -- fp32, or three bf16 terms per sum on the matrix-core path
 * -- plus one fp32 block mass per (query head, query block, key block) on that path (176 MiB for 32/8
 * heads at 128K tokens with S = 16, B = 128), a few MB of per-chunk softmax states where the key
 * strides of a row are shared out among several workgroups (short contexts, steps), or, on the
 * generic path, room for a query block's softmax state when it does not fit in LDS.  Returns 0 on
 * invalid geometry.
 */
size_t rr_workspace_bytes(const rr_shape* shape, int S, int B);

/*
 * Pattern estimation, Sec. 3.1-3.3.
 *   Q, K        device tensors described by `shape` (V is not needed).
 *   S           sampling stride: query head h contributes the query at i*S + S-1-(h mod S)
 *               of every stride i (Sec. 3.1); keys are summed per stride (Sec. 3.2).
 *   B           block size of the mask.
 *   tau         cumulative-mass threshold in (0, 1]: per query block the key blocks are ranked by
 *               mass (ties: smaller index first) and the shortest prefix whose mass reaches
 *               tau times the row total is kept; tau = 1 keeps every causal block.
 *   flags       0 or an OR of RR_FLAG_PROTECT_LAST, RR_FLAG_DIAGONAL_TOKEN.
 *   workspace   device scratch of at least rr_workspace_bytes() bytes, 256-byte aligned; its
 *               contents are undefined afterwards; calls sharing it must be stream-ordered.
 *   out         arrays to fill (see rr_mask); out->Nb must equal ceil(L/B) and out->B must equal B.
 * The stride softmax is causal at stride granularity (key stride j <= query stride i).
 * Arithmetic: fp32 accumulation of exact products; the block ranking is decided in fp32.
 */
int rr_estimate(const rr_shape* shape, const void* Q, const void* K, int S, int B, float tau,
                uint32_t flags, void* workspace, size_t workspace_bytes, rr_mask* out,
                void* hip_stream);

/*
 * Pattern estimation with the variants compared in the ablations of Sec. 4 (round-robin strategy
 * table; last-query-block table).  The paper names them without formulas; this library takes:
 *   offset_mode  which quantity `phase` replaces h in the sampled position i*S + S-1-(phase mod S):
 *                RR_OFFSET_HEAD   phase = h           (the method, Sec. 3.1)
 *                RR_OFFSET_FIXED  phase = 0           (no round-robin: every head samples the last
 *                                                      position of a stride)
 *                RR_OFFSET_LAYER  phase = layer       (one offset per layer)
 *                RR_OFFSET_HYBRID phase = h + layer
 *   layer        layer index, >= 0 (ignored by HEAD and FIXED).
 *   sink_blocks, recent_blocks  >= 0: after Top-tau, key blocks n < sink_blocks and
 *                m - recent_blocks < n <= m are added to every row m (a union, like the
 *                last-query-block protection).
 *   flags        as for rr_estimate.
 *   seq_first    NULL, or packed sequences (below).
 *   ksum_capacity, ksum_valid  0, 0, or (calls that walk one growing context: the chunks of a long prompt, the
 *                steps behind it) the stride key sums of Sec. 3.2 kept in the workspace from call to call, so
 *                that a call only forms the sums of the positions that are new: ksum_capacity = the number of
 *                positions the sums are laid out for (the same in every call, a multiple of B, >= L: size the
 *                workspace with rr_workspace_bytes() of a shape whose L is this number and whose Lq is the
 *                longest chunk), ksum_valid = the leading positions of K whose sums the workspace already holds
 *                (0 in the first call, then the L of the call before).  The calls must use the same workspace,
 *                S, B and capacity, and K must not have changed below ksum_valid; nothing else may write to the
 *                workspace in between.  Same masks, bit for bit.  Shapes outside bf16 / d = 128 / B/S in {4, 8,
 *                16, 32} form all sums in every call, whatever is given here.
 * rr_estimate(..., flags, ...) is rr_estimate_ex with {flags, RR_OFFSET_HEAD, 0, 0, 0, NULL, 0, 0}.
 * opts == NULL or a value out of range returns RR_ERR_NULL / RR_ERR_PARAM.
 */
typedef enum { RR_OFFSET_HEAD = 0, RR_OFFSET_FIXED = 1, RR_OFFSET_LAYER = 2, RR_OFFSET_HYBRID = 3 } rr_offset_mode;
typedef struct {
    uint32_t flags;
    int32_t  offset_mode;      /* rr_offset_mode */
    int32_t  layer;
    int32_t  sink_blocks;
    int32_t  recent_blocks;
    const int32_t* seq_first;  /* device, [Nb]; NULL = the L positions are one sequence */
    int32_t  ksum_capacity;    /* 0, or positions the kept stride sums are laid out for */
    int32_t  ksum_valid;       /* leading positions whose stride sums the workspace holds */
} rr_estimate_opts;
int rr_estimate_ex(const rr_shape* shape, const void* Q, const void* K, int S, int B, float tau,
                   const rr_estimate_opts* opts, void* workspace, size_t workspace_bytes, rr_mask* out,
                   void* hip_stream);

/*
 * rr_estimate for callers that cannot allocate device memory and have no workspace to hand over: code
 * running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and results as rr_estimate without the workspace pair; the scratch is a fixed array of
 * RR_STATIC_SCRATCH_BYTES inside the library's device image (every GPU the library runs on holds its own
 * copy until the process ends).  Nothing is allocated or freed, by the library or by a routine it calls.
 *   - A geometry whose rr_workspace_bytes() exceeds RR_STATIC_SCRATCH_BYTES is refused with
 *     RR_ERR_SCRATCH_LIMIT before any launch (use rr_estimate with a workspace of your own then).
 *   - All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different streams,
 *     different host threads) race and must be ordered by the caller.  The array keeps the previous call's
 *     contents; nothing in it needs clearing, every word the kernels read was written earlier in the same call.
 *   - The first call on a device looks the array's address up (hipGetSymbolAddress) with that device
 *     current; make that first call outside a stream capture.
 */
#define RR_STATIC_SCRATCH_BYTES (32u << 20)
int rr_estimate_static(const rr_shape* shape, const void* Q, const void* K, int S, int B, float tau,
                       uint32_t flags, rr_mask* out, void* hip_stream);

/*
 * Causal block-sparse attention, Sec. 2.1: O = Softmax(Q K^T / sqrt(d) restricted to M_B) V with
 * M_B[i, j] = 1 iff block (floor(i/B), floor(j/B)) is listed and j <= i.
 *   O    [batch, Hq, L, d] in the layout and dtype of Q.
 *   lse  optional [batch, Hq, L] fp32 contiguous: log of the softmax denominator (natural log,
 *        logits already scaled by 1/sqrt(d)); NULL = not written.
 */
int rr_sparse_attn(const rr_shape* shape, const void* Q, const void* K, const void* V,
                   const rr_mask* mask, void* O, float* lse, void* hip_stream);

/*
 * Dense causal attention (the full-attention baseline of the paper's experiments): identical to
 * rr_sparse_attn with every block n <= m listed; B is the tile height used to walk the keys.
 */
int rr_dense_attn(const rr_shape* shape, const void* Q, const void* K, const void* V, int B,
                  void* O, float* lse, void* hip_stream);

/*
 * Packed sequences (a batch of prompts of different lengths in one call).  The L positions of Q, K, V
 * and O hold several sequences back to back.  Every sequence starts at a multiple of B; a sequence whose
 * length is not a multiple of B is followed by filler positions (any finite values) up to the next
 * multiple, whose outputs are meaningless (the LAST sequence may simply end with the tensors, inside a
 * block: see Lengths above).  The table
 *   seq_first  [Nb] int32, device: seq_first[m] = index of the first block of the sequence that block m
 *              belongs to (so seq_first[m] <= m, and block m starts a sequence iff seq_first[m] == m);
 *              with batch > 1 the one table describes every batch entry
 * is all the library needs: the method treats every sequence by itself (Sec. 3.1-3.3 are stated for one
 * sequence), i.e. the sampled query of stride i sees the key strides of its own sequence only, Top-tau
 * ranks the key blocks seq_first[m] .. m, the last query block of EVERY sequence is protected, and
 * sink_blocks counts from the sequence's first block.  The sampling offsets need no change because
 * every sequence starts at a multiple of S.  The mask has the usual [batch, Hq, Nb, Nb] layout with
 * nothing selected outside a row's own sequence, and goes to rr_sparse_attn as it is: token causality
 * inside the diagonal block keeps real queries away from the filler keys of their own block, and with
 * the last query block protected no real row's mask depends on the filler values.  rr_dense_attn_packed
 * is the matching baseline (row m walks seq_first[m] .. m).  Values outside [0, m] are clamped on the
 * device (a wrong table gives wrong rows, no stray access).  Not combined with a step (Lq < L):
 * RR_ERR_PARAM.
 */
int rr_dense_attn_packed(const rr_shape* shape, const void* Q, const void* K, const void* V, int B,
                         const int32_t* seq_first, void* O, float* lse, void* hip_stream);

/*
 * Attention for steps (Lq much smaller than L: a few decoded or speculative tokens, a short chunk; see "Steps"
 * above): rr_sparse_attn / rr_dense_attn with a workspace.  Such a call has only a few (head, query block)
 * rows, each with a long block list; with a workspace of rr_attn_workspace_bytes() bytes (256-byte aligned,
 * contents undefined afterwards) the list of every row is shared out among several workgroups, each computing
 * softmax attention over its share with its own log-sum-exp, and a second kernel merges the shares (Sec. 2.1:
 * the softmax is one sum over the selected keys, so shares combine by their log-sum-exp).  The shares are kept
 * in fp32 and the result is rounded once: it agrees with the one-workgroup-per-row form to the rounding of the
 * tensor type, not bit for bit (the sums are taken in another order).  A step of one or two positions with at
 * most 8 query rows per KV head (the decode stage the paper's "Future Work" names; its experiments decode
 * densely, Sec. 4.1) runs on a kernel of its own: a workgroup reads a range of key blocks of ONE KV head once
 * and serves all its query heads from it (sparse: the union of their lists, every row skipping what it did not
 * select), without matrix instructions; same workspace, same merge, same agreement.
 * A chunk of a long prompt (several query blocks per head against a context of 128 blocks or more, at most 4096
 * rows) has many short rows and a few nearly as long as the context, and an unsplit launch takes as long as its
 * longest row: with a workspace a small kernel first plans, from the row counts, which rows are cut into parts of
 * 64 (128) list entries and where their partial results go (a fixed number of slots: when they run out the
 * remaining rows stay whole); same merge, same agreement.
 * rr_attn_workspace_bytes() returns 0 where a call would not be split (many rows, short lists, shapes outside
 * bf16 / d = 128 / B = 128); a NULL workspace, or a geometry that is not split, gives exactly rr_sparse_attn /
 * rr_dense_attn.  A workspace that is too small or misaligned: RR_ERR_WORKSPACE.
 */
size_t rr_attn_workspace_bytes(const rr_shape* shape, int B);
int rr_sparse_attn_ws(const rr_shape* shape, const void* Q, const void* K, const void* V, const rr_mask* mask,
                      void* O, float* lse, void* workspace, size_t workspace_bytes, void* hip_stream);
int rr_dense_attn_ws(const rr_shape* shape, const void* Q, const void* K, const void* V, int B, void* O, float* lse,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Caller-made masks: fills mask->row_count and mask->row_list (and mask->row_order when non-NULL) from
 * mask->dense, a [batch, Hq, Nb, Nb] 0/1 matrix on the device (any nonzero byte selects; entries with
 * n > m are ignored, the block-sparse attention of Sec. 2.1 being causal).  The result can be handed to
 * rr_sparse_attn and rr_selection_accuracy.  Only shape->batch, Hq, Hkv, L are used besides mask->B.
 */
int rr_mask_from_dense(const rr_shape* shape, rr_mask* mask, void* hip_stream);

/*
 * Block selection accuracy of a mask against full attention (appendix "Block Selection Accuracy
 * Analysis").  For a query i, K*_i is a smallest set of key positions whose causal softmax attention
 * sums to >= tau (descending attention, equal values by smaller position), K_i the positions j <= i
 * of the key blocks the mask selects for the query's block row; precision_i = |K_i n K*_i| / |K_i|
 * (0 for an empty K_i), recall_i = |K_i n K*_i| / |K*_i|.  The averages are taken over the queries
 * i = step-1, 2*step-1, ... (step = 1: every query, as in the paper); F1 = 2 P R / (P + R).
 *   mask       row_count and row_list are read (as by rr_sparse_attn).
 *   tau        in (0, 1) (at 1 the set depends on how the row sum rounds); the paper uses 0.95.
 *   step       >= 1, must divide the number of queries (L, or Lq for a chunk).  This diagnostic
 *              takes whole blocks only: B must divide L and Lq (RR_ERR_PARAM otherwise).
 *   workspace  rr_accuracy_workspace_bytes() bytes, 256-byte aligned: one fp32 attention row per
 *              sampled query (batch * Hq * (L/step) * L * 4 bytes) plus per-query results.
 *   out        [batch, Hq, 3] fp32 device array: precision, recall, F1 per head.
 * A diagnostic: fp32 attention values, O(L^2 d / step) work on the vector ALUs.
 */
size_t rr_accuracy_workspace_bytes(const rr_shape* shape, int step);
int rr_selection_accuracy(const rr_shape* shape, const void* Q, const void* K, const rr_mask* mask,
                          float tau, int step, void* workspace, size_t workspace_bytes, float* out,
                          void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* RR_ATTN_H */
