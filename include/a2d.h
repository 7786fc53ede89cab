/*
 * a2d — per-device compute of Attention2D (arXiv 2503.15758) on MI355X (gfx950).
 *
 * The paper splits self-attention over a sqrt(P) x sqrt(P) device grid along both
 * the query and the key/value dimension.  What one device computes on its share
 * is (i) exact attention of one block of queries against one block of keys and
 * values, kept as an UNNORMALISED partial triple (M, N, D) (Sec. 3.1, Eq. (3);
 * the FlashAttn call of Alg. 1 line 4), (ii) the AttnFix merge of the sqrt(P)
 * partials of a query block followed by the division by D (Alg. 2; Alg. 1
 * lines 5-6), (iii) the per-tile gradient call of Alg. 3 line 3 and (iv) the
 * summing reductions of Alg. 3 lines 4-5.  This header is the whole boundary:
 * four compute entry points plus a workspace query and error reporting.
 *
 * Conventions shared by every call
 *  - Every pointer is caller-owned DEVICE memory unless stated otherwise; the
 *    library allocates nothing and keeps no pointer after a call returns.
 *  - Matrices are row-major [heads][rows][H] with H contiguous and no padding
 *    (the tile calls' inputs in the model's dtype may instead be strided, see
 *    a2d_layout); per-row statistics are [heads][rows].  heads = batch * number of heads (the
 *    method works per head, Sec. 2.1 / Sec. 5).
 *  - Scores are s = scale * <q, k> (the 1/sqrt(H) factor the paper's footnote in
 *    Sec. 2.1 leaves out is the explicit `scale`), then the causal mask of
 *    Sec. 2.1: key r is hidden from query i iff q_off + i < kv_off + r, where
 *    q_off / kv_off are the GLOBAL indices of row 0 / key 0 of the tile.  The
 *    paper's cyclic index sets (Sec. 3.2) map to (q_off, kv_off) = (0, 0) for a
 *    tile with grid row >= grid column and (0, 1) otherwise.
 *  - m, l, lse are in natural-log units of the scaled scores.  A row that sees no
 *    key has m = -inf, l = 0, N = 0; AttnFix gives such a partial weight 0; a row
 *    whose k partials are all empty gets O = 0, lse = -inf.
 *  - Calls only enqueue work on `stream` (a hipStream_t passed as void*, NULL =
 *    the default stream) and return; they do not synchronise.  Outputs are
 *    fully overwritten.  Same inputs give bitwise identical outputs.
 *  - On error a negative status is returned and a2d_last_error() describes the
 *    cause (thread-local, host memory owned by the library).  Every check of
 *    the arguments, and everything else that can fail on the host side, comes
 *    before the call's first kernel launch: with any status other than
 *    A2D_ERR_HIP nothing has been enqueued.  A2D_ERR_HIP from a launch the
 *    runtime refused can leave earlier kernels of the same call on the stream;
 *    the outputs are then undefined.
 *  - Alignment: every device pointer must be 16-byte aligned.
 */
#ifndef A2D_H_
#define A2D_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  A2D_OK = 0,
  A2D_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, k out of range          */
  A2D_ERR_UNSUPPORTED = -2, /* dtype / head size the kernels do not cover               */
  A2D_ERR_MISALIGNED = -3,  /* a device pointer is not 16-byte aligned                  */
  A2D_ERR_WORKSPACE = -4,   /* workspace missing or smaller than a2d_workspace_bytes()  */
  A2D_ERR_HIP = -5          /* the HIP runtime refused a launch                         */
} a2d_status;

typedef enum { A2D_F32 = 0, A2D_BF16 = 1 } a2d_dtype;

typedef enum {
  A2D_OP_PARTIAL_FWD = 0,
  A2D_OP_FIX = 1,
  A2D_OP_PARTIAL_BWD = 2,
  A2D_OP_FIX_BWD = 3,
  A2D_OP_PARTIAL_BWD_DS = 4,   /* workspace query only: a2d_partial_bwd with the dS hand-over */
  A2D_OP_PARTIAL_BWD_SPLIT = 5 /* workspace query only: a2d_partial_bwd_gqa with A2D_TILE_SPLIT_GROUPS */
} a2d_op;

/* Most partials one a2d_fix / a2d_fix_bwd call can merge (sqrt(P) in the paper). */
#define A2D_MAX_PARTS 32

/* Most key/value sub-blocks of one gathered tile (a2d_partial_fwd_seg / a2d_partial_bwd_seg). */
#define A2D_MAX_SEGMENTS 32

/*
 * Where the rows of a [heads][rows][H] tensor of the model's dtype (Q, K, V, O, dO) lie: element
 * (h, r, j) is at base + h * head + r * row + j, strides in ELEMENTS; the H elements of a row are
 * always contiguous.  {0, 0} means the plain layout (row = H, head = rows * H).  Otherwise
 * row >= H, head >= 1, both multiples of 16 bytes' worth of elements (8 for bf16, 4 for fp32), a
 * row stride below 16 MiB, and what one call addresses through one base pointer (the rows of one
 * key/value head; of the query heads that share it) must span less than 4 GiB - e.g. the
 * [rows][heads][H] layout of a fused QKV projection is head = H, row = heads * H (times 3 when
 * Q, K and V are interleaved), with the tensor's base pointer moved to its first element.  The
 * library reads heads * rows rows through these strides and cannot check that they exist.
 * The fp32 partials, statistics and gradient partials the calls write are always plain.
 */
typedef struct {
  int64_t head;
  int64_t row;
} a2d_layout;

/*
 * desc->flags, backward calls: hand dS from the dK/dV kernel to the dQ kernel through the
 * workspace instead of computing it twice (see a2d_workspace_bytes).  The caller ASKS for this
 * path; the size of the workspace never selects it.
 */
#define A2D_DESC_KEEP_DS 1

/* One tile problem: a block of nq queries against a block of nkv keys/values. */
typedef struct {
  int32_t heads;   /* B * M, >= 1                                                     */
  int32_t nq;      /* query rows of the tile, 1 .. 2^22                               */
  int32_t nkv;     /* key/value rows of the tile, 1 .. 2^22                           */
  int32_t hdim;    /* H: 64, 80, 96 or 128 (bf16: MFMA kernels; fp32: vector-ALU ones) */
  int64_t q_off;   /* global index of query row 0 (used only when causal != 0)        */
  int64_t kv_off;  /* global index of key row 0   (used only when causal != 0)        */
  int32_t causal;  /* 0: no mask; 1: hide key r from query i iff q_off+i < kv_off+r   */
  float scale;     /* multiplies <q, k>; 1/sqrt(H) in the paper's setting             */
  int32_t dtype;   /* a2d_dtype of Q, K, V, O, dO                                     */
  int32_t flags;   /* 0 or A2D_DESC_KEEP_DS (backward calls; the forward calls ignore it) */
  a2d_layout lq;   /* layout of Q                                                     */
  a2d_layout lk;   /* layout of K (its heads are the key/value heads)                 */
  a2d_layout lv;   /* layout of V                                                     */
  a2d_layout lo;   /* layout of O  (backward calls)                                   */
  a2d_layout ldo;  /* layout of dO (backward calls)                                   */
} a2d_tile_desc;

/*
 * Bytes of device workspace the given op needs for this tile (0 if none).
 * A2D_OP_PARTIAL_BWD: the minimum (the per-row sums delta = rowsum(dO o O)).
 * A2D_OP_PARTIAL_BWD_DS: the size the backward calls need when desc->flags has A2D_DESC_KEEP_DS:
 * they then ALSO keep dS (bf16, one value per score: about 2 nq nkv bytes per head) in the
 * workspace, so that dQ is one contraction over the stored dS instead of a second recomputation
 * of S and dP.  The hand-over exists for bf16 inputs, sub-blocks of a gathered tile that start at
 * multiples of 64 keys, and less than 4 GiB of dS per key/value head (all the query heads of its
 * group together); where it does not (this query then returns the minimum size for a plain tile)
 * the flag is accepted and the recomputing kernels run.  Same results up to fp32 summation
 * order; faster when the memory is there.
 * A2D_OP_PARTIAL_BWD_SPLIT: the size a2d_partial_bwd_gqa needs with A2D_TILE_SPLIT_GROUPS: that of
 * A2D_OP_PARTIAL_BWD_DS plus fp32 partial dK / dV buffers (at most 2 * heads * nkv * H floats);
 * `k` = the number of key/value heads.
 * `k` is ignored for the other tile ops.  Returns 0 for a NULL or invalid descriptor.
 */
size_t a2d_workspace_bytes(const a2d_tile_desc* desc, int op, int k);

/*
 * Partial attention of one tile (Sec. 3.1, Eq. (3); Alg. 1 line 4).
 *   in : Q [heads][nq][H], K, V [heads][nkv][H] in desc->dtype
 *   out: O_part [heads][nq][H] fp32 = n' (unnormalised), m [heads][nq] fp32 = m'
 *        (the true maximum of the visible scaled scores), l [heads][nq] fp32 = d'.
 * bf16 inputs: products accumulate in fp32, the softmax runs in fp32, the
 * probabilities are rounded to bf16 (nearest-even) before the P*V contraction.
 * fp32 inputs: fp32 throughout.  workspace may be NULL (none is needed).
 */
a2d_status a2d_partial_fwd(const a2d_tile_desc* desc, const void* Q, const void* K,
                           const void* V, float* O_part, float* m, float* l,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * AttnFix over k partials of the same query block, then normalisation
 * (Alg. 2 folded over k inputs; O = Diag(D^-1) N of Alg. 1 line 6; the statistic
 * L = M + log D of the footnote in Sec. 3.2).
 *   in : O_parts, m, l: HOST arrays of k device pointers, each as written by
 *        a2d_partial_fwd for `rows` = heads * nq rows of head size hdim
 *   out: O [rows][hdim] in out_dtype (rounded once, nearest-even), lse [rows] fp32.
 * One pass: M = max_k m_k, w_k = exp(m_k - M), sums taken in index order 0..k-1.
 * 1 <= k <= A2D_MAX_PARTS; hdim a multiple of 4.
 */
a2d_status a2d_fix(int k, int64_t rows, int32_t hdim, int32_t out_dtype,
                   const float* const* O_parts, const float* const* m,
                   const float* const* l, void* O, float* lse, void* stream);

/*
 * AttnFix alone (Alg. 2, folded over k inputs): merges k partials of the same query block into
 * ONE partial of the same unnormalised form - the operator of the reduce-scatter of Alg. 1
 * line 5, one hop of it for k = 2; a2d_fix is this followed by the division of line 6.
 *   in : O_parts, m, l: HOST arrays of k device pointers, each a partial (N, m, l) as written by
 *        a2d_partial_fwd (or by this call) for `rows` rows of head size hdim
 *   out: N_out [rows][hdim], m_out [rows], l_out [rows], fp32:
 *        m_out = max_k m_k, N_out = sum_k exp(m_k - m_out) N_k, l_out = sum_k exp(m_k - m_out) l_k
 *        (sums in index order 0..k-1); a row empty in every input stays empty (0, -inf, 0).
 * The outputs must not be any of the inputs (A2D_ERR_INVALID_ARG).  1 <= k <= A2D_MAX_PARTS;
 * hdim a multiple of 4.
 */
a2d_status a2d_attnfix(int k, int64_t rows, int32_t hdim, const float* const* O_parts,
                       const float* const* m, const float* const* l, float* N_out, float* m_out,
                       float* l_out, void* stream);

/*
 * Gradient share of one tile (the BwdFlashAttn call of Alg. 3 line 3).
 *   in : Q, K, V as for the forward; O [heads][nq][H] and lse [heads][nq]: the
 *        FINAL merged output and log-sum-exp of the query block (what Alg. 1
 *        line 7 saves), not the tile's own partial; dO [heads][nq][H].
 *   out: dQ_part [heads][nq][H], dK_part, dV_part [heads][nkv][H], fp32:
 *        P = exp(S - lse), delta = rowsum(dO o O), dV = P^T dO, dP = dO V^T,
 *        dS = P o (dP - delta), dQ = scale dS K, dK = scale dS^T Q.
 * bf16 inputs: P and dS are rounded to bf16 before their contractions.
 * workspace: at least a2d_workspace_bytes(desc, A2D_OP_PARTIAL_BWD, 0) bytes, or, with
 * A2D_DESC_KEEP_DS in desc->flags (the faster dS hand-over), at least
 * a2d_workspace_bytes(desc, A2D_OP_PARTIAL_BWD_DS, 0) bytes - a smaller one is
 * A2D_ERR_WORKSPACE; contents undefined on entry and exit; calls sharing one workspace
 * must be ordered on one stream.
 */
a2d_status a2d_partial_bwd(const a2d_tile_desc* desc, const void* Q, const void* K,
                           const void* V, const void* O, const void* dO,
                           const float* lse, float* dQ_part, float* dK_part,
                           float* dV_part, void* workspace, size_t workspace_bytes,
                           void* stream);

/*
 * a2d_partial_bwd for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus
 * the workspace), same kernels and bitwise the same results as a2d_partial_bwd with its minimum
 * workspace (A2D_DESC_KEEP_DS is refused: A2D_ERR_UNSUPPORTED).  The per-row sums delta live in
 * a device array inside the library (4 MiB per GPU the library runs on, held until the process
 * ends) of A2D_STATIC_MAX_ROWS floats: heads * nq beyond that is A2D_ERR_WORKSPACE.  The call
 * itself allocates and frees nothing; its first call on a device looks the array's address up.
 * All calls on one GPU share the array: calls that may overlap on that GPU (different streams,
 * different host threads) race and must be ordered by the caller.
 */
#define A2D_STATIC_MAX_ROWS (1 << 20)
a2d_status a2d_partial_bwd_static(const a2d_tile_desc* desc, const void* Q, const void* K,
                                  const void* V, const void* O, const void* dO,
                                  const float* lse, float* dQ_part, float* dK_part,
                                  float* dV_part, void* stream);

/*
 * One sub-block of a GATHERED key/value tile: `rows` consecutive tokens starting at global
 * token index kv_off.
 */
typedef struct {
  int64_t kv_off; /* global index of the sub-block's first key                     */
  int32_t rows;   /* its number of keys, >= 1                                      */
  int32_t pad;    /* must be 0                                                     */
} a2d_kv_segment;

/*
 * The tile calls for a gathered key/value tile: one query block against the concatenation
 * of nseg sub-blocks that come from different places of the sequence - the Compute line of
 * the paper's GatherComputeScatter algorithm (Sec. 3.4), which runs FlashAttn on one query
 * block and the gathered K_g, V_g in one go.  Under the causal mask this is the step-like
 * pattern Sec. 4.1 says the paper's own kernel could not express (it ran one call per
 * sub-block instead).  K, V, dK_part, dV_part are [heads][nkv][H] with
 * nkv = desc->nkv = sum of segs[s].rows, sub-blocks stored in the order of `segs`
 * (a HOST array, read before the call returns); desc->kv_off is ignored; key kk of
 * sub-block s is hidden from query i iff desc->causal and q_off + i < segs[s].kv_off + kk.
 * The paper's cyclic layout maps to kv_off = 0 for a sub-block whose first token does not
 * come after the query block's first token and 1 otherwise (with q_off = 0).
 * Results equal AttnFix over / sums and concatenation of the per-sub-block calls; sub-blocks
 * no query row can see cost nothing.  Everything else is as for a2d_partial_fwd /
 * a2d_partial_bwd.  1 <= nseg <= A2D_MAX_SEGMENTS.
 */
a2d_status a2d_partial_fwd_seg(const a2d_tile_desc* desc, int nseg, const a2d_kv_segment* segs,
                               const void* Q, const void* K, const void* V, float* O_part,
                               float* m, float* l, void* workspace, size_t workspace_bytes,
                               void* stream);
a2d_status a2d_partial_bwd_seg(const a2d_tile_desc* desc, int nseg, const a2d_kv_segment* segs,
                               const void* Q, const void* K, const void* V, const void* O,
                               const void* dO, const float* lse, float* dQ_part,
                               float* dK_part, float* dV_part, void* workspace,
                               size_t workspace_bytes, void* stream);

/*
 * Accumulating forms of the tile calls: the compute-then-reduce pair of the paper's overlapped
 * algorithms (FlashAttn followed by AttnFix in GatherCompute and GatherComputeScatter, Sec. 3.4;
 * "dQ += ..." in their backward counterparts) fused into the tile kernel.
 *   a2d_partial_fwd_acc: O_part, m, l are IN/OUT.  On entry they hold a partial triple of the same
 *     query block (e.g. written by an earlier tile call; m = -inf, l = 0, N = 0 is the empty
 *     one); on exit they hold AttnFix(that triple, the partial of this tile): m the larger
 *     maximum, N and l both rescaled to it and added.  Equal to a2d_partial_fwd into a second
 *     buffer followed by a pairwise merge, up to fp32 rounding.
 *   a2d_partial_bwd_acc: dQ_part is IN/OUT (this tile's dQ share is added to it); dK_part and
 *     dV_part are written as by a2d_partial_bwd.
 * nseg = 0 (segs ignored) means the plain tile of desc->kv_off; nseg >= 1 a gathered tile as for
 * the _seg calls.  Calls that accumulate into the same buffers must be ordered on one stream.
 */
a2d_status a2d_partial_fwd_acc(const a2d_tile_desc* desc, int nseg, const a2d_kv_segment* segs,
                               const void* Q, const void* K, const void* V, float* O_part,
                               float* m, float* l, void* workspace, size_t workspace_bytes,
                               void* stream);
a2d_status a2d_partial_bwd_acc(const a2d_tile_desc* desc, int nseg, const a2d_kv_segment* segs,
                               const void* Q, const void* K, const void* V, const void* O,
                               const void* dO, const float* lse, float* dQ_part,
                               float* dK_part, float* dV_part, void* workspace,
                               size_t workspace_bytes, void* stream);

/*
 * Normalised partial format: a partial as (O' = N / l in the input dtype, lse' = m + ln l), the
 * pair FlashAttention-style kernels return (footnote of Sec. 3.2), instead of the unnormalised
 * fp32 triple.  Half the bytes per partial and a quarter for bf16 inputs, at the price of one
 * rounding of every partial to the input dtype before the merge.
 *   a2d_partial_fwd_norm: as a2d_partial_fwd (nseg = 0) or a2d_partial_fwd_seg (nseg >= 1), but
 *     out: O_norm [heads][nq][H] in desc->dtype, lse_part [heads][nq] fp32 (a row that sees no
 *     key: O' = 0, lse' = -inf).
 *   a2d_fix_norm: merge of k such partials of one query block: L = log sum_k exp(lse_k),
 *     O = sum_k exp(lse_k - L) O'_k, sums in index order; O_norm_parts, lse_parts: HOST arrays of
 *     k device pointers; in_dtype: dtype of the partials; out: O [rows][hdim] in out_dtype,
 *     lse [rows] fp32.  1 <= k <= A2D_MAX_PARTS; hdim a multiple of 4.
 */
a2d_status a2d_partial_fwd_norm(const a2d_tile_desc* desc, int nseg, const a2d_kv_segment* segs,
                                const void* Q, const void* K, const void* V, void* O_norm,
                                float* lse_part, void* workspace, size_t workspace_bytes,
                                void* stream);
a2d_status a2d_fix_norm(int k, int64_t rows, int32_t hdim, int32_t in_dtype, int32_t out_dtype,
                        const void* const* O_norm_parts, const float* const* lse_parts, void* O,
                        float* lse, void* stream);

/*
 * Grouped-query attention (the method works head by head, Sec. 2.1 / Sec. 5; with grouped
 * queries several query heads read the key/value rows of ONE key/value head).  desc->heads
 * counts QUERY heads; K and V hold kv_heads = desc->heads / group heads, query head h reads
 * key/value head h / group (the group's query heads are consecutive).  kv_heads must divide
 * desc->heads; kv_heads == desc->heads is ordinary multi-head attention, kv_heads == 1
 * multi-query attention.
 *   a2d_partial_fwd_gqa: K, V [kv_heads][nkv][H]; everything else as in the call `flags` picks:
 *     0                      a2d_partial_fwd / _seg   (out0 = O_part fp32, out1 = m, out2 = l)
 *     A2D_TILE_ACCUMULATE    a2d_partial_fwd_acc      (the same three buffers, in/out)
 *     A2D_TILE_NORMALISED    a2d_partial_fwd_norm     (out0 = O_norm in desc->dtype, out1 = lse_part,
 *                                                      out2 ignored, may be NULL)
 *   a2d_partial_bwd_gqa: K, V as above; dK_part, dV_part [kv_heads][nkv][H] fp32: the gradient of
 *     a key/value head is the SUM over the query heads of its group (taken inside the kernel, in
 *     head order; one writer per element, no atomics).  flags: 0 or A2D_TILE_ACCUMULATE (dQ +=),
 *     optionally | A2D_TILE_SPLIT_GROUPS: the library may then give a key block to several
 *     workgroups, each summing over a share of the group's query heads into an fp32 partial buffer
 *     in the workspace, and add the partials up in a fixed order afterwards - for key/value head
 *     counts that leave compute units idle (few key/value heads, short key rows).  Same results
 *     up to fp32 summation order, still bitwise reproducible; needs a workspace of
 *     a2d_workspace_bytes(desc, A2D_OP_PARTIAL_BWD_SPLIT, kv_heads) bytes.
 *     workspace otherwise as for a2d_partial_bwd.
 * nseg = 0 (segs ignored): the plain tile of desc->kv_off; nseg >= 1: a gathered tile.
 * group * nq may not exceed 2^22 rows.
 */
#define A2D_TILE_ACCUMULATE 1
#define A2D_TILE_NORMALISED 2
#define A2D_TILE_SPLIT_GROUPS 4
a2d_status a2d_partial_fwd_gqa(const a2d_tile_desc* desc, int32_t kv_heads, int nseg,
                               const a2d_kv_segment* segs, int flags, const void* Q, const void* K,
                               const void* V, void* out0, float* out1, float* out2,
                               void* workspace, size_t workspace_bytes, void* stream);
a2d_status a2d_partial_bwd_gqa(const a2d_tile_desc* desc, int32_t kv_heads, int nseg,
                               const a2d_kv_segment* segs, int flags, const void* Q, const void* K,
                               const void* V, const void* O, const void* dO, const float* lse,
                               float* dQ_part, float* dK_part, float* dV_part, void* workspace,
                               size_t workspace_bytes, void* stream);

/*
 * Sum of k gradient partials (the reduce-scatters of Alg. 3 lines 4-5 use plain
 * summation): out[i] = sum_k parts[k][i], added in index order in fp32, rounded
 * once to out_dtype.  parts: HOST array of k device pointers to n fp32 values;
 * n a multiple of 4.  Call once each for dQ (over a grid row), dK and dV (over a
 * grid column).
 */
a2d_status a2d_fix_bwd(int k, int64_t n, int32_t out_dtype, const float* const* parts,
                       void* out, void* stream);

/*
 * a2d_fix and a2d_fix_bwd with the merged output written through a layout, so that O, dQ, dK, dV
 * land where the model keeps them (e.g. [rows][heads][H] activations, or the Q / K / V slots of a
 * packed gradient buffer) without a transposing copy.  The inputs are the plain fp32 partials of
 * heads * nq (heads * rows) rows as before, lse stays plain [heads][nq]; row r of head h of the
 * output starts h * lo->head + r * lo->row elements from O (multiples of 16 bytes, row >= hdim).
 * lo = NULL or {0, 0}: the plain layout, i.e. exactly a2d_fix / a2d_fix_bwd.  Same arithmetic and
 * same results as those calls; nothing is enqueued on an error.
 */
a2d_status a2d_fix_strided(int k, int32_t heads, int32_t nq, int32_t hdim, int32_t out_dtype,
                           const float* const* O_parts, const float* const* m, const float* const* l,
                           void* O, const a2d_layout* lo, float* lse, void* stream);
a2d_status a2d_fix_bwd_strided(int k, int32_t heads, int32_t rows, int32_t hdim, int32_t out_dtype,
                               const float* const* parts, void* out, const a2d_layout* lout,
                               void* stream);
/* a2d_fix_norm with O written through a layout, as a2d_fix_strided. */
a2d_status a2d_fix_norm_strided(int k, int32_t heads, int32_t nq, int32_t hdim, int32_t in_dtype,
                                int32_t out_dtype, const void* const* O_norm_parts,
                                const float* const* lse_parts, void* O, const a2d_layout* lo,
                                float* lse, void* stream);

/*
 * Diagnostic, not part of the method: the rate the bf16 MFMA units of the current device
 * sustain on their own (register operands only, several wavefronts per SIMD, four independent
 * accumulators per wavefront), for pricing the tile kernels against what the chip delivers
 * rather than the data-sheet number.  The MFMA rate depends on the operand values (power):
 * random_data != 0 uses pseudo-random values of unit scale, 0 uses the constant 0.5.
 * Unlike the compute calls this one is SYNCHRONOUS: it runs on the default stream, waits, and
 * writes HOST results: *tflops (dense bf16 TFLOP/s over the whole chip) and *shader_mhz (the
 * shader clock during the run).  scratch: device memory of at least
 * a2d_mfma_ceiling_scratch_bytes() bytes (0 if the device cannot be queried), overwritten.
 * iters: MFMA groups of 16 per wavefront, 1 .. 2^22 (20000 is about 10 ms).
 */
size_t a2d_mfma_ceiling_scratch_bytes(void);
a2d_status a2d_mfma_ceiling(int iters, int random_data, void* scratch, size_t scratch_bytes,
                            double* tflops, double* shader_mhz);

/*
 * Diagnostic like a2d_mfma_ceiling, one step closer to the forward tile kernel: the same MFMAs on
 * pseudo-random operands, but every MFMA takes a fresh A fragment from LDS and is followed by the
 * softmax arithmetic of one score per lane (fma, exp2, max, add), two wavefronts per SIMD - and
 * nothing else of the kernel (no global traffic, barriers, masks, prologue or epilogue).  What it
 * sustains is what this loop structure can reach on the chip.  Arguments and results as for
 * a2d_mfma_ceiling (same scratch size); synchronous.
 */
a2d_status a2d_forward_mix_ceiling(int iters, void* scratch, size_t scratch_bytes, double* tflops,
                                   double* shader_mhz);

/*
 * The same for the dK/dV kernel of the backward tile call: eight wavefronts in four pairs of a
 * score and a gradient role, per step of 32 query rows 8 MFMAs on natural LDS fragments, the
 * arithmetic that turns their results into the next operand (fma + exp2, or a multiplication with
 * the partner's probabilities, which travel through an LDS mailbox in fp32), 8 MFMAs on
 * transposing LDS reads, one barrier - and nothing else of the kernel (no global traffic, masks,
 * staging, dS hand-over, prologue or epilogue).
 * leave_out: parts of the model to leave out, to see what each costs: bit 0 the mailbox, bit 1
 * the element-wise arithmetic, bit 2 the barrier (accepted only together with bit 0: without the
 * barrier nothing passes between wavefronts); 0 is the whole model.  Other values:
 * A2D_ERR_INVALID_ARG.  Other arguments and results as for a2d_mfma_ceiling (same scratch size);
 * synchronous.
 */
a2d_status a2d_backward_mix_ceiling(int iters, int leave_out, void* scratch, size_t scratch_bytes,
                                    double* tflops, double* shader_mhz);

/*
 * Diagnostic: what the LDS of the chip delivers to eight wavefronts per compute unit that only
 * read it, with the tile kernels' two kinds of fragment reads - 128-bit reads of padded rows
 * (transposing = 0) or 64-bit transposing reads (transposing != 0).  *tbytes_per_s: 10^12 bytes
 * per second over the whole chip.  Against it the kernels' own LDS traffic shows whether LDS
 * bandwidth bounds them.  Other arguments as for a2d_mfma_ceiling (same scratch size; iters:
 * groups of 16 reads per wavefront); synchronous.
 */
a2d_status a2d_lds_read_ceiling(int iters, int transposing, void* scratch, size_t scratch_bytes,
                                double* tbytes_per_s, double* shader_mhz);

/*
 * Debugging aid, not part of the method: on != 0 routes every tile call of the process to the
 * fp32 vector-ALU kernels (also for bf16 inputs), 0 back to the default choice.  The initial
 * value is 1 when A2D_FORCE_GENERIC=1 is in the environment at the first tile call, else 0.
 */
void a2d_debug_force_generic(int on);

/*
 * Diagnostic, not part of the method: per-kernel timing of the calls above.  events: a HOST array
 * of n hipEvent_t handles the caller created with timing enabled (it owns them and the array,
 * which must stay valid until the trace is switched off), or NULL / n = 0 to switch the trace
 * off.  While a trace is set - per host thread - every call of this library made by that thread
 * records the next unused event on the call's stream once before its first kernel and once
 * after each kernel it launches; consecutive events of one call then bracket one kernel each
 * (a tile forward: 2 events; a2d_partial_bwd: 4 - delta, dK/dV, dQ kernels; a merge: 2).  Events
 * beyond n are not recorded.  a2d_debug_trace_count: events recorded since the trace was set.
 */
void a2d_debug_trace(void** events, int n);
int a2d_debug_trace_count(void);

/*
 * Diagnostic, not part of the method: a plain device-to-device copy of `bytes` bytes (a positive
 * multiple of 16; both pointers 16-byte aligned, buffers must not overlap) with 128-bit
 * non-temporal loads and stores, enqueued on `stream`.  It gives the streaming calls (a2d_fix,
 * a2d_fix_bwd) the copy rate this chip reaches as context for their HBM fraction, and a kernel of
 * known traffic for calibrating the HBM byte counters of a profiler run.
 */
a2d_status a2d_copy_probe(void* dst, const void* src, size_t bytes, void* stream);

/* Static string for a status code. */
const char* a2d_status_str(a2d_status status);
/* Detail of the calling thread's last failed call ("" if none). */
const char* a2d_last_error(void);
/* Library version, "major.minor". */
const char* a2d_version(void);

#ifdef __cplusplus
}
#endif
#endif /* A2D_H_ */
