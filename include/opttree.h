/*
 * opttree.h -- C ABI of the MI355X (gfx950) hot path of one OPT-Tree decoding
 * step (arxiv 2406.17276): greedy adaptive draft-tree construction
 * (Sec. 3, Eq. 1-3, Algorithm 1) and the tree-masked attention the target
 * model runs to verify the drafted nodes (Sec. 3, Algorithm 2).
 *
 * Conventions
 *   - every function returns an int status (OT_OK or a negative OT_ERR_*),
 *     never throws, never allocates or frees device memory;
 *   - every tensor argument is a DEVICE pointer owned by the caller; parameter
 *     structs are HOST pointers, read before the call returns;
 *   - all work is enqueued on the caller's hipStream_t (passed as void*, NULL =
 *     the default stream); calls are asynchronous, results are valid after the
 *     stream has been synchronised;
 *   - the library keeps no global device state: scratch lives in a caller-owned
 *     workspace sized by the *_workspace_bytes query.  Concurrent calls must use
 *     distinct workspaces.  (One documented exception: ot_tree_verify_attention_noalloc
 *     works in a fixed array that the library's code object holds on every GPU.);
 *   - alignment of device pointers: workspaces and the attention tensors (Q, K, V, O) 16 bytes; logits
 *     rows the size of one element (rows that are 16-byte aligned, with strides and a vocabulary that are
 *     multiples of 16 bytes, take the vector-load path, anything else a slower element-load path); int32 /
 *     float arrays 4 bytes; uint64 / double arrays 8 bytes;
 *   - arguments are validated on the host before anything is launched; an
 *     invalid call enqueues nothing.
 */
#ifndef OPTTREE_H
#define OPTTREE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OT_API __attribute__((visibility("default")))

#define OT_OK                       0
#define OT_ERR_INVALID_ARG        (-1)  /* null pointer, non-positive size, misaligned pointer, bad stride */
#define OT_ERR_UNSUPPORTED        (-2)  /* outside the limits below */
#define OT_ERR_WORKSPACE_TOO_SMALL (-3)
#define OT_ERR_HIP                (-4)  /* a HIP runtime call failed; see ot_last_hip_error() */
#define OT_ERR_SCRATCH_LIMIT      (-5)  /* the call needs more scratch memory than a *_noalloc entry point owns */

#define OT_F32   0   /* IEEE binary32 */
#define OT_BF16  1   /* bfloat16 */

/* limits of this build */
#define OT_MAX_NODES     256   /* n  */
#define OT_MAX_TOPK       16   /* k  */
#define OT_MAX_DEPTH      32   /* d  */
#define OT_MAX_HEAD_DIM  128
#define OT_MAX_TREE_KEYS 8192     /* tree keys of the attention when they are more than the query rows */
#define OT_MASK_WORDS(n) (((n) + 63) / 64)

OT_API int ot_version(void);                       /* 100*major + minor */
OT_API const char* ot_status_string(int status);   /* static string, never NULL */
OT_API int ot_last_hip_error(void);                /* hipError_t of the last failed HIP call on this thread */

/* ------------------------------------------------------------------------
 * Draft-tree construction (Sec. 3; Algorithm 1 with a fixed number of
 * drafting steps `depth`).
 *
 * Input: for every sequence b, drafting step t (0-based; step 0 expands the
 * root) and frontier slot j < F_t, one row of `vocab` next-token logits of the
 * draft model, where F_0 = 1 and F_{t+1} = min(n, k*F_t).  Row (b,t,j) starts
 * at  logits + b*stride_seq + t*stride_depth + j*stride_row  (strides in
 * elements; rows j >= F_t are never read).  p_d = softmax(row).
 *
 * Per row: the k most probable tokens become the node's children (equal logits:
 * smaller token id first); a child's score is log p^ = score(parent) + log p_d
 * (Eq. 2, root excluded).  Per step the F_{t+1} best candidates are kept (equal
 * scores: smaller parent slot, then smaller rank) and numbered by
 * (parent slot, rank).  Finally the n_out = min(n, sum_t F_t) best nodes of the
 * whole pool are selected (equal scores: shallower, then smaller slot) and
 * emitted in (depth, slot) order, so parents precede children.
 * ---------------------------------------------------------------------- */
typedef struct ot_build_params {
    int32_t batch;          /* sequences, >= 1 */
    int32_t vocab;          /* >= k */
    int32_t depth;          /* drafting steps d, 1..OT_MAX_DEPTH */
    int32_t k;              /* children considered per node, 1..OT_MAX_TOPK */
    int32_t n;              /* node budget, 1..OT_MAX_NODES */
    int32_t logits_dtype;   /* OT_F32 | OT_BF16 */
    int64_t stride_seq, stride_depth, stride_row;   /* elements; stride_row >= vocab */
} ot_build_params;

typedef struct ot_tree_out {      /* device pointers, caller-owned; rows >= n_out are filled as noted */
    int32_t*  token;    /* [batch][n]  vocabulary id of node i            (-1) */
    int32_t*  parent;   /* [batch][n]  output index of the parent, -1 = child of the root (-1) */
    int32_t*  depth;    /* [batch][n]  1..d; position id = position of the root + depth    (0) */
    float*    score;    /* [batch][n]  log p^                                               (-inf) */
    uint64_t* mask;     /* [batch][n][OT_MASK_WORDS(n)] bit j of row i: j is i or an ancestor of i (0) */
    int32_t*  n_out;    /* [batch] */
    double*   expect;   /* [batch]  E(A) = sum_i p^_i  (Eq. 3) */
} ot_tree_out;

OT_API size_t ot_build_workspace_bytes(const ot_build_params* p);   /* 0 if p is invalid */

/* One-shot: all `depth` steps' rows are already in memory. */
OT_API int ot_build_tree(const ot_build_params* p, const void* logits,
                  void* workspace, size_t workspace_bytes,
                  const ot_tree_out* out, void* hip_stream);

/* Measurement aid: ot_build_tree that also records, in two caller-created hipEvent_t (passed as
 * void*, either may be NULL), the begin and the end of its row-scan kernel -- the HBM-bound pass over
 * the logits (softmax normaliser and top-k of every row, Sec. 3).  hipEventElapsedTime between
 * them, after the stream is synchronised, is that kernel's execution time.  Not capturable in a graph. */
OT_API int ot_build_tree_timed(const ot_build_params* p, const void* logits,
                  void* workspace, size_t workspace_bytes,
                  const ot_tree_out* out, void* hip_stream,
                  void* scan_begin_event, void* scan_end_event);

/* ot_build_tree with the stopping rule of Algorithm 1 applied inside the kernel: after every drafting step
 * E_sub(T, n) (the sum of the n largest p^ drafted so far) is compared with its value E one step earlier
 * (E = 0 at the start), and drafting ends when E_sub - E <= delta or after p->depth steps.  The logits of
 * all p->depth steps are passed as for ot_build_tree; rows of steps that are not drafted are scanned but not
 * used.  steps_used[b] (int32, device) receives the number of steps drafted, e_sub[b] (double, device) the
 * last E_sub.  Shapes on the single-wavefront path (n <= 64 and (rows per sequence + 1) * k within the LDS
 * budget -- the 7B, 13B and 70B shapes) run the loop inside one kernel; all other shapes run it step by step on
 * the stream with the kernels of the streaming calls below (the scan of a step's rows, the step, E_sub and the
 * loop condition; a sequence that stops is frozen on the device, nothing is read back, and the rows of the steps
 * it does not draft are not read).  Either way the call returns without waiting for the device. */
OT_API int ot_build_tree_adaptive(const ot_build_params* p, double delta, const void* logits,
                  void* workspace, size_t workspace_bytes,
                  const ot_tree_out* out, int32_t* steps_used, double* e_sub, void* hip_stream);

/* Streaming form of the same computation: what a decoder calls between the
 * draft model's forwards (the loop of Algorithm 1).  The strides of `p` are
 * ignored by begin; each expand call passes its own.
 *   ot_tree_begin   resets the builder kept in `workspace` (a small kernel on `hip_stream`);
 *   ot_tree_expand  consumes the F_t rows of step t (row (b,j) at
 *                   rows + b*stride_seq + j*stride_row) and writes the next
 *                   frontier: token and parent slot of its F_{t+1} slots
 *                   ([batch][n] each, entries >= F_{t+1} untouched) and, if
 *                   frontier_count is not NULL, frontier_count[b] = F_{t+1}, the
 *                   rows the draft model has to produce for sequence b in the
 *                   next step (0 for a sequence that ot_tree_esub has stopped:
 *                   its frontier outputs are left as they were); steps must be
 *                   fed in order t = 0,1,..;
 *   ot_tree_finalize selects and emits the tree over the steps fed so far.
 * The three calls of one tree must use the same workspace and stream order. */
OT_API int ot_tree_begin(const ot_build_params* p, void* workspace, size_t workspace_bytes, void* hip_stream);
OT_API int ot_tree_expand(const ot_build_params* p, int32_t step, const void* rows,
                   int64_t stride_seq, int64_t stride_row,
                   void* workspace, size_t workspace_bytes,
                   int32_t* frontier_token, int32_t* frontier_parent_slot, int32_t* frontier_count,
                   void* hip_stream);
OT_API int ot_tree_finalize(const ot_build_params* p, int32_t steps_done,
                     void* workspace, size_t workspace_bytes,
                     const ot_tree_out* out, void* hip_stream);

/* Drafting-phase attention masks.  The draft model's forward of a drafting step feeds the frontier (at most n
 * tokens) and attends to the K/V of everything drafted so far (Sec. 4, last paragraph); its tree attention
 * mask (Algorithm 2's mask, here per drafting step) is kept incrementally by ot_tree_expand: a node's mask is
 * its parent's plus its own bit.  Pool index of the node in slot s of the layer made by step t (0-based):
 * t*n + s -- the row where the caller stores that node's K/V in a [batch][kv_heads][depth*n][head_dim]
 * tree cache.  ot_tree_frontier_mask, called after the expand of step steps_done-1, writes
 *   mask[b][s][0..W)  W = OT_MASK_WORDS(depth*n): bit j set iff pool node j is frontier node s or one of its
 *                     ancestors; rows s >= F are zero,
 * ready for ot_tree_verify_attention with n_keys = depth*n (at most OT_MAX_DEPTH * OT_MAX_NODES = OT_MAX_TREE_KEYS
 * pool nodes). */
OT_API int ot_tree_frontier_mask(const ot_build_params* p, int32_t steps_done,
                          void* workspace, size_t workspace_bytes, uint64_t* mask, void* hip_stream);

/* Adaptive depth: the loop condition of Algorithm 1 (drafting goes on while E_sub(T,n) - E > delta, and E takes
 * the value of E_sub before every further step).  Called after the expand of step steps_done-1, ot_tree_esub
 * computes, per sequence,
 *   e_sub[b] = E_sub(T, n): the sum of the n largest p^ among the nodes drafted so far (Sec. 3: the best
 *              E over the root-containing n-node subtrees of T; non-decreasing in the steps, Thm. 3.2),
 *   go_on[b] = 1 if e_sub[b] - E[b] > delta, and then E[b] <- e_sub[b]; else 0.   (E[b] = 0 after begin.)
 * e_sub (double[batch]) and go_on (int32[batch]) are device pointers.  A sequence whose go_on was 0 is
 * frozen: later ot_tree_expand calls do not read its rows and leave its tree and its frontier outputs untouched,
 * later ot_tree_esub calls return go_on = 0 for it, and ot_tree_finalize selects among the layers it had when it
 * stopped.
 * The caller ends the loop when no go_on is set or the maximum depth p->depth is reached.
 * Returns OT_ERR_INVALID_ARG for steps_done outside 1..depth, a NaN delta, or null / misaligned pointers. */
OT_API int ot_tree_esub(const ot_build_params* p, int32_t steps_done, double delta,
                 void* workspace, size_t workspace_bytes,
                 double* e_sub, int32_t* go_on, void* hip_stream);

/* ------------------------------------------------------------------------
 * Tree-masked verification attention (Algorithm 2: the target model's forward
 * over T_opt under the tree attention mask that belongs to it).
 *
 * For sequence b, query head h, node i:
 *   O[b,h,i,:] = sum_j softmax_j(scale * Q[b,h,i,:] . K[b,h/g,j,:]) V[b,h/g,j,:]
 * over j in {prefix rows 0..prefix_len[b]-1} U {tree rows j : bit j of mask[b][i]},
 * g = q_heads / kv_heads.  A node whose row has no visible key yields zeros.
 * The root token's K/V is the last prefix row.  Q and K arrive already
 * position-encoded.  bf16 inputs use bf16 MFMA with fp32 accumulation and fp32
 * softmax; f32 inputs use fp32 arithmetic throughout.
 *
 * Element (b,h,r,c) of a tensor is at base + b*s[0] + h*s[1] + r*s[2] + c
 * (strides in elements, multiples of 16 bytes; last dimension contiguous).
 * prefix_len[b] is clamped to [0, max_prefix] on the device; when a value had to be clamped, bit 0 of the
 * 32-bit word at byte OT_ATTN_STATUS_OFFSET of the workspace is set (it stays set until the workspace is
 * prepared again or the caller clears the word), so that a caller can tell a truncated cache from a good one.
 * ---------------------------------------------------------------------- */
typedef struct ot_attn_params {
    int32_t batch, q_heads, kv_heads;   /* q_heads % kv_heads == 0 */
    int32_t head_dim;                   /* 64 or 128 */
    int32_t n;                          /* query rows = tree nodes, 1..OT_MAX_NODES */
    int32_t max_prefix;                 /* rows allocated per (b, kv head) in K_prefix / V_prefix, >= 0 */
    int32_t dtype;                      /* OT_F32 | OT_BF16, of Q, K, V and O */
    float   softmax_scale;              /* 0 => 1/sqrt(head_dim) */
    int64_t q_strides[3], kp_strides[3], vp_strides[3], kt_strides[3], vt_strides[3], o_strides[3];
    int32_t n_keys;                     /* rows of K_tree / V_tree; 0 => n.  Larger than n in the drafting phase,
                                           where the n frontier nodes attend to all nodes drafted so far
                                           (Sec. 4: every drafting step feeds n tokens and reuses the K/V
                                           cache); 1..OT_MAX_TREE_KEYS.  mask is then [batch][n][OT_MASK_WORDS(n_keys)] */
} ot_attn_params;

OT_API size_t ot_attn_workspace_bytes(const ot_attn_params* p);     /* 0 if p is invalid */

/* The first OT_ATTN_SYNC_BYTES bytes of an attention workspace hold the ticket counters with which the
 * workgroups that share output rows (the key ranges a long prefix is split into) find out which of them
 * finishes last and merges the partial results.  They must be zero when ot_tree_verify_attention is
 * called and every completed call leaves them zero, so a workspace is prepared ONCE after it has been
 * allocated (and again only if something else wrote to it, or a launch was aborted):
 * ot_attn_workspace_prepare zeroes them with a small kernel on `hip_stream` (capturable in a graph);
 * a caller may equally clear them itself.  Returns OT_OK, OT_ERR_INVALID_ARG (null or misaligned
 * workspace), OT_ERR_WORKSPACE_TOO_SMALL or OT_ERR_HIP. */
#define OT_ATTN_SYNC_BYTES 4096
#define OT_ATTN_STATUS_OFFSET (OT_ATTN_SYNC_BYTES - 4)   /* status word of the calls made with this workspace */
#define OT_ATTN_STATUS_PREFIX_CLAMPED 1u                 /* some prefix_len[b] was outside [0, max_prefix] */
OT_API int ot_attn_workspace_prepare(void* workspace, size_t workspace_bytes, void* hip_stream);

OT_API int ot_tree_verify_attention(const ot_attn_params* p,
                             const void* Q,                          /* [batch][q_heads][n][head_dim] */
                             const void* K_prefix, const void* V_prefix, /* [batch][kv_heads][max_prefix][head_dim]; may be NULL if max_prefix == 0 */
                             const void* K_tree, const void* V_tree,     /* [batch][kv_heads][n][head_dim] */
                             const int32_t* prefix_len,              /* [batch] */
                             const uint64_t* mask,                   /* [batch][n][OT_MASK_WORDS(n)] */
                             void* O,                                /* [batch][q_heads][n][head_dim] */
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same attention over a K/V cache kept in 8 bits.  The paper states no precision for the cache; the reading built
 * here: K_prefix, V_prefix, K_tree and V_tree hold FP8 E4M3 bytes (the OCP 8-bit format: 4 exponent bits with bias 7,
 * 3 mantissa bits, no infinities, largest value 448), and a byte of sequence b, KV head h stands for
 * k_scale[b][h] * decode(byte) (K) or v_scale[b][h] * decode(byte) (V); k_scale, v_scale: device float
 * [batch][kv_heads], positive and finite.  Q and O are bf16 (p->dtype must be OT_BF16).  The K/V strides of `p` count
 * elements = bytes and must be multiples of 16.  What is computed is the attention defined above on exactly those
 * values (each byte is widened without error; the factors join the softmax scale and the final normalisation);
 * quantising the cache is the caller's step.  Workspace and all other arguments as for ot_tree_verify_attention. */
OT_API int ot_tree_verify_attention_fp8kv(const ot_attn_params* p,
                             const void* Q, const void* K_prefix, const void* V_prefix,
                             const void* K_tree, const void* V_tree,
                             const float* k_scale, const float* v_scale,
                             const int32_t* prefix_len, const uint64_t* mask,
                             void* O, void* workspace, size_t workspace_bytes, void* hip_stream);

/* ot_tree_verify_attention for callers that cannot allocate device memory or keep a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels, with the workspace in
 * a library-owned device array of OT_ATTN_SCRATCH_BYTES that every GPU the library runs on holds until the
 * process ends.  Neither this call nor anything it calls allocates or frees memory, and no
 * ot_attn_workspace_prepare is needed.  The first call on a device looks the array's address up and clears its
 * ticket counters on `hip_stream` (that first call must not be made inside a graph capture; later calls may).
 * The device of `hip_stream` must be the current device.  All calls on one GPU share the one array: calls that
 * may overlap on a GPU (different streams without an ordering between them, or several host threads) race and
 * must use ot_tree_verify_attention with workspaces of their own.  The status word of a clamped prefix length
 * is not observable through this entry point (lengths are still clamped).
 * Returns OT_ERR_SCRATCH_LIMIT when ot_attn_workspace_bytes(p) exceeds OT_ATTN_SCRATCH_BYTES (the split
 * partials of a single sequence with many grouped query heads are the large case, up to 17 MB; a batch-1
 * multi-head shape needs 3-4 MB, batches that fill the chip without splitting only the first
 * OT_ATTN_SYNC_BYTES); other errors as ot_tree_verify_attention. */
#define OT_ATTN_SCRATCH_BYTES (8u << 20)
OT_API int ot_tree_verify_attention_noalloc(const ot_attn_params* p,
                             const void* Q, const void* K_prefix, const void* V_prefix,
                             const void* K_tree, const void* V_tree,
                             const int32_t* prefix_len, const uint64_t* mask,
                             void* O, void* hip_stream);

/* Measurement aid: ot_tree_verify_attention that also records the begin and the end of its
 * K/V-streaming kernel (Algorithm 2's tree-masked attention; for bf16 it includes the split merge) in two
 * caller-created hipEvent_t (void*, either may be NULL).  Not capturable in a graph. */
OT_API int ot_tree_verify_attention_timed(const ot_attn_params* p,
                             const void* Q, const void* K_prefix, const void* V_prefix,
                             const void* K_tree, const void* V_tree,
                             const int32_t* prefix_len, const uint64_t* mask,
                             void* O, void* workspace, size_t workspace_bytes, void* hip_stream,
                             void* kernel_begin_event, void* kernel_end_event);

/* ------------------------------------------------------------------------
 * Greedy verification (Preliminaries, "Speculative Decoding"; Algorithm 2, "Verify" and "Concat").
 *
 * target_logits [batch][n + 1][vocab]: the target model's output rows, row 0 at the root position (the last
 * token of the input), row 1 + i at tree node i (element (b, r, v) at base + b*stride_seq + r*stride_row + v).
 * The ground truth after a position is the most probable token of its row (equal logits: the smaller token
 * id).  Starting at the root, the child of the current node that carries the ground truth is accepted and
 * becomes the current node, until no child does; the ground truth after the last accepted node is produced
 * as well.  Per sequence:
 *   accept_len[b]            A  = tokens produced = accepted nodes + 1            (1..n_out[b] + 1)
 *   accept_node[b][0..A-2]   output indices of the accepted nodes, root side first (rest of [n]: -1)
 *   accept_token[b][0..A-1]  the produced tokens (rest of [n + 1]: -1)
 * token / parent / n_out are the tree builder's outputs ([batch][n], [batch][n], [batch]).
 * ---------------------------------------------------------------------- */
typedef struct ot_verify_params {
    int32_t batch, vocab, n;
    int32_t logits_dtype;               /* OT_F32 | OT_BF16 */
    int64_t stride_seq, stride_row;     /* in elements; stride_row >= vocab */
} ot_verify_params;

OT_API size_t ot_verify_workspace_bytes(const ot_verify_params* p);   /* 0 if p is invalid */

OT_API int ot_verify_greedy(const ot_verify_params* p, const void* target_logits,
                     const int32_t* token, const int32_t* parent, const int32_t* n_out,
                     void* workspace, size_t workspace_bytes,
                     int32_t* accept_len, int32_t* accept_node, int32_t* accept_token, void* hip_stream);

/* Verification under random sampling (Sec. 4, "Performance on Non-greedy Settings": only the acceptable
 * tokens change with respect to the greedy case; the paper gives no rule, this is the reading built here).
 * The ground truth after a position is DRAWN from q = softmax(row / temperature) of that position's target
 * row: the smallest token v with q_0 + ... + q_v > u, u = u[b][r] a uniform number in [0, 1) supplied by the
 * caller per row (device float [batch][n + 1], row index as in target_logits).  The walk and the outputs are
 * those of ot_verify_greedy.  Every produced token is an exact draw from the target's distribution at its
 * position, so the output is distributed as plain sampling from the target.  Logits must be finite or -inf
 * (probability 0; a row without a finite logit draws token 0).  The cumulative sums are taken in fp32 per
 * 16-byte vector and fp64 above: a u closer than ~1e-6 to a boundary of the CDF may fall on either side.
 * temperature > 0 (for temperature -> 0 use ot_verify_greedy).  Unsupported (-2): vocab beyond 512
 * segments of 64 x 16 bytes (131072 f32 / 262144 bf16 logits), batch * (n + 1) > 65535. */
OT_API size_t ot_verify_sample_workspace_bytes(const ot_verify_params* p);   /* 0 if p is invalid or unsupported */

OT_API int ot_verify_sample(const ot_verify_params* p, float temperature, const void* target_logits, const float* u,
                     const int32_t* token, const int32_t* parent, const int32_t* n_out,
                     void* workspace, size_t workspace_bytes,
                     int32_t* accept_len, int32_t* accept_node, int32_t* accept_token, void* hip_stream);

/* The accepted nodes join the cache ("Concat" of Algorithm 2): for j < A - 1 the K and V rows of tree node
 * accept_node[b][j] are copied to prefix row prefix_len[b] + j of every KV head, and
 * new_prefix_len[b] = min(prefix_len[b] + A - 1, max_prefix); rows that do not fit in max_prefix are dropped.
 * Uses batch, kv_heads, head_dim, n, max_prefix, dtype and the K/V strides of `p` (the attention call's
 * parameters).  K_tree / V_tree must not overlap the prefix rows that are written.  new_prefix_len must not
 * overlap prefix_len (workgroups that copy rows still read prefix_len[b] when new_prefix_len[b] is written):
 * a call whose two length arrays overlap returns OT_ERR_INVALID_ARG; a decoder alternates between two arrays.
 * Needs no workspace. */
OT_API int ot_kv_append(const ot_attn_params* p, void* K_prefix, void* V_prefix,
                 const void* K_tree, const void* V_tree,
                 const int32_t* prefix_len, const int32_t* accept_len, const int32_t* accept_node,
                 int32_t* new_prefix_len, void* hip_stream);

/* ------------------------------------------------------------------------
 * Yardsticks for the measurement (for callers that rate the kernels above against what this GPU reaches,
 * not only against published peaks).  Both launch OT_YARDSTICK_WORKGROUPS workgroups of 256 threads.
 *   ot_yardstick_stream_read  reads `bytes` (a multiple of 16, 16-byte aligned) once, 16 bytes per load;
 *                             bytes / time = achievable HBM read bandwidth for a buffer larger than the caches;
 *   ot_yardstick_mfma_loop    per wavefront 4 * iters v_mfma_f32_32x32x16_bf16 on register operands:
 *                             OT_YARDSTICK_WORKGROUPS * 4 wavefronts * 4 * iters * 32768 flop in total.
 * `sink` is a device buffer of at least OT_YARDSTICK_WORKGROUPS 4-byte words that keeps the work observable.
 * ---------------------------------------------------------------------- */
#define OT_YARDSTICK_WORKGROUPS 2048
OT_API int ot_yardstick_stream_read(const void* src, size_t bytes, void* sink, void* hip_stream);
OT_API int ot_yardstick_mfma_loop(int32_t iters, void* sink, void* hip_stream);
/* The streaming read with a caller-chosen number of workgroups (1..2^20, of 256 threads; `sink` holds that many words)
 * and, as in the *_timed calls above, two optional hipEvent_t that receive the kernel's own begin and end time stamps:
 * what a launch of a given size and shape reaches, ramp-up and tail included, measured the way the hot kernels are. */
OT_API int ot_yardstick_stream_read_timed(const void* src, size_t bytes, int32_t workgroups, void* sink, void* hip_stream,
                                   void* kernel_begin_event, void* kernel_end_event);

#ifdef __cplusplus
}
#endif
#endif /* OPTTREE_H */
