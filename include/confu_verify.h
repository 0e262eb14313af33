/*
 * confu_verify.h - C ABI of the MI355X (gfx950) tree-verification library.
 *
 * Two operations of one speculative-decoding iteration's target-model pass:
 *
 *   tree_verify_attention  attention of the M = T + C new rows (T draft-tree nodes,
 *                          C contemplate rows) over the cached prefix and over their
 *                          own tree ancestors, one call per transformer layer;
 *   tree_accept            temperature softmax over the vocabulary and the tree
 *                          acceptance walk that returns the accepted path and the
 *                          bonus / residual token.
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device memory owned by the caller (for instance the
 *     data_ptr() of a PyTorch tensor); "host" pointers are ordinary host memory.
 *     The library never frees or retains them.
 *   - Scratch memory comes from the caller's workspace (device); its size is given by
 *     the matching *_workspace_bytes query for the same descriptor.  The workspace
 *     may be reused by the next call on the same stream; concurrent calls on
 *     different streams need different workspaces.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without synchronising.
 *   - Return value: TV_OK, or an error found on the host before anything was
 *     enqueued.  Errors that depend on device data (a malformed tree, a token id out
 *     of range, a prefix length out of range) are reported per sequence in the
 *     device array `status`, and that sequence's outputs are then zeros
 *     (attention) or -1 (acceptance).
 *   - Global state: cached device properties and launch attributes, the address of the
 *     fixed scratch array of tree_verify_attention_noalloc, and the test hook
 *     tv_set_wait_limit (an atomic integer read by tree_accept).  Calls are thread-safe
 *     for distinct streams and workspaces.
 */
#ifndef CONFU_VERIFY_H
#define CONFU_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- return codes ------------------------------------------------------------ */
#define TV_OK                 0
#define TV_ERR_INVALID_ARG    1   /* null pointer, size out of range, bad struct_size */
#define TV_ERR_WORKSPACE      2   /* workspace missing or too small */
#define TV_ERR_LAUNCH         3   /* HIP reported an error at launch */
#define TV_ERR_UNSUPPORTED    4   /* valid request this build has no kernel for */

/* ---- per-sequence status bits written to `status` (device) --------------------- */
#define TV_STATUS_OK            0
#define TV_STATUS_BAD_PARENT    1   /* parent[i] outside [-1, i), or root missing */
#define TV_STATUS_BAD_KIND      2   /* kind not 0/1, or a draft node hangs off a contemplate row */
#define TV_STATUS_BAD_PREFIX    4   /* prefix_len < soft_len, < 0 or > max_prefix_len */
#define TV_STATUS_BAD_TOKEN     8   /* token id outside [0, V) */
#define TV_STATUS_INTERNAL     16   /* reserved (earlier versions: a bounded wait between workgroups ran out); no longer raised */
#define TV_STATUS_BAD_PATH     32   /* tree_commit: path not a strictly increasing list of nodes starting at the root */

/* ---- limits -------------------------------------------------------------------- */
#define TV_MAX_ROWS   128          /* M (attention) and T (acceptance) */
#define TV_PREPARED_TREE_BYTES 2304 /* device bytes per sequence of a prepared tree (tv_prepare_tree) */

/* ---- enums ---------------------------------------------------------------------- */
#define TV_DTYPE_F32   0
#define TV_DTYPE_BF16  1

#define TV_KIND_NODE         0     /* a draft-tree node (row 0 of a sequence is the root) */
#define TV_KIND_CONTEMPLATE  1     /* a contemplate row: may attend to the soft-prompt slots */

#define TV_RULE_GREEDY         0   /* temperature 0: a child is accepted iff it is the argmax */
#define TV_RULE_DETERMINISTIC  1   /* temp > 0, no draft law: each child is a point-mass proposal */
#define TV_RULE_DRAFT_WOR      2   /* temp > 0, siblings drawn from the draft law without replacement */
#define TV_RULE_DRAFT_WR       3   /* temp > 0, siblings drawn independently (with replacement) */
#define TV_RULE_SAMPLE_MATCH   4   /* temp > 0, target logits only: the target's token is sampled at each node
                                      (inverse CDF at u[T + node]) and a child is accepted iff it proposed that token;
                                      the final token is the sample at the stop node */

#define TV_FINAL_BONUS     0       /* nothing was rejected at the stop node: token from the target law */
#define TV_FINAL_RESIDUAL  1       /* at least one child was rejected there: token from the corrected law */

/* =================================================================================
 * tree_verify_attention
 *
 * Operation (paper: Section 2, tree attention over the draft tree; Section 3.1,
 * contemplate rows appended to the tree and soft-prompt slots at the head of the KV
 * cache that only contemplate rows may attend to; Figure 4).
 *
 * For sequence b, query row i (0 <= i < M) and query head h (KV head g = h / (Hq/Hkv)):
 *
 *   visible cached rows   [soft_len, P_b) if kind[i] = NODE, [0, P_b) if CONTEMPLATE
 *   visible new rows      j in {i, parent[i], parent[parent[i]], ..., root}
 *   out[b,i,h,:] = sum_k softmax_k(softmax_scale * q[b,i,h,:] . K[k,g,:]) * V[k,g,:]
 *
 * The KV pool holds for sequence b the rows kv_offset[b] .. kv_offset[b]+P_b+M-1:
 * the P_b cached rows (the first soft_len of them are the soft-prompt slots) followed
 * by this step's M new rows, already written by the caller.  Row r, KV head g starts
 * at element r*kv_token_stride + g*kv_head_stride; its D elements are contiguous.
 * ================================================================================= */
typedef struct tv_attn_desc {
    uint32_t struct_size;      /* sizeof(tv_attn_desc), checked */
    int32_t  dtype;            /* TV_DTYPE_F32 (D in {64,128}) or TV_DTYPE_BF16 (D = 128) */
    int32_t  B;                /* sequences, 1 .. 65535 */
    int32_t  M;                /* query rows per sequence, 1..TV_MAX_ROWS */
    int32_t  Hq;               /* query heads */
    int32_t  Hkv;              /* KV heads, divides Hq; Hq/Hkv <= 16 */
    int32_t  D;                /* head dimension */
    int32_t  soft_len;         /* s: leading cached rows that are soft-prompt slots, >= 0 */
    int32_t  max_prefix_len;   /* host-known upper bound of prefix_len[b] (sizes the launch) */
    float    softmax_scale;    /* usually 1/sqrt(D) */
    int64_t  kv_token_stride;  /* elements between consecutive rows of the pool; 0 = Hkv*D */
    int64_t  kv_head_stride;   /* elements between KV heads of one row; 0 = D */
    int32_t  num_splits;       /* 0 = library decides how many ranges the keys are cut into */
    int32_t  wg_row_blocks;    /* bf16 path tuning, 0 = library decides: 64-row blocks of the packed query rows that one
                                  workgroup covers (1, 2 or 4) */
    int64_t  sum_prefix_len;   /* hint, B > 1: sum of prefix_len[b] as the host expects it, or 0 = unknown.  The lengths
                                  themselves stay on the device; with the sum the launch is sized for the batch as it
                                  is (all sequences alike, or ragged), without it for a compromise between the two.
                                  0 <= sum_prefix_len <= B * max_prefix_len.  Results do not depend on it. */
} tv_attn_desc;

/* host: writes the workspace size (bytes) tree_verify_attention needs for *desc.
 * Returns TV_OK / TV_ERR_INVALID_ARG / TV_ERR_UNSUPPORTED. */
int tv_attention_workspace_bytes(const tv_attn_desc* desc, size_t* out_bytes);

/* host: the launch shape the library would use for *desc on the current device (bf16 path; the fp32 path
 * reports 1 and 1): *wg_row_blocks = 64-row blocks of the packed query rows per workgroup (1, 2 or 4),
 * *key_ranges = ranges the keys of a sequence are cut into (> 1: partial results in the workspace and a second
 * kernel).  num_splits / wg_row_blocks of the descriptor are honoured (num_splits is capped so that a range
 * keeps at least eight 32-key tiles).  For logging and tuning; nothing has to call it.
 * Returns TV_OK / TV_ERR_INVALID_ARG / TV_ERR_UNSUPPORTED. */
int tv_attention_plan(const tv_attn_desc* desc, int32_t* wg_row_blocks, int32_t* key_ranges);

/* Optional, once per verification step (paper: Section 3.1 / Figure 4 - the tree mask belongs to the step and
 * is the same in every layer): checks the B trees and writes, per sequence, the ancestor mask of every row, the
 * row kinds and the verdict (TV_STATUS_BAD_PARENT / TV_STATUS_BAD_KIND bits) into `prepared` (device, 16-byte
 * aligned, B * TV_PREPARED_TREE_BYTES bytes, owned by the caller).  Layer calls of tree_verify_attention that
 * are handed `prepared` skip their own checks and ancestor walks; results and status are the same either way.
 * parent / kind: device [B, M] as for tree_verify_attention.  Enqueued on hip_stream, no synchronisation; the
 * record must not be rewritten while calls that read it are in flight.
 * Returns TV_OK / TV_ERR_INVALID_ARG / TV_ERR_LAUNCH. */
int tv_prepare_tree(int32_t B, int32_t M, const int32_t* parent, const uint8_t* kind, void* prepared,
                    size_t prepared_bytes, void* hip_stream);

int tree_verify_attention(
    const tv_attn_desc* desc,      /* host */
    const void*    q,              /* device [B, M, Hq, D], dtype, contiguous */
    const void*    k_pool,         /* device, dtype, layout above */
    const void*    v_pool,         /* device, dtype, same layout as k_pool */
    const int64_t* kv_offset,      /* device [B]: first pool row of sequence b */
    const int32_t* prefix_len,     /* device [B]: P_b, soft-prompt slots included */
    const int32_t* parent,         /* device [B, M]: parent row, -1 for the root, parent[i] < i */
    const uint8_t* kind,           /* device [B, M]: TV_KIND_* */
    const void*    prepared_tree,  /* device: what tv_prepare_tree wrote for these B trees (same parent / kind), or NULL:
                                      the call then checks the trees and builds the masks itself.  Used by the bf16
                                      path; the fp32 path always builds its own */
    void*          out,            /* device [B, M, Hq, D], dtype */
    float*         lse,            /* device [B, Hq, M] natural-log sum of exp of the scaled visible scores, or NULL */
    int32_t*       status,         /* device [B]: TV_STATUS_* bits, written by the call */
    void*          workspace,      /* device, 256-byte aligned, may be NULL if 0 bytes are needed */
    size_t         workspace_bytes,
    void*          hip_stream);

/* For callers that cannot allocate device memory or pass a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The same operation, arguments, results and error behaviour as
 * tree_verify_attention, with the partial results of the key ranges kept in a fixed array of
 * TV_NOALLOC_SCRATCH_BYTES inside the library's device image (each GPU the library runs on holds one copy until
 * the process ends) instead of a workspace.  The call allocates and frees nothing.  A launch shape that needs
 * more than the array (tv_attention_workspace_bytes(desc) > TV_NOALLOC_SCRATCH_BYTES: very long contexts, large
 * batches) is refused with TV_ERR_WORKSPACE before anything is enqueued.  All calls on one GPU share that GPU's
 * array: calls that may overlap on one GPU (different streams) race; calls on one stream are safe.  The first
 * call on a device looks the array's address up (do it once outside any graph capture). */
#define TV_NOALLOC_SCRATCH_BYTES (16u << 20)
int tree_verify_attention_noalloc(
    const tv_attn_desc* desc, const void* q, const void* k_pool, const void* v_pool, const int64_t* kv_offset,
    const int32_t* prefix_len, const int32_t* parent, const uint8_t* kind, const void* prepared_tree, void* out,
    float* lse, int32_t* status, void* hip_stream);

/* =================================================================================
 * tree_accept
 *
 * Operation (paper: Section 2 steps 3-4, drafts are checked in order and the first
 * rejected one is replaced by a token from the target's corrected distribution; tree
 * form: the longest accepted path; Section 3.1: the future prediction of the last
 * accepted node is kept; Section 4: temperatures 0 / 0.7 / 1.0, tau counts the bonus
 * token).  With p = softmax(target_logits[node]/temperature) and, for the DRAFT rules,
 * q = softmax(draft_logits[node]/temperature), starting at the root:
 *
 *   for each child c of the current node, in increasing index, x = token[c]:
 *     DETERMINISTIC  accept iff u[c] < p(x);        on reject p(x) = 0, p renormalised
 *     DRAFT_WOR/WR   accept iff u[c]*q(x) < p(x);   on reject p = norm(max(p - q, 0));
 *                    DRAFT_WOR also removes x from q and renormalises q
 *     GREEDY         accept iff x = argmax target_logits[node] (lowest index on ties)
 *     an accepted child becomes the current node;
 *   when no child is accepted: final_token = first v whose running sum of p exceeds
 *   u[T + node] (GREEDY: the argmax), final_kind says whether p had been corrected.
 *
 * Logits may be -infinity (banned tokens, a padded tail): such entries have probability 0.  A row
 * that is -infinity throughout has no law: every child of that node is rejected, and if the walk
 * stops there final_token is -1 (GREEDY: 0, the lowest index of the tie).  NaN and +infinity are
 * not allowed (undefined results).
 * ================================================================================= */
typedef struct tv_accept_desc {
    uint32_t struct_size;        /* sizeof(tv_accept_desc), checked */
    int32_t  B;                  /* sequences, >= 1 */
    int32_t  T;                  /* draft nodes per sequence (root included), 1..TV_MAX_ROWS */
    int32_t  V;                  /* vocabulary size, >= 1 */
    int32_t  C;                  /* entries of con_anchor per sequence (0 if con_anchor is NULL) */
    int32_t  rule;               /* TV_RULE_* */
    float    temperature;        /* > 0 unless rule = GREEDY */
    int64_t  logits_row_stride;  /* elements between consecutive rows of the logits; 0 = V */
    int32_t  logits_dtype;       /* element type of both logits matrices: TV_DTYPE_F32 (0) or TV_DTYPE_BF16 */
    int32_t  reserved;           /* must be 0 */
} tv_accept_desc;

int tv_accept_workspace_bytes(const tv_accept_desc* desc, size_t* out_bytes);

int tree_accept(
    const tv_accept_desc* desc,     /* host */
    const void*    target_logits,   /* device [B, T, V], logits_dtype (rows logits_row_stride elements apart) */
    const void*    draft_logits,    /* device [B, T, V], logits_dtype; required by the DRAFT rules, else NULL */
    const int32_t* token,           /* device [B, T]: token drafted at each node (token[0]: the root's) */
    const int32_t* parent,          /* device [B, T]: parent node, -1 for the root, parent[i] < i */
    const float*   uniforms,        /* device [B, 2T]: u[c] tests node c, u[T+n] draws the final token at stop node n; unused by GREEDY (may be NULL) */
    const int32_t* con_anchor,      /* device [B, C]: node each contemplate row belongs to, or NULL */
    int32_t*       path,            /* device [B, T]: accepted nodes, root first, then -1 */
    int32_t*       n_accepted,      /* device [B]: accepted draft tokens (root not counted) */
    int32_t*       final_token,     /* device [B] */
    int32_t*       final_kind,      /* device [B]: TV_FINAL_* */
    int32_t*       last_node,       /* device [B]: path[n_accepted] */
    int32_t*       selected_con,    /* device [B]: first c with con_anchor[c] == last_node, else -1; may be NULL */
    int32_t*       status,          /* device [B]: TV_STATUS_* bits */
    void*          workspace,       /* device, 256-byte aligned */
    size_t         workspace_bytes,
    void*          hip_stream);

/* =================================================================================
 * Host helpers
 * ================================================================================= */

/* =================================================================================
 * tree_commit
 *
 * Operation (paper: Section 2, step 3 - a rejected draft token and everything after it
 * are discarded; tree form: the longest accepted path is kept; Section 3.1 - after
 * verification the future prediction that belongs to the last accepted token is the one
 * handed to the draft model for the next iteration).
 *
 * After tree_accept: for every layer l < n_layers, sequence b and j = 0 .. n_accepted[b],
 * the K and V rows of tree node path[b][j] (new row node_row[b][path[b][j]] of this step)
 * are moved to new row j, so that the cache holds the accepted tokens contiguously, in
 * order, right behind the old prefix; rows of rejected nodes and of contemplate rows are
 * dropped (left as they are behind the new end).  new_prefix_len[b] = prefix_len[b] +
 * n_accepted[b] + 1.  If hidden is given, f_out[b,:] = hidden[b, con_row[b][selected_con[b]], :]
 * (zeros when selected_con[b] < 0).
 *
 * A sequence with n_accepted[b] < 0 (tree_accept flagged it) is left untouched:
 * new_prefix_len[b] = prefix_len[b], status[b] = 0.  A malformed path (not starting at
 * node 0, not strictly increasing, outside [0,T), or a mapped row outside [0,M)) sets
 * TV_STATUS_BAD_PATH and leaves the sequence untouched.
 * ================================================================================= */
typedef struct tv_commit_desc {
    uint32_t struct_size;      /* sizeof(tv_commit_desc), checked */
    int32_t  dtype;            /* element type of the pools, hidden and f_out: TV_DTYPE_F32 or TV_DTYPE_BF16 */
    int32_t  B;                /* sequences, >= 1 */
    int32_t  T;                /* tree nodes per sequence (row length of path and node_row), 1..TV_MAX_ROWS */
    int32_t  M;                /* new rows per sequence in the pools (nodes + contemplate rows), T..TV_MAX_ROWS */
    int32_t  Hkv;              /* KV heads */
    int32_t  D;                /* head dimension; D * element size is a multiple of 16 bytes */
    int32_t  n_layers;         /* layers compacted by this call, >= 1 */
    int64_t  kv_layer_stride;  /* elements between the pools of consecutive layers (ignored when n_layers = 1) */
    int64_t  kv_token_stride;  /* as in tv_attn_desc; 0 = Hkv*D */
    int64_t  kv_head_stride;   /* as in tv_attn_desc; 0 = D */
    int32_t  C;                /* contemplate rows per sequence (row length of con_row), >= 0 */
    int32_t  d_model;          /* elements of a hidden row; d_model * element size is a multiple of 16 bytes; 0 = no gather */
} tv_commit_desc;

/* Enqueues the work on hip_stream and returns without synchronising; no workspace.
 * Returns TV_OK, TV_ERR_INVALID_ARG, TV_ERR_LAUNCH. */
int tree_commit(
    const tv_commit_desc* desc,
    void*          k_pool,          /* device, updated in place: layer l starts at element l*kv_layer_stride */
    void*          v_pool,          /* device, same layout */
    const int64_t* kv_offset,       /* device [B] */
    const int32_t* prefix_len,      /* device [B]: P_b before this step */
    const int32_t* path,            /* device [B,T]: from tree_accept */
    const int32_t* n_accepted,      /* device [B]: from tree_accept */
    const int32_t* node_row,        /* device [B,T]: new-row index of tree node i (i if the nodes come first, 2i if a
                                       contemplate row follows each node), or NULL for the identity.  Rows must
                                       increase along every accepted path (a child's row comes after its parent's, as
                                       the attention call requires of the same rows): TV_STATUS_BAD_PATH otherwise */
    const void*    hidden,          /* device [B,M,d_model] or NULL: final hidden states of this step's rows */
    const int32_t* con_row,         /* device [B,C]: new-row index of contemplate row c; NULL iff hidden is NULL */
    const int32_t* selected_con,    /* device [B]: from tree_accept; NULL iff hidden is NULL */
    void*          f_out,           /* device [B,d_model]; NULL iff hidden is NULL */
    int32_t*       new_prefix_len,  /* device [B] */
    int32_t*       status,          /* device [B]: TV_STATUS_* bits */
    void*          hip_stream);

/* =================================================================================
 * contemplate_embed
 *
 * Operation (paper: Section 3.2, dynamic contemplate tokens): the embedding of a
 * contemplate (or future) token is a mixture of n_expert learnable embeddings, gated by
 * the hidden state h of the most recently accepted token:
 *
 *   g = softmax(W h)  over the n_expert experts,  S = the k_expert experts with the largest
 *   g (ties: lowest index),  out = sum_{e in S} g_e * E[e,:]
 *
 * (the gates are the softmax scores themselves: they are not renormalised over S).
 * h, W, E and out share one element type; sums are fp32.
 * ================================================================================= */
typedef struct tv_embed_desc {
    uint32_t struct_size;      /* sizeof(tv_embed_desc), checked */
    int32_t  dtype;            /* TV_DTYPE_F32 or TV_DTYPE_BF16 */
    int32_t  B;                /* tokens embedded by this call, >= 1 */
    int32_t  d_in;             /* width of h (the target's concatenated hidden state, or the draft's), multiple of 8 */
    int32_t  d_out;            /* width of an expert embedding, multiple of 8 */
    int32_t  n_expert;         /* 1..64 */
    int32_t  k_expert;         /* 1..n_expert */
    int32_t  reserved;         /* 0 */
} tv_embed_desc;

/* host: writes the workspace size (bytes) contemplate_embed needs for *desc. */
int tv_embed_workspace_bytes(const tv_embed_desc* desc, size_t* out_bytes);

/* Enqueues the work on hip_stream and returns without synchronising.
 * Returns TV_OK, TV_ERR_INVALID_ARG, TV_ERR_WORKSPACE, TV_ERR_LAUNCH. */
int contemplate_embed(
    const tv_embed_desc* desc,
    const void*    h,               /* device [B, d_in] */
    const void*    router_w,        /* device [n_expert, d_in], row major */
    const void*    expert_emb,      /* device [n_expert, d_out] */
    void*          out,             /* device [B, d_out] */
    float*         gates,           /* device [B, n_expert] or NULL: the softmax scores g */
    int32_t*       chosen,          /* device [B, k_expert] or NULL: the selected experts, best first */
    void*          workspace,       /* device, 16-byte aligned, >= tv_embed_workspace_bytes() */
    size_t         workspace_bytes,
    void*          hip_stream);

/* host: checks a parent/kind pair and writes the ancestor-closure bit mask the attention
 * kernels build on the device: bit j of bits[2*i + j/64] is set iff row i may attend to new
 * row j (Section 3.1 / Figure 4).  All pointers are host memory; bits holds 2*M words
 * (pass NULL to validate only).  Returns TV_OK, TV_ERR_INVALID_ARG, or -(TV_STATUS_* bits)
 * when the tree is malformed. */
int tv_build_mask_host(const int32_t* parent, const uint8_t* kind, int M, uint64_t* bits);

/* host: static text for a return code. */
const char* tv_error_string(int code);

/* host: library version, major*100 + minor. */
int tv_version(void);

/* host, for tests: sets how many times a workgroup of tree_accept's sibling-chain kernel (draft rules) looks
 * for a result of another workgroup of its group before it stops waiting and computes that result itself (the
 * same bits, more work).  Results never depend on it; workgroups never wait without bound, whether or not the
 * others are running.  0 restores the default (about a million looks).  Applies to calls made after it;
 * returns the previous setting. */
int tv_set_wait_limit(int polls);

#ifdef __cplusplus
}
#endif
#endif /* CONFU_VERIFY_H */
