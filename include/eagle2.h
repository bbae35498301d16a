/*
 * eagle2.h -- C ABI of the MI355X (gfx950) hot path for one draft-plus-verify
 * round of the context-aware dynamic draft tree of EAGLE-2 (arXiv 2406.16858).
 *
 * One round = depth x eagle2_expand, eagle2_rerank, eagle2_tree_attn (once per
 * attention layer of the verifying model), eagle2_accept; eagle2_commit_kv and
 * eagle2_commit_round carry the accepted tokens over to the next round.
 *
 * Common rules for every entry point
 *   - Every pointer is caller-owned DEVICE memory on the current HIP device,
 *     16-byte aligned, unless the parameter is documented as a host value.  The
 *     library never allocates or frees device memory and keeps no pointer after
 *     the call returns.  Its only mutable global state belongs to the benchmark
 *     timing hooks at the end of this header (a pool of HIP events created by
 *     eagle2_kernel_timing_enable, never inside a call of the method).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).  No entry point synchronises with the host; outputs are
 *     valid once the stream reaches that point.
 *   - `workspace` is scratch owned by the caller, at least
 *     eagle2_workspace_bytes() long, 256-byte aligned.  Its contents carry nothing
 *     from one call to the next.  Calls that share a workspace must be ordered on
 *     one stream.
 *   - Return value: EAGLE2_OK, or a negative error code; on error nothing has
 *     been enqueued and eagle2_last_error() describes the problem.
 *   - Inputs must be finite.  NaN/Inf give unspecified results but never an
 *     out-of-bounds access.
 *   - Batched arrays are [batch, ...] contiguous.
 *
 * Notation (the paper's, Section 4): V vocabulary size, Hd hidden size, D tree
 * depth, k nodes expanded per layer (= children kept per node), N rows of the
 * flattened tree including the root, C = k + (D-1) k^2 candidate nodes of a
 * round, R = 1 + (D-1) k LM-head rows of a round, P length of a sequence's KV
 * prefix.
 *
 * Candidate ids.  Pass d (0-based) expands the layer-d frontier into layer d+1.
 * Layer 1 holds ids 0..k-1 (by rank); layer L >= 2 holds
 * k + (L-2) k^2 + slot*k + rank, where slot is the parent's position in its
 * frontier and rank the child's rank in the parent's distribution.  A larger id
 * is never shallower, so "lower id first" implements the paper's "prefer the
 * shallower node" rule for equal values (Section 4.2).
 */
#ifndef EAGLE2_H
#define EAGLE2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EAGLE2_OK             0
#define EAGLE2_ERR_ARG       (-1)  /* null, misaligned or out-of-range argument        */
#define EAGLE2_ERR_SHAPE     (-2)  /* shape outside the supported set (see eagle2_cfg) */
#define EAGLE2_ERR_WORKSPACE (-3)  /* workspace null or too small                      */
#define EAGLE2_ERR_HIP       (-4)  /* a HIP call failed; see eagle2_last_error()       */

#define EAGLE2_DTYPE_F32  0
#define EAGLE2_DTYPE_BF16 1

#define EAGLE2_MODE_GREEDY 0
#define EAGLE2_MODE_SAMPLE 1

/* Bits of eagle2_cfg.flags: the two switches of the ablation study (Section 5.2, Table 3).
 * RANK_BY_CONFIDENCE ("w/o value"): the expansion phase picks the next frontier by each new
 * node's own confidence instead of its value (the product along the path).
 * NO_RERANK ("w/o reranking"): the draft is what the expansion phase itself selected -- the
 * k nodes expanded in every layer plus the k best nodes of the last layer -- with no global
 * re-selection; the tree then has exactly D*k + 1 rows. */
#define EAGLE2_FLAG_RANK_BY_CONFIDENCE 1
#define EAGLE2_FLAG_NO_RERANK          2
/* STATIC_TREE: the fixed-shape draft tree the method replaces (Section 2.2, "Differences between
 * EAGLE and EAGLE-2": the shape is fixed and the drafting phase fills in the positions).  The
 * caller fixes the shape: frontier[b, d, :] holds the candidate ids expanded by pass d (unused
 * slots -1) and is never written by eagle2_expand; eagle2_rerank takes its N-1 nodes from
 * cfg->static_tree instead of selecting them.  Excludes the other two flags. */
#define EAGLE2_FLAG_STATIC_TREE        4

#define EAGLE2_MAX_TOPK    16
#define EAGLE2_MAX_TREE    128
#define EAGLE2_MAX_CAND    2048

/*
 * Shape of a round.  Supported: 1 <= topk <= 16 <= vocab; depth >= 1;
 * 2 <= n_tree <= 128 and n_tree - 1 <= C <= 2048; hidden * sizeof(dtype) a
 * multiple of 1024 bytes; batch >= 1.
 */
typedef struct eagle2_cfg {
    int32_t batch;   /* B: sequences, each with its own tree                     */
    int32_t vocab;   /* V                                                         */
    int32_t hidden;  /* Hd                                                        */
    int32_t depth;   /* D: LM-head passes per round = deepest layer              */
    int32_t topk;    /* k                                                         */
    int32_t n_tree;  /* N: flattened rows including the root                     */
    int32_t dtype;   /* EAGLE2_DTYPE_*: element type of H, W, Q, K, V and O      */
    int32_t flags;   /* 0 = the method as published; EAGLE2_FLAG_* select ablations;
                        with EAGLE2_FLAG_NO_RERANK n_tree must equal D*k + 1      */
    const int32_t* static_tree;  /* device, [n_tree - 1] candidate ids in increasing order,
                        closed under "parent of"; read only with
                        EAGLE2_FLAG_STATIC_TREE (NULL otherwise)                  */
} eagle2_cfg;

/* Attention geometry.  Supported: head_dim 64 or 128; n_q_heads a multiple of
 * n_kv_heads. */
typedef struct eagle2_attn_cfg {
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    float   scale;         /* multiplies q.k; 0 selects 1/sqrt(head_dim)           */
    int64_t total_prefix;  /* host value: rows of K_prefix/V_prefix; must be >= kv_offsets[B]
                              (grid and workspace are sized from it: key chunks beyond it
                              are ignored, never read out of bounds)                  */
} eagle2_attn_cfg;

/* Library version (major*10000 + minor*100 + patch). */
int eagle2_version(void);

/* Text of the last error raised on the calling thread ("" if none). */
const char* eagle2_last_error(void);

/* Bytes of workspace that is enough for any of the four calls with these shapes
 * (attn may be NULL if eagle2_tree_attn is not used).  0 on invalid shapes. */
size_t eagle2_workspace_bytes(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn);

/*
 * Expansion phase, pass d (Section 4.1).
 *
 * For every sequence b and frontier slot s (F_d rows: F_0 = 1, else k) the draft
 * model's token distribution is softmax(H[b,s,:] . W^T); its k most probable
 * tokens (ties: lower token id) become children of the node in frontier[b,d,s]
 * with joint score = parent score + log-probability (the value equation of
 * Section 4.1, kept as a sum of logs; the root's score is 0).  Children are
 * appended to the candidate arrays at ids base_d + s*k + rank.  If d+1 < D the k
 * new candidates of highest score (ties: lower id) are written to
 * frontier[b,d+1,:], best first (Section 4.1, last paragraph).  With
 * EAGLE2_FLAG_RANK_BY_CONFIDENCE the k new candidates of highest own
 * log-probability are taken instead (Section 5.2); the stored scores stay joint.
 *
 *   H            [B, F_d, Hd] dtype; sequence b starts at element b*h_seq_stride
 *                (h_seq_stride = 0 means F_d*Hd, i.e. contiguous).
 *   W            [V, Hd] dtype, row-major: the LM head.
 *   cand_token   [B, C] int32   in/out: pass d writes ids base_d .. base_d+F_d*k-1
 *   cand_score   [B, C] float64 in/out: reads the parents' scores
 *   cand_parent  [B, C] int32   in/out: candidate id of the parent, -1 = root
 *   frontier     [B, D, k] int32 in/out: row d is read (d >= 1), row d+1 written;
 *                row 0 is never touched.
 *   draft_logits nullable; [B, R, V] float32.  Row (d == 0 ? 0 : 1 + (d-1)k + s)
 *                receives the raw logits of slot s; needed later only by
 *                eagle2_accept in sampling mode.
 */
int eagle2_expand(const eagle2_cfg* cfg, int32_t d,
                  const void* H, int64_t h_seq_stride, const void* W,
                  int32_t* cand_token, double* cand_score, int32_t* cand_parent,
                  int32_t* frontier, float* draft_logits,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Reranking phase and flattening (Section 4.2).
 *
 * Selects the N-1 candidates of highest score (ties: lower id = shallower),
 * lays them out behind the root in increasing id order (parents precede
 * children) and builds, per row, the ancestor bitmask under which the row sees
 * exactly itself and its ancestors (Section 4.2, second paragraph).
 *
 *   root_token   [B] int32: token of the root (the last committed token)
 *   prefix_len   [B] int32: P_b, used for position_ids = P_b + depth
 *   tree_token, tree_parent (flat row of the parent, -1 for the root), tree_depth,
 *   tree_cand (candidate id, -1 for the root), position_ids: [B, N] int32 outputs
 *   mask_bits    [B, N, ceil(N/64)] uint64 output: bit (j % 64) of word j / 64 of
 *                row i is set iff j == i or row j is an ancestor of row i.
 *   frontier     [B, D, k] int32 as left by the D expand passes; read only with
 *                EAGLE2_FLAG_NO_RERANK (may be NULL otherwise).  With that flag the
 *                selection is frontier rows 1..D-1 plus the k best candidates of
 *                layer D (by score, or by own confidence = score - parent's score
 *                with EAGLE2_FLAG_RANK_BY_CONFIDENCE; ties: lower id) (Section 5.2).
 * The candidate arrays must come from D completed eagle2_expand passes (scores
 * non-increasing from parent to child); otherwise tree_parent is unspecified.
 */
int eagle2_rerank(const eagle2_cfg* cfg,
                  const int32_t* cand_token, const double* cand_score, const int32_t* cand_parent,
                  const int32_t* frontier, const int32_t* root_token, const int32_t* prefix_len,
                  int32_t* tree_token, int32_t* tree_parent, int32_t* tree_depth,
                  int32_t* tree_cand, int32_t* position_ids, uint64_t* mask_bits,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Tree attention of the verification pass (Section 4.2, second paragraph).
 *
 * Row i of sequence b, query head h, attends to all P_b prefix keys and to the
 * tree keys j whose bit is set in mask_bits[b,i]; KV head = h / (Hq / Hkv).
 * O = softmax(scale * q.k) v with the softmax taken in float32 (float32 inputs:
 * everything in float32).  With bf16 inputs the probabilities enter the PV
 * product rounded to bf16, the products accumulate in float32, and a key
 * chunk's partial output travels to the final reduction as 16-bit floats under
 * a per-row power-of-two scale (11 significant bits; the output has 8).  No
 * rotary embedding is applied inside.
 *
 *   Q            [B, N, Hq, dh] dtype
 *   K_prefix, V_prefix  [total_prefix, Hkv, dh] dtype; sequence b owns rows
 *                kv_offsets[b] .. kv_offsets[b+1]-1
 *   kv_offsets   [B+1] int64 (device), non-decreasing, kv_offsets[0] = 0
 *   prefix_len   nullable; [B] int32 (device).  With a pre-allocated KV cache
 *                (Appendix "Implementation Details") sequence b's region
 *                kv_offsets[b] .. kv_offsets[b+1]-1 is only partly filled: P_b =
 *                prefix_len[b] (clamped to the region).  NULL: the whole region.
 *   K_tree, V_tree      [B, N, Hkv, dh] dtype
 *   mask_bits    as written by eagle2_rerank
 *   O            [B, N, Hq, dh] dtype output
 *   lse          nullable; [B, N, Hq] float32: log-sum-exp of the scaled scores
 */
int eagle2_tree_attn(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn,
                     const void* Q, const void* K_prefix, const void* V_prefix,
                     const int64_t* kv_offsets, const int32_t* prefix_len,
                     const void* K_tree, const void* V_tree,
                     const uint64_t* mask_bits, void* O, float* lse,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * Tree attention (Section 4.2) over a prefix cache kept in 8 bits.  The paper keeps
 * its cache in the model's 16-bit type; this variant halves the bytes of the
 * prefix stream, which bounds the verification pass at long contexts.
 *
 * Same as eagle2_tree_attn (cfg->dtype must be bf16) except:
 *   K_prefix8, V_prefix8  [total_prefix, Hkv, dh] uint8: E4M3 codes of the OCP 8-bit
 *                floating point format (1 sign, 4 exponent bits of bias 7, 3
 *                mantissa bits, no infinities, largest finite value 448); NaN
 *                codes must not occur
 *   k_scale, v_scale      [Hkv] float32 (device), positive: key (b, t, h, :) is
 *                value(code) * k_scale[h], likewise for V
 * The tree's own keys and values (K_tree, V_tree) stay bf16.  Codes are widened to
 * bf16 exactly; the scales enter in float32 (k_scale with the softmax scale,
 * v_scale on each chunk's partial output).
 */
int eagle2_tree_attn_fp8kv(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn,
                           const void* Q, const void* K_prefix8, const void* V_prefix8,
                           const float* k_scale, const float* v_scale,
                           const int64_t* kv_offsets, const int32_t* prefix_len,
                           const void* K_tree, const void* V_tree,
                           const uint64_t* mask_bits, void* O, float* lse,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Acceptance (Sections 2.1 and 2.2).
 *
 * mode[b] = EAGLE2_MODE_GREEDY: the target's choice after a row is the arg-max of
 * its logits (ties: lower id); starting at the root the walk moves to the child
 * whose token equals the choice while there is one; bonus_token is the choice at
 * the last accepted row.
 * mode[b] = EAGLE2_MODE_SAMPLE: speculative sampling along the tree.  At the
 * current row p = softmax(target_logits / temperature[b]) and q = softmax of the
 * draft logits its children were taken from.  Children are tried in flat order;
 * child c with token x is accepted iff u_accept[b,c] < p(x)/q(x) (Section 2.1);
 * after a rejection p <- norm(max(0, p - q)), x is removed from q and q
 * renormalised, and the next sibling is tried (Section 2.2).  With no child left
 * bonus_token is drawn from p by inverse CDF with u_bonus[b, current row].  The
 * sampling arithmetic is carried out in float64.
 *
 *   target_logits [B, N, V] float32
 *   draft_logits  [B, R, V] float32 (may be NULL if no sequence samples)
 *   temperature   [B] float32 (> 0; read for sampling sequences only)
 *   u_accept, u_bonus [B, N] float32 in [0, 1) (sampling only; may be NULL otherwise)
 *   tree_token, tree_parent, tree_cand  [B, N] int32 from eagle2_rerank
 *   accept_len    [B] int32 output: number of accepted draft tokens
 *   accept_path   [B, D+1] int32 output: flat rows root..last accepted, -1 padded
 *   bonus_token   [B] int32 output
 *
 * Failure reported in the outputs.  The workgroups that share a sampling sequence
 * exchange partial sums through the workspace and wait for each other with a
 * bounded spin, so they must all be resident at the same time: the launch uses at
 * most two workgroups of 256 threads per compute unit in total and assumes that
 * no other kernel occupies the device while it runs (work on other streams may
 * delay it; it cannot deadlock it).  If a wait expires, or the tree arrays are
 * malformed (a cycle, more than k children), the call still returns EAGLE2_OK and
 * that sequence gets accept_len[b] = -1, bonus_token[b] = -1 and an accept_path of
 * all -1; other sequences are unaffected.  Callers check accept_len[b] >= 0.
 * eagle2_commit_kv*, eagle2_commit_round treat a negative accept_len as "nothing
 * to commit" (see there), so a failed sequence can simply be run again.
 */
int eagle2_accept(const eagle2_cfg* cfg, const int32_t* mode,
                  const float* target_logits, const float* draft_logits,
                  const float* temperature, const float* u_accept, const float* u_bonus,
                  const int32_t* tree_token, const int32_t* tree_parent, const int32_t* tree_cand,
                  int32_t* accept_len, int32_t* accept_path, int32_t* bonus_token,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * eagle2_accept for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, results and failure
 * reporting as eagle2_accept, minus the workspace: the scratch (arg-max choices,
 * failure flags, exchange slots of the sampling kernel) is a fixed device array inside
 * the library, eagle2_accept_noalloc_scratch_bytes() long (about 73 KB; every GPU the
 * library runs on holds one copy until the process ends).  The call allocates nothing
 * and frees nothing; on its first use on a device it looks up that device's copy of the
 * array (no allocation) and remembers the address.
 *   - cfg->batch must not exceed EAGLE2_ACCEPT_NOALLOC_MAX_BATCH (n_tree <= 128 as
 *     everywhere); larger shapes return EAGLE2_ERR_SHAPE and nothing is enqueued.
 *   - All calls on one GPU share that GPU's array, on every stream: two calls that
 *     overlap in time on one GPU race.  Order them on one stream (or with events).
 *     The array keeps the last call's contents; the kernels clear what they need.
 */
#define EAGLE2_ACCEPT_NOALLOC_MAX_BATCH 16
size_t eagle2_accept_noalloc_scratch_bytes(void);
int eagle2_accept_noalloc(const eagle2_cfg* cfg, const int32_t* mode,
                          const float* target_logits, const float* draft_logits,
                          const float* temperature, const float* u_accept, const float* u_bonus,
                          const int32_t* tree_token, const int32_t* tree_parent, const int32_t* tree_cand,
                          int32_t* accept_len, int32_t* accept_path, int32_t* bonus_token, void* stream);

/*
 * Commit of a round, part 1: the KV cache (Section 2.1: accepted tokens are kept
 * and the remaining draft is discarded; Appendix "Implementation Details": the KV
 * cache is pre-allocated).
 *
 * For every sequence b and every layer l, the keys and values of the accepted
 * path accept_path[b, 0 .. accept_len[b]] (root first; the root is the last
 * committed token, whose key this verification pass computed) are copied from
 * the tree tensors to rows kv_offsets[b] + prefix_len[b] + i of the cache, behind
 * the prefix_len[b] rows already there.  Rows of rejected branches are not
 * copied.  Rows that would fall at or beyond kv_offsets[b+1] are dropped (the
 * caller sizes each region for prefix + D + 1 more rows).  prefix_len is not
 * changed here: eagle2_commit_round advances it once all layers are committed.
 * A sequence with accept_len[b] < 0 (acceptance reported a failure) is skipped.
 *
 *   n_layers            layers committed by this call (>= 1)
 *   accept_len, accept_path   outputs of eagle2_accept
 *   kv_offsets   [B+1] int64: regions of the cache, as for eagle2_tree_attn
 *   prefix_len   [B] int32: filled rows of each region before the round
 *   K_tree, V_tree      [n_layers][B, N, Hkv, dh] dtype, layers tree_layer_stride
 *                       elements apart
 *   K_cache, V_cache    [n_layers][total_prefix, Hkv, dh] dtype in/out, layers
 *                       cache_layer_stride elements apart (attn->total_prefix =
 *                       kv_offsets[B] rows per layer)
 * Strides are in elements and multiples of 16 bytes; with n_layers = 1 they are
 * ignored.
 */
int eagle2_commit_kv(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn, int32_t n_layers,
                     const int32_t* accept_len, const int32_t* accept_path,
                     const int64_t* kv_offsets, const int32_t* prefix_len,
                     const void* K_tree, const void* V_tree, int64_t tree_layer_stride,
                     void* K_cache, void* V_cache, int64_t cache_layer_stride, void* stream);

/*
 * eagle2_commit_kv into a cache of 8-bit codes (the cache eagle2_tree_attn_fp8kv
 * reads; Section 2.1 and Appendix "Implementation Details" as above).  Every
 * copied bf16 element x of KV head h, layer l becomes the E4M3 code nearest to
 * x / scale[l, h]: the quotient is one correctly rounded float32 division, values
 * beyond +-448 saturate, ties go to the even mantissa.
 *
 *   K_tree, V_tree      [n_layers][B, N, Hkv, dh] bf16, layers tree_layer_stride
 *                       elements apart
 *   K_cache8, V_cache8  [n_layers][total_prefix, Hkv, dh] uint8 in/out, layers
 *                       cache_layer_stride bytes apart
 *   k_scale, v_scale    [n_layers, Hkv] float32 (device), positive
 * Everything else as for eagle2_commit_kv.
 */
int eagle2_commit_kv_fp8(const eagle2_cfg* cfg, const eagle2_attn_cfg* attn, int32_t n_layers,
                         const int32_t* accept_len, const int32_t* accept_path,
                         const int64_t* kv_offsets, const int32_t* prefix_len,
                         const void* K_tree, const void* V_tree, int64_t tree_layer_stride,
                         void* K_cache8, void* V_cache8, int64_t cache_layer_stride,
                         const float* k_scale, const float* v_scale, void* stream);

/*
 * Commit of a round, part 2: tokens and bookkeeping (Section 2.1; Section 2.2,
 * "Drafting Stage": the next draft starts from the target's feature and the token
 * sequence advanced by one step).
 *
 *   out_tokens   [B, D+1] int32 output: the tokens this round adds to the text --
 *                the accept_len[b] accepted draft tokens, then bonus_token[b];
 *                -1 padded
 *   root_token   [B] int32 output: root of the next round's tree (= bonus_token)
 *   prefix_len   [B] int32 in/out: advanced by accept_len[b] + 1 (the root and the
 *                accepted tokens now have KV rows; the bonus token has none yet)
 *   target_hidden  nullable; [B, N, Hd] dtype: the verifying model's feature per
 *                tree row.  next_hidden [B, Hd] dtype output (given together with
 *                target_hidden): the feature at the last accepted row.
 * A sequence with accept_len[b] < 0 (acceptance reported a failure) emits nothing:
 * its out_tokens row is all -1 and root_token[b], prefix_len[b], next_hidden[b]
 * keep their values.
 */
int eagle2_commit_round(const eagle2_cfg* cfg, const int32_t* accept_len, const int32_t* accept_path,
                        const int32_t* tree_token, const int32_t* bonus_token, const void* target_hidden,
                        int32_t* out_tokens, int32_t* root_token, int32_t* prefix_len, void* next_hidden,
                        void* stream);

/*
 * Draft model forward between two expansion passes (Section 2.2, "Drafting Stage":
 * autoregression at the feature level with the token sequence advanced by one
 * step; Section 4.1: all nodes of the current layer pass through the draft model
 * at once under tree attention).  The paper does not print the draft network: this
 * is one LLaMA-style decoder layer -- RMSNorm, rotary grouped-query attention
 * (half-split pairing), SwiGLU MLP, residual connections -- behind a linear fusion
 * of [token embedding ; feature of the previous position].
 *
 * Pass d computes, for every sequence b and frontier slot s (F_d rows), the
 * feature of the node in frontier[b,d,s] (d = 0: the root) from the node's token
 * and the feature of its parent position (d = 0: root_feature, the verifying
 * model's feature at the last committed position, e.g. eagle2_commit_round's
 * next_hidden), attending to the sequence's draft KV prefix and to its own
 * ancestors among the draft rows.  Draft row of (d, s): 0 for the root, else
 * 1 + (d-1)k + s -- the row numbering of draft_logits.  The feature is written
 * to draft_feature[b, row, :]; eagle2_expand(d) can read it in place with
 * H = draft_feature + row_base*Hd and h_seq_stride = Rd*Hd.
 * Rd = max(R, 2) rows per sequence; Rd <= 128.
 *
 *   weights      [out, in] row-major, dtype of cfg: embed [V, Hd]; fc [Hd, 2Hd];
 *                wqkv [(Hq + 2Hkv)dh, Hd] (query rows, key rows, value rows);
 *                wo [Hd, Hq dh]; wgu [2I, Hd] (gate rows, up rows); wdown [Hd, I];
 *                g_attn, g_mlp [Hd] RMSNorm gains.  Every matrix row must be a
 *                multiple of 256 bytes and at least 1024 bytes long.
 *   cand_token, cand_parent, frontier   as left by the expand passes before d
 *   root_token [B] int32, root_feature [B, Hd] dtype, prefix_len [B] int32
 *   K_prefix, V_prefix [total_prefix, Hkv, dh] dtype, kv_offsets [B+1] int64: the
 *                draft model's own KV cache, regions filled to prefix_len[b]
 *   draft_feature [B, Rd, Hd] dtype in/out; K_draft, V_draft [B, Rd, Hkv, dh] dtype
 *                in/out; draft_mask [B, Rd, ceil(Rd/64)] uint64 in/out (ancestor
 *                bits over draft rows).  Pass 0 clears K_draft, V_draft and
 *                draft_mask; passes must run in order on one stream.
 *   workspace    at least eagle2_draft_workspace_bytes()
 * Position of a row: prefix_len[b] + d.  Activations between the matrix products
 * are rounded to dtype; the residual stream and all reductions are float32.
 */
typedef struct eagle2_draft_cfg {
    int32_t n_q_heads, n_kv_heads, head_dim;   /* head_dim 64 or 128                 */
    int32_t intermediate;                      /* I: width of the SwiGLU MLP          */
    float   eps;                               /* RMSNorm epsilon                     */
    float   rope_theta;                        /* rotary base                         */
} eagle2_draft_cfg;

typedef struct eagle2_draft_weights {          /* device pointers, see above          */
    const void *embed, *fc, *g_attn, *wqkv, *wo, *g_mlp, *wgu, *wdown;
} eagle2_draft_weights;

size_t eagle2_draft_workspace_bytes(const eagle2_cfg* cfg, const eagle2_draft_cfg* draft, int64_t total_prefix);

int eagle2_draft_forward(const eagle2_cfg* cfg, const eagle2_draft_cfg* draft, const eagle2_draft_weights* weights, int32_t d,
                         const int32_t* cand_token, const int32_t* cand_parent, const int32_t* frontier,
                         const int32_t* root_token, const void* root_feature, const int32_t* prefix_len,
                         const void* K_prefix, const void* V_prefix, const int64_t* kv_offsets, int64_t total_prefix,
                         void* draft_feature, void* K_draft, void* V_draft, uint64_t* draft_mask,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Kernel timing for benchmarks (not part of the method; the one place where the
 * library holds state: enabling creates a fixed pool of HIP events, 2048 timed
 * launches per slot between two reads, further launches go untimed).  While enabled, every
 * eagle2_expand records a HIP event pair around its LM-head streaming kernel and
 * every eagle2_tree_attn around its split-KV kernel, on the caller's stream.
 * eagle2_kernel_timing_read synchronises those events (host-blocking), returns
 * the summed milliseconds and launch counts since the last read, and resets.
 * which: 0 = LM-head kernel, 1 = tree-attention kernel.
 */
int eagle2_kernel_timing_enable(int32_t enable);
int eagle2_kernel_timing_read(int32_t which, double* total_ms, int32_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* EAGLE2_H */
