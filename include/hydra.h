/*
 * hydra.h - C ABI of the MI355X (gfx950) hot path of Hydra decoding.
 *
 * One speculative step per batch row is four calls, in this order:
 *
 *   hydra_draft_tree     sequentially dependent draft heads fill a static
 *                        candidate tree                  (paper, section 3)
 *   tree_verify_forward  one base-model forward over the packed tree with an
 *                        ancestors-only attention mask   (section 2, "Tree decoding")
 *     tree_attention       the masked attention inside it, exported for tests
 *   accept_greedy        longest path whose candidates equal the base model's
 *                        most likely tokens              (section 2, greedy acceptance)
 *   kv_compact           keep the accepted tokens in the KV cache, drop the rest
 *                        (sections 1-2: accepted tokens are appended, the rest discarded)
 *
 * Notation.  B batch rows; d model width; H attention heads; Dh = d / H; F FFN
 * width; V vocabulary; NL layers; K draft heads (= the deepest candidate the
 * draft can reach); T tree nodes INCLUDING the root.  Node 0 is x_t, the base
 * model's own greedy token, which is always accepted, so every step emits
 * between 1 and (tree depth + 1) tokens.  Per row the carried state is the
 * paper's (x_<=t, h_{t-1}):  seq_len = number of tokens whose K/V are cached
 * (x_<=t-1),  h_last = final hidden state (after the last RMSNorm) of the last
 * cached token,  root = x_t.
 *
 * Conventions.
 *   - Every function returns 0 (HYDRA_OK) or a negative hydra_status;
 *     hydra_last_error() gives a thread-local message for the last failure.
 *   - "device" pointers are HIP device memory of the current device; "host"
 *     pointers are ordinary memory.  The library never frees or keeps ownership
 *     of caller memory; the only device memory it uses is what the caller
 *     passes (weight arena, workspace, KV pages, state, outputs).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls validate arguments on the host, enqueue kernels on `stream` and
 *     return without synchronising.  Two calls that share a workspace must be
 *     ordered on one stream.
 *   - Arguments are validated on the host; a bad argument returns an error and
 *     launches nothing.  Quantities only the device knows (seq_len) are checked
 *     again inside the kernels: a row whose seq_len + T exceeds its page table
 *     is skipped and flagged (see hydra_read_flags), never accessed out of
 *     bounds.
 *   - dtype HYDRA_F32: weights, KV cache and GEMM inputs are fp32.
 *     dtype HYDRA_BF16: weights are given as bfloat16; the KV cache holds 16-bit
 *     elements and GEMM inputs are rounded to 16 bits (the library keeps these
 *     as IEEE half, in which bfloat16 weights are exact); all sums are fp32.
 *     Supported range of that 16-bit interior: weights of magnitude >= 2^-17
 *     are exact, smaller ones lose low bits and below 2^-25 become zero (flag
 *     bit 5 at load time); GEMM inputs are the residual stream times the norm
 *     gain BEFORE the division by its rms (the division commutes with the
 *     contraction and is applied afterwards), so |x * gain| must stay within
 *     65504, as must q, k, v and the SwiGLU activations; a value beyond that is
 *     clamped and flag bit 4 is raised (hydra_read_flags), never silently.
 *     In both, h_last / hidden / logits / margin are fp32 and token ids,
 *     lengths and indices are int32.
 */
#ifndef HYDRA_H
#define HYDRA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HYDRA_OK = 0,
    HYDRA_E_INVALID_ARG = -1,   /* NULL pointer, negative size, bad enum            */
    HYDRA_E_SHAPE = -2,         /* inconsistent shapes (d != H*Dh, bad tree, ...)   */
    HYDRA_E_CAPACITY = -3,      /* page table / workspace / batch too small         */
    HYDRA_E_UNSUPPORTED = -4,   /* T > 128, Dh not in {64,128}, page size != 16 ... */
    HYDRA_E_HIP = -5,           /* a HIP runtime call failed                        */
    HYDRA_E_STATE = -6          /* weights not bound / tensor not loaded            */
} hydra_status;

enum { HYDRA_F32 = 0, HYDRA_BF16 = 1 };
enum { HYDRA_MAX_T = 128, HYDRA_MAX_DRAFT_HEADS = 8, HYDRA_MAX_TOPK = 32, HYDRA_PAGE = 16 };

typedef struct hydra_ctx hydra_ctx;

/* Base model: a LLaMA-family decoder (paper, section 5 "Models"): pre-norm
 * RMSNorm, rotary positions (pairs j, j + Dh/2; frequency rope_theta^(-2j/Dh)),
 * multi-head attention with scale 1/sqrt(Dh), SwiGLU FFN, untied embedding and
 * LM head, no biases. */
typedef struct {
    int32_t d, n_layers, n_heads, head_dim, ffn, vocab;
    int32_t dtype;              /* HYDRA_F32 or HYDRA_BF16                          */
    float   rms_eps, rope_theta;
    int32_t page_size;          /* tokens per KV page; must be HYDRA_PAGE           */
    int32_t max_pos;            /* positions 0..max_pos-1 are representable         */
} hydra_model_desc;

/* Draft heads (section 3).  Head i (1-based) maps
 *   u = [h_last ; E[x_t] ; E[x^_{t+1}] ; ... ; E[x^_{t+i-1}]]   (width (i+1) d)
 * through  z = SiLU(W1 u + b1),  z <- z + SiLU(Wj z + bj) for j = 2..mlp_layers
 * (Hydra++ "Scaling", section 3.1),  logits = Wout z.
 * include_root_embedding = 0 drops E[x_t] from u (width i d).
 * medusa = 1 gives the sequentially independent baseline heads of section 2
 * ("Lightweight heads as a draft model", "Medusa decoding"): u = h_last only
 * (W1 is [d, d]) and the first layer is residual, z = h_last + SiLU(W1 h_last + b1);
 * the candidate path is ignored, so all nodes of one depth receive prefixes of
 * the same ranked list. */
typedef struct {
    int32_t n_draft_heads;      /* K, 0..HYDRA_MAX_DRAFT_HEADS (0: no draft call)   */
    int32_t mlp_layers;         /* >= 1                                             */
    int32_t include_root_embedding;
    int32_t medusa;             /* 0 = Hydra heads, 1 = Medusa-style heads          */
} hydra_heads_desc;

/* Static candidate tree (section 2): host array parent[T], parent[0] = -1,
 * nodes in breadth-first order (depth never decreases with the node index and
 * the children of a node are contiguous, ordered by rank: the first child gets
 * the draft's most likely token).  Copied at hydra_create. */
typedef struct {
    int32_t        T;           /* 1..HYDRA_MAX_T                                   */
    const int32_t *parent;      /* host [T]                                         */
} hydra_tree_desc;

/* Paged KV cache, owned by the caller.  k_pages and v_pages each hold
 * n_layers * n_pages * H * 16 * Dh elements (4 bytes each for HYDRA_F32, 2 bytes
 * each for HYDRA_BF16); page p of layer
 * l, head h starts at element ((l * n_pages + p) * H + h) * 16 * Dh.  The
 * placement of (token, dim) inside a 16 x Dh block is private to the library
 * (it differs between K and V and between dtypes); callers move tokens only
 * through kv_compact.  Row b's logical slot s lives in physical page
 * page_table[b * max_pages + s / 16]. */
typedef struct {
    void          *k_pages, *v_pages;   /* device                                   */
    const int32_t *page_table;          /* device [B, max_pages]                    */
    int32_t        n_pages;             /* physical pages per layer                 */
    int32_t        max_pages;           /* page-table row length                    */
    int32_t        seq_len_hint;        /* host upper bound on max_b seq_len, or 0 = unknown.
                                           Sizes launch grids only; results never depend on it.
                                           If > 0 and seq_len_hint + T > 16 * max_pages the call
                                           returns HYDRA_E_CAPACITY.                            */
} hydra_kv;

typedef enum {
    HYDRA_W_EMBED = 0,      /* [V, d]                                  index, sub ignored      */
    HYDRA_W_LM_HEAD,        /* [V, d]                                                          */
    HYDRA_W_FINAL_NORM,     /* [d]                                                             */
    HYDRA_W_ATTN_NORM,      /* [d]             index = layer                                   */
    HYDRA_W_WQ, HYDRA_W_WK, HYDRA_W_WV, HYDRA_W_WO,   /* [d, d]    index = layer               */
    HYDRA_W_FFN_NORM,       /* [d]                                                             */
    HYDRA_W_GATE, HYDRA_W_UP,   /* [F, d]                                                      */
    HYDRA_W_DOWN,           /* [d, F]                                                          */
    HYDRA_W_HEAD_W1,        /* [d, (i+1) d]    index = head i (1-based)                        */
    HYDRA_W_HEAD_B1,        /* [d]                                                             */
    HYDRA_W_HEAD_WL,        /* [d, d]          index = head, sub = MLP layer j in 2..mlp_layers */
    HYDRA_W_HEAD_BL,        /* [d]                                                             */
    HYDRA_W_HEAD_WOUT,      /* [V, d]          index = head                                    */
    HYDRA_W_KIND_COUNT
} hydra_tensor_kind;

/* ---- life cycle ---------------------------------------------------------- */

/* Validates the descriptors and builds the host-side context (tree tables,
 * rotary table, launch plans).  Allocates no device memory.  max_batch bounds B
 * in every later call.  Errors: INVALID_ARG, SHAPE, UNSUPPORTED. */
int hydra_create(const hydra_model_desc *model, const hydra_heads_desc *heads,
                 const hydra_tree_desc *tree, int max_batch, hydra_ctx **out);
int hydra_destroy(hydra_ctx *ctx);
const char *hydra_last_error(void);

/* Bytes of the weight arena (all weights in the library's internal layout plus
 * the tree and rotary tables).  Depends only on the model and heads
 * descriptors, so contexts that differ in their tree can share one arena. */
size_t hydra_weights_bytes(const hydra_ctx *ctx);

/* Attaches a caller-owned device arena of hydra_weights_bytes() bytes, 256-byte
 * aligned, and uploads this context's tables (tree, rotary angles) into it;
 * synchronises the stream.  Contexts with the same model and heads descriptors
 * may share one arena (for example a chain-tree context for prefill next to the
 * decoding context): each takes its own table_slot in [0, 16). */
int hydra_bind_weights(hydra_ctx *ctx, void *stream, void *arena, int table_slot);

/* Converts one plain row-major tensor (device, model dtype, [out, in]) into the
 * arena's internal layout.  `src` can be freed once the stream has passed the
 * call.  Errors: INVALID_ARG (kind / index / sub out of range), STATE. */
int hydra_load_tensor(hydra_ctx *ctx, void *stream, int kind, int index, int sub,
                      const void *src);

/* Workspace bytes needed by any call with batch B (256-byte aligned device
 * memory, contents irrelevant between calls). */
size_t hydra_workspace_bytes(const hydra_ctx *ctx, int B);

/* Device-side flags raised by kernels of this context since the last call of
 * this function (or since hydra_bind_weights): bit 0 = a row's seq_len + T
 * exceeded its page table or max_pos (row skipped), bit 1 = a token id outside
 * [0, V) (treated as 0), bit 2 = hydra_prefix_attention met an n_acc outside
 * [1, P] or a path entry outside [0, T_src) (clamped), or kv_compact met a path
 * that is not strictly increasing inside [0, T) (the copies stop there),
 * bit 3 = a bounded wait
 * inside the persistent layer kernel expired (see hydra_layer_kernel_info; the
 * outputs of that call are undefined), bit 4 = a value that feeds a GEMM or the
 * cache of the bf16 family exceeded the largest finite half (65504) and was
 * clamped, bit 5 = hydra_load_tensor met a non-zero bfloat16 weight too small
 * for the 16-bit interior (|w| < 2^-25: stored as zero), bit 6 = a page-table
 * entry outside [0, n_pages) (the row's K/V are not written, reads use page 0,
 * copies are skipped).  Reads and clears them; synchronises the stream. */
int hydra_read_flags(hydra_ctx *ctx, void *stream, int32_t *flags_out /* host */);

/* ---- the hot path -------------------------------------------------------- */

/* Section 3 and section 2 ("Tree decoding").  tree_tokens[b,0] = root[b]; for
 * i = 1..depth, every node n of depth i-1 with c > 0 children gets them from
 * head i evaluated on n's root path: the c largest logits, ordered by (logit
 * descending, token id ascending).  Phase i starts after phase i-1's tokens
 * exist.  Requires tree depth <= n_draft_heads (else UNSUPPORTED) and at most
 * HYDRA_MAX_TOPK children per node.
 *   h_last      device [B, d] fp32          root  device [B] int32
 *   tree_tokens device [B, T] int32 (out)                                      */
int hydra_draft_tree(hydra_ctx *ctx, void *stream, int B, void *ws,
                     const float *h_last, const int32_t *root, int32_t *tree_tokens);

/* Section 2 ("Tree decoding"): node n of row b sits at position
 * seq_len[b] + depth[n] and attends to cache slots [0, seq_len[b]) plus its
 * ancestors and itself; its K/V are written to slot seq_len[b] + n.
 *   tree_tokens device [B, T] int32        seq_len device [B] int32
 *   hidden  device [B, T, d] fp32 (out, after the final RMSNorm)
 *   argmax  device [B, T] int32 (out, lowest id among maxima)
 *   margin  device [B, T] fp32 (out, top-1 minus top-2 logit) or NULL
 *   logits  device [B, T, V] fp32 (out) or NULL
 * The caller guarantees page-table capacity for seq_len[b] + T slots. */
int tree_verify_forward(hydra_ctx *ctx, void *stream, int B, void *ws,
                        const int32_t *tree_tokens, const int32_t *seq_len, const hydra_kv *kv,
                        float *hidden, int32_t *argmax, float *margin, float *logits);

/* Section 2 ("Tree decoding": every node attends to the verified prefix, its
 * ancestors and itself).  The attention of one layer of tree_verify_forward on its own:
 *   q   device [B, T, H, Dh] fp32, already rotated
 *   out device [B, T, H, Dh] fp32
 * K/V of the T nodes must already be in slots seq_len[b] .. seq_len[b]+T-1
 * (see hydra_kv_write). */
int tree_attention(hydra_ctx *ctx, void *stream, int B, int layer, void *ws,
                   const float *q, const int32_t *seq_len, const hydra_kv *kv, float *out);

/* Section 2, greedy acceptance.  Per row: cur = 0; while a child c of cur has
 * tree_tokens[c] == argmax[cur] (lowest c if several): cur = c.
 *   n_acc     device [B] int32 (out) = depth[cur] + 1
 *   path      device [B, Dmax+1] int32 (out) root..cur, padded with -1;
 *             Dmax = hydra_tree_depth(ctx)
 *   next_root device [B] int32 (out) = argmax[cur]
 *   last_node device [B] int32 (out) = cur                                      */
int accept_greedy(hydra_ctx *ctx, void *stream, int B,
                  const int32_t *tree_tokens, const int32_t *argmax,
                  int32_t *n_acc, int32_t *path, int32_t *next_root, int32_t *last_node);

/* Section 6.3, typical acceptance: the token of child c of node n passes if
 *   p(tree_tokens[c]) > min(eps, alpha * exp(-H(p))),  p = softmax(logits[n] / tau),
 * H the entropy in nats.  The accepted path ends at the deepest node all of
 * whose path tokens pass (lowest node id among equally deep ones); the root
 * always counts.  next_root = the most likely token at that node (u == NULL,
 * lowest id at ties) or, with u[b] in [0, 1), the token at which the cumulative
 * distribution of softmax(logits[last] / tau), taken in token-id order, first
 * exceeds u[b].  The per-token test is the paper's; path selection and the
 * draw of the next root are this library's reading (the paper states neither).
 *   logits device [B, T, V] fp32: tree_verify_forward's optional output
 *   u      device [B] fp32 or NULL           other outputs as in accept_greedy.
 * Probabilities are computed in fp32.  Requires tau > 0, eps >= 0, alpha >= 0. */
int accept_typical(hydra_ctx *ctx, void *stream, int B, void *ws,
                   const int32_t *tree_tokens, const float *logits,
                   float tau, float eps, float alpha, const float *u,
                   int32_t *n_acc, int32_t *path, int32_t *next_root, int32_t *last_node);

/* accept_typical for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments (without ws), same results.
 * The per-candidate pass flags live in a fixed buffer of 64 KiB inside the library (one per GPU, kept until the
 * process ends; its address is looked up at hydra_bind_weights), which limits a call to B * T <= 16384 tree
 * nodes: beyond that the call returns HYDRA_E_CAPACITY and does nothing.  The call itself allocates nothing.
 * All calls on one GPU share that buffer: calls that overlap in time on one GPU (different streams or threads)
 * race and must be serialised by the caller.  The buffer keeps the last call's contents; every entry a call
 * reads is written by that call first. */
int accept_typical_static(hydra_ctx *ctx, void *stream, int B,
                          const int32_t *tree_tokens, const float *logits, float tau, float eps, float alpha,
                          const float *u, int32_t *n_acc, int32_t *path, int32_t *next_root, int32_t *last_node);

/* Sections 1 and 2 (speculative decoding: the accepted tokens are appended to the
 * sequence, the rest of the candidates is discarded; section 3: the next step's
 * heads read the hidden state of the last accepted token).
 * Keeps the accepted tokens.  Per row, every layer, j = 0..n_acc-1: K/V slot
 * seq_len + path[j] -> slot seq_len + j (in place; sources are read before any
 * destination is written).  Then h_last[b] = hidden[b, last_node[b]],
 * root[b] = next_root[b], seq_len[b] += n_acc[b].  A row that tree_verify_forward
 * skipped for lack of page-table capacity keeps its seq_len, h_last and root (its
 * kv_index is -1).  path must be strictly increasing with path[j] >= j (what
 * accept_greedy and accept_typical produce); otherwise the copies stop at the
 * offending entry and flag bit 2 is raised.
 *   kv_index device [B, Dmax+1, 2] int32 (out) or NULL: (physical page, offset
 *   in page) written for each j, -1 padded.                                     */
int kv_compact(hydra_ctx *ctx, void *stream, int B,
               const int32_t *n_acc, const int32_t *path, const int32_t *next_root,
               const int32_t *last_node, const float *hidden, const hydra_kv *kv,
               int32_t *seq_len, float *h_last, int32_t *root, int32_t *kv_index);

/* Section 3.1 item 3 and the appendix paragraph "Hydra-specific prefix
 * attention" (Hydra++): an extra decoder layer over the verified sequence,
 * queried once per decoding step, whose output at the last verified token the
 * draft heads read in place of the base model's hidden state.
 * `ctx` is a context of its own whose decoder layers are the prefix layer(s)
 * (n_layers = 1 in the paper; its embedding, LM head and draft heads are never
 * read), created with a chain tree of P nodes, with its own weight arena, KV
 * cache and seq_len.  Per row b, with a = n_acc[b] in [1, P]: position
 * seq_len[b] + j (j < a) is fed hidden[b, path[b, j]], the base model's hidden
 * state after its final RMSNorm; its K/V go to slot seq_len[b] + j of `kv`.
 * Then h_out[b] = the residual stream after the layer at position
 * seq_len[b] + a - 1 (no further norm) and seq_len[b] += a.  Rows j >= a are
 * computed on a copy of row a-1 and land in slots past the new length.
 *   hidden  device [B, T_src, d] fp32 (tree_verify_forward's output)
 *   path    device [B, P] int32       n_acc device [B] int32
 *   seq_len device [B] int32 (in/out) h_out device [B, d] fp32 (out)
 * After accept_greedy of a tree of depth Dmax use P = Dmax + 1 and its path;
 * for a prefill chunk of n tokens use P = n, path = 0..n-1, n_acc = n.
 * Readings of the paper taken here: input after the final norm, output before
 * any norm, rotary positions equal to the base model's. */
int hydra_prefix_attention(hydra_ctx *ctx, void *stream, int B, void *ws,
                           const float *hidden, int T_src, const int32_t *path, const int32_t *n_acc,
                           int32_t *seq_len, const hydra_kv *kv, float *h_out);

/* ---- helpers for tests and harnesses -------------------------------------- */

int hydra_tree_depth(const hydra_ctx *ctx);

/* Writes / reads whole tokens of one layer of the cache in plain layout, so a
 * harness can fill or inspect it without knowing the in-page placement.
 *   kv_plain device [B, n_slots, 2, H, Dh] fp32 (K then V per slot), slots
 *   first_slot .. first_slot + n_slots - 1 of every row. */
int hydra_kv_write(hydra_ctx *ctx, void *stream, int B, int layer, const hydra_kv *kv,
                   int first_slot, int n_slots, const float *kv_plain);
int hydra_kv_read(hydra_ctx *ctx, void *stream, int B, int layer, const hydra_kv *kv,
                  int first_slot, int n_slots, float *kv_plain);

/* The persistent layer kernel (bf16 family): a tree_verify_forward of at most 64 rows whose kv->seq_len_hint is
 * positive and at most 1280 - T can run all its decoder layers as one kernel with one workgroup per compute unit
 * (section 2, "Tree decoding": the verification forward; the split into kernels is this library's).  Its grid-wide
 * hand-offs wait with a bound: if not all workgroups become resident (another kernel holds compute units for
 * seconds) the call ends with flag bit 3 set (hydra_read_flags) and undefined outputs, never with a hang.
 *   info[0] = 1 if B rows can take that kernel, info[1] = byte offset inside the workspace of its timeline stamps
 *   ([n_layers][info[3]][info[2]][8] int64 ticks of the 100 MHz wall clock: step begins, work done, arrived, released,
 *   then inside GEMM steps first activations loaded, last MFMA issued, epilogue stores issued;
 *   written only while the environment variable HYDRA_LAYER_KERNEL_STAMPS is 1), info[2] = workgroups, info[3] =
 *   steps per layer.  The kernel is used only while the environment variable
 *   HYDRA_LAYER_KERNEL is 1 (measured, it does not yet beat the multi-kernel path at the 7B shape). */
int hydra_layer_kernel_info(const hydra_ctx *ctx, int B, int64_t *info /* host [4] */);

/* Per-kernel-family timing with HIP events on `stream` (for benchmarks).
 * hydra_profile_begin switches it on and zeroes the counters; every launch of
 * the weight-streaming GEMM kernel then carries an event pair that takes the
 * kernel's own begin and end times on its stream.
 * hydra_profile_end synchronises and returns launches, summed milliseconds and
 * summed weight bytes streamed by those launches. */
int hydra_profile_begin(hydra_ctx *ctx);
int hydra_profile_end(hydra_ctx *ctx, int64_t *launches, double *ms, double *weight_bytes);

#ifdef __cplusplus
}
#endif
#endif /* HYDRA_H */
