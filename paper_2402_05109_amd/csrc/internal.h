// Internal declarations shared by the translation units of libhydra.
// Nothing here is part of the C ABI (see include/hydra.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "hydra.h"

namespace hydra {

typedef uint16_t bf16_t;   // raw bfloat16 bits

// ---------------------------------------------------------------------------
// Device copy of the static candidate tree.
// ---------------------------------------------------------------------------
struct TreeDev {
    int32_t T, max_depth;
    int32_t n_expand[HYDRA_MAX_T];        // per phase i (index i): nodes of depth i-1 that have children
    int32_t expand_off[HYDRA_MAX_T + 1];  // start of phase i's list in expand_nodes
    int16_t expand_nodes[HYDRA_MAX_T];    // node ids, phase by phase, ascending
    int16_t expand_k[HYDRA_MAX_T];        // n_children and first_child of expand_nodes[i], so that one lookup serves a row
    int16_t expand_first[HYDRA_MAX_T];
    int16_t parent[HYDRA_MAX_T];
    int16_t depth[HYDRA_MAX_T];
    int16_t first_child[HYDRA_MAX_T];
    int16_t n_children[HYDRA_MAX_T];
    uint64_t anc[HYDRA_MAX_T][2];         // bit a of anc[n]: a is n or an ancestor of n
};

enum { TABLE_SLOTS = 16, TABLE_SLOT_BYTES = 8192, FLAGS_OFF_IN_SLOT = 8000 };    // a slot: the tree, then (at 8000) the flags word
static_assert(sizeof(TreeDev) <= FLAGS_OFF_IN_SLOT, "tree table slot too small");

// Offsets (bytes) of everything inside the weight arena.
struct LayerOff { size_t attn_norm, wqkv, wo, ffn_norm, wgu, wdown; };
struct HeadOff  { size_t w1, b1, wout; size_t wl[8], bl[8]; };   // wl[j], j = 2..mlp_layers

struct GemmPlan {      // launch shape of one weight-streaming GEMM (bf16 family)
    int mb;            // 32-row blocks per workgroup (1, 2 or 4)
    int nt;            // 32-column bands per wave (1 or 2)
    int nw, kw;        // waves per workgroup along N and along K
    int splits;        // workgroups along K (each writes its own partial output)
    int kpw;           // k-steps (of 16) per wave
    int shared_x;      // 0, or the number of waves (4 or 8) of the many-rows variant that shares X tiles through LDS
    float cost_us;     // the planner's estimate
};

}  // namespace hydra

struct hydra_ctx {
    hydra_model_desc m;
    hydra_heads_desc h;
    int max_batch;
    bool bf16;
    size_t esz;                         // bytes per weight / cache element
    hydra::TreeDev tree;                // host copy
    std::vector<float> rope;            // [max_pos][Dh/2][2] = cos, sin
    // arena
    size_t arena_bytes;
    size_t off_tables, off_rope, off_embed, off_final_norm, off_lm_head;
    std::vector<hydra::LayerOff> layer;
    std::vector<hydra::HeadOff> head;   // index 1..K
    char *arena;                        // device, caller-owned
    int table_slot;
    int n_cus;                          // compute units of the device (workgroups of the persistent layer kernel)
    // profiling
    bool profiling;
    std::vector<hipEvent_t> ev;
    size_t ev_used;
    double prof_bytes;
    int64_t prof_launches;
};

namespace hydra {

void set_error(const std::string &msg);
int  fail(int code, const std::string &msg);
int  hip_fail(hipError_t e, const char *what);

#define HYDRA_HIP(call)                                                     \
    do {                                                                    \
        hipError_t e__ = (call);                                            \
        if (e__ != hipSuccess) return hydra::hip_fail(e__, #call);          \
    } while (0)
#define HYDRA_LAUNCH_CHECK(name)                                            \
    do {                                                                    \
        hipError_t e__ = hipGetLastError();                                 \
        if (e__ != hipSuccess) return hydra::hip_fail(e__, name);           \
    } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int    ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---- workspace ------------------------------------------------------------
struct WsLayout {
    size_t flags, x, xa, xb, part, qbuf, apart, z, ss, topk, mega, total;
    int attn_units;     // split-KV units per (row, head, query group)
};
WsLayout ws_layout(const hydra_ctx *c, int B);
enum { GEMM_KIND_PLAIN = 0, GEMM_KIND_FUSED = 1, GEMM_KIND_PAIRS = 2, GEMM_KIND_SWIGLU = 3 };   // plain output (may split K) / fused epilogue / q|k|v band pairs / gate-up (fused, up to five bands per wave)
GemmPlan plan_gemm(const hydra_ctx *c, int M, int N, int K, int kind);
int      attn_units(const hydra_ctx *c, int B);

// ---- launchers (each enqueues on `s` and returns a hydra_status) -----------
// GEMM:  part[s][m][n] = sum over split s of X[m][k] W[n][k]   (fp32 out, row stride Npad)
//   f32 family: X fp32 row-major [M,K], W fp32 row-major [N,K], one split.
//   bf16 family: X and W in MFMA operand order (see gemm_bf16.hip).
int launch_gemm(hydra_ctx *c, hipStream_t s, const void *X, const void *W, float *part,
                int M, int N, int K, GemmPlan *plan_out);
int gemm_npad(const hydra_ctx *c, int N);   // row stride of `part` for N outputs
// bf16 family, fused epilogues (see bf16_gemm.hip)
int launch_gemm_resid(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K, float *x,
                      const float *gain, void *xg, float *ss, int Mpad, float *part, int *ss_bands);
int launch_gemm_silu(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int F, int K, const float *ss,
                     int nb, int Mpad, void *act);
int launch_gemm_bias_silu(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K,
                          const float *bias, float *z, bool residual, void *xg);
int gemm_max_dynamic_lds(hydra_ctx *c);
int attn_max_dynamic_lds(hydra_ctx *c);
// per-row 1/rms from the per-band sums of squares ss[band][Mpad] (bf16 family); ss == NULL: no scaling
struct RowScale { const float *ss; int nb; int Mpad; int d; float eps; };
int launch_gemm_qkv_rope(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, RowScale rs, int layer,
                         const int32_t *seq_len, const hydra_kv *kv, void *qbuf, float *part, int32_t *flags);
int launch_embed_prep(hydra_ctx *c, hipStream_t s, const int32_t *tokens, float *x, const float *gain, void *xg,
                      float *ss, int Mpad, int M, int32_t *flags);
int launch_final_hidden(hydra_ctx *c, hipStream_t s, const float *x, const float *gain, RowScale rs, float *hidden, int M);

// The decoder layers as one persistent kernel (bf16_layers.hip), for forward passes of up to 64 rows.
struct LayersMegaIO { float *x_first; void *xg_first; float *ss_first; float *x_last; void *xg_last; float *ss_last; int nb_last, Mpad; };
size_t layers_mega_ws_bytes(const hydra_ctx *c, int B);
bool layers_mega_eligible(const hydra_ctx *c, int B, const hydra_kv *kv);
int layers_mega_set_attr(hydra_ctx *c);
void layers_mega_info(const hydra_ctx *c, int B, int64_t *out);
int launch_layers_mega(hydra_ctx *c, hipStream_t s, int B, char *mega, const int32_t *seq_len, const hydra_kv *kv, int32_t *flags,
                       LayersMegaIO *io, bool launch);

// packing (arena loads)
int launch_pack_matrix(hydra_ctx *c, hipStream_t s, const void *src, void *dst, int N, int K,
                       int tile_off, int tile_stride, int rows_per_band, int col_off, int bands_per_head);
int launch_copy_matrix(hydra_ctx *c, hipStream_t s, const void *src, void *dst, size_t rows, size_t cols,
                       size_t dst_row_off, size_t dst_ld);
int launch_to_f32(hydra_ctx *c, hipStream_t s, const void *src, float *dst, int n);

// glue
int launch_gather_prep(hydra_ctx *c, hipStream_t s, int B, const float *hidden, int T_src, const int32_t *path,
                       const int32_t *n_acc, float *x, const float *gain, void *xg, float *ss, int Mpad, int32_t *flags);
int launch_prefix_select(hydra_ctx *c, hipStream_t s, int B, const float *x, const int32_t *n_acc, const hydra_kv *kv,
                         int32_t *seq_len, float *h_out);
struct VerifyArgs;
int launch_embed(hydra_ctx *c, hipStream_t s, const int32_t *tokens, float *x, int M, int32_t *flags);
int launch_rmsnorm(hydra_ctx *c, hipStream_t s, float *x, const float *part, int S, int part_ld, size_t part_split_stride,
                   const float *gain, void *x_out, int M, float *hidden_out);
int launch_rope_append(hydra_ctx *c, hipStream_t s, const float *part, int S, int part_ld, size_t split_stride,
                       RowScale rs, int B, int layer, const int32_t *seq_len, const hydra_kv *kv, void *qbuf,
                       int32_t *flags);
int launch_attention(hydra_ctx *c, hipStream_t s, int B, int layer, const void *qbuf, const int32_t *seq_len,
                     const hydra_kv *kv, float *apart, int units, void *x_out, float *plain_out, int32_t *flags);
int launch_silu_mul(hydra_ctx *c, hipStream_t s, const float *part, int S, int part_ld, size_t split_stride,
                    void *x_out, int M);
int launch_gemm_top2(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K, float *cand, int Mpad, int *fused);
int launch_argmax_bands(hydra_ctx *c, hipStream_t s, const float *cand, int bands, int Mpad, RowScale rs, int M, int32_t *argmax,
                        float *margin);
int launch_argmax(hydra_ctx *c, hipStream_t s, const float *part, int S, int part_ld, size_t split_stride,
                  RowScale rs, int M, int32_t *argmax, float *margin, float *logits);
int launch_q_import(hydra_ctx *c, hipStream_t s, int B, const float *q_plain, void *qbuf);
int launch_kv_plain(hydra_ctx *c, hipStream_t s, int B, int layer, const hydra_kv *kv, int first_slot, int n_slots,
                    float *plain, bool write_cache);
// draft
int launch_draft_root(hydra_ctx *c, hipStream_t s, int B, const int32_t *root, int32_t *tree_tokens);
int launch_draft_gather(hydra_ctx *c, hipStream_t s, int B, int phase, const float *h_last,
                        const int32_t *tree_tokens, void *x_out, float *z_out, int32_t *flags);
int launch_bias_silu(hydra_ctx *c, hipStream_t s, const float *part, int S, int part_ld, size_t split_stride,
                     const float *bias, float *z, bool residual, void *x_out, int M);
int launch_topk(hydra_ctx *c, hipStream_t s, const float *part, int S, int part_ld, size_t split_stride,
                int B, int phase, int32_t *tree_tokens, void *scratch);
size_t topk_scratch_bytes(const hydra_ctx *c, int rows);      // bytes of `scratch` for that many logits rows
// accept / compact
int launch_accept(hydra_ctx *c, hipStream_t s, int B, const int32_t *tree_tokens, const int32_t *argmax,
                  int32_t *n_acc, int32_t *path, int32_t *next_root, int32_t *last_node);
int launch_accept_typical(hydra_ctx *c, hipStream_t s, int B, const int32_t *tree_tokens, const float *logits, float tau,
                          float eps, float alpha, const float *u, int32_t *ok_scratch, int32_t *flags, int32_t *n_acc,
                          int32_t *path, int32_t *next_root, int32_t *last_node);
int typical_static_scratch(int32_t **out);       // the current device's copy of accept_typical_static's fixed buffer
int launch_compact(hydra_ctx *c, hipStream_t s, int B, const int32_t *n_acc, const int32_t *path,
                   const int32_t *next_root, const int32_t *last_node, const float *hidden, const hydra_kv *kv,
                   int32_t *seq_len, float *h_last, int32_t *root, int32_t *kv_index);

inline const TreeDev *tree_dev(const hydra_ctx *c) {
    return reinterpret_cast<const TreeDev *>(c->arena + c->off_tables + (size_t)c->table_slot * TABLE_SLOT_BYTES);
}
inline int32_t *flags_dev(const hydra_ctx *c) {
    return reinterpret_cast<int32_t *>(c->arena + c->off_tables + (size_t)c->table_slot * TABLE_SLOT_BYTES + FLAGS_OFF_IN_SLOT);
}
inline const float *rope_dev(const hydra_ctx *c) { return reinterpret_cast<const float *>(c->arena + c->off_rope); }

}  // namespace hydra
