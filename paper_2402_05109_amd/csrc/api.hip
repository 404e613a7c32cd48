// Host side of libhydra: argument validation, arena and workspace layout, and
// the launch sequences of the four hot-path calls (see include/hydra.h).
#include <math.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "internal.h"

namespace hydra {

static thread_local std::string g_err;
void set_error(const std::string &msg) { g_err = msg; }
int fail(int code, const std::string &msg) { g_err = msg; return code; }
int hip_fail(hipError_t e, const char *what) {
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    return HYDRA_E_HIP;
}


static size_t matrix_bytes(const hydra_ctx *c, size_t N, size_t K) {
    const size_t rows = c->bf16 ? (N + 31) / 32 * 32 : N;
    return align_up(rows * K * c->esz, 256);
}
static size_t vec_bytes(size_t n) { return align_up(n * 4, 256); }

static int head_in_width(const hydra_ctx *c, int i) {
    if (c->h.medusa) return c->m.d;                       // Medusa-style heads read h_last only
    return (c->h.include_root_embedding ? i + 1 : i) * c->m.d;
}

static void layout_arena(hydra_ctx *c) {
    const size_t d = c->m.d, F = c->m.ffn, V = c->m.vocab;
    size_t off = 0;
    c->off_tables = off;      off += (size_t)TABLE_SLOTS * TABLE_SLOT_BYTES;
    c->off_rope = off;        off += align_up((size_t)c->m.max_pos * (c->m.head_dim / 2) * 2 * 4, 256);
    c->off_embed = off;       off += align_up(V * d * c->esz, 256);
    c->off_final_norm = off;  off += vec_bytes(d);
    c->off_lm_head = off;     off += matrix_bytes(c, V, d);
    c->layer.resize(c->m.n_layers);
    for (auto &l : c->layer) {
        l.attn_norm = off; off += vec_bytes(d);
        l.wqkv = off;      off += matrix_bytes(c, 3 * d, d);
        l.wo = off;        off += matrix_bytes(c, d, d);
        l.ffn_norm = off;  off += vec_bytes(d);
        l.wgu = off;       off += matrix_bytes(c, 2 * F, d);
        l.wdown = off;     off += matrix_bytes(c, d, F);
    }
    c->head.resize(c->h.n_draft_heads + 1);
    for (int i = 1; i <= c->h.n_draft_heads; ++i) {
        auto &h = c->head[i];
        h.w1 = off; off += matrix_bytes(c, d, head_in_width(c, i));
        h.b1 = off; off += vec_bytes(d);
        for (int j = 2; j <= c->h.mlp_layers; ++j) {
            h.wl[j - 2] = off; off += matrix_bytes(c, d, d);
            h.bl[j - 2] = off; off += vec_bytes(d);
        }
        h.wout = off; off += matrix_bytes(c, V, d);
    }
    c->arena_bytes = off;
}

static int build_tree(const hydra_tree_desc *t, TreeDev *out, std::string *why) {
    const int T = t->T;
    memset(out, 0, sizeof(*out));
    out->T = T;
    if (t->parent[0] != -1) { *why = "tree: parent[0] must be -1"; return HYDRA_E_SHAPE; }
    for (int n = 0; n < T; ++n) { out->first_child[n] = -1; out->n_children[n] = 0; }
    out->parent[0] = -1;
    out->depth[0] = 0;
    out->anc[0][0] = 1ull;
    for (int n = 1; n < T; ++n) {
        const int p = t->parent[n];
        if (p < 0 || p >= n) { *why = "tree: parent[n] must lie in [0, n)"; return HYDRA_E_SHAPE; }
        if (p < t->parent[n - 1]) { *why = "tree: nodes must be in breadth-first order (children contiguous)"; return HYDRA_E_SHAPE; }
        out->parent[n] = (int16_t)p;
        out->depth[n] = (int16_t)(out->depth[p] + 1);
        if (out->depth[n] < out->depth[n - 1]) { *why = "tree: depth must not decrease with the node index"; return HYDRA_E_SHAPE; }
        if (out->n_children[p] == 0) out->first_child[p] = (int16_t)n;
        else if (out->first_child[p] + out->n_children[p] != n) { *why = "tree: children of a node must be contiguous"; return HYDRA_E_SHAPE; }
        out->n_children[p]++;
        out->anc[n][0] = out->anc[p][0];
        out->anc[n][1] = out->anc[p][1];
        out->anc[n][n >> 6] |= 1ull << (n & 63);
        out->max_depth = std::max<int>(out->max_depth, out->depth[n]);
    }
    int off = 0;
    for (int i = 1; i <= out->max_depth; ++i) {
        out->expand_off[i] = off;
        int cnt = 0;
        for (int n = 0; n < T; ++n)
            if (out->depth[n] == i - 1 && out->n_children[n] > 0) {
                out->expand_k[off] = out->n_children[n];
                out->expand_first[off] = out->first_child[n];
                out->expand_nodes[off++] = (int16_t)n;
                ++cnt;
            }
        out->n_expand[i] = cnt;
    }
    return HYDRA_OK;
}

static int draft_rows_max(const hydra_ctx *c, int B) {
    int mx = 1;
    for (int i = 1; i <= c->tree.max_depth; ++i) mx = std::max(mx, c->tree.n_expand[i]);
    return mx * B;
}

WsLayout ws_layout(const hydra_ctx *c, int B) {
    WsLayout w;
    const size_t d = c->m.d, F = c->m.ffn, V = c->m.vocab, T = c->tree.T;
    const size_t M = (size_t)B * T;
    const size_t Md = draft_rows_max(c, B);
    const size_t rows = align_up(std::max(M, Md), 128);
    const size_t kin_max = (size_t)(c->h.n_draft_heads + 1) * d;
    const size_t cols = std::max(std::max(d, F), kin_max);
    size_t off = 0;
    w.flags = off; off += 256;
    w.x = off;     off += align_up(M * d * 4, 256);
    w.xa = off;    off += align_up(rows * cols * 4, 256);
    w.xb = off;    off += align_up(rows * cols * 4, 256);
    // split-K partial sums: the largest S * Mpad * Npad over every GEMM this context can launch
    size_t part = 0;
    auto need = [&](size_t m, size_t n, size_t k) {
        GemmPlan p = plan_gemm(c, (int)m, (int)n, (int)k, GEMM_KIND_PLAIN);
        const size_t mp = align_up(m, 32), np = (size_t)gemm_npad(c, (int)n);
        part = std::max(part, (size_t)p.splits * mp * np * 4);
    };
    need(M, 3 * d, d); need(M, d, d); need(M, 2 * F, d); need(M, d, F); need(M, V, d);
    for (int i = 1; i <= c->tree.max_depth && i <= c->h.n_draft_heads; ++i) {
        const size_t mi = (size_t)B * c->tree.n_expand[i];
        if (mi == 0) continue;
        need(mi, d, head_in_width(c, i)); need(mi, d, d); need(mi, V, d);
    }
    w.part = off;  off += align_up(part, 256);
    const size_t Tq = align_up(T, 32);
    w.qbuf = off;  off += align_up((size_t)B * c->m.n_heads * Tq * c->m.head_dim * 4, 256);
    w.attn_units = attn_units(c, B);
    const size_t rec = Tq * c->m.head_dim + 2 * Tq;
    w.apart = off; off += c->bf16 ? align_up((size_t)B * c->m.n_heads * w.attn_units * rec * 4, 256) : 256;
    w.z = off;     off += align_up(std::max<size_t>(Md, 1) * d * 4, 256);
    w.ss = off;    off += align_up((d / 32 + 1) * rows * 4, 256);
    w.topk = off;  off += align_up(topk_scratch_bytes(c, (int)std::max<size_t>(Md, 1)), 256);
    w.mega = off;  off += align_up(layers_mega_ws_bytes(c, B), 256);     // per-layer buffers of the persistent layer kernel (0 if the shape cannot take it)
    w.total = off;
    return w;
}

static int check_common(hydra_ctx *c, int B, const void *ws) {
    if (!c) return fail(HYDRA_E_INVALID_ARG, "ctx is NULL");
    if (B < 1 || B > c->max_batch) return fail(HYDRA_E_CAPACITY, "B outside [1, max_batch]");
    if (!ws) return fail(HYDRA_E_INVALID_ARG, "workspace is NULL");
    if (((uintptr_t)ws) & 255) return fail(HYDRA_E_INVALID_ARG, "workspace must be 256-byte aligned");
    if (!c->arena) return fail(HYDRA_E_STATE, "no weight arena bound (hydra_bind_weights)");
    return HYDRA_OK;
}

static int check_kv(hydra_ctx *c, const hydra_kv *kv) {
    if (!kv || !kv->k_pages || !kv->v_pages || !kv->page_table) return fail(HYDRA_E_INVALID_ARG, "kv or one of its pointers is NULL");
    if (kv->n_pages < 1 || kv->max_pages < 1) return fail(HYDRA_E_INVALID_ARG, "kv: n_pages and max_pages must be positive");
    if (kv->seq_len_hint < 0) return fail(HYDRA_E_INVALID_ARG, "kv: seq_len_hint is negative");
    if (kv->seq_len_hint > 0 && kv->seq_len_hint + c->tree.T > kv->max_pages * HYDRA_PAGE)
        return fail(HYDRA_E_CAPACITY, "kv: page table shorter than seq_len_hint + T slots");
    if (kv->seq_len_hint > 0 && kv->seq_len_hint + c->tree.max_depth >= c->m.max_pos)
        return fail(HYDRA_E_CAPACITY, "kv: seq_len_hint + tree depth reaches max_pos");
    return HYDRA_OK;
}

static inline int32_t *flags_ptr(hydra_ctx *c) {
    return reinterpret_cast<int32_t *>(c->arena + c->off_tables + (size_t)c->table_slot * TABLE_SLOT_BYTES + FLAGS_OFF_IN_SLOT);
}

}  // namespace hydra

using namespace hydra;

extern "C" {

const char *hydra_last_error(void) { return g_err.c_str(); }

int hydra_create(const hydra_model_desc *m, const hydra_heads_desc *h, const hydra_tree_desc *t, int max_batch,
                 hydra_ctx **out) {
    if (!m || !h || !t || !out) return fail(HYDRA_E_INVALID_ARG, "hydra_create: NULL argument");
    *out = nullptr;
    if (!t->parent) return fail(HYDRA_E_INVALID_ARG, "tree: parent is NULL");
    if (m->d < 1 || m->n_layers < 1 || m->n_heads < 1 || m->head_dim < 1 || m->ffn < 1 || m->vocab < 2 || m->max_pos < 1)
        return fail(HYDRA_E_INVALID_ARG, "model: non-positive dimension");
    if (m->dtype != HYDRA_F32 && m->dtype != HYDRA_BF16) return fail(HYDRA_E_INVALID_ARG, "model: unknown dtype");
    if (max_batch < 1) return fail(HYDRA_E_INVALID_ARG, "max_batch must be positive");
    if (m->d != m->n_heads * m->head_dim) return fail(HYDRA_E_SHAPE, "model: d != n_heads * head_dim");
    if (m->head_dim != 64 && m->head_dim != 128) return fail(HYDRA_E_UNSUPPORTED, "model: head_dim must be 64 or 128");
    if (m->page_size != HYDRA_PAGE) return fail(HYDRA_E_UNSUPPORTED, "model: page_size must be 16");
    if (!(m->rms_eps >= 0.f) || !(m->rope_theta > 0.f)) return fail(HYDRA_E_INVALID_ARG, "model: bad rms_eps or rope_theta");
    if (m->d > 8192) return fail(HYDRA_E_UNSUPPORTED, "model: d > 8192");
    if (m->dtype == HYDRA_BF16 && (m->d % 128 != 0 || m->ffn % 128 != 0))
        return fail(HYDRA_E_UNSUPPORTED, "bf16 family: d and ffn must be multiples of 128");
    if (t->T < 1 || t->T > HYDRA_MAX_T) return fail(HYDRA_E_UNSUPPORTED, "tree: T outside [1, 128]");
    if (h->n_draft_heads < 0 || h->n_draft_heads > HYDRA_MAX_DRAFT_HEADS) return fail(HYDRA_E_UNSUPPORTED, "heads: n_draft_heads outside [0, 8]");
    if (h->mlp_layers < 1 || h->mlp_layers > 9) return fail(HYDRA_E_UNSUPPORTED, "heads: mlp_layers outside [1, 9]");
    if (h->medusa != 0 && h->medusa != 1) return fail(HYDRA_E_INVALID_ARG, "heads: medusa must be 0 or 1");
    if ((int64_t)m->max_pos * (m->head_dim / 2) * 8 > (int64_t)1 << 31) return fail(HYDRA_E_UNSUPPORTED, "model: max_pos too large");

    hydra_ctx *c = new (std::nothrow) hydra_ctx();
    if (!c) return fail(HYDRA_E_INVALID_ARG, "out of host memory");
    c->m = *m; c->h = *h; c->max_batch = max_batch;
    c->bf16 = m->dtype == HYDRA_BF16;
    c->esz = c->bf16 ? 2 : 4;
    c->arena = nullptr; c->table_slot = 0;
    {   // compute units of the current device; without a device (host-only checks) the MI355X figure
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        (void)hipGetLastError();
        c->n_cus = cus;
    }
    c->profiling = false; c->ev_used = 0; c->prof_bytes = 0; c->prof_launches = 0;
    std::string why;
    int rc = build_tree(t, &c->tree, &why);
    if (rc != HYDRA_OK) { delete c; return fail(rc, why); }
    for (int n = 0; n < t->T; ++n)
        if (c->tree.n_children[n] > HYDRA_MAX_TOPK) { delete c; return fail(HYDRA_E_UNSUPPORTED, "tree: more than 32 children under one node"); }
    // rotary table in double: angle = pos * theta^(-2j/Dh)   (LLaMA pairing j <-> j + Dh/2)
    const int half = m->head_dim / 2;
    c->rope.resize((size_t)m->max_pos * half * 2);
    for (int j = 0; j < half; ++j) {
        const double inv = pow((double)m->rope_theta, -2.0 * j / m->head_dim);
        for (int p = 0; p < m->max_pos; ++p) {
            const double a = (double)p * inv;
            c->rope[((size_t)p * half + j) * 2] = (float)cos(a);
            c->rope[((size_t)p * half + j) * 2 + 1] = (float)sin(a);
        }
    }
    layout_arena(c);
    *out = c;
    return HYDRA_OK;
}

int hydra_destroy(hydra_ctx *c) {
    if (!c) return fail(HYDRA_E_INVALID_ARG, "ctx is NULL");
    for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
    delete c;
    return HYDRA_OK;
}

size_t hydra_weights_bytes(const hydra_ctx *c) { return c ? c->arena_bytes : 0; }
int hydra_tree_depth(const hydra_ctx *c) { return c ? c->tree.max_depth : -1; }
size_t hydra_workspace_bytes(const hydra_ctx *c, int B) {
    if (!c || B < 1 || B > c->max_batch) return 0;
    return ws_layout(c, B).total;
}

int hydra_bind_weights(hydra_ctx *c, void *stream, void *arena, int table_slot) {
    if (!c || !arena) return fail(HYDRA_E_INVALID_ARG, "hydra_bind_weights: NULL argument");
    if (((uintptr_t)arena) & 255) return fail(HYDRA_E_INVALID_ARG, "arena must be 256-byte aligned");
    if (table_slot < 0 || table_slot >= TABLE_SLOTS) return fail(HYDRA_E_INVALID_ARG, "table_slot outside [0, 16)");
    hipStream_t s = (hipStream_t)stream;
    c->arena = (char *)arena;
    c->table_slot = table_slot;
    char *slot = c->arena + c->off_tables + (size_t)table_slot * TABLE_SLOT_BYTES;
    HYDRA_HIP(hipMemsetAsync(slot, 0, TABLE_SLOT_BYTES, s));
    HYDRA_HIP(hipMemcpyAsync(slot, &c->tree, sizeof(TreeDev), hipMemcpyHostToDevice, s));
    HYDRA_HIP(hipMemcpyAsync(c->arena + c->off_rope, c->rope.data(), c->rope.size() * 4, hipMemcpyHostToDevice, s));
    HYDRA_HIP(hipStreamSynchronize(s));     // host buffers may change after return
    {   // set-up of accept_typical_static: the current device's address of its fixed buffer
        int32_t *unused = nullptr;
        int rc = typical_static_scratch(&unused);
        if (rc) return rc;
    }
    if (c->bf16) {
        int rc = gemm_max_dynamic_lds(c);
        if (rc) return rc;
        if ((rc = attn_max_dynamic_lds(c))) return rc;
        if ((rc = layers_mega_set_attr(c))) return rc;
    }
    return HYDRA_OK;
}

int hydra_load_tensor(hydra_ctx *c, void *stream, int kind, int index, int sub, const void *src) {
    if (!c || !src) return fail(HYDRA_E_INVALID_ARG, "hydra_load_tensor: NULL argument");
    if (!c->arena) return fail(HYDRA_E_STATE, "no weight arena bound");
    if (kind < 0 || kind >= HYDRA_W_KIND_COUNT) return fail(HYDRA_E_INVALID_ARG, "unknown tensor kind");
    hipStream_t s = (hipStream_t)stream;
    const int d = c->m.d, F = c->m.ffn, V = c->m.vocab;
    char *A = c->arena;
    const bool layer_kind = kind >= HYDRA_W_ATTN_NORM && kind <= HYDRA_W_DOWN;
    const bool head_kind = kind >= HYDRA_W_HEAD_W1;
    if (layer_kind && (index < 0 || index >= c->m.n_layers)) return fail(HYDRA_E_INVALID_ARG, "layer index out of range");
    if (head_kind && (index < 1 || index > c->h.n_draft_heads)) return fail(HYDRA_E_INVALID_ARG, "head index out of range (1-based)");
    if ((kind == HYDRA_W_HEAD_WL || kind == HYDRA_W_HEAD_BL) && (sub < 2 || sub > c->h.mlp_layers))
        return fail(HYDRA_E_INVALID_ARG, "MLP layer index out of range (2..mlp_layers)");
    auto matrix = [&](size_t off, int N, int K, int f32_row_off, int f32_rows_total, int tile_off, int tile_stride,
                      int rows_per_band = 32, int col_off = 0, int bands_per_head = 0) -> int {
        (void)f32_rows_total;
        if (c->bf16) return launch_pack_matrix(c, s, src, A + off, N, K, tile_off, tile_stride, rows_per_band, col_off, bands_per_head);
        return launch_copy_matrix(c, s, src, A + off, N, K, f32_row_off, K);
    };
    switch (kind) {
        case HYDRA_W_EMBED:      return launch_copy_matrix(c, s, src, A + c->off_embed, V, d, 0, d);
        case HYDRA_W_LM_HEAD:    return matrix(c->off_lm_head, V, d, 0, V, 0, 1);
        case HYDRA_W_FINAL_NORM: return launch_to_f32(c, s, src, (float *)(A + c->off_final_norm), d);
        case HYDRA_W_ATTN_NORM:  return launch_to_f32(c, s, src, (float *)(A + c->layer[index].attn_norm), d);
        case HYDRA_W_FFN_NORM:   return launch_to_f32(c, s, src, (float *)(A + c->layer[index].ffn_norm), d);
        case HYDRA_W_WQ:         return matrix(c->layer[index].wqkv, d, d, 0, 3 * d, 0, 1, 32, 0, c->m.head_dim / 32);        // bf16: rotary
        case HYDRA_W_WK:         return matrix(c->layer[index].wqkv, d, d, d, 3 * d, d / 32, 1, 32, 0, c->m.head_dim / 32);   // pairs adjacent
        case HYDRA_W_WV:         return matrix(c->layer[index].wqkv, d, d, 2 * d, 3 * d, 2 * (d / 32), 1);
        case HYDRA_W_WO:         return matrix(c->layer[index].wo, d, d, 0, d, 0, 1);
        case HYDRA_W_GATE:       return matrix(c->layer[index].wgu, F, d, 0, 2 * F, 0, 1, 16, 0);     // bf16: left half of every band
        case HYDRA_W_UP:         return matrix(c->layer[index].wgu, F, d, F, 2 * F, 0, 1, 16, 16);    // bf16: right half
        case HYDRA_W_DOWN:       return matrix(c->layer[index].wdown, d, F, 0, d, 0, 1);
        case HYDRA_W_HEAD_W1:    return matrix(c->head[index].w1, d, head_in_width(c, index), 0, d, 0, 1);
        case HYDRA_W_HEAD_B1:    return launch_to_f32(c, s, src, (float *)(A + c->head[index].b1), d);
        case HYDRA_W_HEAD_WL:    return matrix(c->head[index].wl[sub - 2], d, d, 0, d, 0, 1);
        case HYDRA_W_HEAD_BL:    return launch_to_f32(c, s, src, (float *)(A + c->head[index].bl[sub - 2]), d);
        case HYDRA_W_HEAD_WOUT:  return matrix(c->head[index].wout, V, d, 0, V, 0, 1);
    }
    return fail(HYDRA_E_INVALID_ARG, "unknown tensor kind");
}

int hydra_read_flags(hydra_ctx *c, void *stream, int32_t *flags_out) {
    if (!c || !flags_out) return fail(HYDRA_E_INVALID_ARG, "hydra_read_flags: NULL argument");
    if (!c->arena) return fail(HYDRA_E_STATE, "no weight arena bound");
    hipStream_t s = (hipStream_t)stream;
    HYDRA_HIP(hipMemcpyAsync(flags_out, flags_ptr(c), 4, hipMemcpyDeviceToHost, s));
    HYDRA_HIP(hipMemsetAsync(flags_ptr(c), 0, 4, s));
    HYDRA_HIP(hipStreamSynchronize(s));
    return HYDRA_OK;
}

int hydra_layer_kernel_info(const hydra_ctx *c, int B, int64_t *info) {
    if (!c || !info) return fail(HYDRA_E_INVALID_ARG, "hydra_layer_kernel_info: NULL argument");
    if (B < 1 || B > c->max_batch) return fail(HYDRA_E_CAPACITY, "B outside [1, max_batch]");
    int64_t v[4];
    layers_mega_info(c, B, v);
    const WsLayout w = ws_layout(c, B);
    info[0] = v[0];
    info[1] = v[0] ? (int64_t)(w.mega + v[1]) : 0;
    info[2] = v[2];
    info[3] = v[3];
    return HYDRA_OK;
}

int hydra_profile_begin(hydra_ctx *c) {
    if (!c) return fail(HYDRA_E_INVALID_ARG, "ctx is NULL");
    c->profiling = true; c->ev_used = 0; c->prof_bytes = 0; c->prof_launches = 0;
    return HYDRA_OK;
}

int hydra_profile_end(hydra_ctx *c, int64_t *launches, double *ms, double *weight_bytes) {
    if (!c) return fail(HYDRA_E_INVALID_ARG, "ctx is NULL");
    c->profiling = false;
    double total = 0;
    if (c->ev_used > 0) HYDRA_HIP(hipEventSynchronize(c->ev[c->ev_used - 1]));
    for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
        float t = 0;
        HYDRA_HIP(hipEventElapsedTime(&t, c->ev[i], c->ev[i + 1]));
        total += t;
    }
    if (launches) *launches = c->prof_launches;
    if (ms) *ms = total;
    if (weight_bytes) *weight_bytes = c->prof_bytes;
    c->ev_used = 0;
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// draft
// ---------------------------------------------------------------------------
int hydra_draft_tree(hydra_ctx *c, void *stream, int B, void *ws, const float *h_last, const int32_t *root,
                     int32_t *tree_tokens) {
    int rc = check_common(c, B, ws);
    if (rc) return rc;
    if (!h_last || !root || !tree_tokens) return fail(HYDRA_E_INVALID_ARG, "hydra_draft_tree: NULL argument");
    if (c->tree.max_depth > c->h.n_draft_heads) return fail(HYDRA_E_UNSUPPORTED, "tree is deeper than the number of draft heads");
    hipStream_t s = (hipStream_t)stream;
    const WsLayout w = ws_layout(c, B);
    char *W = (char *)ws, *A = c->arena;
    float *part = (float *)(W + w.part), *z = (float *)(W + w.z);
    void *xa = W + w.xa, *xb = W + w.xb;
    const int d = c->m.d, V = c->m.vocab;
    if ((rc = launch_draft_root(c, s, B, root, tree_tokens))) return rc;
    for (int i = 1; i <= c->tree.max_depth; ++i) {
        const int Mi = B * c->tree.n_expand[i];
        if (Mi == 0) continue;
        const int Kin = head_in_width(c, i);
        GemmPlan p;
        const bool first_residual = c->h.medusa != 0;       // Medusa-style first layer: z = h_last + SiLU(W1 h_last + b1)
        if ((rc = launch_draft_gather(c, s, B, i, h_last, tree_tokens, xa, first_residual ? z : nullptr, flags_ptr(c)))) return rc;
        void *cur = xb, *other = xa;
        if (c->bf16) {
            // MLP layers: bias + SiLU (+ residual) fused into the GEMM epilogue, unless splitting K over more
            // workgroups (with a small second kernel adding the partials) is estimated to be clearly faster:
            // the wide first layer of the later heads has few output bands and a long K
            auto mlp_layer = [&](const void *xin, size_t w_off, size_t b_off, int K, bool residual, void *xout) -> int {
                const GemmPlan fused = plan_gemm(c, Mi, d, K, GEMM_KIND_FUSED), split = plan_gemm(c, Mi, d, K, GEMM_KIND_PLAIN);
                if (split.splits > 1 && split.cost_us + 5.f < fused.cost_us) {
                    int r2 = launch_gemm(c, s, xin, A + w_off, part, Mi, d, K, &p);
                    if (r2) return r2;
                    return launch_bias_silu(c, s, part, p.splits, gemm_npad(c, d), (size_t)align_up(Mi, 32) * gemm_npad(c, d),
                                            (const float *)(A + b_off), z, residual, xout, Mi);
                }
                return launch_gemm_bias_silu(c, s, xin, A + w_off, Mi, d, K, (const float *)(A + b_off), z, residual, xout);
            };
            if ((rc = mlp_layer(xa, c->head[i].w1, c->head[i].b1, Kin, first_residual, xb))) return rc;
            for (int j = 2; j <= c->h.mlp_layers; ++j) {
                if ((rc = mlp_layer(cur, c->head[i].wl[j - 2], c->head[i].bl[j - 2], d, true, other))) return rc;
                std::swap(cur, other);
            }
        } else {
            if ((rc = launch_gemm(c, s, xa, A + c->head[i].w1, part, Mi, d, Kin, &p))) return rc;
            const size_t ss = (size_t)align_up(Mi, 32) * gemm_npad(c, d);
            if ((rc = launch_bias_silu(c, s, part, p.splits, gemm_npad(c, d), ss, (const float *)(A + c->head[i].b1), z, first_residual, xb, Mi))) return rc;
            for (int j = 2; j <= c->h.mlp_layers; ++j) {
                if ((rc = launch_gemm(c, s, cur, A + c->head[i].wl[j - 2], part, Mi, d, d, &p))) return rc;
                if ((rc = launch_bias_silu(c, s, part, p.splits, gemm_npad(c, d), ss, (const float *)(A + c->head[i].bl[j - 2]), z, true, other, Mi))) return rc;
                std::swap(cur, other);
            }
        }
        if ((rc = launch_gemm(c, s, cur, A + c->head[i].wout, part, Mi, V, d, &p))) return rc;
        const size_t sv = (size_t)align_up(Mi, 32) * gemm_npad(c, V);
        if ((rc = launch_topk(c, s, part, p.splits, gemm_npad(c, V), sv, B, i, tree_tokens, W + w.topk))) return rc;
    }
    return HYDRA_OK;
}

}  // extern "C"

namespace hydra {

// Where the rows of a forward pass come from: token embeddings (tree_verify_forward) or given hidden states
// gathered along an accepted path (hydra_prefix_attention).
struct RowSource {
    const int32_t *tokens;                       // [B, T] or NULL
    const float *hidden; int T_src;              // [B, T_src, d] when tokens == NULL
    const int32_t *path; const int32_t *n_acc;   // [B, T], [B]
};

// The decoder layers of the context over its B * T tree rows.  lm_tail: final RMSNorm, LM head, argmax (the
// verify step); otherwise the residual stream after the last layer is left in the workspace's x.
// LM head, greedy token and margin of the 16-bit family (paper, section 2: the base model's next-token choice at every
// tree node).  Without a logits buffer the GEMM's epilogue reduces every band to its two best columns and a small
// kernel merges the bands; with one, the logits go through memory and argmax_kernel reads them back.
static int lm_head_tail(hydra_ctx *c, hipStream_t s, const void *xg, float *part, int M, RowScale rs, int Mpad, int32_t *argmax,
                        float *margin, float *logits) {
    const int d = c->m.d, V = c->m.vocab;
    const int ld_v = gemm_npad(c, V);
    const size_t mp = align_up(M, 32);
    int rc;
    if (!logits && (size_t)ceil_div(V, 32) * Mpad * 16 <= (size_t)mp * ld_v * 4) {
        int fused = 0;
        if ((rc = launch_gemm_top2(c, s, xg, c->arena + c->off_lm_head, M, V, d, part, Mpad, &fused))) return rc;
        if (fused) return launch_argmax_bands(c, s, part, ceil_div(V, 32), Mpad, rs, M, argmax, margin);
    }
    GemmPlan p;
    if ((rc = launch_gemm(c, s, xg, c->arena + c->off_lm_head, part, M, V, d, &p))) return rc;
    return launch_argmax(c, s, part, p.splits, ld_v, mp * ld_v, rs, M, argmax, margin, logits);
}

static int forward_layers(hydra_ctx *c, hipStream_t s, int B, void *ws, const RowSource &src, const int32_t *seq_len,
                          const hydra_kv *kv, bool lm_tail, float *hidden, int32_t *argmax, float *margin, float *logits) {
    int rc;
    const WsLayout w = ws_layout(c, B);
    char *W = (char *)ws, *A = c->arena;
    float *x = (float *)(W + w.x), *part = (float *)(W + w.part), *apart = (float *)(W + w.apart);
    void *xa = W + w.xa, *xb = W + w.xb, *qbuf = W + w.qbuf;
    int32_t *flags = flags_ptr(c);
    const int d = c->m.d, F = c->m.ffn, V = c->m.vocab, M = B * c->tree.T;
    const size_t mp = align_up(M, 32);
    const int ld_d = gemm_npad(c, d), ld_qkv = gemm_npad(c, 3 * d), ld_gu = gemm_npad(c, 2 * F), ld_v = gemm_npad(c, V);
    GemmPlan p;
    const RowScale none = {nullptr, 0, 0, 0, 0.f};
    if (c->bf16) {
        // Fused flow.  The residual epilogues leave x, xg = half(x * gain of the next norm) and per-band sums of
        // squares; the 1/rms factor of each RMSNorm is applied by the consumer of the following GEMM.
        float *ss = (float *)(W + w.ss);
        const int Mpad = (int)align_up(std::max<size_t>(M, 1), 128);
        RowScale rs = {ss, 1, Mpad, d, c->m.rms_eps};        // rs.nb: rows of ss the last producer filled (1 = a complete sum per row)
        const float *gain0 = (const float *)(A + c->layer[0].attn_norm);
        if (lm_tail && src.tokens && layers_mega_eligible(c, B, kv)) {
            // up to 64 rows and a bounded context: all layers in one persistent kernel (bf16_layers.hip)
            LayersMegaIO io;
            if ((rc = launch_layers_mega(c, s, B, W + w.mega, seq_len, kv, flags, &io, false))) return rc;
            if ((rc = launch_embed_prep(c, s, src.tokens, io.x_first, gain0, io.xg_first, io.ss_first, io.Mpad, M, flags))) return rc;
            if ((rc = launch_layers_mega(c, s, B, W + w.mega, seq_len, kv, flags, &io, true))) return rc;
            const RowScale rl = {io.ss_last, io.nb_last, io.Mpad, d, c->m.rms_eps};
            if ((rc = launch_final_hidden(c, s, io.x_last, (const float *)(A + c->off_final_norm), rl, hidden, M))) return rc;
            return lm_head_tail(c, s, io.xg_last, part, M, rl, io.Mpad, argmax, margin, logits);
        }
        if (src.tokens) { if ((rc = launch_embed_prep(c, s, src.tokens, x, gain0, xa, ss, Mpad, M, flags))) return rc; }
        else            { if ((rc = launch_gather_prep(c, s, B, src.hidden, src.T_src, src.path, src.n_acc, x, gain0, xa, ss, Mpad, flags))) return rc; }
        for (int l = 0; l < c->m.n_layers; ++l) {
            const LayerOff &o = c->layer[l];
            const float *next_gain = (const float *)(A + (l + 1 < c->m.n_layers ? c->layer[l + 1].attn_norm : c->off_final_norm));
            if ((rc = launch_gemm_qkv_rope(c, s, xa, A + o.wqkv, M, rs, l, seq_len, kv, qbuf, part, flags))) return rc;
            if ((rc = launch_attention(c, s, B, l, qbuf, seq_len, kv, apart, w.attn_units, xb, nullptr, flags))) return rc;
            if ((rc = launch_gemm_resid(c, s, xb, A + o.wo, M, d, d, x, (const float *)(A + o.ffn_norm), xa, ss, Mpad, part, &rs.nb))) return rc;
            if ((rc = launch_gemm_silu(c, s, xa, A + o.wgu, M, F, d, ss, rs.nb, Mpad, xb))) return rc;
            if ((rc = launch_gemm_resid(c, s, xb, A + o.wdown, M, d, F, x, next_gain, xa, ss, Mpad, part, &rs.nb))) return rc;
        }
        if (!lm_tail) return HYDRA_OK;
        if ((rc = launch_final_hidden(c, s, x, (const float *)(A + c->off_final_norm), rs, hidden, M))) return rc;
        return lm_head_tail(c, s, xa, part, M, rs, Mpad, argmax, margin, logits);
    }
    if (src.tokens) { if ((rc = launch_embed(c, s, src.tokens, x, M, flags))) return rc; }
    else            { if ((rc = launch_gather_prep(c, s, B, src.hidden, src.T_src, src.path, src.n_acc, x, nullptr, nullptr, nullptr, 0, flags))) return rc; }
    int S_prev = 0;                         // split-K partials of the previous residual branch, still to be added to x
    for (int l = 0; l < c->m.n_layers; ++l) {
        const LayerOff &o = c->layer[l];
        if ((rc = launch_rmsnorm(c, s, x, part, S_prev, ld_d, mp * ld_d, (const float *)(A + o.attn_norm), xa, M, nullptr))) return rc;
        if ((rc = launch_gemm(c, s, xa, A + o.wqkv, part, M, 3 * d, d, &p))) return rc;
        if ((rc = launch_rope_append(c, s, part, p.splits, ld_qkv, mp * ld_qkv, none, B, l, seq_len, kv, qbuf, flags))) return rc;
        if ((rc = launch_attention(c, s, B, l, qbuf, seq_len, kv, apart, w.attn_units, xa, nullptr, flags))) return rc;
        if ((rc = launch_gemm(c, s, xa, A + o.wo, part, M, d, d, &p))) return rc;
        if ((rc = launch_rmsnorm(c, s, x, part, p.splits, ld_d, mp * ld_d, (const float *)(A + o.ffn_norm), xa, M, nullptr))) return rc;
        if ((rc = launch_gemm(c, s, xa, A + o.wgu, part, M, 2 * F, d, &p))) return rc;
        if ((rc = launch_silu_mul(c, s, part, p.splits, ld_gu, mp * ld_gu, xb, M))) return rc;
        if ((rc = launch_gemm(c, s, xb, A + o.wdown, part, M, d, F, &p))) return rc;
        S_prev = p.splits;
    }
    // adds the last residual branch to x; the normalised copy it also writes is what the LM head reads
    if ((rc = launch_rmsnorm(c, s, x, part, S_prev, ld_d, mp * ld_d, (const float *)(A + c->off_final_norm), xa, M, lm_tail ? hidden : nullptr))) return rc;
    if (!lm_tail) return HYDRA_OK;
    if ((rc = launch_gemm(c, s, xa, A + c->off_lm_head, part, M, V, d, &p))) return rc;
    if ((rc = launch_argmax(c, s, part, p.splits, ld_v, mp * ld_v, none, M, argmax, margin, logits))) return rc;
    return HYDRA_OK;
}

}  // namespace hydra

extern "C" {

// ---------------------------------------------------------------------------
// verify
// ---------------------------------------------------------------------------
int tree_verify_forward(hydra_ctx *c, void *stream, int B, void *ws, const int32_t *tree_tokens,
                        const int32_t *seq_len, const hydra_kv *kv, float *hidden, int32_t *argmax, float *margin,
                        float *logits) {
    int rc = check_common(c, B, ws);
    if (rc) return rc;
    if (!tree_tokens || !seq_len || !hidden || !argmax) return fail(HYDRA_E_INVALID_ARG, "tree_verify_forward: NULL argument");
    if ((rc = check_kv(c, kv))) return rc;
    const RowSource src = {tree_tokens, nullptr, 0, nullptr, nullptr};
    return forward_layers(c, (hipStream_t)stream, B, ws, src, seq_len, kv, true, hidden, argmax, margin, logits);
}

// ---------------------------------------------------------------------------
// Hydra++ prefix attention
// ---------------------------------------------------------------------------
int hydra_prefix_attention(hydra_ctx *c, void *stream, int B, void *ws, const float *hidden, int T_src,
                           const int32_t *path, const int32_t *n_acc, int32_t *seq_len, const hydra_kv *kv,
                           float *h_out) {
    int rc = check_common(c, B, ws);
    if (rc) return rc;
    if (!hidden || !path || !n_acc || !seq_len || !h_out) return fail(HYDRA_E_INVALID_ARG, "hydra_prefix_attention: NULL argument");
    if (T_src < 1) return fail(HYDRA_E_INVALID_ARG, "hydra_prefix_attention: T_src must be positive");
    for (int n = 1; n < c->tree.T; ++n)
        if (c->tree.parent[n] != n - 1) return fail(HYDRA_E_SHAPE, "hydra_prefix_attention: the context's tree must be a chain");
    if ((rc = check_kv(c, kv))) return rc;
    hipStream_t s = (hipStream_t)stream;
    const RowSource src = {nullptr, hidden, T_src, path, n_acc};
    if ((rc = forward_layers(c, s, B, ws, src, seq_len, kv, false, nullptr, nullptr, nullptr, nullptr))) return rc;
    const WsLayout w = ws_layout(c, B);
    return launch_prefix_select(c, s, B, (const float *)((char *)ws + w.x), n_acc, kv, seq_len, h_out);
}

int tree_attention(hydra_ctx *c, void *stream, int B, int layer, void *ws, const float *q, const int32_t *seq_len,
                   const hydra_kv *kv, float *out) {
    int rc = check_common(c, B, ws);
    if (rc) return rc;
    if (!q || !seq_len || !out) return fail(HYDRA_E_INVALID_ARG, "tree_attention: NULL argument");
    if (layer < 0 || layer >= c->m.n_layers) return fail(HYDRA_E_INVALID_ARG, "layer out of range");
    if ((rc = check_kv(c, kv))) return rc;
    hipStream_t s = (hipStream_t)stream;
    const WsLayout w = ws_layout(c, B);
    char *W = (char *)ws;
    void *qbuf = W + w.qbuf;
    if ((rc = launch_q_import(c, s, B, q, qbuf))) return rc;
    return launch_attention(c, s, B, layer, qbuf, seq_len, kv, (float *)(W + w.apart), w.attn_units, nullptr, out, flags_ptr(c));
}

// ---------------------------------------------------------------------------
// accept / compact
// ---------------------------------------------------------------------------
int accept_greedy(hydra_ctx *c, void *stream, int B, const int32_t *tree_tokens, const int32_t *argmax,
                  int32_t *n_acc, int32_t *path, int32_t *next_root, int32_t *last_node) {
    if (!c) return fail(HYDRA_E_INVALID_ARG, "ctx is NULL");
    if (B < 1 || B > c->max_batch) return fail(HYDRA_E_CAPACITY, "B outside [1, max_batch]");
    if (!c->arena) return fail(HYDRA_E_STATE, "no weight arena bound");
    if (!tree_tokens || !argmax || !n_acc || !path || !next_root || !last_node)
        return fail(HYDRA_E_INVALID_ARG, "accept_greedy: NULL argument");
    return launch_accept(c, (hipStream_t)stream, B, tree_tokens, argmax, n_acc, path, next_root, last_node);
}

int accept_typical(hydra_ctx *c, void *stream, int B, void *ws, const int32_t *tree_tokens, const float *logits,
                   float tau, float eps, float alpha, const float *u, int32_t *n_acc, int32_t *path,
                   int32_t *next_root, int32_t *last_node) {
    int rc = check_common(c, B, ws);
    if (rc) return rc;
    if (!tree_tokens || !logits || !n_acc || !path || !next_root || !last_node)
        return fail(HYDRA_E_INVALID_ARG, "accept_typical: NULL argument");
    if (!(tau > 0.f) || !(eps >= 0.f) || !(alpha >= 0.f)) return fail(HYDRA_E_INVALID_ARG, "accept_typical: need tau > 0, eps >= 0, alpha >= 0");
    const WsLayout w = ws_layout(c, B);
    int32_t *ok = (int32_t *)((char *)ws + w.part);          // B * T flags; the GEMM partial buffer is free between calls
    return launch_accept_typical(c, (hipStream_t)stream, B, tree_tokens, logits, tau, eps, alpha, u, ok, flags_ptr(c), n_acc, path,
                                 next_root, last_node);
}

int kv_compact(hydra_ctx *c, void *stream, int B, const int32_t *n_acc, const int32_t *path,
               const int32_t *next_root, const int32_t *last_node, const float *hidden, const hydra_kv *kv,
               int32_t *seq_len, float *h_last, int32_t *root, int32_t *kv_index) {
    if (!c) return fail(HYDRA_E_INVALID_ARG, "ctx is NULL");
    if (B < 1 || B > c->max_batch) return fail(HYDRA_E_CAPACITY, "B outside [1, max_batch]");
    if (!c->arena) return fail(HYDRA_E_STATE, "no weight arena bound");
    if (!n_acc || !path || !next_root || !last_node || !hidden || !seq_len || !h_last || !root)
        return fail(HYDRA_E_INVALID_ARG, "kv_compact: NULL argument");
    int rc = check_kv(c, kv);
    if (rc) return rc;
    return launch_compact(c, (hipStream_t)stream, B, n_acc, path, next_root, last_node, hidden, kv, seq_len, h_last, root, kv_index);
}

int hydra_kv_write(hydra_ctx *c, void *stream, int B, int layer, const hydra_kv *kv, int first_slot, int n_slots,
                   const float *kv_plain) {
    if (!c || !kv_plain) return fail(HYDRA_E_INVALID_ARG, "hydra_kv_write: NULL argument");
    if (B < 1 || B > c->max_batch) return fail(HYDRA_E_CAPACITY, "B outside [1, max_batch]");
    if (layer < 0 || layer >= c->m.n_layers) return fail(HYDRA_E_INVALID_ARG, "layer out of range");
    int rc = check_kv(c, kv);
    if (rc) return rc;
    if (first_slot < 0 || n_slots < 0 || first_slot + n_slots > kv->max_pages * HYDRA_PAGE) return fail(HYDRA_E_CAPACITY, "slots outside the page table");
    if (n_slots == 0) return HYDRA_OK;
    return launch_kv_plain(c, (hipStream_t)stream, B, layer, kv, first_slot, n_slots, const_cast<float *>(kv_plain), true);
}

int hydra_kv_read(hydra_ctx *c, void *stream, int B, int layer, const hydra_kv *kv, int first_slot, int n_slots,
                  float *kv_plain) {
    if (!c || !kv_plain) return fail(HYDRA_E_INVALID_ARG, "hydra_kv_read: NULL argument");
    if (B < 1 || B > c->max_batch) return fail(HYDRA_E_CAPACITY, "B outside [1, max_batch]");
    if (layer < 0 || layer >= c->m.n_layers) return fail(HYDRA_E_INVALID_ARG, "layer out of range");
    int rc = check_kv(c, kv);
    if (rc) return rc;
    if (first_slot < 0 || n_slots < 0 || first_slot + n_slots > kv->max_pages * HYDRA_PAGE) return fail(HYDRA_E_CAPACITY, "slots outside the page table");
    if (n_slots == 0) return HYDRA_OK;
    return launch_kv_plain(c, (hipStream_t)stream, B, layer, kv, first_slot, n_slots, kv_plain, false);
}

}  // extern "C"
