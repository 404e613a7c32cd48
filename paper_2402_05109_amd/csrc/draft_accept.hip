// Kernels of the draft phases (gather/concat, bias + SiLU, wave-level top-k)
// and of the integer tail of a step (greedy acceptance, cache compaction,
// state update).
#include "device_common.h"
#include "internal.h"

namespace hydra {

// tree_tokens[b, 0] = root[b]   (node 0 is x_t)
__global__ void draft_root_kernel(const int32_t *root, int32_t *tree_tokens, int B, int T) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) tree_tokens[(size_t)b * T] = root[b];
}

int launch_draft_root(hydra_ctx *c, hipStream_t s, int B, const int32_t *root, int32_t *tree_tokens) {
    hipLaunchKernelGGL(draft_root_kernel, dim3(ceil_div(B, 64)), dim3(64), 0, s, root, tree_tokens, B, c->tree.T);
    HYDRA_LAUNCH_CHECK("draft_root_kernel");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Head input (paper, section 3): for expanding node n of phase i (depth i-1),
//   u = [h_last ; E[tok(p_0)] ; ... ; E[tok(p_{i-1})]],  p_0 = root, p_{i-1} = n,
// concatenated on the feature axis.  Row r = b * n_expand + j.
// grid = (rows, segments); segment 0 copies h_last, segment s >= 1 one embedding.
// Medusa-style heads (section 2) have segment 0 only; z_out then also receives
// h_last in fp32, the residual term of their first layer.
// ---------------------------------------------------------------------------
template <bool BF>
__global__ void draft_gather_kernel(const TreeDev *tree, int phase, int include_root, const float *h_last,
                                    const int32_t *tree_tokens, const typename Elem<BF>::type *E, int d, int V,
                                    int Kin, typename Act<BF>::type *out, float *z_out, int32_t *flags) {
    const int ne = tree->n_expand[phase];
    const int r = blockIdx.x, seg = blockIdx.y;
    const int b = r / ne, j = r - b * ne;
    const int n = tree->expand_nodes[tree->expand_off[phase] + j];
    typedef __attribute__((ext_vector_type(4))) uint32_t u4;
    typedef __attribute__((ext_vector_type(4))) float f4;
    if (seg == 0) {
        if (BF) {                                               // 8 columns per thread: one 16-byte store into the operand tile
            for (int k = threadIdx.x * 8; k < d; k += blockDim.x * 8) {
                const f4 v0 = *reinterpret_cast<const f4 *>(h_last + (size_t)b * d + k);
                const f4 v1 = *reinterpret_cast<const f4 *>(h_last + (size_t)b * d + k + 4);
                const u4 pk = {f2a_pack(v0[0], v0[1]), f2a_pack(v0[2], v0[3]), f2a_pack(v1[0], v1[1]), f2a_pack(v1[2], v1[3])};
                *reinterpret_cast<u4 *>(reinterpret_cast<a16_t *>(out) + x_index<true>(r, k, Kin)) = pk;
                if (z_out) {
                    *reinterpret_cast<f4 *>(z_out + (size_t)r * d + k) = v0;
                    *reinterpret_cast<f4 *>(z_out + (size_t)r * d + k + 4) = v1;
                }
            }
            return;
        }
        for (int k = threadIdx.x; k < d; k += blockDim.x) {
            const float v = h_last[(size_t)b * d + k];
            Act<BF>::st(out, x_index<BF>(r, k, Kin), v);
            if (z_out) z_out[(size_t)r * d + k] = v;
        }
        return;
    }
    // embedding of the path node at depth dd; n itself has depth phase-1
    const int dd = seg - 1 + (include_root ? 0 : 1);
    int a = n;
    for (int up = (phase - 1) - dd; up > 0; --up) a = tree->parent[a];
    int tok = tree_tokens[(size_t)b * tree->T + a];
    if (tok < 0 || tok >= V) {
        if (threadIdx.x == 0) atomicOr(flags, FLAG_BAD_TOKEN);
        tok = 0;
    }
    if (BF) {
        for (int k = threadIdx.x * 8; k < d; k += blockDim.x * 8) {
            const u4 raw = *reinterpret_cast<const u4 *>(reinterpret_cast<const bf16_t *>(E) + (size_t)tok * d + k);     // 8 bfloat16
            u4 pk;
#pragma unroll
            for (int q = 0; q < 4; ++q) pk[q] = f2a_pack(__uint_as_float(raw[q] << 16), __uint_as_float(raw[q] & 0xffff0000u));
            *reinterpret_cast<u4 *>(reinterpret_cast<a16_t *>(out) + x_index<true>(r, seg * d + k, Kin)) = pk;
        }
        return;
    }
    for (int k = threadIdx.x; k < d; k += blockDim.x)
        Act<BF>::st(out, x_index<BF>(r, seg * d + k, Kin), Elem<BF>::ld(E, (size_t)tok * d + k));
}

int launch_draft_gather(hydra_ctx *c, hipStream_t s, int B, int phase, const float *h_last,
                        const int32_t *tree_tokens, void *x_out, float *z_out, int32_t *flags) {
    const int ne = c->tree.n_expand[phase];
    const int inc = c->h.include_root_embedding ? 1 : 0;
    const int nseg = c->h.medusa ? 1 : 1 + (inc ? phase : phase - 1);
    const int Kin = nseg * c->m.d;
    dim3 grid(B * ne, nseg), block(256);
    const void *E = c->arena + c->off_embed;
    if (c->bf16) hipLaunchKernelGGL(draft_gather_kernel<true>, grid, block, 0, s, tree_dev(c), phase, inc, h_last, tree_tokens, (const bf16_t *)E, c->m.d, c->m.vocab, Kin, (a16_t *)x_out, z_out, flags);
    else         hipLaunchKernelGGL(draft_gather_kernel<false>, grid, block, 0, s, tree_dev(c), phase, inc, h_last, tree_tokens, (const float *)E, c->m.d, c->m.vocab, Kin, (float *)x_out, z_out, flags);
    HYDRA_LAUNCH_CHECK("draft_gather_kernel");
    return HYDRA_OK;
}

// z <- (residual ? z : 0) + SiLU(W u + b);  also written as the next GEMM input
template <bool BF>
__global__ void bias_silu_kernel(const float *part, int S, int part_ld, size_t split_stride, const float *bias,
                                 float *z, int residual, int d, typename Act<BF>::type *out) {
    const int m = blockIdx.y;
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= d) return;
    float a = silu_f(part_sum(part, S, split_stride, (size_t)m * part_ld + k) + bias[k]);
    if (residual) a += z[(size_t)m * d + k];
    z[(size_t)m * d + k] = a;
    Act<BF>::st(out, x_index<BF>(m, k, d), a);
}

int launch_bias_silu(hydra_ctx *c, hipStream_t s, const float *part, int S, int part_ld, size_t split_stride,
                     const float *bias, float *z, bool residual, void *x_out, int M) {
    dim3 grid(ceil_div(c->m.d, 256), M), block(256);
    if (c->bf16) hipLaunchKernelGGL(bias_silu_kernel<true>, grid, block, 0, s, part, S, part_ld, split_stride, bias, z, residual ? 1 : 0, c->m.d, (a16_t *)x_out);
    else         hipLaunchKernelGGL(bias_silu_kernel<false>, grid, block, 0, s, part, S, part_ld, split_stride, bias, z, residual ? 1 : 0, c->m.d, (float *)x_out);
    HYDRA_LAUNCH_CHECK("bias_silu_kernel");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Top-k per row, ordered by (logit descending, token id ascending) (paper,
// section 2: children are the m most likely tokens, sorted).  The helpers come
// first (order, monotone keys, wave-wide reductions); the two kernels that use
// them, one wave per 1024-id chunk and one wave per row for the merge, are
// described above topk_chunk_kernel.
// ---------------------------------------------------------------------------
struct Cand { float v; int id; };
__device__ __forceinline__ bool better(float v, int id, float w, int jd) { return v > w || (v == w && id < jd); }

// Monotone 32-bit key of a float: a > b <=> key(a) > key(b).  -0 shares the key of +0 (they compare equal, so the
// token id decides between them) and a NaN gets the key of -infinity (it never wins, as with float comparisons).
__device__ __forceinline__ uint32_t order_key(float v) {
    uint32_t b = __float_as_uint(v);
    if ((b & 0x7fffffffu) > 0x7f800000u) b = 0xff800000u;
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t k) { return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k); }

// Wave-wide max / min of a 32-bit unsigned value, the same in every lane: four cross-lane steps inside each row of
// 16 lanes (swap neighbours, swap pairs, mirror halves of 8, mirror the row), then the four rows meet in scalars.
template <bool MAX>
__device__ __forceinline__ uint32_t wave_reduce_u32(uint32_t x) {
    auto op = [](uint32_t a, uint32_t b) { return MAX ? (a > b ? a : b) : (a < b ? a : b); };
    x = op(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
    x = op(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
    x = op(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x141, 0xf, 0xf, false));   // row_half_mirror
    x = op(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x140, 0xf, 0xf, false));   // row_mirror
    const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)x, 0), r1 = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
    const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)x, 32), r3 = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
    return op(op(r0, r1), op(r2, r3));
}

// best candidate of the wave in the (value descending, id ascending) order; every lane must be active
__device__ __forceinline__ Cand wave_best(Cand c) {
    const uint32_t key = order_key(c.v);
    const uint32_t kmax = wave_reduce_u32<true>(key);
    const uint32_t idmin = wave_reduce_u32<false>(key == kmax ? (uint32_t)c.id : 0xffffffffu);
    return Cand{key_value(kmax), (int)idmin};
}

// Top-k of a logits row in two kernels.  One workgroup on 32000 logits is bound by its own instruction issue (every
// wave rescans its registers once per extracted entry, and the waves of a workgroup share four SIMDs), so the row is
// cut into chunks of 1024 ids, one single-wave workgroup each, spread over the chip: lane l holds ids
// base + l, base + 64 + l, ... as monotone keys (order_key; key 0 is below every real key and marks an absent or
// already extracted entry), and k rounds leave the chunk's k best, in order, as (key, id) pairs.  The second kernel,
// one wave per row, picks the k best of those at most 32 * k survivors in the same (value descending, id
// ascending) order.
enum { TOPK_CHUNK = 1024, TOPK_PER_LANE = 16, TOPK_MAX_CHUNKS = 32 };

__global__ __launch_bounds__(64) void topk_chunk_kernel(const float *part, int S, int part_ld, size_t split_stride, int V,
                                                         const TreeDev *tree, int ne, int expand_off, uint2 *surv) {
    const int r = blockIdx.y, chunk = blockIdx.x, lane = threadIdx.x;
    const int base = chunk * TOPK_CHUNK;
    // the logits first: their addresses need nothing from the tree tables, whose dependent lookups follow
    uint32_t key[TOPK_PER_LANE];
#pragma unroll
    for (int i = 0; i < TOPK_PER_LANE; ++i) {
        const int id = base + i * 64 + lane;
        key[i] = id < V ? order_key(part_sum(part, S, split_stride, (size_t)r * part_ld + id)) : 0u;
    }
    const int k = tree->expand_k[expand_off + r % ne];
    uint2 *out = surv + ((size_t)r * gridDim.x + chunk) * HYDRA_MAX_TOPK;
    for (int t = 0; t < k; ++t) {
        // the lane's best: the first maximum in slot order is also its lowest id
        uint32_t bk = 0u, bs = 0u;
#pragma unroll
        for (int i = 0; i < TOPK_PER_LANE; ++i)
            if (key[i] > bk) { bk = key[i]; bs = (uint32_t)i; }
        const uint32_t kmax = wave_reduce_u32<true>(bk);
        const uint32_t idmin = wave_reduce_u32<false>(bk == kmax && kmax != 0u ? (uint32_t)base + bs * 64u + (uint32_t)lane : 0xffffffffu);
        if (idmin != 0xffffffffu) {                                   // wave-uniform; the winner's owner retires it
            const uint32_t off = idmin - (uint32_t)base;
            const uint32_t slot = off >> 6;
            const bool owner = (off & 63u) == (uint32_t)lane;
#pragma unroll
            for (int i = 0; i < TOPK_PER_LANE; ++i)
                if ((uint32_t)i == slot && owner) key[i] = 0u;
        }
        if (lane == 0) out[t] = make_uint2(kmax, idmin);              // key 0: the chunk ran out of entries
    }
}

__global__ __launch_bounds__(64) void topk_merge_kernel(const uint2 *surv, int chunks, const TreeDev *tree, int ne,
                                                         int expand_off, int32_t *tree_tokens) {
    const int r = blockIdx.x, lane = threadIdx.x;
    const int b = r / ne, j = r - b * ne;
    const int k = tree->expand_k[expand_off + j];
    const int first = tree->expand_first[expand_off + j];
    const uint2 *in = surv + (size_t)r * chunks * HYDRA_MAX_TOPK;
    // chunks * k survivors, at most 32 * 32: lane holds up to 16 of them
    uint32_t mk[16], mi[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int q = i * 64 + lane;                  // survivor index: chunk = q / k, rank = q % k
        mk[i] = 0u; mi[i] = 0xffffffffu;
        if (q < chunks * k) {
            const uint2 e = in[(size_t)(q / k) * HYDRA_MAX_TOPK + (q % k)];
            mk[i] = e.x; mi[i] = e.y;
        }
    }
    for (int t = 0; t < k; ++t) {
        uint32_t bk = 0u, bi = 0xffffffffu;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (mk[i] > bk || (mk[i] == bk && mk[i] != 0u && mi[i] < bi)) { bk = mk[i]; bi = mi[i]; }
        const uint32_t kmax = wave_reduce_u32<true>(bk);
        const uint32_t idmin = wave_reduce_u32<false>(bk == kmax && kmax != 0u ? bi : 0xffffffffu);
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (mi[i] == idmin) mk[i] = 0u;                           // ids are unique among the survivors
        if (lane == 0) tree_tokens[(size_t)b * tree->T + first + t] = (int32_t)idmin;
    }
}

// Any-V fallback: k rounds over memory, each picking the best entry that comes
// strictly after the previous winner in the (value desc, id asc) order.
__global__ __launch_bounds__(256) void topk_scan_kernel(const float *part, int S, int part_ld, size_t split_stride,
                                                         int V, const TreeDev *tree, int phase, int32_t *tree_tokens) {
    const int ne = tree->n_expand[phase];
    const int r = blockIdx.x;
    const int b = r / ne, j = r - b * ne;
    const int n = tree->expand_nodes[tree->expand_off[phase] + j];
    const int k = tree->n_children[n];
    __shared__ Cand red[4];
    __shared__ Cand prev;
    if (threadIdx.x == 0) { prev.v = INFINITY; prev.id = -1; }
    __syncthreads();
    for (int t = 0; t < k; ++t) {
        const Cand p = prev;
        Cand c = {-INFINITY, 0x7fffffff};
        for (int id = threadIdx.x; id < V; id += 256) {
            const float v = part_sum(part, S, split_stride, (size_t)r * part_ld + id);
            const bool after = better(p.v, p.id, v, id);
            if (after && better(v, id, c.v, c.id)) { c.v = v; c.id = id; }
        }
        c = wave_best(c);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = c;
        __syncthreads();
        if (threadIdx.x == 0) {
            Cand w = red[0];
            for (int i = 1; i < 4; ++i) if (better(red[i].v, red[i].id, w.v, w.id)) w = red[i];
            prev = w;
            tree_tokens[(size_t)b * tree->T + tree->first_child[n] + t] = w.id;
        }
        __syncthreads();
    }
}

size_t topk_scratch_bytes(const hydra_ctx *c, int rows) {
    return (size_t)rows * TOPK_MAX_CHUNKS * HYDRA_MAX_TOPK * sizeof(uint2);
}

int launch_topk(hydra_ctx *c, hipStream_t s, const float *part, int S, int part_ld, size_t split_stride, int B,
                int phase, int32_t *tree_tokens, void *scratch) {
    const int ne = c->tree.n_expand[phase], eoff = c->tree.expand_off[phase];
    const int rows = B * ne;
    const int chunks = ceil_div(c->m.vocab, TOPK_CHUNK);
    if (chunks <= TOPK_MAX_CHUNKS) {
        hipLaunchKernelGGL(topk_chunk_kernel, dim3(chunks, rows), dim3(64), 0, s, part, S, part_ld, split_stride, c->m.vocab, tree_dev(c), ne, eoff, (uint2 *)scratch);
        HYDRA_LAUNCH_CHECK("topk_chunk_kernel");
        hipLaunchKernelGGL(topk_merge_kernel, dim3(rows), dim3(64), 0, s, (const uint2 *)scratch, chunks, tree_dev(c), ne, eoff, tree_tokens);
        HYDRA_LAUNCH_CHECK("topk_merge_kernel");
    } else {
        hipLaunchKernelGGL(topk_scan_kernel, dim3(rows), dim3(256), 0, s, part, S, part_ld, split_stride, c->m.vocab, tree_dev(c), phase, tree_tokens);
        HYDRA_LAUNCH_CHECK("topk_scan_kernel");
    }
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Greedy acceptance (paper, section 2): walk down from the root while some
// child carries the base model's most likely token.  One thread per row.
// ---------------------------------------------------------------------------
__global__ void accept_kernel(const TreeDev *tree, int B, const int32_t *tree_tokens, const int32_t *argmax,
                              int32_t *n_acc, int32_t *path, int32_t *next_root, int32_t *last_node) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int T = tree->T, plen = tree->max_depth + 1;
    const int32_t *tok = tree_tokens + (size_t)b * T;
    const int32_t *am = argmax + (size_t)b * T;
    int32_t *p = path + (size_t)b * plen;
    int cur = 0, len = 1;
    p[0] = 0;
    for (;;) {
        const int g = am[cur];
        const int fc = tree->first_child[cur], nc = tree->n_children[cur];
        int nxt = -1;
        for (int i = 0; i < nc; ++i)
            if (tok[fc + i] == g) { nxt = fc + i; break; }
        if (nxt < 0) break;
        cur = nxt;
        p[len++] = cur;
    }
    for (int i = len; i < plen; ++i) p[i] = -1;
    n_acc[b] = len;
    next_root[b] = am[cur];
    last_node[b] = cur;
}

int launch_accept(hydra_ctx *c, hipStream_t s, int B, const int32_t *tree_tokens, const int32_t *argmax,
                  int32_t *n_acc, int32_t *path, int32_t *next_root, int32_t *last_node) {
    hipLaunchKernelGGL(accept_kernel, dim3(ceil_div(B, 64)), dim3(64), 0, s, tree_dev(c), B, tree_tokens, argmax, n_acc, path, next_root, last_node);
    HYDRA_LAUNCH_CHECK("accept_kernel");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Typical acceptance (paper, section 6.3): the child c of node n passes if
//   p(tok[c]) > min(eps, alpha * exp(-H)),  p = softmax(logits[n] / tau), H = entropy(p).
// Kernel 1, one workgroup per (row, node with children): max, Z = sum exp(z - max),
// S = sum exp(z - max) (z - max) with z = logit / tau, so H = ln Z - S / Z; then the
// test for each child.  Kernel 2, one workgroup per row: the deepest node whose whole
// path passes (lowest id among equally deep ones), and the next root: the most likely
// token of that node, or the token at which the cumulative distribution of
// softmax(logits / tau), taken in id order, first exceeds u.
// ---------------------------------------------------------------------------
enum { TYP_THREADS = 1024 };

__device__ __forceinline__ float block_reduce(float v, float *sh, bool is_max) {
    v = is_max ? wave_max(v) : wave_sum(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    float r = sh[0];
    for (int w = 1; w < (int)(blockDim.x >> 6); ++w) r = is_max ? fmaxf(r, sh[w]) : r + sh[w];   // fixed order
    return r;
}

__global__ __launch_bounds__(TYP_THREADS) void typical_stats_kernel(const float *__restrict__ logits, int V,
                                                                     const TreeDev *tree, const int32_t *__restrict__ tree_tokens,
                                                                     float inv_tau, float eps, float alpha,
                                                                     int32_t *__restrict__ ok, int32_t *flags) {
    __shared__ float sh[16];
    const int n = blockIdx.x, b = blockIdx.y, T = tree->T;
    const int nc = tree->n_children[n];
    if (nc == 0) return;                                            // uniform over the workgroup
    const float *row = logits + ((size_t)b * T + n) * V;
    float m = -INFINITY;
    for (int v = threadIdx.x; v < V; v += TYP_THREADS) m = fmaxf(m, row[v]);
    m = block_reduce(m, sh, true);
    float z = 0.f, sz = 0.f;
    for (int v = threadIdx.x; v < V; v += TYP_THREADS) {
        const float t = (row[v] - m) * inv_tau;                     // <= 0
        const float e = __expf(t);
        z += e;
        sz += e > 0.f ? e * t : 0.f;                                // exp underflow: 0 * (-inf) must not appear
    }
    z = block_reduce(z, sh, false);
    sz = block_reduce(sz, sh, false);
    const float H = __logf(z) - sz / z;
    const float th = fminf(eps, alpha * __expf(-H));
    const int first = tree->first_child[n];
    for (int i = threadIdx.x; i < nc; i += TYP_THREADS) {
        const int c = first + i;
        int tok = tree_tokens[(size_t)b * T + c];
        if (tok < 0 || tok >= V) { atomicOr(flags, FLAG_BAD_TOKEN); tok = 0; }
        const float p = __expf((row[tok] - m) * inv_tau) / z;
        ok[(size_t)b * T + c] = p > th ? 1 : 0;
    }
}

__global__ __launch_bounds__(TYP_THREADS) void typical_select_kernel(const float *__restrict__ logits, int V, const TreeDev *tree,
                                                                      const int32_t *__restrict__ ok, float inv_tau,
                                                                      const float *__restrict__ u, int32_t *n_acc,
                                                                      int32_t *path, int32_t *next_root, int32_t *last_node) {
    __shared__ float sh[16];
    __shared__ float wsum[16];
    __shared__ int best_s;
    __shared__ int cand[16];
    const int b = blockIdx.x, T = tree->T, plen = tree->max_depth + 1;
    if (threadIdx.x == 0) {
        // nodes are in breadth-first order: parents first, depth non-decreasing
        uint64_t reach[2] = {1ull, 0ull};
        int best = 0;
        for (int c = 1; c < T; ++c) {
            const int pa = tree->parent[c];
            if (((reach[pa >> 6] >> (pa & 63)) & 1ull) && ok[(size_t)b * T + c]) {
                reach[c >> 6] |= 1ull << (c & 63);
                if (tree->depth[c] > tree->depth[best]) best = c;
            }
        }
        best_s = best;
        const int len = tree->depth[best] + 1;
        int32_t *p = path + (size_t)b * plen;
        int cur = best;
        for (int j = len - 1; j >= 0; --j) { p[j] = cur; cur = tree->parent[cur]; }
        for (int j = len; j < plen; ++j) p[j] = -1;
        n_acc[b] = len;
        last_node[b] = best;
    }
    __syncthreads();
    const int best = best_s;
    const float *row = logits + ((size_t)b * T + best) * V;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (!u) {
        // most likely token, lowest id at ties
        float bv = -INFINITY; int bi = 0x7fffffff;
        for (int v = threadIdx.x; v < V; v += TYP_THREADS) {
            const float x = row[v];
            if (x > bv) { bv = x; bi = v; }                         // ascending v per thread: first maximum kept
        }
        Cand cnd = wave_best(Cand{bv, bi});
        __shared__ Cand red[16];
        if (lane == 0) red[wave] = cnd;
        __syncthreads();
        if (threadIdx.x == 0) {
            Cand w = red[0];
            for (int i = 1; i < 16; ++i) if (better(red[i].v, red[i].id, w.v, w.id)) w = red[i];
            next_root[b] = w.id;
        }
        return;
    }
    float m = -INFINITY;
    for (int v = threadIdx.x; v < V; v += TYP_THREADS) m = fmaxf(m, row[v]);
    m = block_reduce(m, sh, true);
    // thread t owns the contiguous ids [t*C, (t+1)*C): local mass, then an exclusive scan over threads in id order
    const int C = (V + TYP_THREADS - 1) / TYP_THREADS;
    const int v0 = threadIdx.x * C, v1 = min(V, v0 + C);
    float local = 0.f;
    for (int v = v0; v < v1; ++v) local += __expf((row[v] - m) * inv_tau);
    float incl = local;                                             // inclusive scan inside the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const float t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    float before = 0.f, total = 0.f;
    for (int w = 0; w < 16; ++w) { if (w < wave) before += wsum[w]; total += wsum[w]; }
    const float excl = before + incl - local;
    const float target = u[b] * total;
    if (threadIdx.x < 16) cand[threadIdx.x] = 0x7fffffff;
    __syncthreads();
    // the first id whose cumulative mass exceeds the target lies in the first thread range with excl + local > target
    if (local > 0.f && excl + local > target && excl <= target) {
        float c = excl; int pick = v1 - 1;
        for (int v = v0; v < v1; ++v) {
            c += __expf((row[v] - m) * inv_tau);
            if (c > target) { pick = v; break; }
        }
        atomicMin(&cand[0], pick);
    }
    __syncthreads();
    if (threadIdx.x == 0) next_root[b] = cand[0] == 0x7fffffff ? V - 1 : cand[0];
}

int launch_accept_typical(hydra_ctx *c, hipStream_t s, int B, const int32_t *tree_tokens, const float *logits, float tau,
                          float eps, float alpha, const float *u, int32_t *ok_scratch, int32_t *flags, int32_t *n_acc,
                          int32_t *path, int32_t *next_root, int32_t *last_node) {
    const int T = c->tree.T, V = c->m.vocab;
    hipLaunchKernelGGL(typical_stats_kernel, dim3(T, B), dim3(TYP_THREADS), 0, s, logits, V, tree_dev(c), tree_tokens, 1.0f / tau, eps, alpha, ok_scratch, flags);
    HYDRA_LAUNCH_CHECK("typical_stats_kernel");
    hipLaunchKernelGGL(typical_select_kernel, dim3(B), dim3(TYP_THREADS), 0, s, logits, V, tree_dev(c), ok_scratch, 1.0f / tau, u, n_acc, path, next_root, last_node);
    HYDRA_LAUNCH_CHECK("typical_select_kernel");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Cache compaction: slot L + path[j] -> slot L + j for j < n_acc, every layer.
// A thread owns one (layer, head, dim) element column and walks j upwards;
// path[j] >= j and strictly increasing, so within a column every source is read
// before it can be overwritten and no two threads touch the same element.
// A path that is not strictly increasing inside [0, T) (only a caller's own
// path can be: accept_greedy and accept_typical always produce one) ends the
// walk at the offending entry and is reported (FLAG_BAD_PATH); page ids outside
// the cache are reported (FLAG_BAD_PAGE) and their copies skipped.
// ---------------------------------------------------------------------------
template <bool BF>
__global__ void compact_kernel(const TreeDev *tree, const int32_t *n_acc, const int32_t *path,
                               const int32_t *seq_len, const int32_t *page_table, int max_pages, int n_pages,
                               typename Act<BF>::type *kpages, typename Act<BF>::type *vpages, int H, int Dh, int32_t *flags) {
    const int h = blockIdx.x, layer = blockIdx.y, b = blockIdx.z;
    const int dim = threadIdx.x;
    if (dim >= Dh) return;
    const int L = seq_len[b];
    if (L < 0 || L + tree->T > max_pages * 16) return;     // row was skipped by the verify kernels
    const int plen = tree->max_depth + 1;
    int na = n_acc[b];
    na = na < 0 ? 0 : (na > plen ? plen : na);
    int prev = -1;
    for (int j = 0; j < na; ++j) {
        const int n = path[(size_t)b * plen + j];
        if (n <= prev || n < j || n >= tree->T) {          // the same for every thread of the row
            if (dim == 0 && h == 0 && layer == 0) atomicOr(flags, FLAG_BAD_PATH);
            break;
        }
        prev = n;
        if (n == j) continue;
        const int ss = L + n, ds = L + j;
        const int sp = page_table[(size_t)b * max_pages + (ss >> 4)], dp = page_table[(size_t)b * max_pages + (ds >> 4)];
        if ((unsigned)sp >= (unsigned)n_pages || (unsigned)dp >= (unsigned)n_pages) {
            if (dim == 0 && h == 0 && layer == 0) atomicOr(flags, FLAG_BAD_PAGE);
            continue;
        }
        const size_t sb = kv_block_base(layer, n_pages, sp, H, h, Dh);
        const size_t db = kv_block_base(layer, n_pages, dp, H, h, Dh);
        kpages[db + k_in_block<BF>(ds & 15, dim, Dh)] = kpages[sb + k_in_block<BF>(ss & 15, dim, Dh)];
        vpages[db + v_in_block<BF>(ds & 15, dim, Dh)] = vpages[sb + v_in_block<BF>(ss & 15, dim, Dh)];
    }
}

// h_last <- hidden[last accepted node]; root <- next_root; seq_len += n_acc;
// kv_index[j] = (physical page, offset) of slot L + j.  Runs after compact_kernel.
// A row that the verify kernels skipped for lack of cache capacity keeps its state
// (seq_len, h_last, root) and gets kv_index = -1: its n_acc, last_node and hidden
// were computed from nothing.
__global__ void state_update_kernel(const TreeDev *tree, const int32_t *n_acc, const int32_t *next_root,
                                    const int32_t *last_node, const float *hidden, const int32_t *page_table,
                                    int max_pages, int d, int32_t *seq_len, float *h_last, int32_t *root,
                                    int32_t *kv_index) {
    const int b = blockIdx.x;
    const int T = tree->T, plen = tree->max_depth + 1;
    const int L = seq_len[b];
    const bool ok = L >= 0 && L + T <= max_pages * 16;     // uniform over the workgroup
    int na = n_acc[b];
    na = na < 0 ? 0 : (na > plen ? plen : na);
    int last = last_node[b];
    last = last < 0 ? 0 : (last >= T ? T - 1 : last);
    if (ok)
        for (int k = threadIdx.x; k < d; k += blockDim.x) h_last[(size_t)b * d + k] = hidden[((size_t)b * T + last) * d + k];
    __syncthreads();                                        // every thread has read seq_len[b]
    if (threadIdx.x == 0) {
        if (ok) root[b] = next_root[b];
        if (kv_index) {
            for (int j = 0; j < plen; ++j) {
                const bool in = ok && j < na;
                kv_index[((size_t)b * plen + j) * 2 + 0] = in ? page_table[(size_t)b * max_pages + ((L + j) >> 4)] : -1;
                kv_index[((size_t)b * plen + j) * 2 + 1] = in ? ((L + j) & 15) : -1;
            }
        }
        if (ok) seq_len[b] = L + na;
    }
}

int launch_compact(hydra_ctx *c, hipStream_t s, int B, const int32_t *n_acc, const int32_t *path,
                   const int32_t *next_root, const int32_t *last_node, const float *hidden, const hydra_kv *kv,
                   int32_t *seq_len, float *h_last, int32_t *root, int32_t *kv_index) {
    dim3 grid(c->m.n_heads, c->m.n_layers, B), block(c->m.head_dim);
    if (c->bf16) hipLaunchKernelGGL(compact_kernel<true>, grid, block, 0, s, tree_dev(c), n_acc, path, seq_len, kv->page_table, kv->max_pages, kv->n_pages, (a16_t *)kv->k_pages, (a16_t *)kv->v_pages, c->m.n_heads, c->m.head_dim, flags_dev(c));
    else         hipLaunchKernelGGL(compact_kernel<false>, grid, block, 0, s, tree_dev(c), n_acc, path, seq_len, kv->page_table, kv->max_pages, kv->n_pages, (float *)kv->k_pages, (float *)kv->v_pages, c->m.n_heads, c->m.head_dim, flags_dev(c));
    HYDRA_LAUNCH_CHECK("compact_kernel");
    hipLaunchKernelGGL(state_update_kernel, dim3(B), dim3(256), 0, s, tree_dev(c), n_acc, next_root, last_node, hidden, kv->page_table, kv->max_pages, c->m.d, seq_len, h_last, root, kv_index);
    HYDRA_LAUNCH_CHECK("state_update_kernel");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// accept_typical for callers that cannot allocate or pass a workspace (HIP graph capture, tight serving loops):
// the per-candidate pass flags that typical_stats_kernel hands to typical_select_kernel live in a fixed array
// in device memory that belongs to the library.  Each GPU has its own copy of the array at its own address; the
// address is looked up once per device (scratch_pointer) and only that pointer is ever given to kernels or
// memory calls, never the array's name.
// ---------------------------------------------------------------------------
enum { TYP_STATIC_MAX_NODES = 16384, TYP_MAX_DEVICES = 64 };          // B * T <= 16384: 64 KiB per device
static __device__ __align__(256) int32_t scratch[TYP_STATIC_MAX_NODES];
static int32_t *g_scratch_ptr[TYP_MAX_DEVICES];                        // per device; NULL until looked up

// the current device's copy of `scratch`; looked up on first use on that device (hydra_bind_weights does it at set-up)
int typical_static_scratch(int32_t **out) {
    int dev = -1;
    HYDRA_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= TYP_MAX_DEVICES) return fail(HYDRA_E_UNSUPPORTED, "accept_typical_static: device index beyond 63");
    int32_t *p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        void *sym = nullptr;
        HYDRA_HIP(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
        if (!sym) return fail(HYDRA_E_HIP, "accept_typical_static: no device address for the scratch array");
        p = static_cast<int32_t *>(sym);
        __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);    // every thread that races here stores the same address
    }
    *out = p;
    return HYDRA_OK;
}

}  // namespace hydra

extern "C" int accept_typical_static(hydra_ctx *c, void *stream, int B, const int32_t *tree_tokens, const float *logits, float tau,
                                     float eps, float alpha, const float *u, int32_t *n_acc, int32_t *path, int32_t *next_root,
                                     int32_t *last_node) {
    using namespace hydra;
    if (!c) return fail(HYDRA_E_INVALID_ARG, "ctx is NULL");
    if (B < 1 || B > c->max_batch) return fail(HYDRA_E_CAPACITY, "B outside [1, max_batch]");
    if (!c->arena) return fail(HYDRA_E_STATE, "no weight arena bound (hydra_bind_weights)");
    if (!tree_tokens || !logits || !n_acc || !path || !next_root || !last_node)
        return fail(HYDRA_E_INVALID_ARG, "accept_typical_static: NULL argument");
    if (!(tau > 0.f) || !(eps >= 0.f) || !(alpha >= 0.f)) return fail(HYDRA_E_INVALID_ARG, "accept_typical_static: need tau > 0, eps >= 0, alpha >= 0");
    if ((int64_t)B * c->tree.T > TYP_STATIC_MAX_NODES)
        return fail(HYDRA_E_CAPACITY, "accept_typical_static: B * T exceeds the 16384 tree nodes its fixed buffer holds; use accept_typical with a workspace");
    int32_t *ok = nullptr;
    int rc = typical_static_scratch(&ok);
    if (rc) return rc;
    int32_t *flags = reinterpret_cast<int32_t *>(c->arena + c->off_tables + (size_t)c->table_slot * TABLE_SLOT_BYTES + FLAGS_OFF_IN_SLOT);
    // typical_stats_kernel writes the flag of every non-root node before typical_select_kernel reads it, so nothing
    // in the buffer has to start at zero
    return launch_accept_typical(c, (hipStream_t)stream, B, tree_tokens, logits, tau, eps, alpha, u, ok, flags, n_acc, path, next_root, last_node);
}
