// fp32 storage family: a plain VALU GEMM and a one-wave-per-query tree
// attention.  Used by fp32 models (small, launch-bound); written for clarity
// and exactness of fp32 arithmetic, not for bandwidth.
#include "device_common.h"
#include "internal.h"

namespace hydra {

// part[m][n] = sum_k X[m][k] W[n][k].  One wave per output feature n, 16 rows
// of X per workgroup row-block; lanes stride over k, then a wave reduction.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ X, const float *__restrict__ W,
                                                        float *__restrict__ part, int M, int N, int K, int ld) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.x * 4 + wave;
    const int m0 = blockIdx.y * 16;
    if (n >= N) return;
    float acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    for (int k = lane; k < K; k += 64) {
        const float w = W[(size_t)n * K + k];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int m = (m0 + i < M) ? m0 + i : M - 1;
            acc[i] = fmaf(X[(size_t)m * K + k], w, acc[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const float v = wave_sum(acc[i]);
        if (lane == 0 && m0 + i < M) part[(size_t)(m0 + i) * ld + n] = v;
    }
}

int launch_gemm_f32(hydra_ctx *c, hipStream_t s, const float *X, const float *W, float *part, int M, int N, int K) {
    (void)c;
    dim3 grid(ceil_div(N, 4), ceil_div(M, 16)), block(256);
    hipLaunchKernelGGL(gemm_f32_kernel, grid, block, 0, s, X, W, part, M, N, K, N);
    HYDRA_LAUNCH_CHECK("gemm_f32_kernel");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Tree attention (paper, section 2): node n of row b attends to cache slots
// [0, L) and to the tree nodes named by its ancestor bitmask (slots L + a).
// One wave per (node, head, row).  Pass 1 per 64 keys: lane = key, dot with q
// from LDS, mask, online softmax; pass 2: lane = dim, out += p_key * V[key].
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void attn_f32_kernel(const float *__restrict__ q, const float *__restrict__ kpages,
                                                       const float *__restrict__ vpages, const int32_t *page_table,
                                                       int max_pages, int n_pages, int layer, const int32_t *seq_len,
                                                       const TreeDev *tree, int H, int Dh, float scale, float *out,
                                                       int32_t *flags) {
    const int n = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int T = tree->T;
    const int lane = threadIdx.x;
    const int L = seq_len[b];
    if (L < 0 || L + T > max_pages * 16) {
        if (lane == 0) atomicOr(flags, FLAG_CAPACITY);
        return;
    }
    __shared__ float qs[128];
    const size_t qoff = (((size_t)b * T + n) * H + h) * Dh;
    for (int i = lane; i < Dh; i += 64) qs[i] = q[qoff + i] * scale;
    __syncthreads();
    const uint64_t anc0 = tree->anc[n][0], anc1 = tree->anc[n][1];
    const int total = L + T;
    float m_run = -INFINITY, l_run = 0.f, o0 = 0.f, o1 = 0.f;
    for (int base = 0; base < total; base += 64) {
        const int key = base + lane;
        bool valid = key < total;
        if (valid && key >= L) {
            const int a = key - L;
            valid = ((a < 64 ? anc0 >> a : anc1 >> (a - 64)) & 1ull) != 0;
        }
        float sc = -INFINITY;
        if (valid) {
            const int page = checked_page(page_table[(size_t)b * max_pages + (key >> 4)], n_pages, flags);
            const float *kp = kpages + kv_block_base(layer, n_pages, page, H, h, Dh) + (size_t)(key & 15) * Dh;
            float a = 0.f;
            for (int i = 0; i < Dh; ++i) a = fmaf(qs[i], kp[i], a);
            sc = a;
        }
        const float m_new = fmaxf(m_run, wave_max(sc));
        if (m_new == -INFINITY) continue;                       // nothing visible yet (wave-uniform)
        const float p = valid ? __expf(sc - m_new) : 0.f;
        const float alpha = __expf(m_run - m_new);               // exp(-inf) = 0 on the first visible chunk
        l_run = l_run * alpha + wave_sum(p);
        o0 *= alpha;
        o1 *= alpha;
        m_run = m_new;
        const int cnt = min(64, total - base);
        for (int kk = 0; kk < cnt; ++kk) {
            const float pk = __shfl(p, kk, 64);
            if (pk == 0.f) continue;                            // masked keys are never read
            const int ks = base + kk;
            const int page = checked_page(page_table[(size_t)b * max_pages + (ks >> 4)], n_pages, flags);
            const float *vp = vpages + kv_block_base(layer, n_pages, page, H, h, Dh) + (size_t)(ks & 15) * Dh;
            if (lane < Dh) o0 = fmaf(pk, vp[lane], o0);
            if (lane + 64 < Dh) o1 = fmaf(pk, vp[lane + 64], o1);
        }
    }
    const float inv = 1.0f / l_run;
    if (lane < Dh) out[qoff + lane] = o0 * inv;
    if (lane + 64 < Dh) out[qoff + lane + 64] = o1 * inv;
}

int launch_attention_f32(hydra_ctx *c, hipStream_t s, int B, int layer, const float *q, const int32_t *seq_len,
                         const hydra_kv *kv, float *out, int32_t *flags) {
    dim3 grid(c->tree.T, c->m.n_heads, B), block(64);
    const float scale = 1.0f / sqrtf((float)c->m.head_dim);
    hipLaunchKernelGGL(attn_f32_kernel, grid, block, 0, s, q, (const float *)kv->k_pages, (const float *)kv->v_pages,
                       kv->page_table, kv->max_pages, kv->n_pages, layer, seq_len, tree_dev(c), c->m.n_heads,
                       c->m.head_dim, scale, out, flags);
    HYDRA_LAUNCH_CHECK("attn_f32_kernel");
    return HYDRA_OK;
}

}  // namespace hydra
