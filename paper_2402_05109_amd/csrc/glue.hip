// Elementwise / gather / reduce kernels around the GEMMs and the attention:
// embedding gather, residual + RMSNorm, rotary + KV append, SiLU*up,
// LM-head argmax, plain <-> in-page KV conversion.  Each kernel is written once
// and instantiated for the two storage families (BF = bf16, !BF = fp32).
#include "device_common.h"
#include "internal.h"

namespace hydra {

// ---------------------------------------------------------------------------
// x[m, :] = E[token[m], :]      (tree verification feeds all T candidate tokens
// of a row as one packed input; paper, section 2, "Tree decoding")
// ---------------------------------------------------------------------------
template <bool BF>
__global__ void embed_kernel(const typename Elem<BF>::type *E, const int32_t *tokens, float *x, int d, int V,
                             int32_t *flags) {
    const int m = blockIdx.x;
    int tok = tokens[m];
    if (tok < 0 || tok >= V) {
        if (threadIdx.x == 0) atomicOr(flags, FLAG_BAD_TOKEN);
        tok = 0;
    }
    for (int k = threadIdx.x; k < d; k += blockDim.x) x[(size_t)m * d + k] = Elem<BF>::ld(E, (size_t)tok * d + k);
}

// 1 / rms of row m from the per-band sums of squares (one wave's worth of threads adds the bands)
__device__ __forceinline__ float row_rstd_block(const RowScale &rs, int m, float *sh) {
    if (!rs.ss) return 1.0f;
    float a = 0.f;
    if (threadIdx.x < 64)
        for (int b = threadIdx.x; b < rs.nb; b += 64) a += rs.ss[(size_t)b * rs.Mpad + m];
    if (threadIdx.x < 64) {
        a = wave_sum(a);
        if (threadIdx.x == 0) sh[0] = 1.0f / sqrtf(a / (float)rs.d + rs.eps);
    }
    __syncthreads();
    return sh[0];
}

// sum over the 256 threads of a workgroup in a fixed order, written by thread 0
__device__ __forceinline__ void block256_row_sum(float v, float *dst) {
    __shared__ float red[4];
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) *dst = red[0] + red[1] + red[2] + red[3];
}

// bf16 family: x = E[token]; xg = half(x * gain) as GEMM input; ss[row] = sum of x^2 over the row
__global__ __launch_bounds__(256) void embed_prep_kernel(const bf16_t *E, const int32_t *tokens, float *x,
                                                          const float *gain, a16_t *xg, float *ss, int Mpad, int d,
                                                          int V, int32_t *flags) {
    const int m = blockIdx.x;
    int tok = tokens[m];
    if (tok < 0 || tok >= V) {
        if (threadIdx.x == 0) atomicOr(flags, FLAG_BAD_TOKEN);
        tok = 0;
    }
    typedef __attribute__((ext_vector_type(4))) uint32_t u4;
    typedef __attribute__((ext_vector_type(4))) float f4;
    float sq = 0.f;
    // a thread takes 8 consecutive columns (d is a multiple of 128): one 16-byte load, one 16-byte store of xg
    for (int k = threadIdx.x * 8; k < d; k += 256 * 8) {
        const u4 raw = *reinterpret_cast<const u4 *>(E + (size_t)tok * d + k);
        const f4 g0 = *reinterpret_cast<const f4 *>(gain + k), g1 = *reinterpret_cast<const f4 *>(gain + k + 4);
        float v[8];
#pragma unroll
        for (int q = 0; q < 4; ++q) { v[2 * q] = __uint_as_float(raw[q] << 16); v[2 * q + 1] = __uint_as_float(raw[q] & 0xffff0000u); }
        *reinterpret_cast<f4 *>(x + (size_t)m * d + k) = f4{v[0], v[1], v[2], v[3]};
        *reinterpret_cast<f4 *>(x + (size_t)m * d + k + 4) = f4{v[4], v[5], v[6], v[7]};
        const u4 pk = {f2a_pack_f(v[0] * g0[0], v[1] * g0[1], flags), f2a_pack_f(v[2] * g0[2], v[3] * g0[3], flags),
                       f2a_pack_f(v[4] * g1[0], v[5] * g1[1], flags), f2a_pack_f(v[6] * g1[2], v[7] * g1[3], flags)};
        *reinterpret_cast<u4 *>(xg + x_index<true>(m, k, d)) = pk;
#pragma unroll
        for (int q = 0; q < 8; ++q) sq += v[q] * v[q];
    }
    block256_row_sum(sq, ss + m);
}

int launch_embed_prep(hydra_ctx *c, hipStream_t s, const int32_t *tokens, float *x, const float *gain, void *xg,
                      float *ss, int Mpad, int M, int32_t *flags) {
    hipLaunchKernelGGL(embed_prep_kernel, dim3(M), dim3(256), 0, s, (const bf16_t *)(c->arena + c->off_embed), tokens, x,
                       gain, (a16_t *)xg, ss, Mpad, c->m.d, c->m.vocab, flags);
    HYDRA_LAUNCH_CHECK("embed_prep_kernel");
    return HYDRA_OK;
}

// hidden[m][k] = x[m][k] * rstd[m] * gain[k]   (final RMSNorm, fp32 output of tree_verify_forward)
__global__ __launch_bounds__(256) void final_hidden_kernel(const float *x, const float *gain, RowScale rs, float *hidden,
                                                            int d) {
    __shared__ float sh[1];
    const int m = blockIdx.x;
    const float r = row_rstd_block(rs, m, sh);
    for (int k = threadIdx.x; k < d; k += 256) hidden[(size_t)m * d + k] = x[(size_t)m * d + k] * r * gain[k];
}

int launch_final_hidden(hydra_ctx *c, hipStream_t s, const float *x, const float *gain, RowScale rs, float *hidden, int M) {
    hipLaunchKernelGGL(final_hidden_kernel, dim3(M), dim3(256), 0, s, x, gain, rs, hidden, c->m.d);
    HYDRA_LAUNCH_CHECK("final_hidden_kernel");
    return HYDRA_OK;
}

int launch_embed(hydra_ctx *c, hipStream_t s, const int32_t *tokens, float *x, int M, int32_t *flags) {
    const void *E = c->arena + c->off_embed;
    if (c->bf16) hipLaunchKernelGGL(embed_kernel<true>, dim3(M), dim3(256), 0, s, (const bf16_t *)E, tokens, x, c->m.d, c->m.vocab, flags);
    else         hipLaunchKernelGGL(embed_kernel<false>, dim3(M), dim3(256), 0, s, (const float *)E, tokens, x, c->m.d, c->m.vocab, flags);
    HYDRA_LAUNCH_CHECK("embed_kernel");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Residual add + RMSNorm.  x[m,:] += sum_s part[s][m,:]  (if S > 0), then
// out[m,k] = x[m,k] * gain[k] / sqrt(mean_k x^2 + eps), written as the next
// GEMM's input and, for the final norm, also as fp32 `hidden`.
// One workgroup per row; a thread keeps its <= 32 elements in registers.
// ---------------------------------------------------------------------------
template <bool BF>
__global__ __launch_bounds__(256) void rmsnorm_kernel(float *x, const float *part, int S, int part_ld,
                                                       size_t split_stride, const float *gain, float eps, int d,
                                                       typename Act<BF>::type *out, float *hidden) {
    const int m = blockIdx.x;
    float v[32];
    float ss = 0.f;
    int cnt = 0;
    for (int k = threadIdx.x; k < d; k += 256, ++cnt) {
        float a = x[(size_t)m * d + k];
        if (S > 0) {
            a += part_sum(part, S, split_stride, (size_t)m * part_ld + k);
            x[(size_t)m * d + k] = a;
        }
        v[cnt] = a;
        ss += a * a;
    }
    __shared__ float red[4];
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = red[0] + red[1] + red[2] + red[3];
    const float rstd = 1.0f / sqrtf(tot / (float)d + eps);
    cnt = 0;
    for (int k = threadIdx.x; k < d; k += 256, ++cnt) {
        const float y = v[cnt] * rstd * gain[k];
        Act<BF>::st(out, x_index<BF>(m, k, d), y);
        if (hidden) hidden[(size_t)m * d + k] = y;
    }
}

int launch_rmsnorm(hydra_ctx *c, hipStream_t s, float *x, const float *part, int S, int part_ld,
                   size_t split_stride, const float *gain, void *x_out, int M, float *hidden_out) {
    if (c->m.d > 32 * 256) return fail(HYDRA_E_UNSUPPORTED, "rmsnorm: d > 8192");
    if (c->bf16) hipLaunchKernelGGL(rmsnorm_kernel<true>, dim3(M), dim3(256), 0, s, x, part, S, part_ld, split_stride, gain, c->m.rms_eps, c->m.d, (a16_t *)x_out, hidden_out);
    else         hipLaunchKernelGGL(rmsnorm_kernel<false>, dim3(M), dim3(256), 0, s, x, part, S, part_ld, split_stride, gain, c->m.rms_eps, c->m.d, (float *)x_out, hidden_out);
    HYDRA_LAUNCH_CHECK("rmsnorm_kernel");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Rotary embedding of q and k at position seq_len[b] + depth[n], then
//   q -> attention input buffer, (k, v) -> cache slot seq_len[b] + n.
// Input: the QKV GEMM result, columns [0,d) = q, [d,2d) = k, [2d,3d) = v.
// One workgroup per (row m = b*T + n, head); thread j < Dh/2 owns the rotary
// pair (j, j + Dh/2).
//
// q buffer layout.  f32 family: [B][T][H][Dh] fp32.  bf16 family: per (b, head,
// 32-query tile qt) a run of Dh/16 blocks of 1 KiB in MFMA operand order:
// block s, lane = ((dim>>3)&1)*32 + query%32 holds dims (dim>>3)*8 .. +8.
// ---------------------------------------------------------------------------
template <bool BF>
__device__ __forceinline__ size_t q_index(int b, int n, int h, int dim, int H, int Dh, int T) {
    if (BF) {
        const int QT = (T + 31) >> 5, KS = Dh >> 4;
        const size_t blk = (((size_t)b * H + h) * QT + (n >> 5)) * KS + (dim >> 4);
        return ((blk * 64 + ((dim >> 3) & 1) * 32 + (n & 31)) << 3) + (dim & 7);
    } else {
        return (((size_t)b * T + n) * H + h) * Dh + dim;
    }
}

// 16-bit family: rounded to half with the saturation flag, as the fused epilogue of the q|k|v GEMM does
template <bool BF>
__device__ __forceinline__ void qkv_store(typename Act<BF>::type *p, size_t i, float v, int32_t *flags) {
    if constexpr (BF) p[i] = f2a_f(v, flags);
    else p[i] = v;
}

template <bool BF>
__global__ void rope_append_kernel(const float *part, int S, int part_ld, size_t split_stride, RowScale rs, const TreeDev *tree,
                                   const float *rope, const int32_t *seq_len, const int32_t *page_table,
                                   int max_pages, int n_pages, int layer, typename Act<BF>::type *kpages,
                                   typename Act<BF>::type *vpages, typename Act<BF>::type *qbuf, int d, int H,
                                   int Dh, int max_pos, int32_t *flags) {
    const int T = tree->T;
    const int m = blockIdx.x, h = blockIdx.y;
    const int b = m / T, n = m - b * T;
    const int L = seq_len[b];
    const int slot = L + n;
    const int pos = L + tree->depth[n];
    const bool ok = L >= 0 && (L + T) <= max_pages * 16 && (L + tree->max_depth) < max_pos;
    if (!ok) {
        if (threadIdx.x == 0) atomicOr(flags, FLAG_CAPACITY);
        return;
    }
    __shared__ float sh[1];
    const float r = row_rstd_block(rs, m, sh);
    const int half = Dh >> 1;
    const int j = threadIdx.x;
    if (j >= half) return;
    const size_t row = (size_t)m * part_ld;
    const int c0 = h * Dh + j, c1 = c0 + half;                  // v columns (and q, k in the fp32 family): the natural order
    // 16-bit family: the q and k weight bands of a head are packed so that the bands holding dims j and j + Dh/2 are
    // neighbours (pack_weight_kernel, bph > 1): dim j < Dh/2 sits in band 2 * (j / 32), dim j + Dh/2 in the band behind it
    const int p0 = BF ? h * Dh + 2 * (j >> 5) * 32 + (j & 31) : c0, p1 = BF ? p0 + 32 : c1;
    const float q0 = r * part_sum(part, S, split_stride, row + p0), q1 = r * part_sum(part, S, split_stride, row + p1);
    const float k0 = r * part_sum(part, S, split_stride, row + d + p0), k1 = r * part_sum(part, S, split_stride, row + d + p1);
    const float v0 = r * part_sum(part, S, split_stride, row + 2 * d + c0), v1 = r * part_sum(part, S, split_stride, row + 2 * d + c1);
    const float cs = rope[((size_t)pos * half + j) * 2], sn = rope[((size_t)pos * half + j) * 2 + 1];
    qkv_store<BF>(qbuf, q_index<BF>(b, n, h, j, H, Dh, T), q0 * cs - q1 * sn, flags);
    qkv_store<BF>(qbuf, q_index<BF>(b, n, h, j + half, H, Dh, T), q1 * cs + q0 * sn, flags);
    const int page = page_table[(size_t)b * max_pages + (slot >> 4)];
    if ((unsigned)page >= (unsigned)n_pages) { atomicOr(flags, FLAG_BAD_PAGE); return; }      // bad table entry: the row's K/V are not written
    const int tok = slot & 15;
    const size_t base = kv_block_base(layer, n_pages, page, H, h, Dh);
    qkv_store<BF>(kpages, base + k_in_block<BF>(tok, j, Dh), k0 * cs - k1 * sn, flags);
    qkv_store<BF>(kpages, base + k_in_block<BF>(tok, j + half, Dh), k1 * cs + k0 * sn, flags);
    qkv_store<BF>(vpages, base + v_in_block<BF>(tok, j, Dh), v0, flags);
    qkv_store<BF>(vpages, base + v_in_block<BF>(tok, j + half, Dh), v1, flags);
}

int launch_rope_append(hydra_ctx *c, hipStream_t s, const float *part, int S, int part_ld, size_t split_stride,
                       RowScale rs, int B, int layer, const int32_t *seq_len, const hydra_kv *kv, void *qbuf,
                       int32_t *flags) {
    const int T = c->tree.T;
    dim3 grid(B * T, c->m.n_heads), block(64);
    // the bf16 family does this step in the epilogue of its q|k|v GEMM unless the plan splits K (launch_gemm_qkv_rope)
    if (c->bf16) {
        hipLaunchKernelGGL(rope_append_kernel<true>, grid, block, 0, s, part, S, part_ld, split_stride, rs, tree_dev(c), rope_dev(c), seq_len, kv->page_table, kv->max_pages, kv->n_pages, layer, (a16_t *)kv->k_pages, (a16_t *)kv->v_pages, (a16_t *)qbuf, c->m.d, c->m.n_heads, c->m.head_dim, c->m.max_pos, flags);
        HYDRA_LAUNCH_CHECK("rope_append_kernel");
        return HYDRA_OK;
    }
    hipLaunchKernelGGL(rope_append_kernel<false>, grid, block, 0, s, part, S, part_ld, split_stride, rs, tree_dev(c), rope_dev(c), seq_len, kv->page_table, kv->max_pages, kv->n_pages, layer, (float *)kv->k_pages, (float *)kv->v_pages, (float *)qbuf, c->m.d, c->m.n_heads, c->m.head_dim, c->m.max_pos, flags);
    HYDRA_LAUNCH_CHECK("rope_append_kernel");
    return HYDRA_OK;
}

// fp32 [B,T,H,Dh] q (already rotated) -> attention input buffer (tree_attention entry point)
template <bool BF>
__global__ void q_import_kernel(const float *q, typename Act<BF>::type *qbuf, int T, int H, int Dh) {
    const int m = blockIdx.x, h = blockIdx.y;
    const int b = m / T, n = m - b * T;
    for (int dim = threadIdx.x; dim < Dh; dim += blockDim.x)
        Act<BF>::st(qbuf, q_index<BF>(b, n, h, dim, H, Dh, T), q[(((size_t)m) * H + h) * Dh + dim]);
}

int launch_q_import(hydra_ctx *c, hipStream_t s, int B, const float *q_plain, void *qbuf) {
    dim3 grid(B * c->tree.T, c->m.n_heads), block(64);
    if (c->bf16) hipLaunchKernelGGL(q_import_kernel<true>, grid, block, 0, s, q_plain, (a16_t *)qbuf, c->tree.T, c->m.n_heads, c->m.head_dim);
    else         hipLaunchKernelGGL(q_import_kernel<false>, grid, block, 0, s, q_plain, (float *)qbuf, c->tree.T, c->m.n_heads, c->m.head_dim);
    HYDRA_LAUNCH_CHECK("q_import_kernel");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// SwiGLU: act[m,f] = SiLU(gate[m,f]) * up[m,f].  The gate/up GEMM output holds
// gate feature f in column (f / blk) * 2 blk + f % blk and up feature f `blk`
// columns further (blk = 32 for the tile-interleaved bf16 weights, blk = F for
// the fp32 family, where the rows are simply [gate ; up]).
// ---------------------------------------------------------------------------
template <bool BF>
__global__ void silu_mul_kernel(const float *part, int S, int part_ld, size_t split_stride, int F, int blk,
                                typename Act<BF>::type *out) {
    const int m = blockIdx.y;
    const int f = blockIdx.x * blockDim.x + threadIdx.x;
    if (f >= F) return;
    const int gc = (f / blk) * 2 * blk + (f % blk);
    const size_t row = (size_t)m * part_ld;
    const float g = part_sum(part, S, split_stride, row + gc);
    const float u = part_sum(part, S, split_stride, row + gc + blk);
    Act<BF>::st(out, x_index<BF>(m, f, F), silu_f(g) * u);
}

int launch_silu_mul(hydra_ctx *c, hipStream_t s, const float *part, int S, int part_ld, size_t split_stride,
                    void *x_out, int M) {
    const int F = c->m.ffn;
    dim3 grid(ceil_div(F, 256), M), block(256);
    if (c->bf16) hipLaunchKernelGGL(silu_mul_kernel<true>, grid, block, 0, s, part, S, part_ld, split_stride, F, 16, (a16_t *)x_out);
    else         hipLaunchKernelGGL(silu_mul_kernel<false>, grid, block, 0, s, part, S, part_ld, split_stride, F, F, (float *)x_out);
    HYDRA_LAUNCH_CHECK("silu_mul_kernel");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// LM head epilogue: per row, logits = sum of split-K partials; greedy token =
// lowest id among the maxima; margin = top-1 minus top-2 value.
// ---------------------------------------------------------------------------

// One workgroup of 1024 threads per row.  VEC: rows of `part` are 16-byte aligned (row stride a multiple
// of 4), so a thread takes four consecutive logits per load and keeps four loads in flight.
template <bool VEC>
__global__ __launch_bounds__(1024) void argmax_kernel(const float *__restrict__ part, int S, int part_ld, size_t split_stride,
                                                       RowScale rs, int V, int32_t *argmax, float *margin,
                                                       float *__restrict__ logits) {
    typedef __attribute__((ext_vector_type(4))) float f4;
    const int m = blockIdx.x;
    __shared__ float sh[1];
    const float r = row_rstd_block(rs, m, sh);
    Top2 t = {-INFINITY, 0x7fffffff, -INFINITY};
    const float *row = part + (size_t)m * part_ld;
    if (VEC) {
        const int V4 = (V + 3) >> 2;                       // the last group may reach into the row padding (part_ld >= V rounded up to 4)
        for (int g0 = threadIdx.x; g0 < V4; g0 += 4 * 1024) {
            f4 x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int g = g0 + u * 1024;
                x[u] = f4{0.f, 0.f, 0.f, 0.f};
                if (g < V4)
                    for (int sp = 0; sp < S; ++sp) x[u] += *reinterpret_cast<const f4 *>(row + (size_t)sp * split_stride + 4 * g);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int g = g0 + u * 1024;
                if (g >= V4) continue;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int v = 4 * g + e;
                    if (v >= V) continue;
                    const float y = r * x[u][e];
                    if (logits) logits[(size_t)m * V + v] = y;
                    top2_push(t, y, v);
                }
            }
        }
    } else {
        for (int v = threadIdx.x; v < V; v += 1024) {
            const float x = r * part_sum(part, S, split_stride, (size_t)m * part_ld + v);
            if (logits) logits[(size_t)m * V + v] = x;
            top2_push(t, x, v);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        Top2 u = {__shfl_xor(t.v1, o, 64), __shfl_xor(t.i1, o, 64), __shfl_xor(t.v2, o, 64)};
        top2_merge(t, u);
    }
    __shared__ Top2 red[16];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
        Top2 q = red[0];
        for (int w = 1; w < 16; ++w) top2_merge(q, red[w]);
        argmax[m] = q.i1;
        if (margin) margin[m] = q.v1 - q.v2;
    }
}

int launch_argmax(hydra_ctx *c, hipStream_t s, const float *part, int S, int part_ld, size_t split_stride, RowScale rs,
                  int M, int32_t *argmax, float *margin, float *logits) {
    const bool vec = part_ld % 4 == 0 && split_stride % 4 == 0 && part_ld >= (c->m.vocab + 3) / 4 * 4;
    if (vec) hipLaunchKernelGGL(argmax_kernel<true>, dim3(M), dim3(1024), 0, s, part, S, part_ld, split_stride, rs, c->m.vocab, argmax, margin, logits);
    else     hipLaunchKernelGGL(argmax_kernel<false>, dim3(M), dim3(1024), 0, s, part, S, part_ld, split_stride, rs, c->m.vocab, argmax, margin, logits);
    HYDRA_LAUNCH_CHECK("argmax_kernel");
    return HYDRA_OK;
}

// The same result from the per-band candidates that the LM-head GEMM's own epilogue leaves when the logits are not
// asked for (EpiTop2): cand[band][Mpad] = (largest sum of the band, its column, second largest), unscaled.  One
// workgroup per row merges the bands (value descending, then column ascending) after scaling by the row's 1/rms, which
// is computed exactly as argmax_kernel computes it, so the margin has the same bits as on that path; the column can
// differ from it only where two different sums round to the same scaled value (a tie after scaling: that path then
// reports the lower column of the two, this one the column of the larger unscaled sum; the margin is 0 on both).
__global__ __launch_bounds__(256) void argmax_bands_kernel(const float4 *__restrict__ cand, int bands, int Mpad, RowScale rs,
                                                           int32_t *argmax, float *margin) {
    const int m = blockIdx.x;
    __shared__ float sh[1];
    const float r = row_rstd_block(rs, m, sh);
    Top2 t = {-INFINITY, 0x7fffffff, -INFINITY};
    for (int b = threadIdx.x; b < bands; b += 256) {
        const float4 c = cand[(size_t)b * Mpad + m];
        const Top2 u = {r * c.x, __float_as_int(c.y), r * c.z};
        top2_merge(t, u);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        Top2 u = {__shfl_xor(t.v1, o, 64), __shfl_xor(t.i1, o, 64), __shfl_xor(t.v2, o, 64)};
        top2_merge(t, u);
    }
    __shared__ Top2 red[4];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
        Top2 q = red[0];
        for (int w = 1; w < 4; ++w) top2_merge(q, red[w]);
        argmax[m] = q.i1;
        if (margin) margin[m] = q.v1 - q.v2;
    }
}

int launch_argmax_bands(hydra_ctx *c, hipStream_t s, const float *cand, int bands, int Mpad, RowScale rs, int M, int32_t *argmax,
                        float *margin) {
    (void)c;
    hipLaunchKernelGGL(argmax_bands_kernel, dim3(M), dim3(256), 0, s, reinterpret_cast<const float4 *>(cand), bands, Mpad, rs, argmax, margin);
    HYDRA_LAUNCH_CHECK("argmax_bands_kernel");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Plain [B][n_slots][2][H][Dh] fp32 <-> in-page cache placement (test harness).
// ---------------------------------------------------------------------------
template <bool BF, bool WRITE>
__global__ void kv_plain_kernel(typename Act<BF>::type *kpages, typename Act<BF>::type *vpages,
                                const int32_t *page_table, int max_pages, int n_pages, int layer, int first_slot,
                                int n_slots, int H, int Dh, float *plain, int32_t *flags) {
    const int b = blockIdx.z, i = blockIdx.x, h = blockIdx.y;
    const int slot = first_slot + i;
    const int page = page_table[(size_t)b * max_pages + (slot >> 4)];
    if ((unsigned)page >= (unsigned)n_pages) { if (threadIdx.x == 0) atomicOr(flags, FLAG_BAD_PAGE); return; }
    const int tok = slot & 15;
    const size_t base = kv_block_base(layer, n_pages, page, H, h, Dh);
    float *pk = plain + ((((size_t)b * n_slots + i) * 2 + 0) * H + h) * Dh;
    float *pv = plain + ((((size_t)b * n_slots + i) * 2 + 1) * H + h) * Dh;
    for (int dim = threadIdx.x; dim < Dh; dim += blockDim.x) {
        if (WRITE) {
            Act<BF>::st(kpages, base + k_in_block<BF>(tok, dim, Dh), pk[dim]);
            Act<BF>::st(vpages, base + v_in_block<BF>(tok, dim, Dh), pv[dim]);
        } else {
            pk[dim] = Act<BF>::ld(kpages, base + k_in_block<BF>(tok, dim, Dh));
            pv[dim] = Act<BF>::ld(vpages, base + v_in_block<BF>(tok, dim, Dh));
        }
    }
}

int launch_kv_plain(hydra_ctx *c, hipStream_t s, int B, int layer, const hydra_kv *kv, int first_slot, int n_slots,
                    float *plain, bool write_cache) {
    dim3 grid(n_slots, c->m.n_heads, B), block(64);
    const int H = c->m.n_heads, Dh = c->m.head_dim;
#define KVP(BFv, Wv, TY)                                                                                             \
    hipLaunchKernelGGL((kv_plain_kernel<BFv, Wv>), grid, block, 0, s, (TY *)kv->k_pages, (TY *)kv->v_pages,           \
                       kv->page_table, kv->max_pages, kv->n_pages, layer, first_slot, n_slots, H, Dh, plain, flags_dev(c))
    if (c->bf16) { if (write_cache) KVP(true, true, a16_t); else KVP(true, false, a16_t); }
    else         { if (write_cache) KVP(false, true, float); else KVP(false, false, float); }
#undef KVP
    HYDRA_LAUNCH_CHECK("kv_plain_kernel");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Prefix attention (paper, section 3.1 item 3): the extra decoder layer is fed
// the base model's hidden states of the accepted tokens.  Row m = b*P + j of the
// layer input is hidden[b, path[b][min(j, n_acc[b]-1)]]: positions past the
// accepted length repeat the last accepted state (they sit after every valid
// position in the chain, so nothing valid can see them).  Leaves x and, in the
// 16-bit family, the GEMM input xg = half(x * gain) and the row's sum of
// squares, exactly as embed_prep_kernel does for token embeddings.
// ---------------------------------------------------------------------------
template <bool BF>
__global__ __launch_bounds__(256) void gather_prep_kernel(const float *__restrict__ hidden, int T_src,
                                                           const int32_t *__restrict__ path, const int32_t *__restrict__ n_acc,
                                                           int P, float *__restrict__ x, const float *__restrict__ gain,
                                                           a16_t *__restrict__ xg, float *__restrict__ ss, int Mpad, int d,
                                                           int32_t *flags) {
    typedef __attribute__((ext_vector_type(4))) uint32_t u4;
    typedef __attribute__((ext_vector_type(4))) float f4;
    const int m = blockIdx.x;
    const int b = m / P, j = m - b * P;
    int a = n_acc[b];
    if (a < 1 || a > P) {
        if (threadIdx.x == 0) atomicOr(flags, FLAG_BAD_PATH);
        a = a < 1 ? 1 : P;
    }
    int node = path[(size_t)b * P + (j < a ? j : a - 1)];
    if (node < 0 || node >= T_src) {
        if (threadIdx.x == 0) atomicOr(flags, FLAG_BAD_PATH);
        node = 0;
    }
    const float *src = hidden + ((size_t)b * T_src + node) * d;
    if (BF) {
        float sq = 0.f;
        for (int k = threadIdx.x * 8; k < d; k += 256 * 8) {          // d is a multiple of 128
            const f4 v0 = *reinterpret_cast<const f4 *>(src + k), v1 = *reinterpret_cast<const f4 *>(src + k + 4);
            const f4 g0 = *reinterpret_cast<const f4 *>(gain + k), g1 = *reinterpret_cast<const f4 *>(gain + k + 4);
            *reinterpret_cast<f4 *>(x + (size_t)m * d + k) = v0;
            *reinterpret_cast<f4 *>(x + (size_t)m * d + k + 4) = v1;
            const u4 pk = {f2a_pack_f(v0[0] * g0[0], v0[1] * g0[1], flags), f2a_pack_f(v0[2] * g0[2], v0[3] * g0[3], flags),
                           f2a_pack_f(v1[0] * g1[0], v1[1] * g1[1], flags), f2a_pack_f(v1[2] * g1[2], v1[3] * g1[3], flags)};
            *reinterpret_cast<u4 *>(xg + x_index<true>(m, k, d)) = pk;
            sq += v0[0] * v0[0] + v0[1] * v0[1] + v0[2] * v0[2] + v0[3] * v0[3] + v1[0] * v1[0] + v1[1] * v1[1] + v1[2] * v1[2] + v1[3] * v1[3];
        }
        block256_row_sum(sq, ss + m);
    } else {
        for (int k = threadIdx.x; k < d; k += 256) x[(size_t)m * d + k] = src[k];
    }
}

int launch_gather_prep(hydra_ctx *c, hipStream_t s, int B, const float *hidden, int T_src, const int32_t *path,
                       const int32_t *n_acc, float *x, const float *gain, void *xg, float *ss, int Mpad, int32_t *flags) {
    const int P = c->tree.T;
    if (c->bf16) hipLaunchKernelGGL(gather_prep_kernel<true>, dim3(B * P), dim3(256), 0, s, hidden, T_src, path, n_acc, P, x, gain, (a16_t *)xg, ss, Mpad, c->m.d, flags);
    else         hipLaunchKernelGGL(gather_prep_kernel<false>, dim3(B * P), dim3(256), 0, s, hidden, T_src, path, n_acc, P, x, gain, (a16_t *)xg, ss, Mpad, c->m.d, flags);
    HYDRA_LAUNCH_CHECK("gather_prep_kernel");
    return HYDRA_OK;
}

// h_out[b] = layer output at the last accepted position; seq_len[b] += n_acc[b].  Rows the layer kernels
// skipped for lack of cache capacity are left as they are.
__global__ __launch_bounds__(256) void prefix_select_kernel(const float *__restrict__ x, const int32_t *__restrict__ n_acc, int P,
                                                             int max_pages, int d, int32_t *seq_len, float *__restrict__ h_out) {
    const int b = blockIdx.x;
    const int L = seq_len[b];
    if (L < 0 || L + P > max_pages * 16) return;
    int a = n_acc[b];
    a = a < 1 ? 1 : (a > P ? P : a);
    const float *src = x + ((size_t)b * P + a - 1) * d;
    for (int k = threadIdx.x; k < d; k += 256) h_out[(size_t)b * d + k] = src[k];
    __syncthreads();                                        // every thread has read seq_len[b]
    if (threadIdx.x == 0) seq_len[b] = L + a;
}

int launch_prefix_select(hydra_ctx *c, hipStream_t s, int B, const float *x, const int32_t *n_acc, const hydra_kv *kv,
                         int32_t *seq_len, float *h_out) {
    hipLaunchKernelGGL(prefix_select_kernel, dim3(B), dim3(256), 0, s, x, n_acc, c->tree.T, kv->max_pages, c->m.d, seq_len, h_out);
    HYDRA_LAUNCH_CHECK("prefix_select_kernel");
    return HYDRA_OK;
}

}  // namespace hydra
