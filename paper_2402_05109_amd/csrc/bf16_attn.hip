// bf16 storage family: tree attention on MFMA with split-KV, and the merge of
// the split results.
//
// Per (row b, head h) the T tree queries attend to slots [0, L) of the paged
// cache and to the tree slots allowed by each query's ancestor bitmask (paper,
// section 2, "Tree decoding").  All T queries share every K/V byte, so the cache
// is streamed once per (b, h) and both contractions run on the matrix cores:
//
//   S^T[key][query] = K[key][:] . Q[query][:]         A = K tile, B = Q^T
//   O^T[dim][query] += V^T[dim][key] * P^T[key][query] A = V^T tile, B = P^T
//
// Working with the transposes makes a query a COLUMN of every accumulator, so
// its softmax statistics, its ancestor mask and its rescale factor are per-lane
// scalars, and the exponentiated scores are already in the register order the
// second contraction needs for its B operand: no LDS, no shuffles except one
// exchange between the two half-waves.  The in-page placement of K and V (see
// device_common.h) is chosen so that both A operands are single coalesced
// 16-byte-per-lane loads straight from the cache pages.
//
// A wave is one "unit": it walks 32-key tiles unit, unit + U, ... of one
// (b, h, query group) and leaves (max, sum, O) for attn_merge_kernel.
#include "device_common.h"
#include "internal.h"

namespace hydra {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

__device__ __forceinline__ uint32_t pack2bf(float lo, float hi) { return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16); }

// record of one unit in the partial buffer: O[Tq][Dh], m[Tq], l[Tq]   (Tq = 32 * ceil(T/32))
__host__ __device__ inline size_t apart_record(int Tq, int Dh) { return (size_t)Tq * Dh + 2 * (size_t)Tq; }

template <int QT, int DH>
__global__ __launch_bounds__(256) void attn_bf16_kernel(const u32x4_t *__restrict__ qbuf,
                                                         const bf16_t *__restrict__ kpages,
                                                         const bf16_t *__restrict__ vpages,
                                                         const int32_t *__restrict__ page_table, int max_pages,
                                                         int n_pages, int layer, const int32_t *__restrict__ seq_len,
                                                         const TreeDev *__restrict__ tree, int H, int units, int QG,
                                                         float scale, float *__restrict__ apart, int32_t *flags) {
    constexpr int KS = DH / 16;      // k-steps of the score contraction
    constexpr int DT = DH / 32;      // 32-row bands of O^T
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int unit = blockIdx.x * 4 + wave;
    const int h = blockIdx.y;
    const int b = blockIdx.z / QG, qg = blockIdx.z - b * QG;
    const int T = tree->T;
    const int QTtot = (T + 31) >> 5;
    const int L = seq_len[b];
    if (L < 0 || L + T > max_pages * 16) {
        if (threadIdx.x == 0 && blockIdx.x == 0 && h == 0) atomicOr(flags, FLAG_CAPACITY);
        return;
    }
    const int total = L + T;
    const int n_tiles = (total + 31) >> 5;
    const int row_pages = (total + 15) >> 4;
    if (unit >= units || unit >= n_tiles) return;

    const int hl = lane >> 5, col = lane & 31;
    // Q^T operands and this lane's ancestor masks
    u32x4_t qreg[QT][KS];
    uint64_t anc0[QT], anc1[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int qtile = min(qg * QT + qt, QTtot - 1);
        const size_t blk = (((size_t)b * H + h) * QTtot + qtile) * KS;
#pragma unroll
        for (int s = 0; s < KS; ++s) qreg[qt][s] = qbuf[(blk + s) * 64 + lane];
        const int query = (qg * QT + qt) * 32 + col;
        anc0[qt] = query < T ? tree->anc[query][0] : 0ull;
        anc1[qt] = query < T ? tree->anc[query][1] : 0ull;
    }
    f32x16_t o[QT][DT];
    float m_run[QT], l_run[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        m_run[qt] = -INFINITY;
        l_run[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[qt][dt][v] = 0.f;
    }
    const int32_t *pt = page_table + (size_t)b * max_pages;

    for (int t = unit; t < n_tiles; t += units) {
        const int slot0 = t * 32;
        const bool page1_ok = 2 * t + 1 < row_pages;
        const int p0 = pt[2 * t];
        const int p1 = page1_ok ? pt[2 * t + 1] : p0;
        // ---- K tile: lane's key is col (page col/16, token col%16), half hl of every 16-dim step
        const int kpage = (col >> 4) ? p1 : p0;
        const u32x4_t *kp = reinterpret_cast<const u32x4_t *>(kpages + kv_block_base(layer, n_pages, kpage, H, h, DH));
        u32x4_t kreg[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) kreg[s] = kp[(2 * s + hl) * 16 + (col & 15)];
        // ---- V^T tiles: per page g and band dt, lane's dim is 32 dt + col, key half hl
        u32x4_t vreg[2][DT];
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            const u32x4_t *vp = reinterpret_cast<const u32x4_t *>(vpages + kv_block_base(layer, n_pages, g ? p1 : p0, H, h, DH));
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) vreg[g][dt] = vp[(32 * dt + col) * 2 + hl];
        }
        const bool tail = slot0 + 32 > total;
        if (tail) {     // zero V entries of slots >= total (stale or never written), so 0 * garbage cannot appear
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    // dword w holds keys i = 2w, 2w+1 of this half: token = 8*(i/4) + 4*hl + i%4
                    const int i0 = 2 * w, i1 = 2 * w + 1;
                    const int s0 = slot0 + 16 * g + 8 * (i0 >> 2) + 4 * hl + (i0 & 3);
                    const int s1 = slot0 + 16 * g + 8 * (i1 >> 2) + 4 * hl + (i1 & 3);
                    const uint32_t keep = (s0 < total ? 0x0000ffffu : 0u) | (s1 < total ? 0xffff0000u : 0u);
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) vreg[g][dt][w] &= keep;
                }
        }
        const bool need_mask = slot0 + 32 > L;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            f32x16_t sc;
#pragma unroll
            for (int v = 0; v < 16; ++v) sc[v] = 0.f;
#pragma unroll
            for (int s = 0; s < KS; ++s)
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, kreg[s]),
                                                            __builtin_bit_cast(bf16x8_t, qreg[qt][s]), sc, 0, 0, 0);
            float cmax = -INFINITY;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float x = sc[v] * scale;
                if (need_mask) {
                    const int slot = slot0 + 8 * (v >> 2) + 4 * hl + (v & 3);
                    bool ok = slot < L;
                    if (!ok) {
                        const int a = slot - L;
                        ok = a < T && (((a < 64 ? anc0[qt] >> a : anc1[qt] >> (a - 64)) & 1ull) != 0);
                    }
                    x = ok ? x : -INFINITY;
                }
                sc[v] = x;
                cmax = fmaxf(cmax, x);
            }
            cmax = fmaxf(cmax, __shfl_xor(cmax, 32, 64));
            const float m_new = fmaxf(m_run[qt], cmax);
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __expf(m_run[qt] - m_safe);
            float rs = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float p = __expf(sc[v] - m_safe);        // exp(-inf) = 0 for masked keys
                sc[v] = p;
                rs += p;
            }
            rs += __shfl_xor(rs, 32, 64);
            l_run[qt] = l_run[qt] * alpha + rs;
            m_run[qt] = m_new;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[qt][dt][v] *= alpha;
            // P^T operands: page g uses accumulator registers 8g .. 8g+7 in order
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                u32x4_t pb;
#pragma unroll
                for (int w = 0; w < 4; ++w) pb[w] = pack2bf(sc[8 * g + 2 * w], sc[8 * g + 2 * w + 1]);
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
                    o[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vreg[g][dt]),
                                                                       __builtin_bit_cast(bf16x8_t, pb), o[qt][dt], 0, 0, 0);
            }
        }
    }
    // ---- leave (O, m, l) of this unit
    const int Tq = QTtot * 32;
    float *rec = apart + ((((size_t)b * H + h) * units) + unit) * apart_record(Tq, DH);
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int query = (qg * QT + qt) * 32 + col;
        if (query >= Tq) continue;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                f32x4_t v4 = {o[qt][dt][4 * g4], o[qt][dt][4 * g4 + 1], o[qt][dt][4 * g4 + 2], o[qt][dt][4 * g4 + 3]};
                *reinterpret_cast<f32x4_t *>(rec + (size_t)query * DH + 32 * dt + 8 * g4 + 4 * hl) = v4;
            }
        if (hl == 0) {
            rec[(size_t)Tq * DH + query] = m_run[qt];
            rec[(size_t)Tq * DH + Tq + query] = l_run[qt];
        }
    }
}

// out[b, n, h, :] = sum_u w_u O_u[n] / sum_u w_u l_u,  w_u = exp(m_u - max_u m_u)
template <bool PACKED>
__global__ void attn_merge_kernel(const float *__restrict__ apart, const int32_t *__restrict__ seq_len, int T, int H,
                                  int Dh, int units, int max_pages, void *out) {
    const int n = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int L = seq_len[b];
    if (L < 0 || L + T > max_pages * 16) return;
    const int n_tiles = (L + T + 31) >> 5;
    const int nu = min(units, n_tiles);
    const int Tq = ((T + 31) >> 5) * 32;
    const size_t recsz = apart_record(Tq, Dh);
    const float *base = apart + (((size_t)b * H + h) * units) * recsz;
    float mt = -INFINITY;
    for (int u = 0; u < nu; ++u) mt = fmaxf(mt, base[u * recsz + (size_t)Tq * Dh + n]);
    float den = 0.f;
    for (int u = 0; u < nu; ++u) {
        const float *r = base + u * recsz;
        den += __expf(r[(size_t)Tq * Dh + n] - mt) * r[(size_t)Tq * Dh + Tq + n];
    }
    const float inv = 1.0f / den;
    for (int dim = threadIdx.x; dim < Dh; dim += blockDim.x) {
        float acc = 0.f;
        for (int u = 0; u < nu; ++u) {
            const float *r = base + u * recsz;
            acc += __expf(r[(size_t)Tq * Dh + n] - mt) * r[(size_t)n * Dh + dim];
        }
        const int m = b * T + n;
        if (PACKED) reinterpret_cast<bf16_t *>(out)[x_index<true>(m, h * Dh + dim, H * Dh)] = f2bf(acc * inv);
        else        reinterpret_cast<float *>(out)[((size_t)m * H + h) * Dh + dim] = acc * inv;
    }
}

int attn_units(const hydra_ctx *c, int B) {
    const int QG = ceil_div(ceil_div(c->tree.T, 32), 2);
    int u = 1024 / (B * c->m.n_heads * QG);
    if (u < 1) u = 1;
    if (u > 32) u = 32;
    return u;
}

int launch_attention_f32(hydra_ctx *c, hipStream_t s, int B, int layer, const float *q, const int32_t *seq_len,
                         const hydra_kv *kv, float *out, int32_t *flags);

// x_out != NULL: result as the next GEMM's input; plain_out != NULL: fp32 [B,T,H,Dh].
int launch_attention(hydra_ctx *c, hipStream_t s, int B, int layer, const void *qbuf, const int32_t *seq_len,
                     const hydra_kv *kv, float *apart, int units_max, void *x_out, float *plain_out, int32_t *flags) {
    if (!c->bf16) {
        float *dst = plain_out ? plain_out : (float *)x_out;     // the fp32 GEMM input order is [B,T,H,Dh] itself
        return launch_attention_f32(c, s, B, layer, (const float *)qbuf, seq_len, kv, dst, flags);
    }
    const int T = c->tree.T, H = c->m.n_heads, Dh = c->m.head_dim;
    const int QTtot = ceil_div(T, 32);
    const int QT = QTtot >= 2 ? 2 : 1;
    const int QG = ceil_div(QTtot, QT);
    // units: enough waves to fill the chip, but not more than one per two key tiles
    int units = units_max;
    if (kv->seq_len_hint > 0) {
        const int tiles = ceil_div(kv->seq_len_hint + T, 32);
        const int want = ceil_div(tiles, 2);
        if (want < units) units = want;
    }
    if (units < 1) units = 1;
    dim3 grid(ceil_div(units, 4), H, B * QG), block(256);
    const float scale = 1.0f / sqrtf((float)Dh);
#define ATTN_CASE(QTv, DHv)                                                                                          \
    hipLaunchKernelGGL((attn_bf16_kernel<QTv, DHv>), grid, block, 0, s, (const u32x4_t *)qbuf,                        \
                       (const bf16_t *)kv->k_pages, (const bf16_t *)kv->v_pages, kv->page_table, kv->max_pages,      \
                       kv->n_pages, layer, seq_len, tree_dev(c), H, units, QG, scale, apart, flags)
    if (QT == 1 && Dh == 128) ATTN_CASE(1, 128);
    else if (QT == 2 && Dh == 128) ATTN_CASE(2, 128);
    else if (QT == 1 && Dh == 64) ATTN_CASE(1, 64);
    else ATTN_CASE(2, 64);
#undef ATTN_CASE
    HYDRA_LAUNCH_CHECK("attn_bf16_kernel");
    dim3 mgrid(T, H, B), mblock(Dh);
    if (x_out) hipLaunchKernelGGL(attn_merge_kernel<true>, mgrid, mblock, 0, s, apart, seq_len, T, H, Dh, units, kv->max_pages, x_out);
    else       hipLaunchKernelGGL(attn_merge_kernel<false>, mgrid, mblock, 0, s, apart, seq_len, T, H, Dh, units, kv->max_pages, (void *)plain_out);
    HYDRA_LAUNCH_CHECK("attn_merge_kernel");
    return HYDRA_OK;
}

}  // namespace hydra
