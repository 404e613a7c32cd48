// bf16 storage family: tree attention on MFMA.
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
// second contraction needs for its B operand: no LDS and no shuffles in the
// loop except one exchange between the two half-waves.  The in-page placement
// of K and V (device_common.h) makes both A operands single coalesced
// 16-byte-per-lane loads straight from the cache pages.
//
// A workgroup is 8 waves on one (b, h).  Two launch shapes:
//   short contexts (up to ~1200 keys): one workgroup per 32-query tile; its 8
//     waves split the keys (32-key tiles taken round-robin, next tile prefetched
//     while the current one is multiplied), are merged through LDS, and the
//     result goes straight out as the next GEMM's input: one kernel, no partial
//     records.  A CU streams at most ~45 GB/s, which is what bounds this shape;
//   longer contexts: QW waves of a workgroup take different query tiles, 8/QW
//     waves split the keys, and several workgroups per (b, h) split the keys
//     further; each leaves a (max, sum, O) record that attn_merge_kernel combines.
#include <algorithm>

#include "attn_bf16.h"
#include "device_common.h"
#include "internal.h"

namespace hydra {

typedef __attribute__((ext_vector_type(4))) float f32x4_t;

template <int DH, bool PACKED>
__global__ __launch_bounds__(ATTN_WAVES * 64) void attn_bf16_kernel(
    const u32x4_t *__restrict__ qbuf, const a16_t *__restrict__ kpages, const a16_t *__restrict__ vpages,
    const int32_t *__restrict__ page_table, int max_pages, int n_pages, int layer, const int32_t *__restrict__ seq_len,
    const TreeDev *__restrict__ tree, int T, int H, int QW, int qsplit, float scale, float *__restrict__ apart, void *out,
    int32_t *flags) {
    extern __shared__ float lds[];
    attn_bf16_body<DH, PACKED, false, true>(qbuf, kpages, vpages, page_table, max_pages, n_pages, layer, seq_len, tree, T, H, QW, qsplit,
                                      scale, apart, out, flags, (int)blockIdx.x, (int)gridDim.x, (int)blockIdx.y, (int)blockIdx.z, lds, (int)threadIdx.x);
}

// out[b, n, h, :] = sum_u w_u O_u[n] / sum_u w_u l_u,  w_u = exp(m_u - max_u m_u).
// One workgroup per (row, head, 8 queries), one thread per (query, 4 dims); all loads of a thread are
// independent of each other and of the row length, so they make one round trip.
enum { MERGE_MAX_UNITS = 16 };
template <bool PACKED>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float *__restrict__ apart, const int32_t *__restrict__ seq_len,
                                                          int T, int H, int Dh, int units, int max_pages, void *out) {
    const int h = blockIdx.y, b = blockIdx.z;
    const int per_q = Dh >> 2;                              // threads per query
    const int n = blockIdx.x * (256 / per_q) + threadIdx.x / per_q;
    const int dim = (threadIdx.x % per_q) * 4;
    const int Tq = ((T + 31) >> 5) * 32;
    const size_t recsz = apart_record(Tq, Dh);
    const float *base = apart + (((size_t)b * H + h) * units) * recsz;
    const bool live = n < T;
    float mu[MERGE_MAX_UNITS], lu[MERGE_MAX_UNITS];
    f32x4_t ou[MERGE_MAX_UNITS];
#pragma unroll
    for (int u = 0; u < MERGE_MAX_UNITS; ++u) {
        mu[u] = -INFINITY; lu[u] = 0.f; ou[u] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (u < units && live) {
            const float *r = base + u * recsz;
            mu[u] = r[(size_t)Tq * Dh + n];
            lu[u] = r[(size_t)Tq * Dh + Tq + n];
            ou[u] = *reinterpret_cast<const f32x4_t *>(r + (size_t)n * Dh + dim);
        }
    }
    const int L = seq_len[b];
    if (L < 0 || L + T > max_pages * 16 || !live) return;
    float mt = -INFINITY;
#pragma unroll
    for (int u = 0; u < MERGE_MAX_UNITS; ++u) mt = fmaxf(mt, mu[u]);
    float den = 0.f;
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < MERGE_MAX_UNITS; ++u) {
        const float w = u < units ? __expf(mu[u] - mt) : 0.f;
        den += w * lu[u];
        acc += ou[u] * w;
    }
    const float inv = 1.0f / den;
    const int m = b * T + n;
    if (PACKED) {
        u32x2_t pk = {f2a_pack(acc[0] * inv, acc[1] * inv), f2a_pack(acc[2] * inv, acc[3] * inv)};
        *reinterpret_cast<u32x2_t *>(reinterpret_cast<a16_t *>(out) + x_index<true>(m, h * Dh + dim, H * Dh)) = pk;
    } else {
        *reinterpret_cast<f32x4_t *>(reinterpret_cast<float *>(out) + ((size_t)m * H + h) * Dh + dim) = acc * inv;
    }
}

// upper bound of workgroups per (b, h) that the partial buffer is sized for
int attn_units(const hydra_ctx *c, int B) {
    int u = 512 / (B * c->m.n_heads);
    if (u < 1) u = 1;
    if (u > MERGE_MAX_UNITS) u = MERGE_MAX_UNITS;
    return u;
}

int launch_attention_f32(hydra_ctx *c, hipStream_t s, int B, int layer, const float *q, const int32_t *seq_len,
                         const hydra_kv *kv, float *out, int32_t *flags);

static size_t attn_lds_bytes(int Dh) { return ((size_t)ATTN_WAVES * 64 + (size_t)ATTN_WAVES * (Dh / 32) * 16 * 64) * 4; }

int attn_max_dynamic_lds(hydra_ctx *c) {
    (void)c;
    hipError_t e = hipSuccess;
#define ATTR(DHv, Pv) if (e == hipSuccess) e = hipFuncSetAttribute((const void *)attn_bf16_kernel<DHv, Pv>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)
    ATTR(128, true); ATTR(128, false); ATTR(64, true); ATTR(64, false);
#undef ATTR
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(attn_bf16_kernel)");
    return HYDRA_OK;
}

// x_out != NULL: result as the next GEMM's input; plain_out != NULL: fp32 [B,T,H,Dh].
int launch_attention(hydra_ctx *c, hipStream_t s, int B, int layer, const void *qbuf, const int32_t *seq_len,
                     const hydra_kv *kv, float *apart, int units_max, void *x_out, float *plain_out, int32_t *flags) {
    if (!c->bf16) {
        float *dst = plain_out ? plain_out : (float *)x_out;     // the fp32 GEMM input order is [B,T,H,Dh] itself
        return launch_attention_f32(c, s, B, layer, (const float *)qbuf, seq_len, kv, dst, flags);
    }
    const int T = c->tree.T, H = c->m.n_heads, Dh = c->m.head_dim;
    const int QTtot = ceil_div(T, 32);
    int QW = QTtot >= 3 ? 4 : QTtot;                       // 1, 2 or 4 query waves
    int KWV = ATTN_WAVES / QW;
    const int len = kv->seq_len_hint > 0 ? kv->seq_len_hint : c->m.max_pos;
    const int tiles = ceil_div(len + T, 32);
    // Short contexts: one workgroup per 32-query tile, its 8 waves split the keys (up to five 32-key tiles each) and
    // the result goes straight out.  Longer ones: a CU streams at most ~45 GB/s, so the keys of one head are spread
    // over several workgroups (two tiles per wave or more) whose partial records attn_merge_kernel combines.
    int wgs = 1, qsplit = 0;
    // (only while those workgroups fit one round of the chip: at batch 8 and 16 one workgroup per (row, head) that
    // holds all query tiles and reads each K/V byte once measured 2-3 % faster on the whole verify step)
    if (tiles <= ATTN_WAVES * 5 && QTtot * H * B <= 256) {
        qsplit = 1; QW = 1; KWV = ATTN_WAVES; wgs = QTtot;
    } else {
        // ... but never more workgroups than one round of the chip: a workgroup holds a CU by itself (registers), so
        // a second round only repeats the fixed cost of a workgroup (first round trips, LDS merge, partial record).
        // Measured best at about 200 workgroups in all: 7B at 2066 / 4114 keys 4.30 -> 4.01 / 4.63 -> 4.30 ms per verify.
        wgs = ceil_div(tiles, KWV * 2);
        const int cap = std::max(1, 208 / (H * B));
        if (wgs > cap) wgs = cap;
        if (wgs > units_max) wgs = units_max;
        if (wgs < 1) wgs = 1;
    }
    dim3 grid(wgs, H, B), block(ATTN_WAVES * 64);
    const float scale = 1.0f / sqrtf((float)Dh);
    const size_t lds = attn_lds_bytes(Dh);
    void *out = x_out ? x_out : (void *)plain_out;
    const bool packed = x_out != nullptr;
#define ATTN_CASE(DHv, Pv)                                                                                           \
    hipLaunchKernelGGL((attn_bf16_kernel<DHv, Pv>), grid, block, lds, s, (const u32x4_t *)qbuf,                       \
                       (const a16_t *)kv->k_pages, (const a16_t *)kv->v_pages, kv->page_table, kv->max_pages,      \
                       kv->n_pages, layer, seq_len, tree_dev(c), T, H, QW, qsplit, scale, apart, out, flags)
    if (Dh == 128) { if (packed) ATTN_CASE(128, true); else ATTN_CASE(128, false); }
    else           { if (packed) ATTN_CASE(64, true); else ATTN_CASE(64, false); }
#undef ATTN_CASE
    HYDRA_LAUNCH_CHECK("attn_bf16_kernel");
    if (!qsplit && wgs > 1) {
        const int q_per_wg = 256 / (Dh / 4);
        dim3 mgrid(ceil_div(T, q_per_wg), H, B), mblock(256);
        if (packed) hipLaunchKernelGGL(attn_merge_kernel<true>, mgrid, mblock, 0, s, apart, seq_len, T, H, Dh, wgs, kv->max_pages, out);
        else        hipLaunchKernelGGL(attn_merge_kernel<false>, mgrid, mblock, 0, s, apart, seq_len, T, H, Dh, wgs, kv->max_pages, out);
        HYDRA_LAUNCH_CHECK("attn_merge_kernel");
    }
    return HYDRA_OK;
}

}  // namespace hydra
