// bf16 storage family: launch plans and epilogues of the weight-streaming GEMM
// (kernel in gemm_bf16.h), and the kernels that bring plain row-major weights
// into its tile order.
#include "gemm_bf16.h"
#include "internal.h"

namespace hydra {

// rows of a lane's accumulator registers
__device__ __forceinline__ int acc_row(int mb, int v, int lane) { return mb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// rstd[r] for the 32*MB rows of this row group, from the per-band sums of squares
// ss[band][Mpad] left by the residual epilogue:  1 / sqrt(sum_band ss / d + eps).
// Every kw == 0 wave fills the whole scratch itself, so no barrier is needed.
template <int MB>
__device__ __forceinline__ void rstd_to_lds(float *lds, const float *ss, int nb, int Mpad, int row0, int d, float eps,
                                            int lane) {
    for (int r = lane; r < 32 * MB; r += 64) {
        const float *p = ss + row0 + r;
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
        int b = 0;
        for (; b + 4 <= nb; b += 4) {
            s0 += p[(size_t)b * Mpad]; s1 += p[(size_t)(b + 1) * Mpad];
            s2 += p[(size_t)(b + 2) * Mpad]; s3 += p[(size_t)(b + 3) * Mpad];
        }
        for (; b < nb; ++b) s0 += p[(size_t)b * Mpad];
        lds[r] = 1.0f / sqrtf(((s0 + s1) + (s2 + s3)) / (float)d + eps);
    }
}

// ---- epilogues --------------------------------------------------------------
// out[split][row][col] = acc
struct EpiPlain {
    float *out; int ld; size_t split_stride;
    template <int MB, int NT> __device__ void prologue(GemmTile<MB, NT> &, const GemmGeom &, int) const {}
    template <int MB, int NT> __device__ void operator()(GemmTile<MB, NT> &t, const GemmGeom &g) const {
        float *dst = out + (size_t)t.split * split_stride;
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            if (t.tile0 + i >= g.NTiles) continue;
            const int col = (t.tile0 + i) * 32 + (t.lane & 31);
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = acc_row(t.mb0 + a, v, t.lane);
                    if (row < g.M) dst[(size_t)row * ld + col] = t.acc[a][i][v];
                }
        }
    }
};

// Residual branch end: x += acc.  Also leaves what the next RMSNorm'd GEMM needs:
// xg = bf16(x * gain) in GEMM input order (the 1/rms factor commutes with the
// contraction and is applied by the consumer) and ss[band][row] = sum over the
// band's 32 columns of x^2.
struct EpiResid {
    float *x; int d; const float *gain; bf16_t *xg; float *ss; int Mpad;
    template <int MB, int NT> __device__ void prologue(GemmTile<MB, NT> &, const GemmGeom &, int) const {}
    template <int MB, int NT> __device__ void operator()(GemmTile<MB, NT> &t, const GemmGeom &g) const {
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            if (t.tile0 + i >= g.NTiles) continue;
            const int band = t.tile0 + i;
            const int col = band * 32 + (t.lane & 31);
            const float gn = gain[col];
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = acc_row(t.mb0 + a, v, t.lane);
                    float sq = 0.f;
                    if (row < g.M) {
                        const float xn = x[(size_t)row * d + col] + t.acc[a][i][v];
                        x[(size_t)row * d + col] = xn;
                        xg[x_index<true>(row, col, d)] = f2bf(xn * gn);
                        sq = xn * xn;
                    }
#pragma unroll
                    for (int o = 16; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);      // over the 32 columns of the band
                    if ((t.lane & 31) == 0 && row < g.M) ss[(size_t)band * Mpad + row] = sq;
                }
        }
    }
};

// SwiGLU: bands (2j, 2j+1) hold gate and up of features 32j..32j+31.
// act = SiLU(r * gate) * (r * up) with r = rstd[row] of the RMSNorm that feeds this GEMM.
struct EpiSilu {
    const float *ss; int nb; int Mpad; int dmodel; float eps; bf16_t *act; int F;
    template <int MB, int NT> __device__ void prologue(GemmTile<MB, NT> &t, const GemmGeom &, int wave) const {
        (void)wave;
        rstd_to_lds<MB>(t.lds, ss, nb, Mpad, t.mb0 * 32, dmodel, eps, t.lane);
    }
    template <int MB, int NT> __device__ void operator()(GemmTile<MB, NT> &t, const GemmGeom &g) const {
        static_assert(NT == 2, "gate/up pairs need two bands per wave");
        const int f = (t.tile0 >> 1) * 32 + (t.lane & 31);
#pragma unroll
        for (int a = 0; a < MB; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = acc_row(t.mb0 + a, v, t.lane);
                if (row >= g.M) continue;
                const float r = t.lds[row - t.mb0 * 32];
                act[x_index<true>(row, f, F)] = f2bf(silu_f(r * t.acc[a][0][v]) * (r * t.acc[a][1][v]));
            }
    }
};

// Draft-head MLP layer: z = (residual ? z : 0) + SiLU(acc + bias), fp32 and as next GEMM input
struct EpiBiasSilu {
    const float *bias; float *z; int d; int residual; bf16_t *xg;
    template <int MB, int NT> __device__ void prologue(GemmTile<MB, NT> &, const GemmGeom &, int) const {}
    template <int MB, int NT> __device__ void operator()(GemmTile<MB, NT> &t, const GemmGeom &g) const {
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            if (t.tile0 + i >= g.NTiles) continue;
            const int col = (t.tile0 + i) * 32 + (t.lane & 31);
            const float bv = bias[col];
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = acc_row(t.mb0 + a, v, t.lane);
                    if (row >= g.M) continue;
                    float y = silu_f(t.acc[a][i][v] + bv);
                    if (residual) y += z[(size_t)row * d + col];
                    z[(size_t)row * d + col] = y;
                    xg[x_index<true>(row, col, d)] = f2bf(y);
                }
        }
    }
};

// ---- launch plans ---------------------------------------------------------------
int gemm_npad(const hydra_ctx *c, int N) { return c->bf16 ? ceil_div(N, 32) * 32 : N; }

// A workgroup is NW x KW waves of up to 8; the grid should cover every CU (256) at
// least once, and a wave should own at least 8 k-steps.  `pairs`: NT must be 2.
GemmPlan plan_gemm(const hydra_ctx *c, int M, int N, int K, bool pairs, bool allow_split) {
    GemmPlan p;
    p.splits = 1;
    if (!c->bf16) { p.mb = 1; p.nt = 1; p.nw = 1; p.kw = 1; p.kpw = K; return p; }
    const int mblocks = ceil_div(M, 32);
    p.mb = mblocks >= 4 ? 4 : (mblocks >= 2 ? 2 : 1);
    const int bands = ceil_div(N, 32), KT = K / 16;
    p.nt = (pairs || bands >= 512) ? 2 : 1;
    const int groups = ceil_div(bands, p.nt);
    p.nw = 1;
    p.kw = 4;
    while (p.kw > 1 && KT / p.kw < 8) p.kw >>= 1;
    // many row groups (large batch): workgroups are plentiful, share X between N-waves instead of splitting K
    const int mgroups = ceil_div(mblocks, p.mb);
    if (mgroups >= 2) { p.nw = 2; p.kw = 2; }
    int wgs = ceil_div(groups, p.nw) * mgroups;
    if (wgs < 256 && p.kw == 4 && KT / 8 >= 8) p.kw = 8;      // few workgroups: more waves (bytes in flight) per CU
    if (allow_split && wgs < 192) {
        int s = (256 + wgs - 1) / wgs;
        while (s > 1 && KT / (p.kw * s) < 8) --s;
        p.splits = s;
    }
    p.kpw = ceil_div(KT, p.kw * p.splits);
    return p;
}

int launch_gemm_f32(hydra_ctx *c, hipStream_t s, const float *X, const float *W, float *part, int M, int N, int K);

template <class Epi>
static int launch_bf16(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K,
                       const GemmPlan &p, const Epi &epi) {
    GemmGeom g;
    g.X = (const u32x4_t *)X; g.W = (const u32x4_t *)W;
    g.M = M; g.NTiles = ceil_div(N, 32); g.KT = K / 16; g.kpw = p.kpw; g.NW = p.nw; g.KW = p.kw;
    const int groups = ceil_div(g.NTiles, p.nt);
    dim3 grid(ceil_div(groups, p.nw), p.splits, ceil_div(ceil_div(M, 32), p.mb)), block(p.nw * p.kw * 64);
    const size_t lds = ((size_t)GEMM_LDS_SCRATCH + (size_t)(p.kw / 2) * p.nw * p.mb * p.nt * 16 * 64) * 4;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (c->profiling) {
        if (c->ev_used + 2 > c->ev.size())
            for (int i = 0; i < 2; ++i) { hipEvent_t e; HYDRA_HIP(hipEventCreate(&e)); c->ev.push_back(e); }
        e0 = c->ev[c->ev_used++]; e1 = c->ev[c->ev_used++];
        HYDRA_HIP(hipEventRecord(e0, s));
    }
#define GEMM_CASE(MBv, NTv)                                                                                          \
    hipLaunchKernelGGL((gemm_bf16_kernel<MBv, NTv, 512, Epi>), grid, block, lds, s, g, epi)
    if (p.mb == 1 && p.nt == 1) GEMM_CASE(1, 1);
    else if (p.mb == 1 && p.nt == 2) GEMM_CASE(1, 2);
    else if (p.mb == 2 && p.nt == 1) GEMM_CASE(2, 1);
    else if (p.mb == 2 && p.nt == 2) GEMM_CASE(2, 2);
    else if (p.mb == 4 && p.nt == 1) GEMM_CASE(4, 1);
    else GEMM_CASE(4, 2);
#undef GEMM_CASE
    HYDRA_LAUNCH_CHECK("gemm_bf16_kernel");
    if (c->profiling) {
        HYDRA_HIP(hipEventRecord(e1, s));
        c->prof_bytes += (double)N * K * 2;
        c->prof_launches += 1;
    }
    return HYDRA_OK;
}

// SiLU epilogue needs NT == 2: instantiate only those
static int launch_bf16_silu(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K,
                            const GemmPlan &p, const EpiSilu &epi) {
    GemmGeom g;
    g.X = (const u32x4_t *)X; g.W = (const u32x4_t *)W;
    g.M = M; g.NTiles = ceil_div(N, 32); g.KT = K / 16; g.kpw = p.kpw; g.NW = p.nw; g.KW = p.kw;
    const int groups = ceil_div(g.NTiles, 2);
    dim3 grid(ceil_div(groups, p.nw), 1, ceil_div(ceil_div(M, 32), p.mb)), block(p.nw * p.kw * 64);
    const size_t lds = ((size_t)GEMM_LDS_SCRATCH + (size_t)(p.kw / 2) * p.nw * p.mb * 2 * 16 * 64) * 4;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (c->profiling) {
        if (c->ev_used + 2 > c->ev.size())
            for (int i = 0; i < 2; ++i) { hipEvent_t e; HYDRA_HIP(hipEventCreate(&e)); c->ev.push_back(e); }
        e0 = c->ev[c->ev_used++]; e1 = c->ev[c->ev_used++];
        HYDRA_HIP(hipEventRecord(e0, s));
    }
    if (p.mb == 1) hipLaunchKernelGGL((gemm_bf16_kernel<1, 2, 512, EpiSilu>), grid, block, lds, s, g, epi);
    else if (p.mb == 2) hipLaunchKernelGGL((gemm_bf16_kernel<2, 2, 512, EpiSilu>), grid, block, lds, s, g, epi);
    else hipLaunchKernelGGL((gemm_bf16_kernel<4, 2, 512, EpiSilu>), grid, block, lds, s, g, epi);
    HYDRA_LAUNCH_CHECK("gemm_bf16_kernel<silu>");
    if (c->profiling) {
        HYDRA_HIP(hipEventRecord(e1, s));
        c->prof_bytes += (double)N * K * 2;
        c->prof_launches += 1;
    }
    return HYDRA_OK;
}

// part[split][m][n]  (fp32 family: one split, plain row-major operands)
int launch_gemm(hydra_ctx *c, hipStream_t s, const void *X, const void *W, float *part, int M, int N, int K,
                GemmPlan *plan_out) {
    GemmPlan p = plan_gemm(c, M, N, K, false, true);
    if (plan_out) *plan_out = p;
    if (!c->bf16) return launch_gemm_f32(c, s, (const float *)X, (const float *)W, part, M, N, K);
    const int npad = gemm_npad(c, N);
    EpiPlain epi{part, npad, (size_t)ceil_div(M, 32) * 32 * npad};
    return launch_bf16(c, s, X, W, M, N, K, p, epi);
}

int launch_gemm_resid(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K, float *x,
                      const float *gain, void *xg, float *ss, int Mpad) {
    GemmPlan p = plan_gemm(c, M, N, K, false, false);
    EpiResid epi{x, N, gain, (bf16_t *)xg, ss, Mpad};
    return launch_bf16(c, s, X, W, M, N, K, p, epi);
}

int launch_gemm_silu(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int F, int K, const float *ss,
                     int nb, int Mpad, void *act) {
    GemmPlan p = plan_gemm(c, M, 2 * F, K, true, false);
    EpiSilu epi{ss, nb, Mpad, K, c->m.rms_eps, (bf16_t *)act, F};
    return launch_bf16_silu(c, s, X, W, M, 2 * F, K, p, epi);
}

int launch_gemm_bias_silu(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K,
                          const float *bias, float *z, bool residual, void *xg) {
    GemmPlan p = plan_gemm(c, M, N, K, false, false);
    EpiBiasSilu epi{bias, z, N, residual ? 1 : 0, (bf16_t *)xg};
    return launch_bf16(c, s, X, W, M, N, K, p, epi);
}

int gemm_max_dynamic_lds(hydra_ctx *c) {
    (void)c;
    // opt in to the full LDS for every instantiation (a no-op for those that need less)
    hipError_t e = hipSuccess;
#define ATTR(MBv, NTv, E)                                                                                            \
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)gemm_bf16_kernel<MBv, NTv, 512, E>,                    \
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)
    ATTR(1, 1, EpiPlain); ATTR(1, 2, EpiPlain); ATTR(2, 1, EpiPlain); ATTR(2, 2, EpiPlain); ATTR(4, 1, EpiPlain); ATTR(4, 2, EpiPlain);
    ATTR(1, 1, EpiResid); ATTR(1, 2, EpiResid); ATTR(2, 1, EpiResid); ATTR(2, 2, EpiResid); ATTR(4, 1, EpiResid); ATTR(4, 2, EpiResid);
    ATTR(1, 1, EpiBiasSilu); ATTR(1, 2, EpiBiasSilu); ATTR(2, 1, EpiBiasSilu); ATTR(2, 2, EpiBiasSilu); ATTR(4, 1, EpiBiasSilu); ATTR(4, 2, EpiBiasSilu);
    ATTR(1, 2, EpiSilu); ATTR(2, 2, EpiSilu); ATTR(4, 2, EpiSilu);
#undef ATTR
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(gemm_bf16_kernel)");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Row-major [N][K] bf16 -> tile order.  Destination band = tile_off +
// band * tile_stride, so several source matrices can be interleaved band by
// band (q|k|v stacked; gate and up alternating).  Rows >= N of the last band
// are zero.  One thread writes one 16-byte lane entry.
// ---------------------------------------------------------------------------
__global__ void pack_weight_kernel(const bf16_t *__restrict__ src, u32x4_t *__restrict__ dst, int N, int K,
                                   int tile_off, int tile_stride) {
    const int KT = K >> 4;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;      // (band, kt, lane)
    const size_t total = (size_t)((N + 31) >> 5) * KT * 64;
    if (idx >= total) return;
    const int lane = (int)(idx & 63);
    const int kt = (int)((idx >> 6) % KT);
    const int band = (int)((idx >> 6) / KT);
    const int n = band * 32 + (lane & 31);
    const int k = kt * 16 + (lane >> 5) * 8;
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (n < N) v = *reinterpret_cast<const u32x4_t *>(src + (size_t)n * K + k);
    dst[((size_t)(tile_off + band * tile_stride) * KT + kt) * 64 + lane] = v;
}

int launch_pack_matrix(hydra_ctx *c, hipStream_t s, const void *src, void *dst, int N, int K, int tile_off,
                       int tile_stride, int) {
    (void)c;
    const size_t total = (size_t)ceil_div(N, 32) * (K / 16) * 64;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t *)src,
                       (u32x4_t *)dst, N, K, tile_off, tile_stride);
    HYDRA_LAUNCH_CHECK("pack_weight_kernel");
    return HYDRA_OK;
}

// plain copies into the arena (fp32 family matrices, embedding tables)
template <typename T>
__global__ void copy_rows_kernel(const T *src, T *dst, size_t rows, size_t cols, size_t dst_row_off, size_t dst_ld) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * cols) return;
    const size_t r = i / cols, cidx = i - r * cols;
    dst[(dst_row_off + r) * dst_ld + cidx] = src[i];
}

int launch_copy_matrix(hydra_ctx *c, hipStream_t s, const void *src, void *dst, size_t rows, size_t cols,
                       size_t dst_row_off, size_t dst_ld) {
    const size_t total = rows * cols;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (c->bf16) hipLaunchKernelGGL(copy_rows_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t *)src, (bf16_t *)dst, rows, cols, dst_row_off, dst_ld);
    else         hipLaunchKernelGGL(copy_rows_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float *)src, (float *)dst, rows, cols, dst_row_off, dst_ld);
    HYDRA_LAUNCH_CHECK("copy_rows_kernel");
    return HYDRA_OK;
}

template <bool BF>
__global__ void to_f32_kernel(const typename Elem<BF>::type *src, float *dst, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = Elem<BF>::ld(src, i);
}

int launch_to_f32(hydra_ctx *c, hipStream_t s, const void *src, float *dst, int n) {
    if (c->bf16) hipLaunchKernelGGL(to_f32_kernel<true>, dim3(ceil_div(n, 256)), dim3(256), 0, s, (const bf16_t *)src, dst, n);
    else         hipLaunchKernelGGL(to_f32_kernel<false>, dim3(ceil_div(n, 256)), dim3(256), 0, s, (const float *)src, dst, n);
    HYDRA_LAUNCH_CHECK("to_f32_kernel");
    return HYDRA_OK;
}

}  // namespace hydra
