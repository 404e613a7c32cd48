// bf16 storage family: launch plans and epilogues of the weight-streaming GEMM
// (kernel in gemm_bf16.h), and the kernels that bring plain row-major weights
// into its tile order.
#include <stdlib.h>

#include "gemm_bf16.h"
#include "internal.h"

namespace hydra {

// rows of a lane's accumulator registers
__device__ __forceinline__ int acc_row(int mb, int v, int lane) { return mb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// rstd[r] for the 32*MB rows of this row group, from the per-band sums of squares
// ss[band][Mpad] left by the residual epilogue:  1 / sqrt(sum_band ss / d + eps).
// All waves of the workgroup cooperate: wave w adds bands w, w + nwaves, ... for row = lane
// (independent loads, one round trip), the partial sums meet in LDS in a fixed order.
template <int MB>
__device__ __forceinline__ void rstd_to_lds(float *lds, const float *__restrict__ ss, int nb, int Mpad, int row0, int d,
                                            float eps, int lane, int wave) {
    const int nwaves = blockDim.x >> 6;
    float *partial = lds + 128;                               // [nwaves <= 8][up to 128 rows] would not fit: rows are done 64 at a time
    for (int r0 = 0; r0 < 32 * MB; r0 += 64) {
        const int r = r0 + lane;
        float acc = 0.f;
        if (r < 32 * MB) {
            float v[16];
            for (int b0 = wave; b0 < nb; b0 += 16 * nwaves) {
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int b = b0 + j * nwaves;
                    v[j] = b < nb ? ss[(size_t)b * Mpad + row0 + r] : 0.f;
                }
#pragma unroll
                for (int j = 0; j < 16; ++j) acc += v[j];
            }
        }
        partial[wave * 64 + lane] = acc;
        __syncthreads();
        if (wave == 0 && r < 32 * MB) {
            float t = 0.f;
            for (int w = 0; w < nwaves; ++w) t += partial[w * 64 + lane];
            lds[r] = 1.0f / sqrtf(t / (float)d + eps);
        }
        __syncthreads();
    }
}

// ---- epilogues (one 32x32 tile at a time; see gemm_bf16.h) -------------------------
// out[split][row][col] = acc
struct EpiPlain {
    float *out; int ld; size_t split_stride;
    template <int MB, int NT> __device__ void prologue(GemmTile<MB, NT> &, const GemmGeom &, int) const {}
    template <int MB, int NT>
    __device__ void tile(const f32x16_t &acc, int a, int i, const GemmTile<MB, NT> &t, const GemmGeom &g) const {
        if (t.tile0 + i >= g.NTiles) return;
        float *dst = out + (size_t)t.split * split_stride + (t.tile0 + i) * 32 + (t.lane & 31);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = acc_row(t.mb0 + a, v, t.lane);
            if (row < g.M) dst[(size_t)row * ld] = acc[v];
        }
    }
};

// Residual branch end: x += acc.  Also leaves what the next RMSNorm'd GEMM needs:
// xg = bf16(x * gain) in GEMM input order (the 1/rms factor commutes with the
// contraction and is applied by the consumer) and ss[band][row] = sum over the
// band's 32 columns of x^2.
struct EpiResid {
    float *x; int d; const float *gain; a16_t *xg; float *ss; int Mpad;
    template <int MB, int NT> __device__ void prologue(GemmTile<MB, NT> &, const GemmGeom &, int) const {}
    template <int MB, int NT>
    __device__ void tile(const f32x16_t &acc, int a, int i, const GemmTile<MB, NT> &t, const GemmGeom &g) const {
        if (t.tile0 + i >= g.NTiles) return;
        float *__restrict__ xp = x;
        a16_t *__restrict__ xgp = xg;
        float *__restrict__ ssp = ss;
        const int band = t.tile0 + i;
        const int col = band * 32 + (t.lane & 31);
        const float gn = gain[col];
        float xo[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {                                 // all loads first: one round trip
            const int row = acc_row(t.mb0 + a, v, t.lane);
            xo[v] = row < g.M ? xp[(size_t)row * d + col] : 0.f;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = acc_row(t.mb0 + a, v, t.lane);
            const float xn = xo[v] + acc[v];
            float sq = 0.f;
            if (row < g.M) {
                xp[(size_t)row * d + col] = xn;
                xgp[x_index<true>(row, col, d)] = f2a(xn * gn);
                sq = xn * xn;
            }
#pragma unroll
            for (int o = 16; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);      // over the 32 columns of the band
            if ((t.lane & 31) == 0 && row < g.M) ssp[(size_t)band * Mpad + row] = sq;
        }
    }
};

// SwiGLU.  The gate/up weight bands are interleaved at half-band granularity: band b holds
// gate features 16b..16b+15 in columns 0-15 and the same up features in columns 16-31, so every
// band is self-contained:  act = SiLU(r * gate) * (r * up)  with r = rstd[row] of the RMSNorm that
// feeds this GEMM.  Lanes of the left half finish rows v < 8 of a register set, lanes of the right
// half rows v >= 8, each fetching the partner value from the lane 16 columns away.
struct EpiSilu {
    const float *ss; int nb; int Mpad; int dmodel; float eps; a16_t *act; int F;
    template <int MB, int NT> __device__ void prologue(GemmTile<MB, NT> &t, const GemmGeom &, int wave) const {
        rstd_to_lds<MB>(t.lds, ss, nb, Mpad, t.mb0 * 32, dmodel, eps, t.lane, wave);
    }
    template <int MB, int NT>
    __device__ void tile(const f32x16_t &acc, int a, int i, const GemmTile<MB, NT> &t, const GemmGeom &g) const {
        if (t.tile0 + i >= g.NTiles) return;
        const int c = t.lane & 31;
        const bool left = c < 16;
        const int f = (t.tile0 + i) * 16 + (c & 15);
        a16_t *__restrict__ ap = act;
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            // left lanes need (gate = own acc[v], up = partner acc[v]); right lanes (gate = partner acc[v+8], up = own acc[v+8])
            const float send = left ? acc[v + 8] : acc[v];
            const float got = __shfl_xor(send, 16, 64);
            const float gate = left ? acc[v] : got;
            const float up = left ? got : acc[v + 8];
            const int row = acc_row(t.mb0 + a, left ? v : v + 8, t.lane);
            if (row >= g.M) continue;
            const float r = t.lds[row - t.mb0 * 32];
            ap[x_index<true>(row, f, F)] = f2a(silu_f(r * gate) * (r * up));
        }
    }
};

// Draft-head MLP layer: z = (residual ? z : 0) + SiLU(acc + bias), fp32 and as next GEMM input
struct EpiBiasSilu {
    const float *bias; float *z; int d; int residual; a16_t *xg;
    template <int MB, int NT> __device__ void prologue(GemmTile<MB, NT> &, const GemmGeom &, int) const {}
    template <int MB, int NT>
    __device__ void tile(const f32x16_t &acc, int a, int i, const GemmTile<MB, NT> &t, const GemmGeom &g) const {
        if (t.tile0 + i >= g.NTiles) return;
        const int col = (t.tile0 + i) * 32 + (t.lane & 31);
        const float bv = bias[col];
        float *__restrict__ zp = z;
        a16_t *__restrict__ xgp = xg;
        float zo[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = acc_row(t.mb0 + a, v, t.lane);
            zo[v] = (residual && row < g.M) ? zp[(size_t)row * d + col] : 0.f;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = acc_row(t.mb0 + a, v, t.lane);
            if (row >= g.M) continue;
            const float y = silu_f(acc[v] + bv) + zo[v];
            zp[(size_t)row * d + col] = y;
            xgp[x_index<true>(row, col, d)] = f2a(y);
        }
    }
};

// ---- launch plans ---------------------------------------------------------------
int gemm_npad(const hydra_ctx *c, int N) { return c->bf16 ? ceil_div(N, 32) * 32 : N; }

// Launch shapes.  Measured on MI355X: one CU pulls at most ~45 GB/s of L1-miss traffic, and the
// X tiles a wave reads count against it like the W tiles do; HBM needs ~24 GB/s of W per CU on all
// 256 CUs.  So a plan wants ~256 equally loaded workgroups and X bytes <= W bytes per workgroup:
// more bands per wave (NT) amortise X, and splitting K over workgroups (S) both adds workgroups and
// shrinks the X slice each one reads.  S > 1 leaves S partial outputs for the consumer to add.
static double env_or(const char *name, double dflt) {
    const char *v = getenv(name);
    return v ? atof(v) : dflt;
}

GemmPlan plan_gemm(const hydra_ctx *c, int M, int N, int K, int kind) {
    // model constants; the environment overrides exist for tuning runs only
    static const double cap_gbps = env_or("HYDRA_PLAN_CAP", 45.0);        // L1-miss bytes one CU can pull, GB/s
    static const double hbm_tbps = env_or("HYDRA_PLAN_HBM", 6.0);         // achievable HBM stream, TB/s
    static const double split_us = env_or("HYDRA_PLAN_SPLIT_US", 0.5);    // cost of reading one more partial back, us
    static const int max_split = (int)env_or("HYDRA_PLAN_MAX_SPLIT", 8);
    GemmPlan p;
    p.splits = 1;
    if (!c->bf16) { p.mb = 1; p.nt = 1; p.nw = 1; p.kw = 1; p.kpw = K; return p; }
    const int mblocks = ceil_div(M, 32);
    p.mb = mblocks >= 4 ? 4 : (mblocks >= 2 ? 2 : 1);
    const int mgroups = ceil_div(mblocks, p.mb);
    const int bands = ceil_div(N, 32), KT = K / 16;
    const bool pairs = false;
    const bool may_split = kind == GEMM_KIND_PLAIN;
    p.nw = 1;
    // bands per wave: accumulators MB*NT*16 plus two prefetch sets must fit the register file
    int nt_max = p.mb == 4 ? 2 : 4;
    int best_nt = pairs ? 2 : 1, best_s = 1;
    double best_cost = 1e30;
    for (int nt = pairs ? 2 : 1; nt <= nt_max; nt += pairs ? 2 : 1) {
        const int groups = ceil_div(bands, nt);
        for (int s = 1; s <= (may_split ? max_split : 1); ++s) {
            if (KT / s < 16 && s > 1) break;
            const int wgs = groups * s * mgroups;
            const int rounds = ceil_div(wgs, 256);                     // workgroups on the busiest CU
            const double w_bytes = (double)nt * 32 * K * 2 / s;         // per workgroup
            const double x_bytes = (double)p.mb * 32 * K * 2 / s;
            double cost = rounds * (w_bytes + x_bytes) / (cap_gbps * 1e3);   // us at the per-CU limit
            const double hbm = (double)N * K * 2 / (hbm_tbps * 1e6);         // us at the HBM limit
            if (cost < hbm) cost = hbm;
            cost += (s > 1 ? 1.0 + split_us * s : 0.0);                      // reading S partials back costs a little
            if (cost < best_cost - 1e-9) { best_cost = cost; best_nt = nt; best_s = s; }
        }
    }
    p.nt = best_nt;
    p.splits = best_s;
    const int max_waves = (p.mb * p.nt >= 6) ? 4 : 8;                   // 256-thread workgroups get 512 VGPRs per wave
    p.kw = max_waves;
    while (p.kw > 1 && KT / (p.kw * p.splits) < 4) p.kw >>= 1;
    while (p.kw > 1 && ((size_t)GEMM_LDS_SCRATCH + (size_t)p.kw * p.mb * p.nt * 16 * 64) * 4 > 150 * 1024) p.kw >>= 1;   // LDS: KW accumulator copies
    if (mgroups >= 2 && p.kw >= 2) { p.nw = 2; p.kw >>= 1; }            // large batch: share X between two N-waves
    p.kpw = ceil_div(KT, p.kw * p.splits);
    return p;
}

int launch_gemm_f32(hydra_ctx *c, hipStream_t s, const float *X, const float *W, float *part, int M, int N, int K);

template <int MB, int NT, class Epi>
static void launch_one(dim3 grid, dim3 block, size_t lds, hipStream_t s, const GemmGeom &g, const Epi &epi) {
    constexpr int MAXT = (MB * NT >= 6) ? 256 : 512;
    hipLaunchKernelGGL((gemm_bf16_kernel<MB, NT, MAXT, Epi>), grid, block, lds, s, g, epi);
}

template <class Epi, bool EVEN_ONLY>
static int launch_bf16(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K,
                       const GemmPlan &p, const Epi &epi) {
    GemmGeom g;
    g.X = (const u32x4_t *)X; g.W = (const u32x4_t *)W;
    g.M = M; g.NTiles = ceil_div(N, 32); g.KT = K / 16; g.kpw = p.kpw; g.NW = p.nw; g.KW = p.kw;
    const int groups = ceil_div(g.NTiles, p.nt);
    dim3 grid(ceil_div(groups, p.nw), p.splits, ceil_div(ceil_div(M, 32), p.mb)), block(p.nw * p.kw * 64);
    const size_t lds = ((size_t)GEMM_LDS_SCRATCH + (p.kw > 1 ? (size_t)p.kw * p.nw * p.mb * p.nt * 16 * 64 : 0)) * 4;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (c->profiling) {
        if (c->ev_used + 2 > c->ev.size())
            for (int i = 0; i < 2; ++i) { hipEvent_t e; HYDRA_HIP(hipEventCreate(&e)); c->ev.push_back(e); }
        e0 = c->ev[c->ev_used++]; e1 = c->ev[c->ev_used++];
        HYDRA_HIP(hipEventRecord(e0, s));
    }
    const int key = p.mb * 10 + p.nt;
    if constexpr (EVEN_ONLY) {
        switch (key) {
            case 12: launch_one<1, 2>(grid, block, lds, s, g, epi); break;
            case 14: launch_one<1, 4>(grid, block, lds, s, g, epi); break;
            case 22: launch_one<2, 2>(grid, block, lds, s, g, epi); break;
            case 24: launch_one<2, 4>(grid, block, lds, s, g, epi); break;
            case 42: launch_one<4, 2>(grid, block, lds, s, g, epi); break;
            default: return fail(HYDRA_E_UNSUPPORTED, "gemm: no kernel for this plan");
        }
    } else {
        switch (key) {
            case 11: launch_one<1, 1>(grid, block, lds, s, g, epi); break;
            case 12: launch_one<1, 2>(grid, block, lds, s, g, epi); break;
            case 13: launch_one<1, 3>(grid, block, lds, s, g, epi); break;
            case 14: launch_one<1, 4>(grid, block, lds, s, g, epi); break;
            case 21: launch_one<2, 1>(grid, block, lds, s, g, epi); break;
            case 22: launch_one<2, 2>(grid, block, lds, s, g, epi); break;
            case 23: launch_one<2, 3>(grid, block, lds, s, g, epi); break;
            case 24: launch_one<2, 4>(grid, block, lds, s, g, epi); break;
            case 41: launch_one<4, 1>(grid, block, lds, s, g, epi); break;
            case 42: launch_one<4, 2>(grid, block, lds, s, g, epi); break;
            default: return fail(HYDRA_E_UNSUPPORTED, "gemm: no kernel for this plan");
        }
    }
    HYDRA_LAUNCH_CHECK("gemm_bf16_kernel");
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
    GemmPlan p = plan_gemm(c, M, N, K, GEMM_KIND_PLAIN);
    if (plan_out) *plan_out = p;
    if (!c->bf16) return launch_gemm_f32(c, s, (const float *)X, (const float *)W, part, M, N, K);
    const int npad = gemm_npad(c, N);
    EpiPlain epi{part, npad, (size_t)ceil_div(M, 32) * 32 * npad};
    return launch_bf16<EpiPlain, false>(c, s, X, W, M, N, K, p, epi);
}

// x += X W^T, then xg = bf16(x * gain) and the per-band sums of squares.  Either fused into the GEMM
// epilogue (one workgroup owns a band for all of K) or, when the plan splits K over workgroups to fill
// the chip, as S partial outputs added by a small second kernel.
__global__ __launch_bounds__(256) void resid_norm_kernel(float *__restrict__ x, const float *__restrict__ part, int S,
                                                          int ld, size_t split_stride, const float *__restrict__ gain,
                                                          a16_t *__restrict__ xg, float *__restrict__ ss, int Mpad,
                                                          int d) {
    const int m = blockIdx.y;
    const int k = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (k >= d) return;                                       // d % 32 == 0: a 32-lane group is all in or all out
    f32x4_t a = *reinterpret_cast<const f32x4_t *>(x + (size_t)m * d + k);
    for (int sp = 0; sp < S; ++sp) {
        const f32x4_t q = *reinterpret_cast<const f32x4_t *>(part + (size_t)sp * split_stride + (size_t)m * ld + k);
        a[0] += q[0]; a[1] += q[1]; a[2] += q[2]; a[3] += q[3];
    }
    *reinterpret_cast<f32x4_t *>(x + (size_t)m * d + k) = a;
    const f32x4_t gn = *reinterpret_cast<const f32x4_t *>(gain + k);
    const uint32_t lo = f2a_pack(a[0] * gn[0], a[1] * gn[1]);
    const uint32_t hi = f2a_pack(a[2] * gn[2], a[3] * gn[3]);
    uint32_t *dst = reinterpret_cast<uint32_t *>(xg + x_index<true>(m, k, d));     // 4 consecutive k share an 8-run
    dst[0] = lo; dst[1] = hi;
    float sq = a[0] * a[0] + a[1] * a[1] + a[2] * a[2] + a[3] * a[3];
    sq += __shfl_xor(sq, 1, 64); sq += __shfl_xor(sq, 2, 64); sq += __shfl_xor(sq, 4, 64);   // 8 lanes = one 32-column band
    if ((threadIdx.x & 7) == 0) ss[(size_t)(k >> 5) * Mpad + m] = sq;
}

int launch_gemm_resid(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K, float *x,
                      const float *gain, void *xg, float *ss, int Mpad, float *part) {
    GemmPlan p = plan_gemm(c, M, N, K, GEMM_KIND_PLAIN);
    if (p.splits > 1) {
        const int npad = gemm_npad(c, N);
        const size_t stride = (size_t)ceil_div(M, 32) * 32 * npad;
        EpiPlain epi{part, npad, stride};
        int rc = launch_bf16<EpiPlain, false>(c, s, X, W, M, N, K, p, epi);
        if (rc) return rc;
        hipLaunchKernelGGL(resid_norm_kernel, dim3(ceil_div(N, 1024), M), dim3(256), 0, s, x, part, p.splits, npad, stride,
                           gain, (a16_t *)xg, ss, Mpad, N);
        HYDRA_LAUNCH_CHECK("resid_norm_kernel");
        return HYDRA_OK;
    }
    p = plan_gemm(c, M, N, K, GEMM_KIND_FUSED);
    EpiResid epi{x, N, gain, (a16_t *)xg, ss, Mpad};
    return launch_bf16<EpiResid, false>(c, s, X, W, M, N, K, p, epi);
}

int launch_gemm_silu(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int F, int K, const float *ss,
                     int nb, int Mpad, void *act) {
    GemmPlan p = plan_gemm(c, M, 2 * F, K, GEMM_KIND_FUSED);
    EpiSilu epi{ss, nb, Mpad, K, c->m.rms_eps, (a16_t *)act, F};
    return launch_bf16<EpiSilu, false>(c, s, X, W, M, 2 * F, K, p, epi);
}

int launch_gemm_bias_silu(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K,
                          const float *bias, float *z, bool residual, void *xg) {
    GemmPlan p = plan_gemm(c, M, N, K, GEMM_KIND_FUSED);
    EpiBiasSilu epi{bias, z, N, residual ? 1 : 0, (a16_t *)xg};
    return launch_bf16<EpiBiasSilu, false>(c, s, X, W, M, N, K, p, epi);
}

template <int MB, int NT, class Epi>
static hipError_t set_attr() {
    constexpr int MAXT = (MB * NT >= 6) ? 256 : 512;
    return hipFuncSetAttribute((const void *)gemm_bf16_kernel<MB, NT, MAXT, Epi>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}
template <class Epi>
static hipError_t set_attr_all() {
    hipError_t e = hipSuccess;
    if (e == hipSuccess) e = set_attr<1, 1, Epi>(); if (e == hipSuccess) e = set_attr<1, 2, Epi>();
    if (e == hipSuccess) e = set_attr<1, 3, Epi>(); if (e == hipSuccess) e = set_attr<1, 4, Epi>();
    if (e == hipSuccess) e = set_attr<2, 1, Epi>(); if (e == hipSuccess) e = set_attr<2, 2, Epi>();
    if (e == hipSuccess) e = set_attr<2, 3, Epi>(); if (e == hipSuccess) e = set_attr<2, 4, Epi>();
    if (e == hipSuccess) e = set_attr<4, 1, Epi>(); if (e == hipSuccess) e = set_attr<4, 2, Epi>();
    return e;
}

// opt in to the full LDS for every instantiation (a no-op for those that need less)
int gemm_max_dynamic_lds(hydra_ctx *c) {
    (void)c;
    hipError_t e = set_attr_all<EpiPlain>();
    if (e == hipSuccess) e = set_attr_all<EpiResid>();
    if (e == hipSuccess) e = set_attr_all<EpiBiasSilu>();
    if (e == hipSuccess) e = set_attr_all<EpiSilu>();
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(gemm_bf16_kernel)");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Row-major [N][K] bfloat16 -> tile order, converted to the a16 element (see device_common.h).  Source row n goes to band
// tile_off + (n / rows_per_band) * tile_stride, column col_off + n % rows_per_band, so
// several source matrices can share the bands of one packed matrix (q|k|v stacked band
// after band; gate and up side by side inside every band with rows_per_band = 16).
// Columns of the last band that have no source row are zero.  One thread writes one
// 16-byte lane entry.
// ---------------------------------------------------------------------------
__global__ void pack_weight_kernel(const bf16_t *__restrict__ src, u32x4_t *__restrict__ dst, int N, int K,
                                   int tile_off, int tile_stride, int rows_per_band, int col_off) {
    const int KT = K >> 4;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;      // (band, kt, lane)
    const int nbands = (N + rows_per_band - 1) / rows_per_band;
    const size_t total = (size_t)nbands * KT * 64;
    if (idx >= total) return;
    const int lane = (int)(idx & 63);
    const int kt = (int)((idx >> 6) % KT);
    const int band = (int)((idx >> 6) / KT);
    const int c = (lane & 31) - col_off;
    if (c < 0 || c >= rows_per_band) return;                               // this column belongs to another source
    const int n = band * rows_per_band + c;
    const int k = kt * 16 + (lane >> 5) * 8;
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (n < N) {
        const u32x4_t raw = *reinterpret_cast<const u32x4_t *>(src + (size_t)n * K + k);     // 8 bfloat16
#pragma unroll
        for (int q = 0; q < 4; ++q)                                                          // -> 8 half (exact from 2^-17 up)
            v[q] = f2a_pack(__uint_as_float(raw[q] << 16), __uint_as_float(raw[q] & 0xffff0000u));
    }
    dst[((size_t)(tile_off + band * tile_stride) * KT + kt) * 64 + lane] = v;
}

int launch_pack_matrix(hydra_ctx *c, hipStream_t s, const void *src, void *dst, int N, int K, int tile_off,
                       int tile_stride, int rows_per_band, int col_off) {
    (void)c;
    const size_t total = (size_t)ceil_div(N, rows_per_band) * (K / 16) * 64;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t *)src,
                       (u32x4_t *)dst, N, K, tile_off, tile_stride, rows_per_band, col_off);
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
