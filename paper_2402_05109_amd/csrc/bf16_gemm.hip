// bf16 storage family: launch plans and epilogues of the weight-streaming GEMM
// (kernel in gemm_bf16.h), and the kernels that bring plain row-major weights
// into its tile order.
#include <stdio.h>
#include <stdlib.h>

#include <type_traits>

#include <algorithm>

#include <hip/hip_ext.h>

#include "gemm_bf16.h"
#include "gemm_epilogues.h"
#include "internal.h"

namespace hydra {

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
    p.shared_x = 0;
    p.cost_us = 0.f;
    if (!c->bf16) { p.mb = 1; p.nt = 1; p.nw = 1; p.kw = 1; p.kpw = K; return p; }
    const int mblocks = ceil_div(M, 32);
    // three row blocks go into one group of four (a quarter of its MFMAs idle) rather than into two groups of two, which
    // would stream W twice: measured 5.5 against 5.8 ms per step at 96 rows, 7B shape
    p.mb = mblocks >= 3 ? 4 : (mblocks >= 2 ? 2 : 1);
    const int mgroups = ceil_div(mblocks, p.mb);
    const int bands = ceil_div(N, 32), KT = K / 16;
    const bool pairs = kind == GEMM_KIND_PAIRS;                        // band pairs: exactly two bands per wave
    // a partial output is M x N floats written and read back: the charge per split was fitted at 64 rows and grows
    // with the rows beyond that (measured at 128 and 256 rows: verify 6.08 -> 5.74 and 10.05 -> 9.3 ms with 4x / 8x)
    const double split_charge = split_us * (M > 64 ? M / 32.0 : 1.0);
    const bool may_split = kind == GEMM_KIND_PLAIN;
    p.nw = 1;
    // bands per wave: accumulators MB*NT*16 plus two prefetch sets must fit the register file
    int nt_max = pairs ? (p.mb == 4 ? 2 : 4) : (p.mb == 4 ? 3 : 4);   // pairs: one or two band pairs per wave
    if (kind == GEMM_KIND_SWIGLU && p.mb == 2) nt_max = 5;             // the widest instantiation (very wide FFNs: one round instead of two)
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
            cost += (s > 1 ? 1.0 + split_charge * s : 0.0);                  // writing and reading S partials back
            if (cost < best_cost - 1e-9) { best_cost = cost; best_nt = nt; best_s = s; }
        }
    }
    if (kind == GEMM_KIND_SWIGLU && p.mb == 2 && env_or("HYDRA_PLAN_SWIGLU_NT", 0.0) == 5.0) best_nt = 5, best_s = 1;   // tests: force the widest shape
    if (pairs && p.mb <= 2) {                                          // tests: force one or two band pairs per wave
        const int forced = (int)env_or("HYDRA_PLAN_PAIRS_NT", 0.0);
        if (forced == 2 || forced == 4) best_nt = forced;
    }
    p.nt = best_nt;
    p.splits = best_s;
    p.cost_us = (float)best_cost;
    const int max_waves = (p.mb * p.nt >= 6) ? 4 : 8;                   // 256-thread workgroups get 512 VGPRs per wave
    p.kw = max_waves;
    if (p.kw == 8 && p.splits > 1 && KT / (8 * p.splits) >= 16) p.kw = 4;   // split K with long runs left: four waves with twice the run each measured faster
    while (p.kw > 1 && KT / (p.kw * p.splits) < 4) p.kw >>= 1;
    while (p.kw > 1 && ((size_t)GEMM_LDS_SCRATCH + (size_t)p.kw * p.mb * p.nt * 16 * 64) * 4 > 150 * 1024) p.kw >>= 1;   // LDS: KW accumulator copies
    // Two band groups per workgroup only pay for many row groups (measured: slower at 2-4 row groups of 128 rows,
    // faster at 8): the X tiles both groups read count against the CU's request path even when they hit in L1.
    if (mgroups >= 6 && p.kw >= 2) { p.nw = 2; p.kw >>= 1; }
    p.kpw = ceil_div(KT, p.kw * p.splits);
    // Four row blocks per workgroup: the X tiles dominate what a workgroup pulls, and where enough workgroups remain 4 or 8
    // waves take different band pairs and share X through LDS (gemm_bf16_sharedx_kernel).  A workgroup then pulls NWT
    // pairs of W and X once.  Where the output may be split (plain partial outputs), K is also split over workgroups:
    // that multiplies the workgroups and shortens each one's slice of X (a single row group of 128 rows has only
    // bands / (2 NWT) workgroups otherwise).  The shape is taken where it costs less than the plan above.
    if (p.mb == 4 && (mgroups >= 2 || may_split) && KT >= 16) {
        const int groups2 = ceil_div(bands, 2);
        int pick = 0, pick_s = 1;
        if (getenv("HYDRA_PLAN_SHARED_X_MIN_WGS")) {                  // tests: the shape wherever this many workgroups remain
            const int min_wgs = (int)env_or("HYDRA_PLAN_SHARED_X_MIN_WGS", 160.0);
            for (int nwt = 8; nwt >= 4 && !pick && mgroups >= 4; nwt >>= 1)
                if (ceil_div(groups2, nwt) * mgroups >= min_wgs) pick = nwt;
            const int sp = (int)env_or("HYDRA_PLAN_SHARED_X_SPLITS", 1.0);       // tests: with this many K splits where the output may be split
            if (pick && may_split && sp > 1 && KT / sp >= 4) pick_s = sp;
        } else {
            double best = p.cost_us;
            const double hbm = (double)N * K * 2 / (hbm_tbps * 1e6);
            const int s_max = (may_split && env_or("HYDRA_PLAN_SHARED_X_SPLIT", 1.0) != 0.0) ? max_split : 1;
            for (int nwt = 8; nwt >= 4; nwt >>= 1)
                for (int sp = 1; sp <= s_max; ++sp) {
                    if (sp > 1 && KT / sp < 16) break;
                    if (sp == 1 && mgroups < 2) continue;              // one row group, no split: too few workgroups by construction
                    const int wgs = ceil_div(groups2, nwt) * mgroups * sp;
                    const double bytes = ((double)nwt * 64 + 128.0) * K * 2 / sp;
                    double cost = ceil_div(wgs, 256) * bytes / (cap_gbps * 1e3);
                    if (cost < hbm) cost = hbm;
                    cost += (sp > 1 ? 1.0 + split_charge * sp : 0.0);
                    if (wgs >= 128 && cost < 0.97 * best) { best = cost; pick = nwt; pick_s = sp; }      // a tie goes to the plan with more workgroups
                }
            if (pick) p.cost_us = (float)best;
        }
        if (pick) {
            p.shared_x = pick; p.nt = 2; p.nw = pick; p.kw = 1; p.splits = pick_s;
            p.kpw = ceil_div(ceil_div(KT, pick_s), 4) * 4;           // k-steps per split: whole blocks of four
            p.splits = ceil_div(KT, p.kpw);
        }
    }
    static const bool debug = getenv("HYDRA_PLAN_DEBUG") != nullptr;       // tuning aid: every plan to stderr
    if (debug)
        fprintf(stderr, "plan M=%d N=%d K=%d kind=%d -> mb=%d nt=%d nw=%d kw=%d splits=%d shared_x=%d cost=%.1f\n", M, N, K, kind, p.mb, p.nt, p.nw,
                p.kw, p.splits, p.shared_x, p.cost_us);
    return p;
}

int launch_gemm_f32(hydra_ctx *c, hipStream_t s, const float *X, const float *W, float *part, int M, int N, int K);

// e0/e1 non-null (profiling): the events take the kernel's own begin and end times, not the stream's before and after
template <int MB, int NT, class Epi>
static void launch_one(dim3 grid, dim3 block, size_t lds, hipStream_t s, const GemmGeom &g, const Epi &epi, hipEvent_t e0, hipEvent_t e1) {
    constexpr int MAXT = (MB * NT >= 6) ? 256 : 512;
    if constexpr (MB == 4) {                       // several row groups exist only with four row blocks per workgroup
        if (g.gz > 1) {
            if (e0) hipExtLaunchKernelGGL((gemm_bf16_kernel<MB, NT, MAXT, Epi, true>), grid, block, lds, s, e0, e1, 0, g, epi);
            else    hipLaunchKernelGGL((gemm_bf16_kernel<MB, NT, MAXT, Epi, true>), grid, block, lds, s, g, epi);
            return;
        }
    }
    if (e0) hipExtLaunchKernelGGL((gemm_bf16_kernel<MB, NT, MAXT, Epi>), grid, block, lds, s, e0, e1, 0, g, epi);
    else    hipLaunchKernelGGL((gemm_bf16_kernel<MB, NT, MAXT, Epi>), grid, block, lds, s, g, epi);
}

enum { NT_ANY = 0, NT_TWO = 2 };
template <class Epi, int NT_SET>
static int launch_bf16(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K,
                       const GemmPlan &p, const Epi &epi, int extra_blocks = 0) {
    GemmGeom g;
    g.X = (const u32x4_t *)X; g.W = (const u32x4_t *)W;
    g.M = M; g.NTiles = ceil_div(N, 32); g.KT = K / 16; g.kpw = p.kpw; g.NW = p.nw; g.KW = p.kw;
    const int groups = ceil_div(g.NTiles, p.nt);
    dim3 grid(ceil_div(groups, p.nw), p.splits, ceil_div(ceil_div(M, 32), p.mb)), block(p.nw * p.kw * 64);
    g.gx = (int)grid.x; g.gy = (int)grid.y; g.gz = (int)grid.z;
    if (grid.z > 1) grid = dim3((unsigned)(ceil_div(g.gx * g.gy, 8) * 8 * g.gz), 1, 1);          // see gemm_block()
    if (Epi::EXTRA_BLOCKS && !p.shared_x && g.gy == 1 && g.gz == 1) grid.x += extra_blocks;      // see Epilogue::extra_block
    size_t lds = ((size_t)GEMM_LDS_SCRATCH + (p.kw > 1 ? (size_t)p.kw * p.nw * p.mb * p.nt * 16 * 64 : 0)) * 4;
    if (p.shared_x) {
        if (p.mb != 4 || p.nt != 2 || p.kw != 1 || p.splits < 1 || (p.splits > 1 && !std::is_same<Epi, EpiPlain>::value) || p.nw != p.shared_x || (p.shared_x != 4 && p.shared_x != 8))
            return fail(HYDRA_E_UNSUPPORTED, "gemm: inconsistent shared-X plan");
        lds = ((size_t)GEMM_LDS_SCRATCH + 2 * 4 * 4 * 256) * 4;          // two blocks of 4 k-steps x 4 row blocks of 1 KiB
    }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (c->profiling) {
        if (c->ev_used + 2 > c->ev.size())
            for (int i = 0; i < 2; ++i) { hipEvent_t e; HYDRA_HIP(hipEventCreate(&e)); c->ev.push_back(e); }
        e0 = c->ev[c->ev_used++]; e1 = c->ev[c->ev_used++];
    }
    const int key = p.mb * 10 + p.nt;
    if (p.shared_x) {
        if constexpr (std::is_same<Epi, EpiTop2>::value) {           // never planned for this epilogue (launch_gemm_top2): no such kernel is built
            return fail(HYDRA_E_UNSUPPORTED, "gemm: the band-wise top-2 epilogue has no shared-X kernel");
        } else if (p.shared_x == 8) {
            if (e0) hipExtLaunchKernelGGL((gemm_bf16_sharedx_kernel<4, 2, 8, Epi>), grid, block, lds, s, e0, e1, 0, g, epi);
            else    hipLaunchKernelGGL((gemm_bf16_sharedx_kernel<4, 2, 8, Epi>), grid, block, lds, s, g, epi);
        } else {
            if (e0) hipExtLaunchKernelGGL((gemm_bf16_sharedx_kernel<4, 2, 4, Epi>), grid, block, lds, s, e0, e1, 0, g, epi);
            else    hipLaunchKernelGGL((gemm_bf16_sharedx_kernel<4, 2, 4, Epi>), grid, block, lds, s, g, epi);
        }
    } else if constexpr (NT_SET == NT_TWO) {
        switch (key) {
            case 12: launch_one<1, 2>(grid, block, lds, s, g, epi, e0, e1); break;
            case 14: launch_one<1, 4>(grid, block, lds, s, g, epi, e0, e1); break;
            case 22: launch_one<2, 2>(grid, block, lds, s, g, epi, e0, e1); break;
            case 24: launch_one<2, 4>(grid, block, lds, s, g, epi, e0, e1); break;
            case 42: launch_one<4, 2>(grid, block, lds, s, g, epi, e0, e1); break;
            default: return fail(HYDRA_E_UNSUPPORTED, "gemm: no kernel for this plan");
        }
    } else {
        switch (key) {
            case 11: launch_one<1, 1>(grid, block, lds, s, g, epi, e0, e1); break;
            case 12: launch_one<1, 2>(grid, block, lds, s, g, epi, e0, e1); break;
            case 13: launch_one<1, 3>(grid, block, lds, s, g, epi, e0, e1); break;
            case 14: launch_one<1, 4>(grid, block, lds, s, g, epi, e0, e1); break;
            case 21: launch_one<2, 1>(grid, block, lds, s, g, epi, e0, e1); break;
            case 22: launch_one<2, 2>(grid, block, lds, s, g, epi, e0, e1); break;
            case 23: launch_one<2, 3>(grid, block, lds, s, g, epi, e0, e1); break;
            case 24: launch_one<2, 4>(grid, block, lds, s, g, epi, e0, e1); break;
            case 25:
                if constexpr (std::is_same<Epi, EpiSilu>::value) { launch_one<2, 5>(grid, block, lds, s, g, epi, e0, e1); break; }
                else return fail(HYDRA_E_UNSUPPORTED, "gemm: no kernel for this plan");
            case 41: launch_one<4, 1>(grid, block, lds, s, g, epi, e0, e1); break;
            case 42: launch_one<4, 2>(grid, block, lds, s, g, epi, e0, e1); break;
            case 43: launch_one<4, 3>(grid, block, lds, s, g, epi, e0, e1); break;
            default: return fail(HYDRA_E_UNSUPPORTED, "gemm: no kernel for this plan");
        }
    }
    HYDRA_LAUNCH_CHECK("gemm_bf16_kernel");
    if (c->profiling) {
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
    return launch_bf16<EpiPlain, NT_ANY>(c, s, X, W, M, N, K, p, epi);
}

// x += X W^T, then xg = half(x * gain) and the sums of squares (*ss_bands rows of ss: one per band, or one per 1024-column chunk).  Either fused into the GEMM
// epilogue (one workgroup owns a band for all of K) or, when the plan splits K over workgroups to fill
// the chip, as S partial outputs added by a small second kernel.
// One workgroup per (row, 1024-column chunk): the chunk's sum of squares goes to ss[chunk][row], so the consumers'
// row-scale gathering reads d / 1024 values per row instead of one per 32-column band.
__global__ __launch_bounds__(256) void resid_norm_kernel(float *__restrict__ x, const float *__restrict__ part, int S,
                                                          int ld, size_t split_stride, const float *__restrict__ gain,
                                                          a16_t *__restrict__ xg, float *__restrict__ ss, int Mpad,
                                                          int d, int32_t *flags) {
    __shared__ float red[4];
    const int m = blockIdx.y;
    const int k = (blockIdx.x * 256 + threadIdx.x) * 4;
    float sq = 0.f;
    if (k < d) {                                              // d % 32 == 0: a group of 8 lanes is all in or all out
        f32x4_t a = *reinterpret_cast<const f32x4_t *>(x + (size_t)m * d + k);
        const f32x4_t gn = *reinterpret_cast<const f32x4_t *>(gain + k);
        const float *src = part + (size_t)m * ld + k;
        for (int s0 = 0; s0 < S; s0 += 4) {                    // four partials per round trip (surplus loads re-read the last split)
            f32x4_t q[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) q[u] = *reinterpret_cast<const f32x4_t *>(src + (size_t)min(s0 + u, S - 1) * split_stride);
#pragma unroll
            for (int u = 0; u < 4; ++u)                        // added in split order
                if (s0 + u < S) { a[0] += q[u][0]; a[1] += q[u][1]; a[2] += q[u][2]; a[3] += q[u][3]; }
        }
        *reinterpret_cast<f32x4_t *>(x + (size_t)m * d + k) = a;
        const uint32_t lo = f2a_pack_f(a[0] * gn[0], a[1] * gn[1], flags);
        const uint32_t hi = f2a_pack_f(a[2] * gn[2], a[3] * gn[3], flags);
        uint32_t *dst = reinterpret_cast<uint32_t *>(xg + x_index<true>(m, k, d));     // 4 consecutive k share an 8-run
        dst[0] = lo; dst[1] = hi;
        sq = a[0] * a[0] + a[1] * a[1] + a[2] * a[2] + a[3] * a[3];
    }
    sq = wave_sum(sq);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sq;
    __syncthreads();
    if (threadIdx.x == 0) ss[(size_t)blockIdx.x * Mpad + m] = red[0] + red[1] + red[2] + red[3];
}

int launch_gemm_resid(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K, float *x,
                      const float *gain, void *xg, float *ss, int Mpad, float *part, int *ss_bands) {
    GemmPlan p = plan_gemm(c, M, N, K, GEMM_KIND_PLAIN);
    if (p.splits > 1) {
        const int npad = gemm_npad(c, N);
        const size_t stride = (size_t)ceil_div(M, 32) * 32 * npad;
        EpiPlain epi{part, npad, stride};
        int rc = launch_bf16<EpiPlain, NT_ANY>(c, s, X, W, M, N, K, p, epi);
        if (rc) return rc;
        hipLaunchKernelGGL(resid_norm_kernel, dim3(ceil_div(N, 1024), M), dim3(256), 0, s, x, part, p.splits, npad, stride,
                           gain, (a16_t *)xg, ss, Mpad, N, flags_dev(c));
        HYDRA_LAUNCH_CHECK("resid_norm_kernel");
        *ss_bands = ceil_div(N, 1024);       // one partial sum per 1024-column chunk
        return HYDRA_OK;
    }
    *ss_bands = N / 32;                      // the fused epilogue leaves one partial sum per 32-column band
    p = plan_gemm(c, M, N, K, GEMM_KIND_FUSED);
    EpiResid epi{x, N, gain, (a16_t *)xg, ss, Mpad, flags_dev(c)};
    return launch_bf16<EpiResid, NT_ANY>(c, s, X, W, M, N, K, p, epi);
}

// LM head straight to per-band top-2 candidates (no logits): *fused = 0 and nothing launched where the plan that splits K
// over workgroups is estimated clearly faster than one workgroup per band group (the candidates need complete sums).
// Opt-in (HYDRA_LM_HEAD_TOP2=1): measured at the 7B shape it is a wash, 50.3 + 5.8 us against 47.0 + 11.6 us at 64 rows and
// 52.1 + 5.7 against 41.8 + ~8 us for the one-node tree, so by default the logits go through memory.
int launch_gemm_top2(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K, float *cand, int Mpad, int *fused) {
    const GemmPlan ps = plan_gemm(c, M, N, K, GEMM_KIND_PLAIN);
    const GemmPlan p = plan_gemm(c, M, N, K, GEMM_KIND_FUSED);
    *fused = (p.shared_x == 0 && p.cost_us <= ps.cost_us + 4.0f && env_or("HYDRA_LM_HEAD_TOP2", 0.0) != 0.0) ? 1 : 0;
    if (!*fused) return HYDRA_OK;
    EpiTop2 epi{cand, Mpad, N};
    return launch_bf16<EpiTop2, NT_ANY>(c, s, X, W, M, N, K, p, epi);
}

int launch_gemm_silu(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int F, int K, const float *ss,
                     int nb, int Mpad, void *act) {
    GemmPlan p = plan_gemm(c, M, 2 * F, K, GEMM_KIND_SWIGLU);
    EpiSilu epi{ss, nb, Mpad, K, c->m.rms_eps, (a16_t *)act, F, flags_dev(c)};
    return launch_bf16<EpiSilu, NT_ANY>(c, s, X, W, M, 2 * F, K, p, epi);
}

int launch_gemm_bias_silu(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K,
                          const float *bias, float *z, bool residual, void *xg) {
    GemmPlan p = plan_gemm(c, M, N, K, GEMM_KIND_FUSED);
    EpiBiasSilu epi{bias, z, N, residual ? 1 : 0, (a16_t *)xg, flags_dev(c)};
    return launch_bf16<EpiBiasSilu, NT_ANY>(c, s, X, W, M, N, K, p, epi);
}

// q|k|v projection, rotary embedding and cache append in one kernel (bf16 family)
int launch_gemm_qkv_rope(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, RowScale rs, int layer,
                         const int32_t *seq_len, const hydra_kv *kv, void *qbuf, float *part, int32_t *flags) {
    {
        // Beyond 128 rows a plan that splits K over workgroups (plain partial sums, then rotary embedding and cache append
        // as a kernel of their own) can beat the fused one: each workgroup pulls a shorter slice of X (measured: steps at
        // 192 rows 7.7 -> 7.3 ms, the 33B shape at 256 rows 30.8 -> 29.5 ms; at 96 and 128 rows it lost 1.5 %).  It is taken where
        // the planner's estimate plus the cost of the second kernel is lower (HYDRA_PLAN_QKV_UNFUSED: 0 never, 1 always).
        const int dd = c->m.d;
        const GemmPlan pf = plan_gemm(c, M, 3 * dd, dd, GEMM_KIND_PAIRS), pu = plan_gemm(c, M, 3 * dd, dd, GEMM_KIND_PLAIN);
        const int mode = (int)env_or("HYDRA_PLAN_QKV_UNFUSED", -1.0);
        // the second kernel: its launch, and S partial outputs of M x 3d floats read back at about 4 TB/s
        const float second = 5.0f + (float)((double)pu.splits * M * 3 * dd * 4 / 4e6);
        const bool unfused = mode == 1 || (mode != 0 && M > 128 && pu.splits > 1 && pu.cost_us + second < pf.cost_us);
        if (unfused) {
            const int npad = gemm_npad(c, 3 * dd);
            const size_t stride = (size_t)ceil_div(M, 32) * 32 * npad;
            EpiPlain epi{part, npad, stride};
            int rc = launch_bf16<EpiPlain, NT_ANY>(c, s, X, W, M, 3 * dd, dd, pu, epi);
            if (rc) return rc;
            return launch_rope_append(c, s, part, pu.splits, npad, stride, rs, M / c->tree.T, layer, seq_len, kv, qbuf, flags);
        }
    }
    const int d = c->m.d;
    GemmPlan p = plan_gemm(c, M, 3 * d, d, GEMM_KIND_PAIRS);
    EpiQkvRope epi{rs.ss, rs.nb, rs.Mpad, d, rs.eps, seq_len, tree_dev(c), kv->page_table, kv->max_pages, kv->n_pages, layer,
                   (a16_t *)kv->k_pages, (a16_t *)kv->v_pages, (a16_t *)qbuf, rope_dev(c), c->m.n_heads, c->m.head_dim,
                   c->tree.T, c->m.max_pos, flags, (int)env_or("HYDRA_KV_TOUCH_MAX_KEYS", 1280.0)};
    // CUs that get no band group pre-read the layer's K/V pages: only where an eighth of the chip or more is idle
    // (7B: 64 CUs; measured at the 13B shape, 16 idle CUs: the GEMM is close to the HBM limit there and the pre-read
    // costs more than attention gains, verify 6.35 -> 6.52 ms)
    const int wgs = ceil_div(ceil_div(ceil_div(3 * d, 32), p.nt), p.nw);
    const int idle = std::min(64, 256 - wgs);
    const int extra = (idle >= 32 && env_or("HYDRA_KV_TOUCH", 1.0) != 0.0) ? idle : 0;
    return launch_bf16<EpiQkvRope, NT_TWO>(c, s, X, W, M, 3 * d, d, p, epi, extra);
}

template <int MB, int NT, class Epi>
static hipError_t set_attr() {
    constexpr int MAXT = (MB * NT >= 6) ? 256 : 512;
    if constexpr (MB == 4) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_bf16_kernel<MB, NT, MAXT, Epi, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
    }
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
    if (e == hipSuccess) e = set_attr_all<EpiTop2>();
    if (e == hipSuccess) e = set_attr_all<EpiBiasSilu>();
    if (e == hipSuccess) e = set_attr_all<EpiSilu>();
    if (e == hipSuccess) e = set_attr<1, 2, EpiQkvRope>();
    if (e == hipSuccess) e = set_attr<2, 2, EpiQkvRope>();
    if (e == hipSuccess) e = set_attr<4, 2, EpiQkvRope>();
    if (e == hipSuccess) e = set_attr<2, 5, EpiSilu>();
    if (e == hipSuccess) e = set_attr<1, 4, EpiQkvRope>();
    if (e == hipSuccess) e = set_attr<2, 4, EpiQkvRope>();
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(gemm_bf16_kernel)");
    return HYDRA_OK;
}

// ---------------------------------------------------------------------------
// Row-major [N][K] bfloat16 -> tile order, converted to the a16 element (see device_common.h).  Source row n goes to band
// tile_off + (n / rows_per_band) * tile_stride, column col_off + n % rows_per_band, so
// several source matrices can share the bands of one packed matrix (q|k|v stacked band
// after band; gate and up side by side inside every band with rows_per_band = 16).
// bph > 1 (q and k): within each group of bph bands (one head) the bands that hold the two
// members of the rotary pairs (o and o + bph/2) are stored next to each other.
// Columns of the last band that have no source row are zero.  One thread writes one
// 16-byte lane entry.
// ---------------------------------------------------------------------------
__global__ void pack_weight_kernel(const bf16_t *__restrict__ src, u32x4_t *__restrict__ dst, int N, int K,
                                   int tile_off, int tile_stride, int rows_per_band, int col_off, int bph, int32_t *flags) {
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
        for (int q = 0; q < 4; ++q) {                                                        // -> 8 half (exact from 2^-17 up)
            v[q] = f2a_pack(__uint_as_float(raw[q] << 16), __uint_as_float(raw[q] & 0xffff0000u));
            // a non-zero weight below 2^-25 becomes zero in half: reported (flag bit 5), not silent
            const bool lost = ((raw[q] & 0x7fffu) != 0u && (v[q] & 0x7fffu) == 0u) || ((raw[q] & 0x7fff0000u) != 0u && (v[q] & 0x7fff0000u) == 0u);
            if (lost) atomicOr(flags, FLAG_WEIGHT_UNDERFLOW);
        }
    }
    int dband = band;
    if (bph > 1) {                      // rotary pairing: bands o and o + bph/2 of a head become neighbours
        const int h = band / bph, o = band - h * bph, hb = bph >> 1;
        dband = h * bph + (o % hb) * 2 + o / hb;
    }
    dst[((size_t)(tile_off + dband * tile_stride) * KT + kt) * 64 + lane] = v;
}

int launch_pack_matrix(hydra_ctx *c, hipStream_t s, const void *src, void *dst, int N, int K, int tile_off,
                       int tile_stride, int rows_per_band, int col_off, int bph) {
    const size_t total = (size_t)ceil_div(N, rows_per_band) * (K / 16) * 64;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t *)src,
                       (u32x4_t *)dst, N, K, tile_off, tile_stride, rows_per_band, col_off, bph, flags_dev(c));
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
