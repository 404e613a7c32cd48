// bf16 storage family: launch plans and epilogues of the weight-streaming GEMM
// (kernel in gemm_bf16.h), and the kernels that bring plain row-major weights
// into its tile order.
#include <stdio.h>
#include <stdlib.h>

#include <type_traits>

#include <algorithm>

#include <hip/hip_ext.h>

#include "gemm_bf16.h"
#include "internal.h"

namespace hydra {

// rows of a lane's accumulator registers
__device__ __forceinline__ int acc_row(int mb, int v, int lane) { return mb * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// Per-row 1/rms for the 32*MB rows of a workgroup, from the per-band sums of squares ss[band][Mpad]
// left by the producer of the GEMM input:  rstd = 1 / sqrt(sum_band ss / d + eps).
// The waves of the workgroup share the bands.  A load instruction covers G = 64 / (8*MB) bands: lane
// l reads the four rows 4*(l % (8*MB)) .. +3 of band group l / (8*MB).  rowsum_issue() starts the
// first eight such loads of a wave; rowsum_finish() adds them (and any further batches, which only
// very wide models need), folds the band groups together with lane shuffles and leaves this wave's
// partial sums in LDS at lds[wave*128 + row].  rstd_row() adds the partials in wave order.
struct RowSumRegs { f32x4_t v[8]; };
struct NoPre {};

template <int MB>
__device__ __forceinline__ RowSumRegs rowsum_issue(const float *__restrict__ ss, int nb, int Mpad, int row0, int lane,
                                                   int wave, int base) {
    constexpr int LPR = 8 * MB, G = 64 / LPR;
    const int nwaves = blockDim.x >> 6;
    const int grp = lane / LPR, r4 = (lane % LPR) * 4;
    RowSumRegs r;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int b = base + (j * nwaves + wave) * G + grp;
        if (b < nb) r.v[j] = *reinterpret_cast<const f32x4_t *>(ss + (size_t)b * Mpad + row0 + r4);
        else        r.v[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    return r;
}

template <int MB>
__device__ __forceinline__ void rowsum_finish(RowSumRegs r, float *lds, const float *__restrict__ ss, int nb, int Mpad,
                                              int row0, int lane, int wave) {
    constexpr int LPR = 8 * MB, G = 64 / LPR;
    const int nwaves = blockDim.x >> 6;
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    for (int base = 0;;) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc += r.v[j];
        base += 8 * nwaves * G;
        if (base >= nb) break;
        r = rowsum_issue<MB>(ss, nb, Mpad, row0, lane, wave, base);
    }
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) {
        acc[0] += __shfl_xor(acc[0], o, 64); acc[1] += __shfl_xor(acc[1], o, 64);
        acc[2] += __shfl_xor(acc[2], o, 64); acc[3] += __shfl_xor(acc[3], o, 64);
    }
    if (lane < LPR) *reinterpret_cast<f32x4_t *>(lds + GEMM_LDS_ROWSUM + wave * 128 + lane * 4) = acc;
}

// after the barrier: every wave fills its own table of row scales, rstd[row] at wave_stage(t)[256 + row]
__device__ __forceinline__ float *wave_stage(float *lds, int wave) { return lds + GEMM_LDS_STAGE + wave * GEMM_LDS_STAGE_WAVE; }
template <int MB>
__device__ __forceinline__ void rstd_table(float *lds, int lane, int wave, int d, float eps) {
    const int nwaves = blockDim.x >> 6;
    float *tab = wave_stage(lds, wave) + 256;
    for (int r = lane; r < 32 * MB; r += 64) {
        float s = 0.f;
        for (int w = 0; w < nwaves; ++w) s += lds[GEMM_LDS_ROWSUM + w * 128 + r];
        tab[r] = 1.0f / sqrtf(s / (float)d + eps);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- epilogues (one 32x32 tile at a time; see gemm_bf16.h) -------------------------
// out[split][row][col] = acc
struct EpiPlain {
    float *out; int ld; size_t split_stride;
    static constexpr bool LDS_PROLOGUE = false, PAIRED = false, EXTRA_BLOCKS = false;
    template <int MB, int NT> __device__ __forceinline__ NoPre issue(const GemmTile<MB, NT> &, const GemmGeom &) const { return NoPre{}; }
    template <int MB, int NT> __device__ __forceinline__ NoPre prologue(NoPre, const GemmTile<MB, NT> &, const GemmGeom &) const { return NoPre{}; }
    template <int MB, int NT> __device__ __forceinline__ void before_barrier(NoPre, const GemmTile<MB, NT> &, const GemmGeom &) const {}
    template <int MB, int NT> __device__ __forceinline__ void begin(const GemmTile<MB, NT> &, const GemmGeom &) const {}
    template <int MB, int NT>
    __device__ __forceinline__ void tile(const f32x16_t &acc, int a, int i, const GemmTile<MB, NT> &t, const GemmGeom &g) const {
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
// xg = half(x * gain) in GEMM input order (the 1/rms factor commutes with the
// contraction and is applied by the consumer) and ss[band][row] = sum over the
// band's 32 columns of x^2.
struct EpiResid {
    float *x; int d; const float *gain; a16_t *xg; float *ss; int Mpad;
    static constexpr bool LDS_PROLOGUE = false, PAIRED = false, EXTRA_BLOCKS = false;
    template <int MB, int NT> __device__ __forceinline__ NoPre issue(const GemmTile<MB, NT> &, const GemmGeom &) const { return NoPre{}; }
    template <int MB, int NT> __device__ __forceinline__ NoPre prologue(NoPre, const GemmTile<MB, NT> &, const GemmGeom &) const { return NoPre{}; }
    template <int MB, int NT> __device__ __forceinline__ void before_barrier(NoPre, const GemmTile<MB, NT> &, const GemmGeom &) const {}
    template <int MB, int NT> __device__ __forceinline__ void begin(const GemmTile<MB, NT> &, const GemmGeom &) const {}
    template <int MB, int NT>
    __device__ __forceinline__ void tile(const f32x16_t &acc, int a, int i, const GemmTile<MB, NT> &t, const GemmGeom &g) const {
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
    static constexpr bool LDS_PROLOGUE = true, PAIRED = false, EXTRA_BLOCKS = false;
    template <int MB, int NT> __device__ __forceinline__ RowSumRegs issue(const GemmTile<MB, NT> &t, const GemmGeom &) const {
        return rowsum_issue<MB>(ss, nb, Mpad, t.mb0 * 32, t.lane, t.wave, 0);
    }
    template <int MB, int NT> __device__ __forceinline__ NoPre prologue(RowSumRegs r, const GemmTile<MB, NT> &t, const GemmGeom &) const {
        rowsum_finish<MB>(r, t.lds, ss, nb, Mpad, t.mb0 * 32, t.lane, t.wave);
        return NoPre{};
    }
    template <int MB, int NT> __device__ __forceinline__ void before_barrier(NoPre, const GemmTile<MB, NT> &, const GemmGeom &) const {}
    template <int MB, int NT> __device__ __forceinline__ void begin(const GemmTile<MB, NT> &t, const GemmGeom &) const {
        rstd_table<MB>(t.lds, t.lane, t.wave, dmodel, eps);
    }
    // One band of gate|up columns gives 32 rows x 16 features of the activation: exactly one 1 KiB tile of
    // the next GEMM's input.  The wave assembles it in its LDS staging block and writes it with a single
    // 16-byte-per-lane store (rows past M hold don't-care values in the padded part of the buffer).
    template <int MB, int NT>
    __device__ __forceinline__ void tile(const f32x16_t &acc, int a, int i, const GemmTile<MB, NT> &t, const GemmGeom &g) const {
        if (t.tile0 + i >= g.NTiles) return;
        const int c = t.lane & 31, hl = t.lane >> 5;
        const bool left = c < 16;
        const int fo = c & 15;
        float *ws = wave_stage(t.lds, t.wave);
        a16_t *stage = reinterpret_cast<a16_t *>(ws);
        const float *rstd = ws + 256 + a * 32 + 4 * hl;
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            // left lanes need (gate = own acc[v], up = partner acc[v]); right lanes (gate = partner acc[v+8], up = own acc[v+8])
            const float send = left ? acc[v + 8] : acc[v];
            const float got = __shfl_xor(send, 16, 64);
            const float gate = left ? acc[v] : got;
            const float up = left ? got : acc[v + 8];
            const int vv = left ? v : v + 8;
            const int rl = 8 * (vv >> 2) + 4 * hl + (vv & 3);            // row inside the 32-row block
            const float r = left ? rstd[8 * (v >> 2) + (v & 3)] : rstd[8 * ((v + 8) >> 2) + (v & 3)];
            stage[((fo >> 3) * 32 + rl) * 8 + (fo & 7)] = f2a(silu_f(r * gate) * (r * up));
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");           // LDS is in order within a wave; keep the compiler from reordering
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const u32x4_t blk = reinterpret_cast<const u32x4_t *>(stage)[t.lane];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        reinterpret_cast<u32x4_t *>(act)[((size_t)(t.mb0 + a) * (F >> 4) + (t.tile0 + i)) * 64 + t.lane] = blk;
    }
};

// q|k|v projection with the rotary embedding and the cache append fused in (paper, section 2, "Tree
// decoding": node n of row b sits at position seq_len[b] + depth[n] and its K/V go to slot seq_len[b] + n).
// The q and k weight bands of a head are packed so that the bands holding dims j and j + Dh/2 are
// neighbours: a band pair (NT = 2) then holds both members of every rotary pair in the same lane.  The
// v bands keep their order.  r = 1/rms of the RMSNorm that feeds this GEMM (see rowsum_issue).
// Wave 0 looks up position and cache page of the workgroup's rows while the weights stream and leaves
// them in LDS: pos (or -1: row absent or over capacity), page*16 + slot%16, b*128 + n.
struct QkvRopePre { RowSumRegs rs; int L[2]; int dep[2]; int max_depth; };
struct QkvRopeCarry { int pos[2]; int pagetok[2]; int bn[2]; };
struct EpiQkvRope {
    const float *ss; int nb; int Mpad; int dmodel; float eps;
    const int32_t *seq_len; const TreeDev *tree; const int32_t *page_table; int max_pages, n_pages, layer;
    a16_t *kpages, *vpages, *qbuf; const float *rope; int H, Dh, T, max_pos; int32_t *flags;
    int kv_touch_max;       // rows with more keys than this are not pre-read (see extra_block)
    static constexpr bool LDS_PROLOGUE = true, PAIRED = true, EXTRA_BLOCKS = true;
    // Workgroups behind the last band group (the q|k|v GEMM of up to 64 rows leaves a quarter of the CUs without
    // one) read this layer's cached K and V pages once, so that tree attention, which follows and is a chain of
    // dependent round trips, finds them in the memory-side cache.  Nothing is computed from the values.  Only for
    // short rows: with more keys attention is a throughput problem spread over many workgroups, and the extra
    // pass over K/V costs this GEMM more than attention gains (measured at 2066 and 4114 keys: +0.13 and +0.63 ms).
    __device__ __forceinline__ void extra_block(int w, int n, const GemmGeom &g) const {
        const int rows = (g.M + T - 1) / T;
        const int n16 = H * Dh * 2;                                  // 16-byte pieces of one page of one layer (16 tokens, all heads)
        uint32_t sink = 0u;
        for (int b = 0; b < rows; ++b) {
            const int L = seq_len[b];
            if (L <= 0 || L + T > max_pages * 16 || L + T > kv_touch_max) continue;      // uniform over the workgroup
            const int pages = (L + 15) >> 4;
            for (int pi = (w + n - b % n) % n; pi < pages; pi += n) {
                const int page = page_table[(size_t)b * max_pages + pi];
                if ((unsigned)page >= (unsigned)n_pages) continue;
                const u32x4_t *kp = reinterpret_cast<const u32x4_t *>(kpages + kv_block_base(layer, n_pages, page, H, 0, Dh));
                const u32x4_t *vp = reinterpret_cast<const u32x4_t *>(vpages + kv_block_base(layer, n_pages, page, H, 0, Dh));
                for (int i = threadIdx.x; i < n16; i += blockDim.x) {
                    const u32x4_t a = kp[i], c = vp[i];
                    sink ^= a[0] ^ c[0];
                }
            }
        }
        asm volatile("" : : "v"(sink));                              // the loads must be issued although nothing uses them
    }
    template <int MB, int NT> __device__ __forceinline__ QkvRopePre issue(const GemmTile<MB, NT> &t, const GemmGeom &g) const {
        QkvRopePre p;
        p.rs = rowsum_issue<MB>(ss, nb, Mpad, t.mb0 * 32, t.lane, t.wave, 0);
        p.max_depth = 0;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            p.L[q] = -1; p.dep[q] = 0;
            const int r = t.lane + 64 * q, m = t.mb0 * 32 + r;
            if (t.wave == 0 && r < 32 * MB && m < g.M) {
                const int b = m / T, n = m - b * T;
                p.L[q] = seq_len[b];
                p.dep[q] = tree->depth[n];
                p.max_depth = tree->max_depth;
            }
        }
        return p;
    }
    template <int MB, int NT> __device__ __forceinline__ QkvRopeCarry prologue(const QkvRopePre &p, const GemmTile<MB, NT> &t, const GemmGeom &g) const {
        rowsum_finish<MB>(p.rs, t.lds, ss, nb, Mpad, t.mb0 * 32, t.lane, t.wave);
        QkvRopeCarry c;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            c.pos[q] = -1; c.pagetok[q] = 0; c.bn[q] = 0;
            const int r = t.lane + 64 * q, m = t.mb0 * 32 + r;
            if (t.wave == 0 && r < 32 * MB && m < g.M) {
                const int b = m / T, n = m - b * T, L = p.L[q];
                const bool ok = L >= 0 && L + T <= max_pages * 16 && L + p.max_depth < max_pos;
                if (ok) {
                    const int slot = L + n;
                    c.pos[q] = L + p.dep[q];
                    c.pagetok[q] = page_table[(size_t)b * max_pages + (slot >> 4)] * 16 + (slot & 15);
                    c.bn[q] = b * 128 + n;
                } else if (blockIdx.x == 0) {
                    atomicOr(flags, FLAG_CAPACITY);
                }
            }
        }
        return c;
    }
    template <int MB, int NT> __device__ __forceinline__ void before_barrier(const QkvRopeCarry &c, const GemmTile<MB, NT> &t, const GemmGeom &) const {
        if (t.wave != 0) return;
        int *info = reinterpret_cast<int *>(t.lds + GEMM_LDS_ROWINFO);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int r = t.lane + 64 * q;
            if (r < 32 * MB) { info[r] = c.pos[q]; info[128 + r] = c.pagetok[q]; info[256 + r] = c.bn[q]; }
        }
    }
    template <int MB, int NT> __device__ __forceinline__ void begin(const GemmTile<MB, NT> &t, const GemmGeom &) const {
        rstd_table<MB>(t.lds, t.lane, t.wave, dmodel, eps);
    }
    template <int MB, int NT>
    __device__ __forceinline__ void pair4(const float (&x0)[4], const float (&x1)[4], int a, int v0, const GemmTile<MB, NT> &t, const GemmGeom &g) const {
        if (t.tile0 + 1 >= g.NTiles) return;
        const int c = t.lane & 31, hl = t.lane >> 5;
        const int nbs = dmodel >> 5, bph = Dh >> 5, half = Dh >> 1;
        const int sec = t.tile0 / nbs, hb = t.tile0 - sec * nbs;
        const int h = hb / bph, pb = hb - h * bph;                       // pb is even: first band of a pair
        const int *info = reinterpret_cast<const int *>(t.lds + GEMM_LDS_ROWINFO);
        const float *rstd = wave_stage(t.lds, t.wave) + 256;
        const int rl0 = a * 32 + 8 * (v0 >> 2) + 4 * hl;
        int pos[4], pagetok[4], bn[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) { pos[q] = info[rl0 + q]; pagetok[q] = info[128 + rl0 + q]; bn[q] = info[256 + rl0 + q]; }
        a16_t *__restrict__ kp = kpages;
        a16_t *__restrict__ vp = vpages;
        a16_t *__restrict__ qp = qbuf;
        if (sec == 2) {
            const int dim0 = pb * 32 + c, dim1 = dim0 + 32;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (pos[q] < 0) continue;
                const float r = rstd[rl0 + q];
                const size_t base = kv_block_base(layer, n_pages, pagetok[q] >> 4, H, h, Dh);
                const int tok = pagetok[q] & 15;
                vp[base + v_in_block<true>(tok, dim0, Dh)] = f2a(r * x0[q]);
                vp[base + v_in_block<true>(tok, dim1, Dh)] = f2a(r * x1[q]);
            }
            return;
        }
        const int j = (pb >> 1) * 32 + c;                                // rotary pair (j, j + Dh/2)
        float cs[4], sn[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float2 t2 = pos[q] >= 0 ? *reinterpret_cast<const float2 *>(rope + ((size_t)pos[q] * half + j) * 2) : float2{1.f, 0.f};
            cs[q] = t2.x; sn[q] = t2.y;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (pos[q] < 0) continue;
            const float r = rstd[rl0 + q];
            const float u0 = r * x0[q], u1 = r * x1[q];
            const float y0 = u0 * cs[q] - u1 * sn[q], y1 = u1 * cs[q] + u0 * sn[q];
            if (sec == 0) {
                const int b = bn[q] >> 7, n = bn[q] & 127;
                const int QT = (T + 31) >> 5, KS = Dh >> 4;
                const size_t blk = (((size_t)b * H + h) * QT + (n >> 5)) * KS;
                qp[(((blk + (j >> 4)) * 64 + ((j >> 3) & 1) * 32 + (n & 31)) << 3) + (j & 7)] = f2a(y0);
                const int j1 = j + half;
                qp[(((blk + (j1 >> 4)) * 64 + ((j1 >> 3) & 1) * 32 + (n & 31)) << 3) + (j1 & 7)] = f2a(y1);
            } else {
                const size_t base = kv_block_base(layer, n_pages, pagetok[q] >> 4, H, h, Dh);
                const int tok = pagetok[q] & 15;
                kp[base + k_in_block<true>(tok, j, Dh)] = f2a(y0);
                kp[base + k_in_block<true>(tok, j + half, Dh)] = f2a(y1);
            }
        }
    }
    template <int MB, int NT>
    __device__ __forceinline__ void tile(const f32x16_t &, int, int, const GemmTile<MB, NT> &, const GemmGeom &) const {}
};

// Draft-head MLP layer: z = (residual ? z : 0) + SiLU(acc + bias), fp32 and as next GEMM input
struct EpiBiasSilu {
    const float *bias; float *z; int d; int residual; a16_t *xg;
    static constexpr bool LDS_PROLOGUE = false, PAIRED = false, EXTRA_BLOCKS = false;
    template <int MB, int NT> __device__ __forceinline__ NoPre issue(const GemmTile<MB, NT> &, const GemmGeom &) const { return NoPre{}; }
    template <int MB, int NT> __device__ __forceinline__ NoPre prologue(NoPre, const GemmTile<MB, NT> &, const GemmGeom &) const { return NoPre{}; }
    template <int MB, int NT> __device__ __forceinline__ void before_barrier(NoPre, const GemmTile<MB, NT> &, const GemmGeom &) const {}
    template <int MB, int NT> __device__ __forceinline__ void begin(const GemmTile<MB, NT> &, const GemmGeom &) const {}
    template <int MB, int NT>
    __device__ __forceinline__ void tile(const f32x16_t &acc, int a, int i, const GemmTile<MB, NT> &t, const GemmGeom &g) const {
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
    p.shared_x = 0;
    p.cost_us = 0.f;
    if (!c->bf16) { p.mb = 1; p.nt = 1; p.nw = 1; p.kw = 1; p.kpw = K; return p; }
    const int mblocks = ceil_div(M, 32);
    p.mb = mblocks >= 4 ? 4 : (mblocks >= 2 ? 2 : 1);
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
    // Two or more row groups of 128 rows: the X tiles dominate, and where enough workgroups remain 4 or 8 waves take
    // different band pairs and share X through LDS (gemm_bf16_sharedx_kernel; no K split in that shape).  A workgroup
    // then pulls NWT pairs of W and X once; the shape is taken where that costs less than the plan above.
    if (p.mb == 4 && mgroups >= 2 && KT >= 16) {
        const int groups2 = ceil_div(bands, 2);
        int pick = 0;
        if (getenv("HYDRA_PLAN_SHARED_X_MIN_WGS")) {                  // tests: the shape wherever this many workgroups remain
            const int min_wgs = (int)env_or("HYDRA_PLAN_SHARED_X_MIN_WGS", 160.0);
            for (int nwt = 8; nwt >= 4 && !pick && mgroups >= 4; nwt >>= 1)
                if (ceil_div(groups2, nwt) * mgroups >= min_wgs) pick = nwt;
        } else {
            double best = p.cost_us;
            const double hbm = (double)N * K * 2 / (hbm_tbps * 1e6);
            for (int nwt = 8; nwt >= 4; nwt >>= 1) {
                const int wgs = ceil_div(groups2, nwt) * mgroups;
                const double bytes = (double)nwt * 64 * K * 2 + 128.0 * K * 2;
                double cost = ceil_div(wgs, 256) * bytes / (cap_gbps * 1e3);
                if (cost < hbm) cost = hbm;
                if (wgs >= 128 && cost < 0.97 * best) { best = cost; pick = nwt; }      // a tie goes to the plan with more workgroups
            }
            if (pick) p.cost_us = (float)best;
        }
        if (pick) { p.shared_x = pick; p.nt = 2; p.nw = pick; p.kw = 1; p.splits = 1; p.kpw = KT; }
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
    if (Epi::EXTRA_BLOCKS && !p.shared_x && grid.y == 1 && grid.z == 1) grid.x += extra_blocks;    // see Epilogue::extra_block
    size_t lds = ((size_t)GEMM_LDS_SCRATCH + (p.kw > 1 ? (size_t)p.kw * p.nw * p.mb * p.nt * 16 * 64 : 0)) * 4;
    if (p.shared_x) {
        if (p.mb != 4 || p.nt != 2 || p.kw != 1 || p.splits != 1 || p.nw != p.shared_x || (p.shared_x != 4 && p.shared_x != 8))
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
    if (p.shared_x == 8) {
        if (e0) hipExtLaunchKernelGGL((gemm_bf16_sharedx_kernel<4, 2, 8, Epi>), grid, block, lds, s, e0, e1, 0, g, epi);
        else    hipLaunchKernelGGL((gemm_bf16_sharedx_kernel<4, 2, 8, Epi>), grid, block, lds, s, g, epi);
    } else if (p.shared_x == 4) {
        if (e0) hipExtLaunchKernelGGL((gemm_bf16_sharedx_kernel<4, 2, 4, Epi>), grid, block, lds, s, e0, e1, 0, g, epi);
        else    hipLaunchKernelGGL((gemm_bf16_sharedx_kernel<4, 2, 4, Epi>), grid, block, lds, s, g, epi);
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
                                                          int d) {
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
        const uint32_t lo = f2a_pack(a[0] * gn[0], a[1] * gn[1]);
        const uint32_t hi = f2a_pack(a[2] * gn[2], a[3] * gn[3]);
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
                           gain, (a16_t *)xg, ss, Mpad, N);
        HYDRA_LAUNCH_CHECK("resid_norm_kernel");
        *ss_bands = ceil_div(N, 1024);       // one partial sum per 1024-column chunk
        return HYDRA_OK;
    }
    *ss_bands = N / 32;                      // the fused epilogue leaves one partial sum per 32-column band
    p = plan_gemm(c, M, N, K, GEMM_KIND_FUSED);
    EpiResid epi{x, N, gain, (a16_t *)xg, ss, Mpad};
    return launch_bf16<EpiResid, NT_ANY>(c, s, X, W, M, N, K, p, epi);
}

int launch_gemm_silu(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int F, int K, const float *ss,
                     int nb, int Mpad, void *act) {
    GemmPlan p = plan_gemm(c, M, 2 * F, K, GEMM_KIND_SWIGLU);
    EpiSilu epi{ss, nb, Mpad, K, c->m.rms_eps, (a16_t *)act, F};
    return launch_bf16<EpiSilu, NT_ANY>(c, s, X, W, M, 2 * F, K, p, epi);
}

int launch_gemm_bias_silu(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, int N, int K,
                          const float *bias, float *z, bool residual, void *xg) {
    GemmPlan p = plan_gemm(c, M, N, K, GEMM_KIND_FUSED);
    EpiBiasSilu epi{bias, z, N, residual ? 1 : 0, (a16_t *)xg};
    return launch_bf16<EpiBiasSilu, NT_ANY>(c, s, X, W, M, N, K, p, epi);
}

// q|k|v projection, rotary embedding and cache append in one kernel (bf16 family)
int launch_gemm_qkv_rope(hydra_ctx *c, hipStream_t s, const void *X, const void *W, int M, RowScale rs, int layer,
                         const int32_t *seq_len, const hydra_kv *kv, void *qbuf, int32_t *flags) {
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
                                   int tile_off, int tile_stride, int rows_per_band, int col_off, int bph) {
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
    int dband = band;
    if (bph > 1) {                      // rotary pairing: bands o and o + bph/2 of a head become neighbours
        const int h = band / bph, o = band - h * bph, hb = bph >> 1;
        dband = h * bph + (o % hb) * 2 + o / hb;
    }
    dst[((size_t)(tile_off + dband * tile_stride) * KT + kt) * 64 + lane] = v;
}

int launch_pack_matrix(hydra_ctx *c, hipStream_t s, const void *src, void *dst, int N, int K, int tile_off,
                       int tile_stride, int rows_per_band, int col_off, int bph) {
    (void)c;
    const size_t total = (size_t)ceil_div(N, rows_per_band) * (K / 16) * 64;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t *)src,
                       (u32x4_t *)dst, N, K, tile_off, tile_stride, rows_per_band, col_off, bph);
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
