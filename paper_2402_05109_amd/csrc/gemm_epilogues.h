// Epilogues of the weight-streaming bf16 GEMM (see gemm_bf16.h for the interface) and the row-scale helpers they
// share.  Used by the stand-alone GEMM kernels (bf16_gemm.hip) and by the persistent layer kernel (bf16_layers.hip).
//
// Epilogues with a DEV parameter write their results either with ordinary stores (DEV = false: the consumer is a
// later kernel) or with device-scope write-through stores (DEV = true: the consumer is another workgroup of the
// same kernel, which reads them after a grid-wide hand-off; see bf16_layers.hip).
#pragma once

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
template <bool DEV>
struct EpiPlainT {
    float *out; int ld; size_t split_stride;
    static constexpr bool LDS_PROLOGUE = false, PAIRED = false, EXTRA_BLOCKS = false, ROWWISE = false;
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
            if (row < g.M) st_dev<DEV>(dst + (size_t)row * ld, acc[v]);
        }
    }
};

// top2_merge without branches (the sixteen rows of a tile are independent chains that the compiler may interleave)
__device__ __forceinline__ void top2_join(Top2 &a, const Top2 &b) {
    const bool take = b.v1 > a.v1 || (b.v1 == a.v1 && b.i1 < a.i1);
    const float loser = take ? a.v1 : b.v1;
    a.v2 = fmaxf(take ? b.v2 : a.v2, loser);
    a.v1 = take ? b.v1 : a.v1;
    a.i1 = take ? b.i1 : a.i1;
}
template <int CTRL>
__device__ __forceinline__ Top2 top2_dpp(const Top2 &q) {
    Top2 u;
    u.v1 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(q.v1), CTRL, 0xf, 0xf, false));
    u.i1 = __builtin_amdgcn_update_dpp(0, q.i1, CTRL, 0xf, 0xf, false);
    u.v2 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(q.v2), CTRL, 0xf, 0xf, false));
    return u;
}

// LM head when only the greedy token and its margin are wanted: instead of the 32x32 tile of logits, each band leaves
// per row (largest sum, its column, second largest sum) of its 32 columns, cand[band][Mpad] as four floats (the
// column as integer bits).  Columns at or beyond V (padding of the last band) do not take part.  The sums are left
// unscaled: argmax_bands_kernel applies the row's 1/rms and merges the bands.
struct EpiTop2 {
    float *cand; int Mpad; int V;
    static constexpr bool LDS_PROLOGUE = false, PAIRED = false, EXTRA_BLOCKS = false, ROWWISE = true;
    template <int MB, int NT> __device__ __forceinline__ NoPre issue(const GemmTile<MB, NT> &, const GemmGeom &) const { return NoPre{}; }
    template <int MB, int NT> __device__ __forceinline__ NoPre prologue(NoPre, const GemmTile<MB, NT> &, const GemmGeom &) const { return NoPre{}; }
    template <int MB, int NT> __device__ __forceinline__ void before_barrier(NoPre, const GemmTile<MB, NT> &, const GemmGeom &) const {}
    template <int MB, int NT> __device__ __forceinline__ void begin(const GemmTile<MB, NT> &, const GemmGeom &) const {}
    // The same from the workgroup's LDS reduction buffer (waves that split K): copies[w * copy_stride + v * 64 + lane] is
    // accumulator register v of K-split wave w.  Here a lane takes one ROW of the tile and half of its 32 columns, adds
    // the copies in wave order and keeps a running top-2, so one exchange between the two halves finishes the row (the
    // column-wise way above needs a reduction across lanes for each of the 16 registers).  Row r of the tile lives in
    // register 4 * (r / 8) + r % 4 of the lanes 32 * ((r % 8) / 4) + column; the columns are visited in an order rotated
    // by the row, so that the 32 lanes of a half read 32 different LDS banks.
    template <int MB, int NT>
    __device__ __forceinline__ void rows(const float *copies, size_t copy_stride, int KW, int a, int i, const GemmTile<MB, NT> &t,
                                         const GemmGeom &g) const {
        const int band = t.tile0 + i;
        if (band >= g.NTiles) return;
        const int r = t.lane & 31, h = t.lane >> 5;
        const float *src = copies + (4 * (r >> 3) + (r & 3)) * 64 + 32 * ((r & 7) >> 2);
        float x[16];
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) x[jj] = 0.f;
        for (int w = 0; w < KW; ++w) {                                         // sixteen independent reads per copy, added in wave order
#pragma unroll
            for (int jj = 0; jj < 16; ++jj) x[jj] += src[(size_t)w * copy_stride + ((jj + r + 16 * h) & 31)];
        }
        Top2 q = {-INFINITY, 0x7fffffff, -INFINITY};
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const int col = band * 32 + ((jj + r + 16 * h) & 31);
            top2_join(q, Top2{col < V ? x[jj] : -INFINITY, col < V ? col : 0x7fffffff, -INFINITY});
        }
        top2_join(q, Top2{__shfl_xor(q.v1, 32, 64), __shfl_xor(q.i1, 32, 64), __shfl_xor(q.v2, 32, 64)});
        const int row = 32 * (t.mb0 + a) + r;
        if (h == 0 && row < g.M) reinterpret_cast<f32x4_t *>(cand)[(size_t)band * Mpad + row] = f32x4_t{q.v1, __int_as_float(q.i1), q.v2, 0.f};
    }
    template <int MB, int NT>
    __device__ __forceinline__ void tile(const f32x16_t &acc, int a, int i, const GemmTile<MB, NT> &t, const GemmGeom &g) const {
        const int band = t.tile0 + i;
        if (band >= g.NTiles) return;
        const int col = band * 32 + (t.lane & 31);
        f32x4_t *dst = reinterpret_cast<f32x4_t *>(cand) + (size_t)band * Mpad;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = acc_row(t.mb0 + a, v, t.lane);
            Top2 q = {col < V ? acc[v] : -INFINITY, col < V ? col : 0x7fffffff, -INFINITY};
            // over the 32 columns of the band: four data-parallel-primitive steps inside the rows of 16 lanes (each joins
            // two disjoint sets of lanes, so no column is counted twice), then one exchange between the two rows
            top2_join(q, top2_dpp<0xB1>(q));                                   // quad_perm [1,0,3,2]
            top2_join(q, top2_dpp<0x4E>(q));                                   // quad_perm [2,3,0,1]
            top2_join(q, top2_dpp<0x141>(q));                                  // row_half_mirror
            top2_join(q, top2_dpp<0x140>(q));                                  // row_mirror
            top2_join(q, Top2{__shfl_xor(q.v1, 16, 64), __shfl_xor(q.i1, 16, 64), __shfl_xor(q.v2, 16, 64)});
            if ((t.lane & 31) == 0 && row < g.M) dst[row] = f32x4_t{q.v1, __int_as_float(q.i1), q.v2, 0.f};
        }
    }
};

// Residual branch end: x += acc.  Also leaves what the next RMSNorm'd GEMM needs:
// xg = half(x * gain) in GEMM input order (the 1/rms factor commutes with the
// contraction and is applied by the consumer) and ss[band][row] = sum over the
// band's 32 columns of x^2.
struct EpiResid {
    float *x; int d; const float *gain; a16_t *xg; float *ss; int Mpad; int32_t *flags;
    static constexpr bool LDS_PROLOGUE = false, PAIRED = false, EXTRA_BLOCKS = false, ROWWISE = false;
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
                xgp[x_index<true>(row, col, d)] = f2a_f(xn * gn, flags);
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
template <bool DEV>
struct EpiSiluT {
    const float *ss; int nb; int Mpad; int dmodel; float eps; a16_t *act; int F; int32_t *flags;
    static constexpr bool LDS_PROLOGUE = true, PAIRED = false, EXTRA_BLOCKS = false, ROWWISE = false;
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
            const float y = silu_f(r * gate) * (r * up);
            if ((t.mb0 + a) * 32 + rl < g.M) flag_saturation(y, 0.f, flags);     // rows past M hold don't-care values: not reported
            stage[((fo >> 3) * 32 + rl) * 8 + (fo & 7)] = f2a(y);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");           // LDS is in order within a wave; keep the compiler from reordering
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const u32x4_t blk = reinterpret_cast<const u32x4_t *>(stage)[t.lane];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        st_dev128<DEV>(reinterpret_cast<u32x4_t *>(act) + ((size_t)(t.mb0 + a) * (F >> 4) + (t.tile0 + i)) * 64 + t.lane, blk);
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
template <bool DEV>
struct EpiQkvRopeT {
    const float *ss; int nb; int Mpad; int dmodel; float eps;
    const int32_t *seq_len; const TreeDev *tree; const int32_t *page_table; int max_pages, n_pages, layer;
    a16_t *kpages, *vpages, *qbuf; const float *rope; int H, Dh, T, max_pos; int32_t *flags;
    int kv_touch_max;       // no pre-read when the rows of the call hold more keys than this in all (see extra_block)
    static constexpr bool LDS_PROLOGUE = true, PAIRED = true, EXTRA_BLOCKS = true, ROWWISE = false;
    // Workgroups behind the last band group (the q|k|v GEMM of up to 64 rows leaves a quarter of the CUs without
    // one) read this layer's cached K and V pages once, so that tree attention, which follows and is a chain of
    // dependent round trips, finds them in the memory-side cache.  Nothing is computed from the values.  Only for
    // short rows: with more keys attention is a throughput problem spread over many workgroups, and the extra
    // pass over K/V costs this GEMM more than attention gains (measured at 2066 and 4114 keys: +0.13 and +0.63 ms).
    __device__ __forceinline__ void extra_block(int w, int n, const GemmGeom &g) const {
        const int rows = (g.M + T - 1) / T;
        const int n16 = H * Dh * 2;                                  // 16-byte pieces of one page of one layer (16 tokens, all heads)
        // the limit is on the keys of all rows together: a batch of rows makes attention a throughput problem as a long
        // row does (at 16 rows of 512 keys the pre-read was 134 MB per layer and took six times as long as the GEMM)
        int total = 0;
        for (int b = 0; b < rows; ++b) total += max(seq_len[b], 0) + T;
        if (total > kv_touch_max) return;                            // uniform over the workgroup
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
                    const int page = page_table[(size_t)b * max_pages + (slot >> 4)];
                    if ((unsigned)page >= (unsigned)n_pages) {            // bad table entry: the row is skipped and flagged
                        if (t.tile0 == 0) atomicOr(flags, FLAG_BAD_PAGE);
                        c.pos[q] = -1;
                    }
                    c.pagetok[q] = page * 16 + (slot & 15);
                    c.bn[q] = b * 128 + n;
                } else if (t.tile0 == 0) {
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
                st_dev<DEV>(vp + base + v_in_block<true>(tok, dim0, Dh), f2a_f(r * x0[q], flags));
                st_dev<DEV>(vp + base + v_in_block<true>(tok, dim1, Dh), f2a_f(r * x1[q], flags));
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
                st_dev<DEV>(qp + ((((blk + (j >> 4)) * 64 + ((j >> 3) & 1) * 32 + (n & 31)) << 3) + (j & 7)), f2a_f(y0, flags));
                const int j1 = j + half;
                st_dev<DEV>(qp + ((((blk + (j1 >> 4)) * 64 + ((j1 >> 3) & 1) * 32 + (n & 31)) << 3) + (j1 & 7)), f2a_f(y1, flags));
            } else {
                const size_t base = kv_block_base(layer, n_pages, pagetok[q] >> 4, H, h, Dh);
                const int tok = pagetok[q] & 15;
                st_dev<DEV>(kp + base + k_in_block<true>(tok, j, Dh), f2a_f(y0, flags));
                st_dev<DEV>(kp + base + k_in_block<true>(tok, j + half, Dh), f2a_f(y1, flags));
            }
        }
    }
    template <int MB, int NT>
    __device__ __forceinline__ void tile(const f32x16_t &, int, int, const GemmTile<MB, NT> &, const GemmGeom &) const {}
};

// Draft-head MLP layer: z = (residual ? z : 0) + SiLU(acc + bias), fp32 and as next GEMM input
struct EpiBiasSilu {
    const float *bias; float *z; int d; int residual; a16_t *xg; int32_t *flags;
    static constexpr bool LDS_PROLOGUE = false, PAIRED = false, EXTRA_BLOCKS = false, ROWWISE = false;
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
            xgp[x_index<true>(row, col, d)] = f2a_f(y, flags);
        }
    }
};

typedef EpiPlainT<false> EpiPlain;
typedef EpiSiluT<false> EpiSilu;
typedef EpiQkvRopeT<false> EpiQkvRope;

}  // namespace hydra
