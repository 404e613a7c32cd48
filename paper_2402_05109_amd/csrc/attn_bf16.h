// Tree attention on MFMA, 16-bit family: the body of one workgroup (see bf16_attn.hip for the method and the
// launch shapes).  Shared by the stand-alone kernel and by the persistent layer kernel (bf16_layers.hip).
#pragma once

#include "device_common.h"
#include "internal.h"

namespace hydra {

typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;


// record of one workgroup in the partial buffer: O[Tq][Dh], m[Tq], l[Tq]   (Tq = 32 * ceil(T/32))
__host__ __device__ inline size_t apart_record(int Tq, int Dh) { return (size_t)Tq * Dh + 2 * (size_t)Tq; }

enum { ATTN_WAVES = 8 };

template <int DH>
struct KVTile { u32x4_t k[DH / 16]; u32x4_t v[2][DH / 32]; };

template <int DH>
__device__ __forceinline__ void load_kv_tile(KVTile<DH> &kv, const a16_t *kpages, const a16_t *vpages,
                                             int p0, int p1, int layer, int n_pages, int H, int h, int lane) {
    const int hl = lane >> 5, col = lane & 31;
    const u32x4_t *kp = reinterpret_cast<const u32x4_t *>(kpages + kv_block_base(layer, n_pages, (col >> 4) ? p1 : p0, H, h, DH));
#pragma unroll
    for (int s = 0; s < DH / 16; ++s) kv.k[s] = kp[(2 * s + hl) * 16 + (col & 15)];
#pragma unroll
    for (int g = 0; g < 2; ++g) {
        const u32x4_t *vp = reinterpret_cast<const u32x4_t *>(vpages + kv_block_base(layer, n_pages, g ? p1 : p0, H, h, DH));
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt) kv.v[g][dt] = vp[(32 * dt + col) * 2 + hl];
    }
}

// One workgroup of tree attention: (bx of nbx, h, b) are its coordinates in the launch shape described at the top of
// bf16_attn.hip, lds its ATTN_WAVES * 64 + ATTN_WAVES * (DH / 32) * 1024 floats of shared memory.  DEV: the final
// output is written with device-scope stores (the reader is another workgroup of the same kernel).  The function
// contains two workgroup barriers that every wave reaches unless the row is over capacity (uniform early return).
// tid: the thread's index in the workgroup.  QLDS: the query tiles are kept in LDS instead of registers, which takes
// 8 * DH / 32 registers per lane off a kernel that sits at the limit of 256.  They lie in the space of the O merge
// buffers (QW * DH * 64 bytes, never more than those), which are first written behind the barrier that follows the
// key loops of all waves.
template <int DH, bool PACKED, bool DEV, bool QLDS>
__device__ __forceinline__ void attn_bf16_body(
    const u32x4_t *__restrict__ qbuf, const a16_t *__restrict__ kpages, const a16_t *__restrict__ vpages,
    const int32_t *__restrict__ page_table, int max_pages, int n_pages, int layer, const int32_t *__restrict__ seq_len,
    const TreeDev *__restrict__ tree, int T, int H, int QW, int qsplit, float scale, float *__restrict__ apart, void *out,
    int32_t *flags, int bx, int nbx, int h, int b, float *lds, int tid) {
    constexpr int KS = DH / 16, DT = DH / 32;
    const int lane = tid & 63, wave = tid >> 6;
    const int hl = lane >> 5, col = lane & 31;
    const int KWV = ATTN_WAVES / QW;
    const int qw = wave % QW, kwv = wave / QW;
    const int QTtot = (T + 31) >> 5;
    const int Tq = QTtot * 32;
    // qsplit: the workgroups of a (row, head) take different 32-query tiles and each sees all keys (no partial
    // records, no merge kernel); otherwise they split the keys and every workgroup holds all query tiles
    const int qtile = qsplit ? bx * QW + qw : qw;
    const int key_wgs = qsplit ? 1 : nbx;
    const int units = key_wgs * KWV;
    const int unit = (qsplit ? 0 : bx) * KWV + kwv;
    const bool active = qtile < QTtot;                     // idle waves only take part in the barriers
    const int32_t *pt = page_table + (size_t)b * max_pages;
    // Everything whose address does not depend on the row's length is requested before the length is known:
    // the queries, the ancestor masks and the page-table entries of this wave's first key tiles (the table
    // has max_pages entries for every row, so the reads are in bounds; entries past the row's pages are not used).
    enum { PG_AHEAD = 5 };                                 // page ids of this many key tiles per wave are fetched up front
    u32x4_t qreg[KS];
    uint64_t anc0 = 0ull, anc1 = 0ull;
    int pg[PG_AHEAD][2];
    if (active) {
        const size_t blk = (((size_t)b * H + h) * QTtot + qtile) * KS;
#pragma unroll
        for (int s = 0; s < KS; ++s) qreg[s] = qbuf[(blk + s) * 64 + lane];
        if (QLDS && kwv == 0) {                            // one copy per query tile, written by the first wave of its key split
            u32x4_t *qs = reinterpret_cast<u32x4_t *>(lds + ATTN_WAVES * 64) + (size_t)qw * KS * 64;
#pragma unroll
            for (int s = 0; s < KS; ++s) qs[s * 64 + lane] = qreg[s];
        }
        const int query = qtile * 32 + col;
        if (query < T) { anc0 = tree->anc[query][0]; anc1 = tree->anc[query][1]; }
#pragma unroll
        for (int j = 0; j < PG_AHEAD; ++j) {
            const int t = unit + j * units;
            pg[j][0] = pt[min(2 * t, max_pages - 1)];             // checked below, where they are used
            pg[j][1] = pt[min(2 * t + 1, max_pages - 1)];
        }
    }
    const int L = seq_len[b];
    if (QLDS) __syncthreads();                             // the query tiles are in LDS (before any early return: every wave reaches it)
    const u32x4_t *qlds = reinterpret_cast<const u32x4_t *>(lds + ATTN_WAVES * 64) + (size_t)qw * KS * 64 + lane;
    if (L < 0 || L + T > max_pages * 16) {                 // uniform over the workgroup
        if (tid == 0 && bx == 0 && h == 0) atomicOr(flags, FLAG_CAPACITY);
        return;
    }
    const int total = L + T;
    const int n_tiles = (total + 31) >> 5;
    const int row_pages = (total + 15) >> 4;

    f32x16_t o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[dt][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    if (active && unit < n_tiles) {
        KVTile<DH> cur, nxt;
        // second page of a tile: absent when the row ends inside the first one (its keys are masked; any valid page will do)
        {
            const int p0 = checked_page(pg[0][0], n_pages, flags);
            const int p1 = (2 * unit + 1 < row_pages) ? checked_page(pg[0][1], n_pages, flags) : p0;
            load_kv_tile<DH>(cur, kpages, vpages, p0, p1, layer, n_pages, H, h, lane);
        }
        int it = 0;                                        // index of tile t among this wave's tiles
        for (int t = unit; t < n_tiles; t += units, ++it) {
            const bool more = t + units < n_tiles;
            if (more) {
                const int tn = t + units;
                int p0, p1;
                switch (it + 1) {                          // wave-uniform; keeps the page ids in scalar registers
                    case 1: p0 = pg[1][0]; p1 = pg[1][1]; break;
                    case 2: p0 = pg[2][0]; p1 = pg[2][1]; break;
                    case 3: p0 = pg[3][0]; p1 = pg[3][1]; break;
                    case 4: p0 = pg[4][0]; p1 = pg[4][1]; break;
                    default: p0 = pt[2 * tn]; p1 = (2 * tn + 1 < row_pages) ? pt[2 * tn + 1] : p0; break;
                }
                if (2 * tn + 1 >= row_pages) p1 = p0;
                p0 = checked_page(p0, n_pages, flags);                  // wave-uniform
                p1 = checked_page(p1, n_pages, flags);
                load_kv_tile<DH>(nxt, kpages, vpages, p0, p1, layer, n_pages, H, h, lane);
            }
            const int slot0 = t * 32;
            if (slot0 + 32 > total) {   // zero V of slots >= total (stale or never written): 0 * garbage must not appear
#pragma unroll
                for (int g = 0; g < 2; ++g)
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        // dword w holds keys i = 2w, 2w+1 of this half-wave: token = 8*(i/4) + 4*hl + i%4
                        const int i0 = 2 * w, i1 = 2 * w + 1;
                        const int s0 = slot0 + 16 * g + 8 * (i0 >> 2) + 4 * hl + (i0 & 3);
                        const int s1 = slot0 + 16 * g + 8 * (i1 >> 2) + 4 * hl + (i1 & 3);
                        const uint32_t keep = (s0 < total ? 0x0000ffffu : 0u) | (s1 < total ? 0xffff0000u : 0u);
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt) cur.v[g][dt][w] &= keep;
                    }
            }
            f32x16_t sc;
#pragma unroll
            for (int v = 0; v < 16; ++v) sc[v] = 0.f;
            int qoff = 0;
            if (QLDS) asm volatile("" : "+v"(qoff));           // keeps the LDS reads of the queries inside the loop (hoisted, they are registers again)
#pragma unroll
            for (int s = 0; s < KS; ++s)
                sc = HYDRA_MFMA16(__builtin_bit_cast(a16x8_t, cur.k[s]), __builtin_bit_cast(a16x8_t, QLDS ? qlds[qoff + s * 64] : qreg[s]), sc);
            const bool need_mask = slot0 + 32 > L;
            float cmax = -INFINITY;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float x = sc[v] * scale;
                if (need_mask) {
                    const int slot = slot0 + 8 * (v >> 2) + 4 * hl + (v & 3);
                    bool ok = slot < L;
                    if (!ok) {
                        const int a = slot - L;
                        ok = a < T && (((a < 64 ? anc0 >> a : anc1 >> (a - 64)) & 1ull) != 0);
                    }
                    x = ok ? x : -INFINITY;
                }
                sc[v] = x;
                cmax = fmaxf(cmax, x);
            }
            cmax = fmaxf(cmax, __shfl_xor(cmax, 32, 64));
            const float m_new = fmaxf(m_run, cmax);
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __expf(m_run - m_safe);
            float rs = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float p = __expf(sc[v] - m_safe);        // exp(-inf) = 0 for masked keys
                sc[v] = p;
                rs += p;
            }
            rs += __shfl_xor(rs, 32, 64);
            l_run = l_run * alpha + rs;
            m_run = m_new;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[dt][v] *= alpha;
            // P^T operands: page g uses accumulator registers 8g .. 8g+7 in order
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                u32x4_t pb;
#pragma unroll
                for (int w = 0; w < 4; ++w) pb[w] = f2a_pack(sc[8 * g + 2 * w], sc[8 * g + 2 * w + 1]);
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
                    o[dt] = HYDRA_MFMA16(__builtin_bit_cast(a16x8_t, cur.v[g][dt]), __builtin_bit_cast(a16x8_t, pb), o[dt]);
            }
            if (more) cur = nxt;
        }
    }

    // ---- merge the KWV key-split waves of each query tile through LDS
    // layout: ml[QW][KWV][2][32] then O[QW][KWV][DT*16][64]
    float *ml = lds;
    float *ob = lds + ATTN_WAVES * 64;
    if (hl == 0) {
        ml[((qw * KWV + kwv) * 2 + 0) * 32 + col] = m_run;
        ml[((qw * KWV + kwv) * 2 + 1) * 32 + col] = l_run;
    }
    __syncthreads();
    float m_tot = -INFINITY;
    for (int w = 0; w < KWV; ++w) m_tot = fmaxf(m_tot, ml[((qw * KWV + w) * 2 + 0) * 32 + col]);
    float l_tot = 0.f;
    for (int w = 0; w < KWV; ++w) {
        const float mw = ml[((qw * KWV + w) * 2 + 0) * 32 + col];
        l_tot += __expf(mw - (m_tot == -INFINITY ? 0.f : m_tot)) * ml[((qw * KWV + w) * 2 + 1) * 32 + col];
    }
    const float mine = __expf(m_run - (m_tot == -INFINITY ? 0.f : m_tot));
    {
        float *dst = ob + (size_t)(qw * KWV + kwv) * DT * 16 * 64 + lane;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) dst[(dt * 16 + v) * 64] = o[dt][v] * mine;
    }
    __syncthreads();
    if (!active) return;
    // the (band, group of 4 registers = 4 consecutive dims) items are shared out over the KWV waves of the query tile
    const int query = qtile * 32 + col;
    const bool final_out = key_wgs == 1;
    const float inv = final_out ? 1.0f / l_tot : 1.0f;
    float *rec = apart + ((((size_t)b * H + h) * nbx) + bx) * apart_record(Tq, DH);
    for (int id = kwv; id < DT * 4; id += KWV) {
        const int dt = id >> 2, g4 = id & 3;
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int w = 0; w < KWV; ++w) {
            const float *src = ob + (size_t)(qw * KWV + w) * DT * 16 * 64 + lane;
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] += src[(dt * 16 + 4 * g4 + q) * 64];
        }
        const int dim = 32 * dt + 8 * g4 + 4 * hl;
        if (final_out) {
            if (query < T) {
                const int m = b * T + query;
                if (PACKED) {
                    st_dev64<DEV>(reinterpret_cast<a16_t *>(out) + x_index<true>(m, h * DH + dim, H * DH),
                                  f2a_pack(acc[0] * inv, acc[1] * inv), f2a_pack(acc[2] * inv, acc[3] * inv));
                } else {
                    f32x4_t v4 = {acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv};
                    *reinterpret_cast<f32x4_t *>(reinterpret_cast<float *>(out) + ((size_t)m * H + h) * DH + dim) = v4;
                }
            }
        } else {
            f32x4_t v4 = {acc[0], acc[1], acc[2], acc[3]};
            *reinterpret_cast<f32x4_t *>(rec + (size_t)query * DH + dim) = v4;
        }
    }
    if (!final_out && kwv == 0 && hl == 0) {
        rec[(size_t)Tq * DH + query] = m_tot;
        rec[(size_t)Tq * DH + Tq + query] = l_tot;
    }
}

}  // namespace hydra
