// The weight-streaming bf16 GEMM of the bf16 storage family (device code).
//
//   C[m][n] = sum_k X[m][k] * W[n][k]       fp32 accumulation
//
// At M <= 128 rows every weight byte is used once, so the kernel is a stream
// over W that has to keep HBM busy.  W (N x K, 16-bit) is stored as 32 x 16
// (n x k) tiles of 1 KiB in the register order of the 32x32x16 MFMA "B" operand
// (lane = (k%16)/8*32 + n%32 holds 8 consecutive k); the tiles of one 32-row
// band are contiguous along k.  X uses the same tile order ("A" operand).
//
// Work split.  A wave owns NT bands and every KW-th block of GEMM_U k-steps; it loads
// its W tiles (and the matching X tiles, which hit in L1/L2) straight into
// registers with fully coalesced 16-byte-per-lane loads, U k-steps ahead of
// the MFMAs, and never synchronises with other waves while streaming.  A
// workgroup is NW x KW waves: KW waves share a band group and split K.  All of
// them leave their accumulators in LDS; then wave kw adds the KW copies of the
// 32x32 tiles j = kw, kw + KW, ... in wave order (a fixed order, so results do
// not depend on scheduling) and runs the epilogue on those tiles, which spreads
// the epilogue over the workgroup.  grid.y = S > 1 splits K over workgroups as
// well; then each split hands its own partial tiles to the epilogue (only
// epilogues that write per-split outputs accept S > 1).
//
// The epilogue is a functor with
//   tile(acc, a, i, t, g): one finished 32x32 tile in the MFMA layout,
//       acc[v] -> row = 32*(mb0+a) + 8*(v/4) + 4*(lane/32) + v%4,  col = 32*(tile0+i) + lane%32;
//   issue(t, g) / prologue(pre, t, g): run in every wave while the first two blocks of W are in
//       flight: issue() only starts loads (returned in registers), prologue() consumes them after the
//       second block has been requested and may start further loads whose registers it returns;
//   before_barrier(carry, t, g): after streaming; receives what prologue() returned.  None of the
//       three may contain a workgroup barrier; what they leave in LDS is visible to tile() because a
//       barrier separates streaming from the epilogue;
//   begin(t, g): once per wave after that barrier, before its first tile.
// An epilogue with ROWWISE = true also has rows(copies, copy_stride, KW, a, i, t, g): where waves split K it is handed the
// LDS reduction buffer of tile (a, i) instead of the summed registers and reads it in whatever order suits it.
// An epilogue with PAIRED = true (NT = 2 or 4: one or two band pairs per wave) instead receives both tiles of a
// band pair, four accumulator registers (rows) at a time:  pair4(x0, x1, a, v0, t, g) with x0[q], x1[q] the
// registers v0 + q of the pair's tiles in row block a, and t.tile0 the pair's first band.  The 4*MB items of
// each pair are shared out over the KW waves.
#pragma once

#include <type_traits>
#include <utility>

#include "device_common.h"

namespace hydra {

typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

struct GemmGeom {
    const u32x4_t *X, *W;
    int M;          // valid rows
    int NTiles;     // 32-column bands of W (N padded up)
    int KT;         // k-steps of 16 in K
    int kpw;        // k-steps per wave
    int NW, KW;     // waves per workgroup along N and K (KW a power of two)
    int gx, gy, gz; // gz > 1 (several row groups): the grid is one-dimensional and gemm_block() maps it onto (gx, gy, gz)
};

// Which (band group, K split, row group) a workgroup takes.  With several row groups the workgroups that stream the
// same weight bands should meet in one L2: workgroups are handed to the 8 XCDs in turn, so workgroup i runs on XCD
// i % 8, and the row groups of one (band group, split) take consecutive places on one XCD.  The grid is rounded up
// to whole sets of 8 (band group, split) pairs; false: no such pair (the whole workgroup leaves).
__device__ __forceinline__ bool gemm_block(const GemmGeom &g, int &bx, int &by, int &bz) {
    if (g.gz <= 1) { bx = (int)blockIdx.x; by = (int)blockIdx.y; bz = 0; return true; }
    const int i = (int)blockIdx.x, xcd = i & 7, j = i >> 3;
    bz = j % g.gz;
    const int q = (j / g.gz) * 8 + xcd;
    bx = q % g.gx;
    by = q / g.gx;
    return q < g.gx * g.gy;
}

// floats reserved in front of the reduction buffer: per-wave partial row sums [8 waves][128 rows], then per
// wave a 1 KiB staging block (epilogues that assemble whole operand tiles) and a 128-row table of row scales
// and three 128-row tables of per-row integers shared by the workgroup
enum { GEMM_LDS_ROWSUM = 0, GEMM_LDS_ROWINFO = 8 * 128, GEMM_LDS_STAGE = 8 * 128 + 3 * 128, GEMM_LDS_STAGE_WAVE = 256 + 128,
       GEMM_LDS_SCRATCH = 8 * 128 + 3 * 128 + 8 * (256 + 128) };

// prefetch distance in k-steps: two register sets of U*(NT+MB) KiB per wave
template <int MB, int NT> struct GemmU {
    enum { value = (MB * NT >= 12) ? 2 : (MB * NT == 8) ? 4 : (MB * NT >= 6) ? 2 : ((MB + NT >= 5) ? 2 : 4) };
};

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a compile-time constant
// whatever the unroller decides, so that register arrays indexed by it never have to live in memory
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

template <int MB, int NT>
struct GemmTile {
    int tile0;      // first band of this wave
    int mb0;        // first 32-row block
    int lane, wave;
    int split;      // blockIdx.y
    float *lds;     // GEMM_LDS_SCRATCH floats of per-workgroup scratch
};

// One workgroup of the GEMM: (bx, by, bz) are its band-group, K-split and row-group indices (the plain kernel passes
// its block indices), red its dynamic LDS.
// ROWGROUPS: the launch has several row groups (see the load of W and the K walk below)
template <int MB, int NT, class Epilogue, int GEMM_U, bool ROWGROUPS = false>
__device__ __forceinline__ void gemm_bf16_body(const GemmGeom &g, const Epilogue &epi, int bx, int by, int bz, float *red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nw = wave % g.NW, kw = wave / g.NW;
    const int group = bx * g.NW + nw;               // band group of this wave
    GemmTile<MB, NT> t;
    t.tile0 = group * NT;
    t.mb0 = bz * MB;
    t.lane = lane;
    t.wave = wave;
    t.split = by;
    t.lds = red;
    float *redbuf = red + GEMM_LDS_SCRATCH;
    // the KW waves of a workgroup share the k-range of their split block by block (wave kw takes the blocks
    // kw, kw + KW, ... of GEMM_U steps), so that together they sweep each band as one contiguous front
    const int s_begin = min(g.KT, by * g.KW * g.kpw);
    const int k_end = min(g.KT, s_begin + g.KW * g.kpw);

    const u32x4_t *wrow[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) wrow[i] = g.W + (size_t)min(t.tile0 + i, g.NTiles - 1) * g.KT * 64 + lane;
    const u32x4_t *xrow[MB];
#pragma unroll
    for (int a = 0; a < MB; ++a) xrow[a] = g.X + (size_t)(t.mb0 + a) * g.KT * 64 + lane;
    f32x16_t acc[MB][NT];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][i][v] = 0.f;

    u32x4_t wa[GEMM_U][NT], xa[GEMM_U][MB], wb[GEMM_U][NT], xb[GEMM_U][MB];
    auto load = [&](u32x4_t (&w)[GEMM_U][NT], u32x4_t (&x)[GEMM_U][MB], int k0) {
#pragma unroll
        for (int u = 0; u < GEMM_U; ++u) {
            const int k = min(k0 + u, g.KT - 1);         // clamped: a ragged tail re-reads a valid tile and skips its MFMA
#pragma unroll
            for (int i = 0; i < NT; ++i)            // a streaming load where each byte is used once; with several row groups the
                w[u][i] = ROWGROUPS ? wrow[i][(size_t)k * 64] : __builtin_nontemporal_load(wrow[i] + (size_t)k * 64);   // others on this XCD read the same lines: keep them in L2
#pragma unroll
            for (int a = 0; a < MB; ++a) x[u][a] = xrow[a][(size_t)k * 64];
        }
    };
    auto compute = [&](u32x4_t (&w)[GEMM_U][NT], u32x4_t (&x)[GEMM_U][MB], int k0) {
#pragma unroll
        for (int u = 0; u < GEMM_U; ++u) {
            if (k0 + u < k_end) {
#pragma unroll
                for (int a = 0; a < MB; ++a)
#pragma unroll
                    for (int i = 0; i < NT; ++i)
                        acc[a][i] = HYDRA_MFMA16(__builtin_bit_cast(a16x8_t, x[u][a]), __builtin_bit_cast(a16x8_t, w[u][i]), acc[a][i]);
            }
        }
    };
    // One row group (X is small): k-blocks of U steps are visited in an order rotated by the band-group index, so
    // that the workgroups streaming different bands do not all ask the L2 for the same X lines at once.  With several
    // row groups X is large (M x K), and every band group re-reads it: there all workgroups walk K in the same order,
    // so that the part of X in use at any time fits in L2 (rotated, each band group's X reads missed: at 1024 rows
    // the GEMMs fetched 11-13 times their weight bytes from memory).
    const int nblk = ((k_end - s_begin + GEMM_U - 1) / GEMM_U - kw + g.KW - 1) / g.KW;
    const int rot = (!ROWGROUPS && nblk > 0) ? (int)(((unsigned)bx * 5u) % (unsigned)nblk) : 0;
    auto kof = [&](int j) { int q = j + rot; if (q >= nblk) q -= nblk; return s_begin + (q * g.KW + kw) * GEMM_U; };
    // Two register sets alternate.  The long-run case is its own straight-line region whose refills are
    // unconditional: only then can the compiler count how many loads are younger than the set it is about to
    // use, and wait for exactly that set instead of draining the queue (a refill behind a condition makes it
    // assume the worst, which turns the double buffer into issue-then-wait).
    auto stream = [&](auto steady) {
        constexpr bool STEADY = decltype(steady)::value;
        if (STEADY || nblk > 0) load(wa, xa, kof(0));
        auto pre = epi.issue(t, g);
        if (STEADY || nblk > 1) load(wb, xb, kof(1));
        auto carry = epi.prologue(pre, t, g);
        int j = 0;
        if constexpr (STEADY) {
            for (; j + 3 < nblk; j += 2) {
                compute(wa, xa, kof(j));
                load(wa, xa, kof(j + 2));
                compute(wb, xb, kof(j + 1));
                load(wb, xb, kof(j + 3));
            }
        }
        // at most three blocks left: j in wa, j + 1 in wb, j + 2 still to fetch
        if (j < nblk) compute(wa, xa, kof(j));
        if (j + 2 < nblk) load(wa, xa, kof(j + 2));
        if (j + 1 < nblk) compute(wb, xb, kof(j + 1));
        if (j + 2 < nblk) compute(wa, xa, kof(j + 2));
        return carry;
    };
    auto carry = nblk >= 4 ? stream(std::true_type{}) : stream(std::false_type{});

    // ---- finish: KW == 1 keeps everything in registers; otherwise meet in LDS and share the tiles out
    epi.before_barrier(carry, t, g);
    const bool live = t.tile0 < g.NTiles;                         // surplus waves streamed a clamped band: discard
    constexpr int TILES = MB * NT;
    if (g.KW == 1) {
        if (Epilogue::LDS_PROLOGUE && (g.NW > 1 || Epilogue::PAIRED)) __syncthreads();
        if (!live) return;
        epi.begin(t, g);
        if constexpr (Epilogue::PAIRED) {
            static_for<NT / 2>([&](auto PR) {
                constexpr int pr = decltype(PR)::value;
                GemmTile<MB, NT> tp = t;
                tp.tile0 = t.tile0 + 2 * pr;
                static_for<MB>([&](auto A) {
                    static_for<4>([&](auto Q4) {
                        constexpr int a = decltype(A)::value, q4 = decltype(Q4)::value;
                        float x0[4], x1[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) { x0[q] = acc[a][2 * pr][4 * q4 + q]; x1[q] = acc[a][2 * pr + 1][4 * q4 + q]; }
                        epi.pair4(x0, x1, a, 4 * q4, tp, g);
                    });
                });
            });
        } else {
            static_for<MB * NT>([&](auto J) {
                constexpr int a = decltype(J)::value / NT, i = decltype(J)::value % NT;
                const f32x16_t tile_acc = acc[a][i];                    // a copy: no address of an accumulator escapes
                epi.tile(tile_acc, a, i, t, g);
            });
        }
        return;
    }
    {
        float *dst = redbuf + ((size_t)(kw * g.NW + nw) * TILES) * 16 * 64 + lane;
#pragma unroll
        for (int a = 0; a < MB; ++a)
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) dst[((a * NT + i) * 16 + v) * 64] = acc[a][i][v];
    }
    __syncthreads();
    if (!live) return;
    epi.begin(t, g);
    if constexpr (Epilogue::ROWWISE) {                             // the epilogue reads the tile row by row out of the reduction buffer itself
        for (int j = kw; j < TILES; j += g.KW)                     // wave-uniform
            epi.rows(redbuf + ((size_t)nw * TILES + j) * 16 * 64, (size_t)g.NW * TILES * 16 * 64, g.KW, j / NT, j % NT, t, g);
    } else if constexpr (Epilogue::PAIRED) {
        for (int id = kw; id < MB * 4 * (NT / 2); id += g.KW) {    // wave-uniform
            const int pr = id / (MB * 4), r = id - pr * (MB * 4);
            const int a = r >> 2, v0 = (r & 3) * 4;
            float x0[4] = {0.f, 0.f, 0.f, 0.f}, x1[4] = {0.f, 0.f, 0.f, 0.f};
            for (int w = 0; w < g.KW; ++w) {
                const float *src = redbuf + ((size_t)(w * g.NW + nw) * TILES + a * NT + 2 * pr) * 16 * 64 + lane;
#pragma unroll
                for (int q = 0; q < 4; ++q) { x0[q] += src[(v0 + q) * 64]; x1[q] += src[(16 + v0 + q) * 64]; }
            }
            GemmTile<MB, NT> tp = t;
            tp.tile0 = t.tile0 + 2 * pr;
            epi.pair4(x0, x1, a, v0, tp, g);
        }
    } else {
#pragma unroll
        for (int a = 0; a < MB; ++a)
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                const int j = a * NT + i;
                if (j % g.KW != kw) continue;                          // wave-uniform
                f32x16_t sum;
#pragma unroll
                for (int v = 0; v < 16; ++v) sum[v] = 0.f;
                for (int w = 0; w < g.KW; ++w) {
                    const float *src = redbuf + ((size_t)(w * g.NW + nw) * TILES + j) * 16 * 64 + lane;
#pragma unroll
                    for (int v = 0; v < 16; ++v) sum[v] += src[v * 64];
                }
                epi.tile(sum, a, i, t, g);
            }
    }
}


template <int MB, int NT, int MAXT, class Epilogue, bool ROWGROUPS = false, int GEMM_U = GemmU<MB, NT>::value>
__global__ __launch_bounds__(MAXT) void gemm_bf16_kernel(GemmGeom g, Epilogue epi) {
    extern __shared__ float red[];                 // [scratch] + [KW][NW][MB*NT][16][64]
    if constexpr (Epilogue::EXTRA_BLOCKS) {        // workgroups behind the last band group: side work of the epilogue's choosing
        const int wgs = ((g.NTiles + NT - 1) / NT + g.NW - 1) / g.NW;
        if (g.gz <= 1 && (int)blockIdx.x >= wgs) { epi.extra_block((int)blockIdx.x - wgs, (int)gridDim.x - wgs, g); return; }
    }
    int bx, by, bz;
    if (!gemm_block(g, bx, by, bz)) return;
    gemm_bf16_body<MB, NT, Epilogue, GEMM_U, ROWGROUPS>(g, epi, bx, by, bz, red);
}

// Variant for many rows (four row blocks per workgroup): the X tiles dominate what a workgroup pulls through its CU's
// request path, so here the NWT waves of a workgroup take different band groups, all walk the workgroup's K range
// block by block in step, and share the X tiles of a block through LDS: each wave fetches 1/NWT of them, two blocks
// live in LDS, one workgroup barrier per block.  W still goes straight to registers, two sets alternating.  No wave
// splits K, so the epilogue runs on the wave's own accumulators; grid.y may split K over workgroups (g.kpw k-steps
// each) for epilogues that write per-split outputs.
//   iteration j: multiply block j (X from LDS buffer j % 2) | refill the W set just used with block j + 2 |
//   barrier (every wave is done with buffer j % 2) | store the fetched X share of block j + 2 there |
//   request the share of block j + 3.
// The store becomes visible to the others at the barrier of iteration j + 1, in front of block j + 2.  Every load
// is unconditional (blocks past the end re-read the last one and their MFMAs are skipped), so waits are exact and
// every wave meets the same number of barriers.
template <int MB, int NT, int NWT, class Epilogue, int GEMM_U = 4>
__global__ __launch_bounds__(NWT * 64) void gemm_bf16_sharedx_kernel(GemmGeom g, Epilogue epi) {
    extern __shared__ float red[];                 // [scratch] + 2 x [GEMM_U][MB] X tiles of 1 KiB
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int bx, by, bz;
    if (!gemm_block(g, bx, by, bz)) return;
    GemmTile<MB, NT> t;
    t.tile0 = (bx * NWT + wave) * NT;
    t.mb0 = bz * MB;
    t.lane = lane;
    t.wave = wave;
    t.split = by;
    t.lds = red;
    constexpr int XT = GEMM_U * MB;                 // X tiles per block
    constexpr int XS = (XT + NWT - 1) / NWT;        // of which this wave fetches up to XS
    u32x4_t *xbuf = reinterpret_cast<u32x4_t *>(red + GEMM_LDS_SCRATCH);

    const u32x4_t *wrow[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) wrow[i] = g.W + (size_t)min(t.tile0 + i, g.NTiles - 1) * g.KT * 64 + lane;
    const u32x4_t *xbase = g.X + (size_t)t.mb0 * g.KT * 64 + lane;
    f32x16_t acc[MB][NT];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][i][v] = 0.f;

    // grid.y > 1 splits K over workgroups (g.kpw k-steps each; only epilogues that write per-split outputs)
    const int s_begin = min(g.KT, by * g.kpw), k_end = min(g.KT, s_begin + g.kpw);
    const int nblk = (k_end - s_begin + GEMM_U - 1) / GEMM_U;
    auto kof = [&](int j) { return j >= nblk ? k_end : s_begin + j * GEMM_U; };      // every workgroup of a split walks its K range in the same order: the part of X in use fits in L2
    u32x4_t wa[GEMM_U][NT], wb[GEMM_U][NT], xs[XS];
    auto load_w = [&](u32x4_t (&w)[GEMM_U][NT], int k0) {
#pragma unroll
        for (int u = 0; u < GEMM_U; ++u) {
            const int k = min(k0 + u, g.KT - 1);
#pragma unroll
            for (int i = 0; i < NT; ++i) w[u][i] = wrow[i][(size_t)k * 64];      // not a streaming load: the other row groups on this XCD read the same lines
        }
    };
    // tile q of a block: k-step q / MB, row block q % MB; this wave fetches q = wave, wave + NWT, ...
    auto load_x = [&](int k0) {
#pragma unroll
        for (int e = 0; e < XS; ++e) {
            const int q = min(wave + e * NWT, XT - 1);
            const int k = min(k0 + q / MB, g.KT - 1);
            xs[e] = xbase[((size_t)(q % MB) * g.KT + k) * 64];
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int e = 0; e < XS; ++e) {
            const int q = wave + e * NWT;
            if (q < XT) xbuf[((size_t)buf * XT + q) * 64 + lane] = xs[e];
        }
    };
    // the X tiles of k-step u + 1 are read from LDS while the MFMAs of k-step u run
    auto compute = [&](u32x4_t (&w)[GEMM_U][NT], int buf, int k0) {
        const u32x4_t *xb = xbuf + (size_t)buf * XT * 64 + lane;
        u32x4_t xr[2][MB];
#pragma unroll
        for (int a = 0; a < MB; ++a) xr[0][a] = xb[a * 64];
#pragma unroll
        for (int u = 0; u < GEMM_U; ++u) {
            if (u + 1 < GEMM_U) {
#pragma unroll
                for (int a = 0; a < MB; ++a) xr[(u + 1) & 1][a] = xb[((u + 1) * MB + a) * 64];
            }
            if (k0 + u < k_end) {
#pragma unroll
                for (int a = 0; a < MB; ++a)
#pragma unroll
                    for (int i = 0; i < NT; ++i)
                        acc[a][i] = HYDRA_MFMA16(__builtin_bit_cast(a16x8_t, xr[u & 1][a]), __builtin_bit_cast(a16x8_t, w[u][i]), acc[a][i]);
            }
        }
    };

    load_w(wa, kof(0));
    load_x(kof(0));
    auto pre = epi.issue(t, g);
    load_w(wb, kof(1));
    auto carry = epi.prologue(pre, t, g);
    store_x(0);
    load_x(kof(1));
    store_x(1);
    load_x(kof(2));
    __syncthreads();
    for (int j = 0; j < nblk; j += 2) {
        compute(wa, 0, kof(j));
        load_w(wa, kof(j + 2));
        __syncthreads();
        store_x(0);
        load_x(kof(j + 3));
        if (j + 1 < nblk) compute(wb, 1, kof(j + 1));
        load_w(wb, kof(j + 3));
        __syncthreads();
        store_x(1);
        load_x(kof(j + 4));
    }

    epi.before_barrier(carry, t, g);
    if (Epilogue::LDS_PROLOGUE) __syncthreads();
    if (t.tile0 >= g.NTiles) return;                                // surplus waves streamed a clamped band: discard
    epi.begin(t, g);
    if constexpr (Epilogue::PAIRED) {
        static_for<MB>([&](auto A) {
            static_for<4>([&](auto Q4) {
                constexpr int a = decltype(A)::value, q4 = decltype(Q4)::value;
                float x0[4], x1[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) { x0[q] = acc[a][0][4 * q4 + q]; x1[q] = acc[a][NT - 1][4 * q4 + q]; }
                epi.pair4(x0, x1, a, 4 * q4, t, g);
            });
        });
    } else {
#pragma unroll
        for (int a = 0; a < MB; ++a)
#pragma unroll
            for (int i = 0; i < NT; ++i) epi.tile(acc[a][i], a, i, t, g);
    }
}

}  // namespace hydra
