// bf16 storage family: all decoder layers of one tree_verify_forward as ONE persistent kernel.
//
// Why.  At up to 64 rows a decoder layer is a stream over its weights (paper, section 1: decoding is bound by moving
// the weights), and as separate kernels its seven steps (q|k|v + rotary + cache append, tree attention, O
// projection, add + norm, gate/up + SwiGLU, down projection, add + norm) each pay a start (kernel arguments, first
// HBM round trip) and an end (LDS reduction, epilogue, store drain, the spread between the first and the last
// workgroup) during which HBM idles: measured, about 45 % of a layer.  Here one workgroup per CU stays resident for
// the whole pass.  The steps are separated by grid-wide hand-offs instead of kernel boundaries, and because weights
// do not depend on activations every workgroup requests the first two weight blocks of its NEXT GEMM item as soon
// as the accumulators of the current one have left the registers, i.e. before the hand-off: the LDS reduction, the
// epilogue, the hand-off itself and the first activation loads of the next step then run under the weight stream.
//
// Hand-off.  A counter that all 256 workgroups bump and poll at one address serialises in the memory system
// (~30 ns per access to the same address: ~8 us per hand-off, measured).  So arrival and release go through a
// two-level tree: workgroup w belongs to group w % 8; it bumps its group's counter; the last arriver of a group
// bumps the grid counter and alone polls it; when all groups have arrived it sets the group's release word, which
// the other members poll (measured: ~0.8 us from the last arrival to the first release).  Every poll loop is
// bounded: on expiry the workgroup sets FLAG_TIMEOUT and the abort word, which the others notice in their own
// loops, and every workgroup leaves the kernel.  The counters are zeroed by a small kernel before each launch.
//
// Visibility.  The L2 caches of the dies are not coherent with each other inside a kernel.  What one step writes
// for the next is written with device-scope (write-through) stores; each wave waits for its stores to be
// acknowledged before its workgroup arrives; and every such buffer has its own address per layer and step, so no
// L2 can hold a line of it from before it was written (the caches are invalidated when the kernel starts).  After
// the release the readers use ordinary loads, which the L2 of their die then shares among its workgroups.
//
// Work split.  A GEMM item is (band group, K split) as in gemm_bf16.h, with the 8 waves of a workgroup splitting
// the item's K range block by block and meeting in LDS; item i of a step runs on workgroup (i + offset) % grid, and
// the steps' plans keep every step at one item per workgroup at most.  Attention items are (row, head, 32-query
// tile), one workgroup each, the 8 waves splitting the keys (contexts up to ~1280 keys; longer ones take the
// multi-kernel path).  The O projection's items start behind the attention items, so that workgroups without an
// attention item hold the O weights in registers by the time attention is done.  Results are bit-identical from
// run to run: every sum has a fixed order.
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>

#include <hip/hip_ext.h>

#include "attn_bf16.h"
#include "gemm_bf16.h"
#include "gemm_epilogues.h"
#include "internal.h"

namespace hydra {

enum { LK_WAVES = 8, LK_THREADS = LK_WAVES * 64, LK_GROUPS = 8, LK_WORDS = 32, LK_BARRIER_WORDS = (1 + 2 * LK_GROUPS) * LK_WORDS,
       LK_STAGES = 7 };

struct GridSync {
    unsigned *base;         // word 0: abort; barrier k at base + LK_WORDS + k * LK_BARRIER_WORDS: grid counter, group counters, release words
    int32_t *flags;
    int spin_limit;
    int groups_expected;    // groups that have members (a test passes one more: no hand-off can then complete)
};

struct StagePlan { int groups, splits, ksplit, n_items, off; };      // item -> (band group = item % groups, split = item / groups), k-steps per split

struct LayerKernelArgs {
    const char *arena;
    size_t attn_norm, wqkv, wo, ffn_norm, wgu, wdown;   // layer 0; layer l adds l * layer_stride
    size_t layer_stride, final_norm;
    int NL, M, Mpad, d, F, H, T, B, nb_first, nb;
    float eps, scale;
    StagePlan q, o, gu, dn;
    int n_attn, QT;
    char *blk;                                          // per-layer buffer blocks: layer l reads block l and writes block l + 1
    size_t blk_stride, x_a, x_b, xg_a, xg_b, ss_a, ss_b, attn, act, part_o, part_d, qbuf;
    const int32_t *seq_len, *page_table;
    int max_pages, n_pages;
    a16_t *kpages, *vpages;
    const TreeDev *tree;
    const float *rope;
    int max_pos;
    int32_t *flags;
    long long *stamps;                                  // NULL, or [NL][LK_STAGES][grid][8] wall-clock stamps (timeline for tuning)
    GridSync sync;
};

// ---- workgroup barrier that orders LDS only (weight loads stay in flight across it) ----
__device__ __forceinline__ void wg_barrier_lds() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
template <int N> __device__ __forceinline__ void wait_vmem_older_than() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

__device__ __forceinline__ unsigned *gs_barrier(const GridSync &s, int k) { return s.base + LK_WORDS + (size_t)k * LK_BARRIER_WORDS; }

// Every wave has waited for its own stores.  ctl: two ints of LDS.
__device__ __forceinline__ void gs_arrive(const GridSync &s, int k, int *ctl) {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (threadIdx.x == 0) {
        const int grp = (int)blockIdx.x % LK_GROUPS;
        const int n_local = ((int)gridDim.x - grp + LK_GROUPS - 1) / LK_GROUPS;
        unsigned *g = gs_barrier(s, k);
        const unsigned old = __hip_atomic_fetch_add(g + (1 + grp) * LK_WORDS, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int leader = old == (unsigned)(n_local - 1);
        if (leader) __hip_atomic_fetch_add(g, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ctl[0] = leader;
    }
}

// false: give up (a wait expired here or elsewhere); uniform over the workgroup
__device__ __forceinline__ bool gs_wait(const GridSync &s, int k, int *ctl) {
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        const int leader = ctl[0];
        unsigned *g = gs_barrier(s, k);
        unsigned *lf = g + (1 + LK_GROUPS + (int)blockIdx.x % LK_GROUPS) * LK_WORDS;
        int ok = 1;
        if (leader) {
            for (int it = 0;;) {
                if (__hip_atomic_load(g, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= (unsigned)s.groups_expected) break;
                ++it;
                if ((it & 15) == 0 && __hip_atomic_load(s.base, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) { ok = 0; break; }
                if (it > s.spin_limit) {
                    ok = 0;
                    if (lane == 0) { atomicOr(s.flags, FLAG_TIMEOUT); __hip_atomic_store(s.base, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            if (lane == 0) __hip_atomic_store(lf, ok ? 1u : 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            unsigned v = 0u;
            for (int it = 0;;) {
                v = __hip_atomic_load(lf, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (v != 0u) break;
                if (++it > 2 * s.spin_limit) {
                    v = 2u;
                    if (lane == 0) { atomicOr(s.flags, FLAG_TIMEOUT); __hip_atomic_store(s.base, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            ok = v == 1u;
        }
        if (lane == 0) ctl[1] = ok;
    }
    wg_barrier_lds();
    const bool ok = ctl[1] != 0;
    asm volatile("" ::: "memory");
    return ok;
}

// ---- weight walk of one wave through its GEMM item ----
// Everything in it is uniform over the wave (the wave index is read with readfirstlane), so it lives in scalar
// registers; the lane's share of an address is added at the load.
template <int NT, int U>
struct WaveWalk {
    const u32x4_t *w0;          // tile (band tile0, k-step 0)
    size_t band_stride;         // 16-byte elements between bands (0 past the last band: the surplus bands re-read it)
    int nt_valid;               // bands of the item that exist
    int bx, by, s_begin, k_end, nblk, rot, kw, KT;
    bool valid;
    __device__ __forceinline__ int kof(int j) const {
        int q = j + rot;
        if (q >= nblk) q -= nblk;
        return s_begin + (q * LK_WAVES + kw) * U;
    }
    __device__ __forceinline__ const u32x4_t *tile(int i, int k) const {
        return w0 + (size_t)min(i, nt_valid - 1) * band_stride + (size_t)k * 64;
    }
};
// The two weight register sets of a wave.  ONE object serves every step: a step's sets are dead once its last MFMA
// has been issued, which is when the next step's first blocks are requested into them.
enum { LK_WSET = 8 };                               // tiles per set: NT * U <= 8 for every step
struct WRegs { u32x4_t a[LK_WSET], b[LK_WSET]; };

// The thread index as a value the optimiser cannot see through: what is derived from it is computed where it is used,
// in every layer, instead of being kept in registers across the whole layer loop (which made the kernel spill).
__device__ __forceinline__ int opaque_tid() {
    int t = (int)threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
}
__device__ __forceinline__ int wave_index() { return __builtin_amdgcn_readfirstlane(opaque_tid() >> 6); }

template <int NT, int U>
__device__ __forceinline__ WaveWalk<NT, U> make_walk(const void *W, const StagePlan &p, int NTiles, int KT) {
    WaveWalk<NT, U> w;
    w.kw = wave_index();
    int item = (int)blockIdx.x - p.off;
    if (item < 0) item += (int)gridDim.x;
    w.valid = item < p.n_items;
    w.bx = w.valid ? item % p.groups : 0;
    w.by = w.valid ? item / p.groups : 0;
    const int tile0 = min(w.bx * NT, NTiles - 1);
    w.nt_valid = max(1, min(NT, NTiles - tile0));
    w.band_stride = (size_t)KT * 64;
    w.w0 = reinterpret_cast<const u32x4_t *>(W) + (size_t)tile0 * KT * 64;
    w.KT = KT;
    w.s_begin = min(KT, w.by * p.ksplit);
    w.k_end = min(KT, w.s_begin + p.ksplit);
    const int tot = (w.k_end - w.s_begin + U - 1) / U;
    w.nblk = tot > w.kw ? (tot - w.kw + LK_WAVES - 1) / LK_WAVES : 0;
    w.rot = w.nblk > 0 ? (int)(((unsigned)w.bx * 5u) % (unsigned)w.nblk) : 0;
    return w;
}

template <int NT, int U>
__device__ __forceinline__ void load_w(u32x4_t (&w)[LK_WSET], const WaveWalk<NT, U> &wk, int k0) {
    static_assert(NT * U <= LK_WSET, "weight set too small");
    const int lane = opaque_tid() & 63;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int k = min(k0 + u, wk.KT - 1);            // clamped: a ragged tail re-reads a valid tile and skips its MFMA
#pragma unroll
        for (int i = 0; i < NT; ++i) w[u * NT + i] = __builtin_nontemporal_load(wk.tile(i, k) + lane);
    }
}

// What a step does for the one after it: request the next item's first two weight blocks (a: when the accumulators
// have left the registers; b: after this step's last store), then wait for this step's stores.
template <int NT, int U>
struct Prefetch {
    WRegs &r;
    const WaveWalk<NT, U> &wk;
    __device__ __forceinline__ void a() const { if (wk.valid) load_w<NT, U>(r.a, wk, wk.kof(0)); }
    __device__ __forceinline__ void b() const { if (wk.valid) load_w<NT, U>(r.b, wk, wk.kof(1)); }
    __device__ __forceinline__ void wait_stores() const {
        if (wk.valid) wait_vmem_older_than<NT * U>();    // the stores are older than the NT * U loads of b()
        else wait_vmem_older_than<0>();
    }
};
struct NoPrefetch {
    __device__ __forceinline__ void a() const {}
    __device__ __forceinline__ void b() const {}
    __device__ __forceinline__ void wait_stores() const { wait_vmem_older_than<0>(); }
};

// One GEMM item.  r holds the weights of the wave's first two blocks (requested by the previous step's Prefetch).
template <int MB, int NT, int U, class Epilogue, class Next>
__device__ __forceinline__ void gemm_stage(const GemmGeom &g, const Epilogue &epi, const WaveWalk<NT, U> &wk, WRegs &r,
                                           float *lds, const Next &next, long long *stamp = nullptr) {
    if (!wk.valid) {                                    // uniform over the workgroup
        next.a(); next.b(); next.wait_stores();
        return;
    }
    const int lane = opaque_tid() & 63, kw = wk.kw;
    GemmTile<MB, NT> t;
    t.tile0 = wk.bx * NT; t.mb0 = 0; t.lane = lane; t.wave = kw; t.split = wk.by; t.lds = lds;
    float *redbuf = lds + GEMM_LDS_SCRATCH;
    f32x16_t acc[MB][NT];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][i][v] = 0.f;
    u32x4_t xa[U][MB], xb[U][MB];
    auto load_x = [&](u32x4_t (&x)[U][MB], int k0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = min(k0 + u, g.KT - 1);
#pragma unroll
            for (int a = 0; a < MB; ++a) x[u][a] = g.X[((size_t)a * g.KT + k) * 64 + lane];
        }
    };
    auto load = [&](u32x4_t (&w)[LK_WSET], u32x4_t (&x)[U][MB], int k0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = min(k0 + u, g.KT - 1);
#pragma unroll
            for (int i = 0; i < NT; ++i) w[u * NT + i] = __builtin_nontemporal_load(wk.tile(i, k) + lane);
#pragma unroll
            for (int a = 0; a < MB; ++a) x[u][a] = g.X[((size_t)a * g.KT + k) * 64 + lane];
        }
    };
    auto compute = [&](u32x4_t (&w)[LK_WSET], u32x4_t (&x)[U][MB], int k0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (k0 + u < wk.k_end) {
#pragma unroll
                for (int a = 0; a < MB; ++a)
#pragma unroll
                    for (int i = 0; i < NT; ++i)
                        acc[a][i] = HYDRA_MFMA16(__builtin_bit_cast(a16x8_t, x[u][a]), __builtin_bit_cast(a16x8_t, w[u * NT + i]), acc[a][i]);
            }
        }
    };
    const int nblk = wk.nblk;
    load_x(xa, wk.kof(0));
    auto pre = epi.issue(t, g);
    load_x(xb, wk.kof(1));
    auto carry = epi.prologue(pre, t, g);
    if (stamp && threadIdx.x == 0) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); stamp[4] = wall_clock64(); }
    int j = 0;
    if (nblk >= 4) {                                    // long run: unconditional refills, exact waits (see gemm_bf16.h)
        for (; j + 3 < nblk; j += 2) {
            compute(r.a, xa, wk.kof(j));
            load(r.a, xa, wk.kof(j + 2));
            compute(r.b, xb, wk.kof(j + 1));
            load(r.b, xb, wk.kof(j + 3));
        }
    }
    if (j < nblk) compute(r.a, xa, wk.kof(j));
    if (j + 2 < nblk) load(r.a, xa, wk.kof(j + 2));
    if (j + 1 < nblk) compute(r.b, xb, wk.kof(j + 1));
    if (j + 2 < nblk) compute(r.a, xa, wk.kof(j + 2));

    if (stamp && threadIdx.x == 0) stamp[5] = wall_clock64();
    // ---- finish: the waves meet in LDS, at most PASS tiles at a time, and share the tiles out
    epi.before_barrier(carry, t, g);
    const bool live = t.tile0 < g.NTiles;
    constexpr int TILES = MB * NT;
    constexpr int PASS = TILES <= 4 ? TILES : (TILES + 1) / 2;
    constexpr int NPASS = (TILES + PASS - 1) / PASS;
    static_assert(NPASS == 1 || !Epilogue::PAIRED, "paired epilogues take their tiles in one pass");
    static_for<NPASS>([&](auto P) {
        constexpr int p = decltype(P)::value;
        constexpr int J0 = p * PASS, J1 = (J0 + PASS < TILES) ? J0 + PASS : TILES;
        {
            float *dst = redbuf + (size_t)kw * PASS * 16 * 64 + lane;
            static_for<J1 - J0>([&](auto JJ) {
                constexpr int jl = decltype(JJ)::value, jt = J0 + jl, a = jt / NT, i = jt % NT;
#pragma unroll
                for (int v = 0; v < 16; ++v) dst[(jl * 16 + v) * 64] = acc[a][i][v];
            });
        }
        if (p == 0) next.a();
        wg_barrier_lds();
        if (p == 0 && live) epi.begin(t, g);
        if (live) {
            if constexpr (Epilogue::PAIRED) {
                for (int id = kw; id < MB * 4 * (NT / 2); id += LK_WAVES) {          // wave-uniform
                    const int pr = id / (MB * 4), rr = id - pr * (MB * 4);
                    const int a = rr >> 2, v0 = (rr & 3) * 4;
                    float x0[4] = {0.f, 0.f, 0.f, 0.f}, x1[4] = {0.f, 0.f, 0.f, 0.f};
                    for (int w = 0; w < LK_WAVES; ++w) {
                        const float *src = redbuf + ((size_t)w * PASS + a * NT + 2 * pr) * 16 * 64 + lane;
#pragma unroll
                        for (int q = 0; q < 4; ++q) { x0[q] += src[(v0 + q) * 64]; x1[q] += src[(16 + v0 + q) * 64]; }
                    }
                    GemmTile<MB, NT> tp = t;
                    tp.tile0 = t.tile0 + 2 * pr;
                    epi.pair4(x0, x1, a, v0, tp, g);
                }
            } else {
                static_for<J1 - J0>([&](auto JJ) {
                    constexpr int jl = decltype(JJ)::value, jt = J0 + jl, a = jt / NT, i = jt % NT;
                    if (jl % LK_WAVES == kw) {                                         // wave-uniform
                        f32x16_t sum;
#pragma unroll
                        for (int v = 0; v < 16; ++v) sum[v] = 0.f;
                        for (int w = 0; w < LK_WAVES; ++w) {
                            const float *src = redbuf + ((size_t)w * PASS + jl) * 16 * 64 + lane;
#pragma unroll
                            for (int v = 0; v < 16; ++v) sum[v] += src[v * 64];
                        }
                        epi.tile(sum, a, i, t, g);
                    }
                });
            }
        }
        if (p + 1 < NPASS) wg_barrier_lds();            // the next pass overwrites the buffer
    });
    if (stamp && threadIdx.x == 0) stamp[6] = wall_clock64();
    next.b();
    next.wait_stores();
}

// x_out = x_in + sum of S split-K partials; xg = half(x_out * gain) as GEMM input; ss[chunk][row] = sum of squares
// over the 1024-column chunk.  One half workgroup (256 threads) per (row, chunk).
__device__ __forceinline__ void resid_stage(const float *__restrict__ part, int S, size_t split_stride, int ld,
                                            const float *__restrict__ x_in, float *__restrict__ x_out, const float *__restrict__ gain,
                                            a16_t *__restrict__ xg, float *__restrict__ ss, int Mpad, int M, int d, float *lds, int32_t *flags) {
    const int tix = opaque_tid();
    const int half = tix >> 8, tid = tix & 255, wave = tix >> 6;
    const int n_chunks = (d + 1023) >> 10, n_units = M * n_chunks;
    for (int u0 = (int)blockIdx.x * 2; u0 < n_units; u0 += 2 * (int)gridDim.x) {      // uniform over the workgroup
        const int u = u0 + half;
        const bool live = u < n_units;
        const int m = live ? u / n_chunks : 0, c = live ? u - m * n_chunks : 0;
        const int k = c * 1024 + tid * 4;
        float sq = 0.f;
        if (live && k < d) {
            f32x4_t a = *reinterpret_cast<const f32x4_t *>(x_in + (size_t)m * d + k);
            const f32x4_t gn = *reinterpret_cast<const f32x4_t *>(gain + k);
            const float *src = part + (size_t)m * ld + k;
            for (int s0 = 0; s0 < S; s0 += 4) {                    // four partials per round trip (surplus loads re-read the last split)
                f32x4_t q[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) q[e] = *reinterpret_cast<const f32x4_t *>(src + (size_t)min(s0 + e, S - 1) * split_stride);
#pragma unroll
                for (int e = 0; e < 4; ++e)                        // added in split order
                    if (s0 + e < S) { a[0] += q[e][0]; a[1] += q[e][1]; a[2] += q[e][2]; a[3] += q[e][3]; }
            }
            float *xo = x_out + (size_t)m * d + k;
            st_dev64<true>(xo, __float_as_uint(a[0]), __float_as_uint(a[1]));
            st_dev64<true>(xo + 2, __float_as_uint(a[2]), __float_as_uint(a[3]));
            st_dev64<true>(xg + x_index<true>(m, k, d), f2a_pack_f(a[0] * gn[0], a[1] * gn[1], flags), f2a_pack_f(a[2] * gn[2], a[3] * gn[3], flags));
            sq = a[0] * a[0] + a[1] * a[1] + a[2] * a[2] + a[3] * a[3];
        }
        sq = wave_sum(sq);
        if ((tix & 63) == 0) lds[wave] = sq;
        wg_barrier_lds();
        if (tid == 0 && live) st_dev<true>(ss + (size_t)c * Mpad + m, lds[half * 4] + lds[half * 4 + 1] + lds[half * 4 + 2] + lds[half * 4 + 3]);
        wg_barrier_lds();
    }
    wait_vmem_older_than<0>();
}

// timeline: what = 0 step begins, 1 work done (stores acknowledged), 2 arrived, 3 released; inside a GEMM step:
// 4 first activations in registers, 5 last MFMA issued, 6 epilogue stores issued
__device__ __forceinline__ void lk_stamp(const LayerKernelArgs &A, int l, int stage, int what) {
    if (A.stamps && threadIdx.x == 0)
        A.stamps[(((size_t)l * LK_STAGES + stage) * gridDim.x + blockIdx.x) * 8 + what] = wall_clock64();
}

__device__ __forceinline__ long long *lk_stamp_ptr(const LayerKernelArgs &A, int l, int stage) {
    return A.stamps ? A.stamps + (((size_t)l * LK_STAGES + stage) * gridDim.x + blockIdx.x) * 8 : nullptr;
}

template <int MB> struct LkShape {
    static constexpr int NT_Q = 2, NT_O = 2, NT_G = 3, NT_D = 2;
    // k-steps per register set.  With two row blocks the accumulators, two weight sets and two activation sets of
    // four k-steps fill all 256 registers of a wave, and anything else that is live pushes weight tiles into scratch
    // memory (whose reloads wait for every older load: the end of the software pipeline); three k-steps leave room.
    static constexpr int U_Q = 3, U_O = 3, U_G = 2, U_D = 3;
};

template <int MB, int DH>
__global__ __launch_bounds__(LK_THREADS) void layers_kernel(LayerKernelArgs A) {
    typedef LkShape<MB> S;
    extern __shared__ float lds[];
    int *ctl = reinterpret_cast<int *>(lds + GEMM_LDS_SCRATCH + LK_WAVES * 4 * 16 * 64);    // behind the reduction buffer
    const int d = A.d, F = A.F, KTd = d >> 4, KTf = F >> 4;
    const int bands_q = 3 * d / 32, bands_d = d / 32, bands_g = 2 * F / 32;
    const int npad_d = bands_d * 32;
    const size_t part_stride = (size_t)MB * 32 * npad_d;
    const bool attn_wg = (int)blockIdx.x < A.n_attn;

    auto layer_w = [&](size_t off, int l) { return A.arena + off + (size_t)l * A.layer_stride; };
    WRegs r;
    WaveWalk<S::NT_Q, S::U_Q> wq = make_walk<S::NT_Q, S::U_Q>(layer_w(A.wqkv, 0), A.q, bands_q, KTd);
    {
        Prefetch<S::NT_Q, S::U_Q> first{r, wq};
        first.a(); first.b();
    }
    int bar = 0;
    for (int l = 0; l < A.NL; ++l) {
        char *bin = A.blk + (size_t)l * A.blk_stride, *bout = bin + A.blk_stride;
        const float *x_in = reinterpret_cast<const float *>(bin + A.x_b);
        const float *ss_in = reinterpret_cast<const float *>(bin + A.ss_b);
        const int nb_in = l == 0 ? A.nb_first : A.nb;
        float *x_a = reinterpret_cast<float *>(bout + A.x_a), *x_b = reinterpret_cast<float *>(bout + A.x_b);
        a16_t *xg_a = reinterpret_cast<a16_t *>(bout + A.xg_a), *xg_b = reinterpret_cast<a16_t *>(bout + A.xg_b);
        float *ss_a = reinterpret_cast<float *>(bout + A.ss_a), *ss_b = reinterpret_cast<float *>(bout + A.ss_b);
        a16_t *attn = reinterpret_cast<a16_t *>(bout + A.attn), *act = reinterpret_cast<a16_t *>(bout + A.act);
        float *part_o = reinterpret_cast<float *>(bout + A.part_o), *part_d = reinterpret_cast<float *>(bout + A.part_d);
        a16_t *qbuf = reinterpret_cast<a16_t *>(bout + A.qbuf);
        const float *gain_ffn = reinterpret_cast<const float *>(layer_w(A.ffn_norm, l));
        const float *gain_next = reinterpret_cast<const float *>(l + 1 < A.NL ? layer_w(A.attn_norm, l + 1) : A.arena + A.final_norm);

        const WaveWalk<S::NT_O, S::U_O> wo = make_walk<S::NT_O, S::U_O>(layer_w(A.wo, l), A.o, bands_d, KTd);

        // ---- q|k|v + rotary + cache append
        {
            GemmGeom g;
            g.X = reinterpret_cast<const u32x4_t *>(bin + A.xg_b); g.W = nullptr; g.M = A.M; g.NTiles = bands_q; g.KT = KTd; g.kpw = 0; g.NW = 1; g.KW = LK_WAVES;
            EpiQkvRopeT<true> epi{ss_in, nb_in, A.Mpad, d, A.eps, A.seq_len, A.tree, A.page_table, A.max_pages, A.n_pages, l,
                                  A.kpages, A.vpages, qbuf, A.rope, A.H, DH, A.T, A.max_pos, A.flags, 0};
            gemm_stage<MB, S::NT_Q, S::U_Q>(g, epi, wq, r, lds, NoPrefetch{}, lk_stamp_ptr(A, l, 0));
        }
        lk_stamp(A, l, 0, 1);
        gs_arrive(A.sync, bar, ctl);
        lk_stamp(A, l, 0, 2);
        if (!gs_wait(A.sync, bar, ctl)) return;
        lk_stamp(A, l, 0, 3);
        lk_stamp(A, l, 1, 0);
        ++bar;
        // ---- tree attention
        if (attn_wg) {
            const int it = (int)blockIdx.x;
            const int qt = it % A.QT, h = (it / A.QT) % A.H, b = it / (A.QT * A.H);
            attn_bf16_body<DH, true, true, false>(reinterpret_cast<const u32x4_t *>(qbuf), A.kpages, A.vpages, A.page_table, A.max_pages, A.n_pages, l,
                                           A.seq_len, A.tree, A.T, A.H, 1, 1, A.scale, nullptr, attn, A.flags, qt, A.QT, h, b, lds, opaque_tid());
            wg_barrier_lds();                           // the attention body's LDS is the next step's
        }
        {   // the O weights: requested here by every workgroup (those without an attention item have the whole attention
            // step to receive them), so that they are not live in registers while attention runs
            Prefetch<S::NT_O, S::U_O> pf{r, wo};
            pf.a(); pf.b(); pf.wait_stores();
        }
        lk_stamp(A, l, 1, 1);
        gs_arrive(A.sync, bar, ctl);
        lk_stamp(A, l, 1, 2);
        if (!gs_wait(A.sync, bar, ctl)) return;
        lk_stamp(A, l, 1, 3);
        lk_stamp(A, l, 2, 0);
        ++bar;
        // ---- O projection, K split over workgroups
        const WaveWalk<S::NT_G, S::U_G> wg = make_walk<S::NT_G, S::U_G>(layer_w(A.wgu, l), A.gu, bands_g, KTd);
        {
            GemmGeom g;
            g.X = reinterpret_cast<const u32x4_t *>(attn); g.W = nullptr; g.M = A.M; g.NTiles = bands_d; g.KT = KTd; g.kpw = 0; g.NW = 1; g.KW = LK_WAVES;
            EpiPlainT<true> epi{part_o, npad_d, part_stride};
            gemm_stage<MB, S::NT_O, S::U_O>(g, epi, wo, r, lds, Prefetch<S::NT_G, S::U_G>{r, wg}, lk_stamp_ptr(A, l, 2));
        }
        lk_stamp(A, l, 2, 1);
        gs_arrive(A.sync, bar, ctl);
        lk_stamp(A, l, 2, 2);
        if (!gs_wait(A.sync, bar, ctl)) return;
        lk_stamp(A, l, 2, 3);
        lk_stamp(A, l, 3, 0);
        ++bar;
        // ---- residual + norm input of the FFN
        resid_stage(part_o, A.o.splits, part_stride, npad_d, x_in, x_a, gain_ffn, xg_a, ss_a, A.Mpad, A.M, d, lds, A.flags);
        lk_stamp(A, l, 3, 1);
        gs_arrive(A.sync, bar, ctl);
        lk_stamp(A, l, 3, 2);
        if (!gs_wait(A.sync, bar, ctl)) return;
        lk_stamp(A, l, 3, 3);
        lk_stamp(A, l, 4, 0);
        ++bar;
        // ---- gate/up + SwiGLU
        const WaveWalk<S::NT_D, S::U_D> wd = make_walk<S::NT_D, S::U_D>(layer_w(A.wdown, l), A.dn, bands_d, KTf);
        {
            GemmGeom g;
            g.X = reinterpret_cast<const u32x4_t *>(xg_a); g.W = nullptr; g.M = A.M; g.NTiles = bands_g; g.KT = KTd; g.kpw = 0; g.NW = 1; g.KW = LK_WAVES;
            EpiSiluT<true> epi{ss_a, A.nb, A.Mpad, d, A.eps, act, F, A.flags};
            gemm_stage<MB, S::NT_G, S::U_G>(g, epi, wg, r, lds, Prefetch<S::NT_D, S::U_D>{r, wd}, lk_stamp_ptr(A, l, 4));
        }
        lk_stamp(A, l, 4, 1);
        gs_arrive(A.sync, bar, ctl);
        lk_stamp(A, l, 4, 2);
        if (!gs_wait(A.sync, bar, ctl)) return;
        lk_stamp(A, l, 4, 3);
        lk_stamp(A, l, 5, 0);
        ++bar;
        // ---- down projection, K split over workgroups
        wq = make_walk<S::NT_Q, S::U_Q>(layer_w(A.wqkv, l + 1 < A.NL ? l + 1 : l), A.q, bands_q, KTd);
        const bool q_valid = wq.valid;
        if (l + 1 >= A.NL) wq.valid = false;            // behind the last layer there is nothing to request
        {
            GemmGeom g;
            g.X = reinterpret_cast<const u32x4_t *>(act); g.W = nullptr; g.M = A.M; g.NTiles = bands_d; g.KT = KTf; g.kpw = 0; g.NW = 1; g.KW = LK_WAVES;
            EpiPlainT<true> epi{part_d, npad_d, part_stride};
            gemm_stage<MB, S::NT_D, S::U_D>(g, epi, wd, r, lds, Prefetch<S::NT_Q, S::U_Q>{r, wq}, lk_stamp_ptr(A, l, 5));
            wq.valid = q_valid;
        }
        lk_stamp(A, l, 5, 1);
        gs_arrive(A.sync, bar, ctl);
        lk_stamp(A, l, 5, 2);
        if (!gs_wait(A.sync, bar, ctl)) return;
        lk_stamp(A, l, 5, 3);
        lk_stamp(A, l, 6, 0);
        ++bar;
        // ---- residual + norm input of the next layer (or of the LM head)
        resid_stage(part_d, A.dn.splits, part_stride, npad_d, x_a, x_b, gain_next, xg_b, ss_b, A.Mpad, A.M, d, lds, A.flags);
        lk_stamp(A, l, 6, 1);
        if (l + 1 < A.NL) {
            gs_arrive(A.sync, bar, ctl);
            lk_stamp(A, l, 6, 2);
            if (!gs_wait(A.sync, bar, ctl)) return;
            lk_stamp(A, l, 6, 3);
            lk_stamp(A, l + 1, 0, 0);
            ++bar;
        }
    }
}

__global__ void zero_words_kernel(unsigned *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// ---------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------
static int env_int(const char *name, int dflt) {
    const char *v = getenv(name);
    return v ? atoi(v) : dflt;
}

static size_t lk_lds_bytes() { return ((size_t)GEMM_LDS_SCRATCH + (size_t)LK_WAVES * 4 * 16 * 64 + 64) * 4; }

// bytes of the per-layer buffer block and the offsets inside it
struct LkBlock { size_t x_a, x_b, xg_a, xg_b, ss_a, ss_b, attn, act, part_o, part_d, qbuf, bytes; };
static LkBlock lk_block(const hydra_ctx *c, int B, int splits_o, int splits_d) {
    LkBlock k;
    const size_t d = c->m.d, F = c->m.ffn, M = (size_t)B * c->tree.T, Mp = align_up(M, 32), Mpad = align_up(M, 128);
    const size_t Tq = align_up((size_t)c->tree.T, 32);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    k.x_a = take(Mp * d * 4); k.x_b = take(Mp * d * 4);
    k.xg_a = take(Mp * d * 2); k.xg_b = take(Mp * d * 2);
    k.ss_a = take((d / 1024 + 1) * Mpad * 4); k.ss_b = take((d / 1024 + 1) * Mpad * 4);
    k.attn = take(Mp * d * 2); k.act = take(Mp * F * 2);
    k.part_o = take((size_t)splits_o * Mp * d * 4); k.part_d = take((size_t)splits_d * Mp * d * 4);
    k.qbuf = take((size_t)B * c->m.n_heads * Tq * c->m.head_dim * 2);
    k.bytes = off;
    return k;
}

struct LkPlan { bool ok; int G, MB; StagePlan q, o, gu, dn; int n_attn, QT; };

static StagePlan split_plan(int groups, int KT, int want_items, int U) {
    StagePlan p;
    p.groups = groups;
    int s = std::max(1, want_items / groups);
    s = std::min(s, 8);
    while (s > 1 && KT / s < 16) --s;
    p.splits = s;
    p.ksplit = ceil_div(ceil_div(KT, s), U) * U;         // whole blocks per split
    p.splits = ceil_div(KT, p.ksplit);
    p.n_items = groups * p.splits;
    p.off = 0;
    return p;
}

static LkPlan lk_plan(const hydra_ctx *c, int B) {
    LkPlan p;
    p.ok = false;
    const int T = c->tree.T, M = B * T, d = c->m.d, F = c->m.ffn, H = c->m.n_heads;
    if (!c->bf16 || M > 64 || c->n_cus < LK_GROUPS) return p;
    p.G = c->n_cus;
    p.MB = M > 32 ? 2 : 1;
    p.QT = ceil_div(T, 32);
    p.n_attn = B * H * p.QT;
    const int G = p.G;
    if (p.n_attn > G) return p;
    // q|k|v: band pairs, whole K
    p.q.groups = 3 * d / 64; p.q.splits = 1; p.q.ksplit = d / 16; p.q.n_items = p.q.groups; p.q.off = 0;
    if (p.q.n_items > G) return p;
    // gate/up: three bands per wave, whole K
    p.gu.groups = ceil_div(2 * F / 32, 3); p.gu.splits = 1; p.gu.ksplit = d / 16; p.gu.n_items = p.gu.groups; p.gu.off = 0;
    if (p.gu.n_items > G) return p;
    // O: two bands per wave, K split so that the items fit behind the attention workgroups when possible
    const int groups_d = ceil_div(d / 32, 2);
    if (groups_d > G) return p;
    const int room = G - p.n_attn >= groups_d ? G - p.n_attn : G;
    p.o = split_plan(groups_d, d / 16, room, 3);
    p.o.off = (room == G) ? 0 : p.n_attn;
    p.dn = split_plan(groups_d, F / 16, G, 3);
    if (p.o.n_items > G || p.dn.n_items > G) return p;
    // the gate/up items leave workgroups idle: start them where the O items end, so that other workgroups idle in the two steps
    p.gu.off = 0;
    p.ok = true;
    return p;
}

static size_t lk_sync_words(const hydra_ctx *c) { return (size_t)LK_WORDS + (size_t)(LK_STAGES * c->m.n_layers + 1) * LK_BARRIER_WORDS; }
static size_t lk_sync_bytes(const hydra_ctx *c) { return align_up(lk_sync_words(c) * 4, 256); }
static size_t lk_stamp_bytes(const hydra_ctx *c, int G) { return align_up((size_t)c->m.n_layers * LK_STAGES * G * 8 * 8, 256); }

size_t layers_mega_ws_bytes(const hydra_ctx *c, int B) {
    const LkPlan p = lk_plan(c, B);
    if (!p.ok) return 0;
    const LkBlock k = lk_block(c, B, p.o.splits, p.dn.splits);
    return lk_sync_bytes(c) + lk_stamp_bytes(c, p.G) + (size_t)(c->m.n_layers + 1) * k.bytes;
}

// Can this forward pass take the persistent kernel?  (bf16 family, at most 64 rows, a known upper bound of the row
// lengths that keeps attention at one workgroup per query tile, plans of one item per workgroup.)
bool layers_mega_eligible(const hydra_ctx *c, int B, const hydra_kv *kv) {
    // Off unless HYDRA_LAYER_KERNEL=1 (read at every call: tests compare the two paths).  Measured at the 7B shape it
    // is not yet faster than the multi-kernel path: the hand-offs cost ~2 us, but the waves of a workgroup end their
    // streams up to ~4 us apart and the LDS reduction behind that spread is as exposed here as at a kernel boundary.
    if (!env_int("HYDRA_LAYER_KERNEL", 0) || !c->bf16) return false;
    if (kv->seq_len_hint <= 0) return false;
    if (ceil_div(kv->seq_len_hint + c->tree.T, 32) > ATTN_WAVES * 5) return false;
    return lk_plan(c, B).ok;
}

// out[0] = 1 if forward passes of B rows can take the persistent kernel (given a bounded context), out[1] = bytes from
// the start of that kernel's workspace region to its timeline stamps, out[2] = workgroups, out[3] = steps per layer
void layers_mega_info(const hydra_ctx *c, int B, int64_t *out) {
    const LkPlan p = lk_plan(c, B);
    out[0] = p.ok ? 1 : 0;
    out[1] = p.ok ? (int64_t)lk_sync_bytes(c) : 0;
    out[2] = p.ok ? p.G : 0;
    out[3] = LK_STAGES;
}

int layers_mega_set_attr(hydra_ctx *c) {
    (void)c;
    hipError_t e = hipSuccess;
    const int bytes = (int)lk_lds_bytes();
#define LK_ATTR(MBv, DHv) if (e == hipSuccess) e = hipFuncSetAttribute((const void *)layers_kernel<MBv, DHv>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes)
    LK_ATTR(1, 64); LK_ATTR(1, 128); LK_ATTR(2, 64); LK_ATTR(2, 128);
#undef LK_ATTR
    if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(layers_kernel)");
    return HYDRA_OK;
}

// mega: the workspace region of layers_mega_ws_bytes().  Block 0 receives the embedding step's outputs (x, xg, ss)
// from the caller before this launch; the results of the last layer are in block NL (pointers returned).
int launch_layers_mega(hydra_ctx *c, hipStream_t s, int B, char *mega, const int32_t *seq_len, const hydra_kv *kv, int32_t *flags,
                       LayersMegaIO *io, bool launch) {
    const LkPlan p = lk_plan(c, B);
    if (!p.ok) return fail(HYDRA_E_UNSUPPORTED, "layer kernel: shape not eligible");
    const LkBlock k = lk_block(c, B, p.o.splits, p.dn.splits);
    const int NL = c->m.n_layers, M = B * c->tree.T;
    const size_t sync_words = lk_sync_words(c);
    char *blocks = mega + lk_sync_bytes(c) + lk_stamp_bytes(c, p.G);
    io->x_first = reinterpret_cast<float *>(blocks + k.x_b);
    io->xg_first = blocks + k.xg_b;
    io->ss_first = reinterpret_cast<float *>(blocks + k.ss_b);
    char *last = blocks + (size_t)NL * k.bytes;
    io->x_last = reinterpret_cast<float *>(last + k.x_b);
    io->xg_last = last + k.xg_b;
    io->ss_last = reinterpret_cast<float *>(last + k.ss_b);
    io->nb_last = ceil_div(c->m.d, 1024);
    io->Mpad = (int)align_up((size_t)std::max(M, 1), 128);
    if (!launch) return HYDRA_OK;

    LayerKernelArgs A;
    A.arena = c->arena;
    const LayerOff &o0 = c->layer[0];
    A.attn_norm = o0.attn_norm; A.wqkv = o0.wqkv; A.wo = o0.wo; A.ffn_norm = o0.ffn_norm; A.wgu = o0.wgu; A.wdown = o0.wdown;
    A.layer_stride = NL > 1 ? c->layer[1].attn_norm - o0.attn_norm : 0;
    A.final_norm = c->off_final_norm;
    A.NL = NL; A.M = M; A.Mpad = io->Mpad; A.d = c->m.d; A.F = c->m.ffn; A.H = c->m.n_heads; A.T = c->tree.T; A.B = B;
    A.nb_first = 1; A.nb = io->nb_last;
    A.eps = c->m.rms_eps; A.scale = 1.0f / sqrtf((float)c->m.head_dim);
    A.q = p.q; A.o = p.o; A.gu = p.gu; A.dn = p.dn; A.n_attn = p.n_attn; A.QT = p.QT;
    A.blk = blocks; A.blk_stride = k.bytes;
    A.x_a = k.x_a; A.x_b = k.x_b; A.xg_a = k.xg_a; A.xg_b = k.xg_b; A.ss_a = k.ss_a; A.ss_b = k.ss_b; A.attn = k.attn; A.act = k.act;
    A.part_o = k.part_o; A.part_d = k.part_d; A.qbuf = k.qbuf;
    A.seq_len = seq_len; A.page_table = kv->page_table; A.max_pages = kv->max_pages; A.n_pages = kv->n_pages;
    A.kpages = (a16_t *)kv->k_pages; A.vpages = (a16_t *)kv->v_pages;
    A.tree = tree_dev(c); A.rope = rope_dev(c); A.max_pos = c->m.max_pos; A.flags = flags;
    A.stamps = env_int("HYDRA_LAYER_KERNEL_STAMPS", 0) ? reinterpret_cast<long long *>(mega + lk_sync_bytes(c)) : nullptr;
    A.sync.base = reinterpret_cast<unsigned *>(mega);
    A.sync.flags = flags;
    // Tests of the give-up path: a short spin limit and one group more than exists, so that no hand-off can complete
    // and every workgroup leaves through the bounded wait (the kernel still exits normally).
    A.sync.spin_limit = std::max(1, env_int("HYDRA_LAYER_KERNEL_SPIN", 1 << 20));
    A.sync.groups_expected = std::min(p.G, (int)LK_GROUPS) + (env_int("HYDRA_LAYER_KERNEL_TEST_STALL", 0) ? 1 : 0);

    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)ceil_div((int)sync_words, 256)), dim3(256), 0, s, A.sync.base, (int)sync_words);
    HYDRA_LAUNCH_CHECK("zero_words_kernel");
    dim3 grid(p.G), block(LK_THREADS);
    const size_t lds = lk_lds_bytes();
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (c->profiling) {
        if (c->ev_used + 2 > c->ev.size())
            for (int i = 0; i < 2; ++i) { hipEvent_t e; HYDRA_HIP(hipEventCreate(&e)); c->ev.push_back(e); }
        e0 = c->ev[c->ev_used++]; e1 = c->ev[c->ev_used++];
    }
#define LK_LAUNCH(MBv, DHv)                                                                                              \
    do {                                                                                                                 \
        if (e0) hipExtLaunchKernelGGL((layers_kernel<MBv, DHv>), grid, block, lds, s, e0, e1, 0, A);                      \
        else    hipLaunchKernelGGL((layers_kernel<MBv, DHv>), grid, block, lds, s, A);                                    \
    } while (0)
    if (p.MB == 1) { if (c->m.head_dim == 128) LK_LAUNCH(1, 128); else LK_LAUNCH(1, 64); }
    else           { if (c->m.head_dim == 128) LK_LAUNCH(2, 128); else LK_LAUNCH(2, 64); }
#undef LK_LAUNCH
    HYDRA_LAUNCH_CHECK("layers_kernel");
    if (c->profiling) {
        c->prof_bytes += (double)NL * (4.0 * c->m.d * c->m.d + 3.0 * c->m.d * c->m.ffn) * 2;
        c->prof_launches += 1;
    }
    return HYDRA_OK;
}

}  // namespace hydra
