// Device-side helpers shared by all kernels: 16-bit conversions, the MFMA operand
// order used for GEMM inputs, in-page placement of K and V, wave reductions.
//
// Number formats of the bf16 storage family.  Weights arrive as bfloat16.  Inside
// the library every 16-bit value that feeds a matrix core (packed weights, GEMM
// inputs, q, the KV cache, softmax probabilities) is held as IEEE half ("a16"):
// a bfloat16 weight of magnitude >= 2^-17 is exactly representable in half, and
// half keeps 11 significant bits of the activations where bfloat16 keeps 8, which
// is what keeps a 32-layer forward inside the 2e-2 parity tolerance (rounding
// every GEMM input to bfloat16 measured 4e-2 on the 7B shape).  Conversions
// saturate at the largest finite half (65504).  Sums are fp32 throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hydra {

typedef uint16_t bf16_t;

// round to nearest even; the cast compiles to the hardware converter of gfx950
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
__device__ __forceinline__ uint32_t f2bf_pack(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_;
    const f32x2_ v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_));
}
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// ---- a16: the 16-bit activation / cache / packed-weight element (IEEE half) ----
typedef uint16_t a16_t;
typedef __attribute__((ext_vector_type(8))) _Float16 a16x8_t;      // one lane's MFMA operand
#define HYDRA_MFMA16(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0)
__device__ __forceinline__ float a16_sat(float f) { return fminf(fmaxf(f, -65504.f), 65504.f); }
__device__ __forceinline__ a16_t f2a(float f) { return __builtin_bit_cast(a16_t, (_Float16)a16_sat(f)); }
__device__ __forceinline__ uint32_t f2a_pack(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_;
    typedef __attribute__((ext_vector_type(2))) _Float16 h16x2_;
    const f32x2_ v = {a16_sat(lo), a16_sat(hi)};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, h16x2_));
}
__device__ __forceinline__ float a2f(a16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
// The same conversions for values that feed a GEMM or the cache: a value beyond the largest finite half is still
// clamped, but the clamp is reported (flag bit 4), so a residual stream with channels too large for the 16-bit
// interior never passes silently.
__device__ __forceinline__ void flag_saturation(float a, float b, int32_t *flags) {
    if (fmaxf(fabsf(a), fabsf(b)) > 65504.f) atomicOr(flags, 16 /* FLAG_SATURATED */);
}
__device__ __forceinline__ a16_t f2a_f(float f, int32_t *flags) { flag_saturation(f, 0.f, flags); return f2a(f); }
__device__ __forceinline__ uint32_t f2a_pack_f(float lo, float hi, int32_t *flags) { flag_saturation(lo, hi, flags); return f2a_pack(lo, hi); }

template <bool BF> struct Elem;
template <> struct Elem<true>  { typedef bf16_t type; static __device__ __forceinline__ float ld(const bf16_t *p, size_t i) { return bf2f(p[i]); }
                                 static __device__ __forceinline__ void st(bf16_t *p, size_t i, float v) { p[i] = f2bf(v); } };
template <> struct Elem<false> { typedef float type;  static __device__ __forceinline__ float ld(const float *p, size_t i) { return p[i]; }
                                 static __device__ __forceinline__ void st(float *p, size_t i, float v) { p[i] = v; } };
// Elem: the format weights are GIVEN in (bf16 / fp32).  Act: the format of activations and cache (a16 / fp32).
template <bool BF> struct Act;
template <> struct Act<true>  { typedef a16_t type; static __device__ __forceinline__ float ld(const a16_t *p, size_t i) { return a2f(p[i]); }
                                static __device__ __forceinline__ void st(a16_t *p, size_t i, float v) { p[i] = f2a(v); } };
template <> struct Act<false> { typedef float type; static __device__ __forceinline__ float ld(const float *p, size_t i) { return p[i]; }
                                static __device__ __forceinline__ void st(float *p, size_t i, float v) { p[i] = v; } };

// ---- GEMM input order ------------------------------------------------------
// bf16 family: activations X[M][K] are stored as 32-row x 16-column tiles in
// the register order of the 32x32x16 MFMA "A" operand: lane = (k%16)/8*32 + m%32
// holds 8 consecutive k.  Tile (mb, kt) is the 1 KiB block number mb*KT + kt.
// f32 family: plain row-major.
template <bool BF>
__device__ __forceinline__ size_t x_index(int m, int k, int K) {
    if (BF) {
        const int KT = K >> 4;
        return ((((size_t)(m >> 5) * KT + (k >> 4)) * 64 + ((k >> 3) & 1) * 32 + (m & 31)) << 3) + (k & 7);
    } else {
        return (size_t)m * K + k;
    }
}

// ---- KV cache placement ------------------------------------------------------
// One (layer, page, head) block holds 16 tokens x Dh dims.
//   f32 : K and V row-major [token][dim].
//   bf16: K as [dim/8][token][dim%8]   (16-byte runs = MFMA operand rows for S^T = K Q^T),
//         V as [dim][perm(token)]      (16-byte runs = MFMA operand rows for O^T = V^T P^T)
//         with perm(t) = ((t>>2)&1)*8 + (t>>3)*4 + (t&3), the order in which a lane
//         of the 32x32 accumulator holds the 16 keys of a page.
template <bool BF> __device__ __forceinline__ int k_in_block(int tok, int dim, int Dh) {
    return BF ? (((dim >> 3) * 16 + tok) << 3) + (dim & 7) : tok * Dh + dim;
}
__device__ __forceinline__ int v_perm(int t) { return ((t >> 2) & 1) * 8 + (t >> 3) * 4 + (t & 3); }
template <bool BF> __device__ __forceinline__ int v_in_block(int tok, int dim, int Dh) {
    return BF ? dim * 16 + v_perm(tok) : tok * Dh + dim;
}
__device__ __forceinline__ size_t kv_block_base(int layer, int n_pages, int page, int H, int head, int Dh) {
    return ((((size_t)layer * n_pages + page) * H) + head) * (size_t)(16 * Dh);
}

// A page id from the caller's page table: ids outside [0, n_pages) are reported (flag bit 6) and replaced by page 0,
// so that a bad table entry gives a flagged wrong result instead of an access outside the cache.
__device__ __forceinline__ int checked_page(int page, int n_pages, int32_t *flags) {
    if ((unsigned)page >= (unsigned)n_pages) { atomicOr(flags, 64 /* FLAG_BAD_PAGE */); return 0; }
    return page;
}

// ---- wave reductions (64 lanes) ------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// sum of S split-K partial results of one output element
// Four partials per memory round trip: the loads of a group are unconditional (surplus ones re-read the last split), so
// they are all in flight before the first add; the adds keep the split order.
__device__ __forceinline__ float part_sum(const float *part, int S, size_t split_stride, size_t idx) {
    float a = 0.f;
    for (int s0 = 0; s0 < S; s0 += 4) {
        float q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) q[u] = part[(size_t)min(s0 + u, S - 1) * split_stride + idx];
        a = s0 == 0 ? q[0] : a + q[0];
#pragma unroll
        for (int u = 1; u < 4; ++u)
            if (s0 + u < S) a += q[u];
    }
    return a;
}

// ---- stores whose result another workgroup of the SAME kernel reads --------------------------------
// The L2 caches of the chip's dies are not kept coherent with each other while a kernel runs.  A value that a
// workgroup on another die reads after a grid-wide hand-off is therefore written with a device-scope store, which
// goes through to memory (DEV = true); DEV = false is an ordinary store.  The reader must not have touched the
// line earlier in the same kernel (the layer kernel gives every such buffer its own address per layer and stage).
template <bool DEV, typename T>
__device__ __forceinline__ void st_dev(T *p, T v) {
    if (DEV) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
}
template <bool DEV>
__device__ __forceinline__ void st_dev64(void *p, uint32_t lo, uint32_t hi) {
    typedef __attribute__((ext_vector_type(2))) uint32_t u2;
    if (DEV) __hip_atomic_store(reinterpret_cast<uint64_t *>(p), ((uint64_t)hi << 32) | lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *reinterpret_cast<u2 *>(p) = u2{lo, hi};
}
// 16 bytes as two 8-byte stores.  The elements are copied into named scalars first: a bit-cast applied directly to
// an element of the vector was compiled (hipcc 7.2) into reads of element 0 for every element.
template <bool DEV>
__device__ __forceinline__ void st_dev128(void *p, __attribute__((ext_vector_type(4))) uint32_t v) {
    typedef __attribute__((ext_vector_type(4))) uint32_t u4;
    if (DEV) {
        const uint32_t e0 = v[0], e1 = v[1], e2 = v[2], e3 = v[3];
        st_dev64<true>(p, e0, e1);
        st_dev64<true>(reinterpret_cast<char *>(p) + 8, e2, e3);
    } else {
        *reinterpret_cast<u4 *>(p) = v;
    }
}

// running (largest value, its index, second largest value); ties go to the lower index
struct Top2 { float v1; int i1; float v2; };
__device__ __forceinline__ void top2_push(Top2 &t, float v, int i) {
    if (v > t.v1 || (v == t.v1 && i < t.i1)) { t.v2 = t.v1; t.v1 = v; t.i1 = i; }
    else if (v > t.v2) t.v2 = v;
}
__device__ __forceinline__ void top2_merge(Top2 &a, const Top2 &b) {
    if (b.v1 > a.v1 || (b.v1 == a.v1 && b.i1 < a.i1)) { a.v2 = fmaxf(a.v1, b.v2); a.v1 = b.v1; a.i1 = b.i1; }
    else a.v2 = fmaxf(a.v2, b.v1);
}

__device__ __forceinline__ float silu_f(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

enum { FLAG_CAPACITY = 1, FLAG_BAD_TOKEN = 2, FLAG_BAD_PATH = 4, FLAG_TIMEOUT = 8, FLAG_SATURATED = 16, FLAG_WEIGHT_UNDERFLOW = 32, FLAG_BAD_PAGE = 64 };

}  // namespace hydra
