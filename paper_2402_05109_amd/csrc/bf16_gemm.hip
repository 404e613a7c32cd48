// bf16 storage family: the weight-streaming GEMM on MFMA, and the kernels that
// bring plain row-major weights into its operand order.
//
//   part[split][m][n] = sum_{k in split} X[m][k] * W[n][k]      (fp32)
//
// The matrix W (N x K, bf16) is the only large operand: at M <= 128 rows every
// weight byte is used once, so the kernel is a stream over W that must keep
// enough bytes in flight to cover HBM latency.  Layout: W is stored as 32 x 16
// (n x k) tiles of 1 KiB in the register order of the 32x32x16 MFMA "B"
// operand (lane = (k%16)/8*32 + n%32 holds 8 consecutive k), tiles of one
// 32-row band contiguous along k.  A wave owns NT bands; its load of one tile
// is one fully coalesced 16-byte-per-lane instruction and goes straight to
// registers.  X (M x K, bf16, same tile order, "A" operand) is small and shared
// by all waves of a workgroup: it is staged through LDS in chunks.
// Split-K partial sums are left to the consumer kernel (fixed order => the
// result does not depend on scheduling).
#include "device_common.h"
#include "internal.h"

namespace hydra {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

enum { GEMM_U = 4 };   // k-steps per register block (prefetch distance)

template <int MB, int NT, int CHUNK>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const u32x4_t *__restrict__ Xp, const u32x4_t *__restrict__ Wp,
                                                         float *__restrict__ part, int M, int Npad, int NTiles, int KT,
                                                         int kt_per_split, size_t split_stride) {
    __shared__ u32x4_t xs[MB * CHUNK * 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int tile0 = (blockIdx.x * nwaves + wave) * NT;
    const int kt_begin = blockIdx.y * kt_per_split;
    const int kt_end = min(KT, kt_begin + kt_per_split);
    const int mb0 = blockIdx.z * MB;

    const u32x4_t *wrow[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tile = min(tile0 + t, NTiles - 1);            // clamped: surplus waves stream a valid band and discard it
        wrow[t] = Wp + (size_t)tile * KT * 64 + lane;
    }
    f32x16_t acc[MB][NT];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][t][v] = 0.f;

    u32x4_t wa[GEMM_U][NT], wb[GEMM_U][NT];
    auto load_w = [&](u32x4_t (&w)[GEMM_U][NT], int k0) {
#pragma unroll
        for (int u = 0; u < GEMM_U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t) w[u][t] = wrow[t][(size_t)(k0 + u) * 64];
    };
    auto refill = [&](int k0) {     // stage X k-steps [k0, k0+CHUNK) of the MB row blocks into LDS
        const int cn = min(CHUNK, kt_end - k0);
        __syncthreads();
#pragma unroll
        for (int a = 0; a < MB; ++a)
            for (int i = threadIdx.x; i < cn * 64; i += blockDim.x)
                xs[a * CHUNK * 64 + i] = Xp[((size_t)(mb0 + a) * KT + k0) * 64 + i];
        __syncthreads();
    };
    auto compute = [&](u32x4_t (&w)[GEMM_U][NT], int kl) {     // kl = k-step offset inside the LDS chunk
#pragma unroll
        for (int u = 0; u < GEMM_U; ++u)
#pragma unroll
            for (int a = 0; a < MB; ++a) {
                const bf16x8_t xa = __builtin_bit_cast(bf16x8_t, xs[(a * CHUNK + kl + u) * 64 + lane]);
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[a][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, __builtin_bit_cast(bf16x8_t, w[u][t]), acc[a][t], 0, 0, 0);
            }
    };

    load_w(wa, kt_begin);
    for (int k0 = kt_begin; k0 < kt_end; k0 += 2 * GEMM_U) {
        if ((k0 - kt_begin) % CHUNK == 0) refill(k0);
        const bool has_b = k0 + GEMM_U < kt_end;
        if (has_b) load_w(wb, k0 + GEMM_U);
        compute(wa, (k0 - kt_begin) % CHUNK);
        if (has_b) {
            if ((k0 + GEMM_U - kt_begin) % CHUNK == 0) refill(k0 + GEMM_U);
            if (k0 + 2 * GEMM_U < kt_end) load_w(wa, k0 + 2 * GEMM_U);
            compute(wb, (k0 + GEMM_U - kt_begin) % CHUNK);
        }
    }

    float *dst = part + (size_t)blockIdx.y * split_stride;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (tile0 + t >= NTiles) continue;
        const int col = (tile0 + t) * 32 + (lane & 31);
#pragma unroll
        for (int a = 0; a < MB; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = (mb0 + a) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < M) dst[(size_t)row * Npad + col] = acc[a][t][v];
            }
    }
}

int gemm_npad(const hydra_ctx *c, int N) { return c->bf16 ? ceil_div(N, 32) * 32 : N; }

GemmPlan plan_gemm(const hydra_ctx *c, int M, int N, int K) {
    GemmPlan p;
    if (!c->bf16) { p.mb = 1; p.nt = 1; p.waves = 4; p.splits = 1; p.kt_per_split = K; return p; }
    const int mblocks = ceil_div(M, 32);
    p.mb = mblocks >= 4 ? 4 : (mblocks >= 2 ? 2 : 1);
    const int ntiles = ceil_div(N, 32), KT = K / 16;
    p.waves = 4;
    p.nt = (ntiles >= 512) ? 2 : 1;
    const int wg_n = ceil_div(ntiles, p.waves * p.nt);
    const int mgroups = ceil_div(mblocks, p.mb);
    int S = 1;
    if (M <= 128) {
        S = (640 + wg_n * mgroups - 1) / (wg_n * mgroups);
        const int smax = KT / 16 > 0 ? KT / 16 : 1;
        if (S > smax) S = smax;
        if (S < 1) S = 1;
    }
    int kps = ceil_div(ceil_div(KT, S), 2 * GEMM_U) * 2 * GEMM_U;
    if (kps > KT) kps = KT;
    p.kt_per_split = kps;
    p.splits = ceil_div(KT, kps);
    return p;
}

int launch_gemm_f32(hydra_ctx *c, hipStream_t s, const float *X, const float *W, float *part, int M, int N, int K);

int launch_gemm(hydra_ctx *c, hipStream_t s, const void *X, const void *W, float *part, int M, int N, int K,
                GemmPlan *plan_out) {
    GemmPlan p = plan_gemm(c, M, N, K);
    if (plan_out) *plan_out = p;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (c->profiling) {
        if (c->ev_used + 2 > c->ev.size()) {
            for (int i = 0; i < 2; ++i) { hipEvent_t e; HYDRA_HIP(hipEventCreate(&e)); c->ev.push_back(e); }
        }
        e0 = c->ev[c->ev_used++]; e1 = c->ev[c->ev_used++];
        HYDRA_HIP(hipEventRecord(e0, s));
    }
    int rc = HYDRA_OK;
    if (!c->bf16) {
        rc = launch_gemm_f32(c, s, (const float *)X, (const float *)W, part, M, N, K);
    } else {
        const int ntiles = ceil_div(N, 32), KT = K / 16, npad = ntiles * 32;
        const int mblocks = ceil_div(M, 32);
        dim3 grid(ceil_div(ntiles, p.waves * p.nt), p.splits, ceil_div(mblocks, p.mb)), block(p.waves * 64);
        const size_t split_stride = (size_t)ceil_div(M, 32) * 32 * npad;
        const u32x4_t *Xp = (const u32x4_t *)X, *Wp = (const u32x4_t *)W;
#define GEMM_CASE(MBv, NTv, CHv)                                                                                     \
    hipLaunchKernelGGL((gemm_bf16_kernel<MBv, NTv, CHv>), grid, block, 0, s, Xp, Wp, part, M, npad, ntiles, KT,      \
                       p.kt_per_split, split_stride)
        if (p.mb == 1 && p.nt == 1) GEMM_CASE(1, 1, 32);
        else if (p.mb == 1 && p.nt == 2) GEMM_CASE(1, 2, 32);
        else if (p.mb == 2 && p.nt == 1) GEMM_CASE(2, 1, 32);
        else if (p.mb == 2 && p.nt == 2) GEMM_CASE(2, 2, 32);
        else if (p.mb == 4 && p.nt == 1) GEMM_CASE(4, 1, 16);
        else GEMM_CASE(4, 2, 16);
#undef GEMM_CASE
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) rc = hip_fail(e, "gemm_bf16_kernel");
    }
    if (c->profiling) {
        HYDRA_HIP(hipEventRecord(e1, s));
        c->prof_bytes += (double)N * K * c->esz;
        c->prof_launches += 1;
    }
    return rc;
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
