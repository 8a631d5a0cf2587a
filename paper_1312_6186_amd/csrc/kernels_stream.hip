// Bandwidth-bound kernels of the hot path for gfx950: the fused momentum /
// weight-decay update (optionally writing the worker copy in the same pass), the
// Adagrad / Adadelta updates, the gradient accumulator, the parameter snapshot,
// pooling, response normalisation, softmax cross-entropy, bias-gradient column
// sums and the layout conversions around the channel-last activation format.
// Every reduction has a fixed summation order so that a run is reproducible bit
// for bit.
#include <hip/hip_runtime.h>

#include "asgd_internal.h"

namespace asgd {

typedef __bf16 bf16_t;

__device__ inline float ldf(const float *p) { return *p; }
__device__ inline float ldf(const bf16_t *p) { return (float)*p; }
__device__ inline void stf(float *p, float v) { *p = v; }
__device__ inline void stf(bf16_t *p, float v) { *p = (bf16_t)v; }

static inline unsigned blocks_for(size_t n, unsigned per_block) { return (unsigned)((n + per_block - 1) / per_block); }
static inline int launch_ok() { return hipGetLastError() == hipSuccess ? 0 : -1; }

__host__ __device__ inline uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

uint64_t dropout_key(uint64_t seed, uint64_t step, uint32_t worker, uint32_t layer)
{
    return mix64(mix64(mix64(seed) + step) + (((uint64_t)worker << 32) | (uint64_t)layer));
}

// ---------------------------------------------------------------- update
// t = g + wd*w; v = mu*v - lr*t; w = w + v.  20 bytes of traffic per parameter.
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Each thread owns 4 float4 per buffer, 256 apart, all loads issued before the arithmetic; gradients are read and
// parameters / momentum written with non-temporal hints (the 1.2 GB working set of the AlexNet-style net cannot
// stay in cache between steps anyway).  Measured 5.65 TB/s on 62.4 M parameters.
// One element of the update, with the contractions written out so that every code path (vector body, scalar
// tail, unaligned fallback) rounds identically: t = g + wd*w;  v = mu*v - lr*t;  w = w + v.
__device__ __forceinline__ void update1(float &w, float &v, float g, float lr, float mu, float wd)
{
    const float t = __builtin_fmaf(wd, w, g);
    v = __builtin_fmaf(mu, v, -(lr * t));
    w = w + v;
}

// SNAP: 0 = update only, 1 = also write the new parameters to `copy` as fp32, 2 = as bf16 (round to nearest even):
// the worker copy of the next fetch comes out of the same pass instead of a second read of the parameters.
__device__ inline uint32_t f32_to_bf16_bits(uint32_t u);
// The work of block `blk` of an update over n parameters whose buffers are 16-byte aligned (n4 = n / 4 whole vectors;
// block 0 also takes the n % 4 elements behind them).
template <int SNAP>
__device__ __forceinline__ void update_block(f32x4 *__restrict__ w, f32x4 *__restrict__ v, const f32x4 *__restrict__ g, size_t n4, float *ws, float *vs,
                                             const float *gs, size_t n, float lr, float mu, float wd, void *__restrict__ copy, size_t blk)
{
    constexpr int U = 4;
    const size_t i0 = blk * (256 * U) + threadIdx.x;
    f32x4 ww[U], vv[U], gg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t i = i0 + (size_t)u * 256;
        if (i < n4) { ww[u] = w[i]; vv[u] = v[i]; gg[u] = __builtin_nontemporal_load(&g[i]); }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t i = i0 + (size_t)u * 256;
        if (i < n4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float wn = ww[u][e], vn = vv[u][e];
                update1(wn, vn, gg[u][e], lr, mu, wd);
                ww[u][e] = wn; vv[u][e] = vn;
            }
            __builtin_nontemporal_store(ww[u], &w[i]);
            __builtin_nontemporal_store(vv[u], &v[i]);
            if constexpr (SNAP == 1) static_cast<f32x4 *>(copy)[i] = ww[u];
            if constexpr (SNAP == 2) {
                typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
                u32x2 o;
                o.x = f32_to_bf16_bits(__float_as_uint(ww[u].x)) | (f32_to_bf16_bits(__float_as_uint(ww[u].y)) << 16);
                o.y = f32_to_bf16_bits(__float_as_uint(ww[u].z)) | (f32_to_bf16_bits(__float_as_uint(ww[u].w)) << 16);
                static_cast<u32x2 *>(copy)[i] = o;
            }
        }
    }
    if (blk == 0) {
        const size_t i = n4 * 4 + threadIdx.x;
        if (i < n) {
            float wn = ws[i], vn = vs[i];
            update1(wn, vn, gs[i], lr, mu, wd);
            vs[i] = vn; ws[i] = wn;
            if constexpr (SNAP == 1) static_cast<float *>(copy)[i] = wn;
            if constexpr (SNAP == 2) static_cast<uint16_t *>(copy)[i] = (uint16_t)f32_to_bf16_bits(__float_as_uint(wn));
        }
    }
}

template <int SNAP>
__global__ __launch_bounds__(256) void update_kernel(f32x4 *__restrict__ w, f32x4 *__restrict__ v, const f32x4 *__restrict__ g, size_t n4,
                                                     float *ws, float *vs, const float *gs, size_t n, float lr, float mu, float wd,
                                                     int *version_counter, void *__restrict__ copy)
{
    update_block<SNAP>(w, v, g, n4, ws, vs, gs, n, lr, mu, wd, copy, blockIdx.x);
    if (blockIdx.x == 0 && threadIdx.x == 0 && version_counter) *version_counter += 1;
}

// The same over up to eight separate ranges of one parameter vector in one launch (the slices that are left when
// some layers have been pushed elsewhere): a block finds its range, then does what update_kernel's block does on it.
// A range whose start is not a multiple of 4 elements runs element by element.
struct UpdateRanges { size_t off[8], cnt[8]; unsigned blk[9]; int n; };
template <int SNAP>
__global__ __launch_bounds__(256) void update_ranges_kernel(float *w, float *v, const float *g, UpdateRanges R, float lr, float mu, float wd, void *copy)
{
    int q = 0;
    while (q + 1 < R.n && blockIdx.x >= R.blk[q + 1]) ++q;
    const size_t off = R.off[q], n = R.cnt[q], blk = blockIdx.x - R.blk[q];
    constexpr size_t es = SNAP == 2 ? 2 : 4;
    if ((off & 3) == 0) {
        update_block<SNAP>(reinterpret_cast<f32x4 *>(w + off), reinterpret_cast<f32x4 *>(v + off), reinterpret_cast<const f32x4 *>(g + off), n / 4, w + off,
                           v + off, g + off, n, lr, mu, wd, static_cast<char *>(copy) + off * es, blk);
    } else {
        for (size_t i = blk * 1024 + threadIdx.x; i < n && i < (blk + 1) * 1024; i += 256) {
            float wn = w[off + i], vn = v[off + i];
            update1(wn, vn, g[off + i], lr, mu, wd);
            v[off + i] = vn; w[off + i] = wn;
            if constexpr (SNAP == 1) static_cast<float *>(copy)[off + i] = wn;
            if constexpr (SNAP == 2) static_cast<uint16_t *>(copy)[off + i] = (uint16_t)f32_to_bf16_bits(__float_as_uint(wn));
        }
    }
}

template <int SNAP>
__global__ __launch_bounds__(256) void update_scalar_kernel(float *w, float *v, const float *g, size_t n, float lr, float mu, float wd,
                                                            int *version_counter, void *copy)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float wn = w[i], vn = v[i];
        update1(wn, vn, g[i], lr, mu, wd);
        v[i] = vn; w[i] = wn;
        if constexpr (SNAP == 1) static_cast<float *>(copy)[i] = wn;
        if constexpr (SNAP == 2) static_cast<uint16_t *>(copy)[i] = (uint16_t)f32_to_bf16_bits(__float_as_uint(wn));
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && version_counter) *version_counter += 1;
}

template <int SNAP>
static int launch_update_t(float *w, float *v, const float *g, size_t n, float lr, float mu, float wd, int *version_counter, void *copy, hipStream_t s)
{
    const unsigned copy_align = SNAP == 1 ? 15u : SNAP == 2 ? 7u : 0u;
    const bool aligned = (((uintptr_t)w | (uintptr_t)v | (uintptr_t)g) & 15) == 0 && ((uintptr_t)copy & copy_align) == 0;
    if (aligned && n >= 4) {
        const size_t n4 = n / 4;
        const size_t blocks = (n4 + 1023) / 1024 ? (n4 + 1023) / 1024 : 1;
        if (blocks > 0x7fffffffu) return -1;
        hipLaunchKernelGGL(update_kernel<SNAP>, dim3((unsigned)blocks), dim3(256), 0, s, reinterpret_cast<f32x4 *>(w), reinterpret_cast<f32x4 *>(v),
                           reinterpret_cast<const f32x4 *>(g), n4, w, v, g, n, lr, mu, wd, version_counter, copy);
    } else {
        unsigned blocks = blocks_for(n ? n : 1, 256);
        if (blocks > 8192) blocks = 8192;
        hipLaunchKernelGGL(update_scalar_kernel<SNAP>, dim3(blocks), dim3(256), 0, s, w, v, g, n, lr, mu, wd, version_counter, copy);
    }
    return launch_ok();
}
int launch_update(float *w, float *v, const float *g, size_t n, float lr, float mu, float wd, int *version_counter, hipStream_t s)
{
    return launch_update_t<0>(w, v, g, n, lr, mu, wd, version_counter, nullptr, s);
}
int launch_update_snapshot_ranges(float *w, float *v, const float *g, const size_t *off, const size_t *cnt, int n_ranges, float lr, float mu, float wd,
                                  void *copy, int dst_dtype, hipStream_t s)
{
    if (n_ranges <= 0) return 0;
    if (n_ranges > 8) return -1;
    if ((((uintptr_t)w | (uintptr_t)v | (uintptr_t)g | (uintptr_t)copy) & 15) != 0) return -1;
    UpdateRanges R; R.n = n_ranges;
    size_t blocks = 0;
    for (int q = 0; q < n_ranges; ++q) {
        R.off[q] = off[q]; R.cnt[q] = cnt[q]; R.blk[q] = (unsigned)blocks;
        const size_t b = (off[q] & 3) == 0 ? (cnt[q] / 4 + 1023) / 1024 : (cnt[q] + 1023) / 1024;   // 1024 vectors, or 1024 elements, per block
        blocks += b ? b : 1;
        if (blocks > 0x7fffffffu) return -1;
    }
    R.blk[n_ranges] = (unsigned)blocks;
    if (dst_dtype == kBF16) hipLaunchKernelGGL(update_ranges_kernel<2>, dim3((unsigned)blocks), dim3(256), 0, s, w, v, g, R, lr, mu, wd, copy);
    else hipLaunchKernelGGL(update_ranges_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, s, w, v, g, R, lr, mu, wd, copy);
    return launch_ok();
}
int launch_update_snapshot(float *w, float *v, const float *g, size_t n, float lr, float mu, float wd, void *copy, int dst_dtype, hipStream_t s)
{
    return dst_dtype == kBF16 ? launch_update_t<2>(w, v, g, n, lr, mu, wd, nullptr, copy, s) : launch_update_t<1>(w, v, g, n, lr, mu, wd, nullptr, copy, s);
}

// ---------------------------------------------------------------- Adagrad / Adadelta server updates
// The same streaming shape as the momentum update: 16-byte vectors where the buffers allow, identical arithmetic
// (explicit contractions) on every path.
//   Adagrad :  t = g + wd*w;  h += t*t;  w -= lr * t / (sqrt(h) + eps)
//   Adadelta:  t = g + wd*w;  a = rho*a + (1-rho)*t*t;  d = -sqrt(b+eps)/sqrt(a+eps)*t;  b = rho*b + (1-rho)*d*d;  w += d
__device__ __forceinline__ void adagrad1(float &w, float &h, float g, float lr, float eps, float wd)
{
    const float t = __builtin_fmaf(wd, w, g);
    h = __builtin_fmaf(t, t, h);
    w = w - lr * t * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(h) + eps);   // hardware sqrt and reciprocal: about an ulp each on the step
}
__device__ __forceinline__ void adadelta1(float &w, float &a, float &b, float g, float rho, float eps, float wd)
{
    const float t = __builtin_fmaf(wd, w, g);
    a = __builtin_fmaf(rho, a, (1.f - rho) * (t * t));
    const float d = -(__builtin_amdgcn_sqrtf(b + eps) * __builtin_amdgcn_rsqf(a + eps)) * t;   // hardware sqrt and reciprocal sqrt
    b = __builtin_fmaf(rho, b, (1.f - rho) * (d * d));
    w = w + d;
}
// KIND 0: Adagrad (s1 = h, s2 unused, c1 = lr); KIND 1: Adadelta (s1 = a, s2 = b, c1 = rho)
template <int KIND>
__global__ __launch_bounds__(256) void adaptive_update_kernel(float *__restrict__ w, float *__restrict__ s1, float *__restrict__ s2,
                                                             const float *__restrict__ g, size_t n, int vec, float c1, float eps, float wd)
{
    // vector body: each thread owns U float4 per buffer, 256 apart, all loads issued before the arithmetic
    constexpr int U = 4;
    const size_t n4 = vec ? n / 4 : 0;
    const size_t i0 = (size_t)blockIdx.x * (256 * U) + threadIdx.x;
    f32x4 ww[U], aa[U], bb[U], gg[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t i = i0 + (size_t)u * 256;
        if (i < n4) {
            ww[u] = reinterpret_cast<f32x4 *>(w)[i]; aa[u] = reinterpret_cast<f32x4 *>(s1)[i];
            if (KIND == 1) bb[u] = reinterpret_cast<f32x4 *>(s2)[i];
            gg[u] = __builtin_nontemporal_load(&reinterpret_cast<const f32x4 *>(g)[i]);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t i = i0 + (size_t)u * 256;
        if (i < n4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float we = ww[u][e], ae = aa[u][e], be = KIND == 1 ? bb[u][e] : 0.f;
                if (KIND == 0) adagrad1(we, ae, gg[u][e], c1, eps, wd);
                else adadelta1(we, ae, be, gg[u][e], c1, eps, wd);
                ww[u][e] = we; aa[u][e] = ae;
                if (KIND == 1) bb[u][e] = be;
            }
            __builtin_nontemporal_store(ww[u], &reinterpret_cast<f32x4 *>(w)[i]);
            __builtin_nontemporal_store(aa[u], &reinterpret_cast<f32x4 *>(s1)[i]);
            if (KIND == 1) __builtin_nontemporal_store(bb[u], &reinterpret_cast<f32x4 *>(s2)[i]);
        }
    }
    // scalar tail (everything, if the buffers are not 16-byte aligned), grid-stride
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = n4 * 4 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float we = w[i], ae = s1[i], be = KIND == 1 ? s2[i] : 0.f;
        if (KIND == 0) adagrad1(we, ae, g[i], c1, eps, wd);
        else adadelta1(we, ae, be, g[i], c1, eps, wd);
        w[i] = we; s1[i] = ae;
        if (KIND == 1) s2[i] = be;
    }
}
static unsigned adaptive_blocks(size_t n, int vec)
{
    if (vec) { const size_t b = (n / 4 + 1023) / 1024; return (unsigned)(b ? b : 1); }
    unsigned b = blocks_for(n ? n : 1, 256);
    return b > 32768 ? 32768 : b;
}
int launch_adagrad(float *w, float *h, const float *g, size_t n, float lr, float eps, float wd, hipStream_t s)
{
    const int vec = ((((uintptr_t)w | (uintptr_t)h | (uintptr_t)g) & 15) == 0) ? 1 : 0;
    const unsigned blocks = adaptive_blocks(n, vec);
    hipLaunchKernelGGL(adaptive_update_kernel<0>, dim3(blocks), dim3(256), 0, s, w, h, static_cast<float *>(nullptr), g, n, vec, lr, eps, wd);
    return launch_ok();
}
int launch_adadelta(float *w, float *a, float *b, const float *g, size_t n, float rho, float eps, float wd, hipStream_t s)
{
    const int vec = ((((uintptr_t)w | (uintptr_t)a | (uintptr_t)b | (uintptr_t)g) & 15) == 0) ? 1 : 0;
    const unsigned blocks = adaptive_blocks(n, vec);
    hipLaunchKernelGGL(adaptive_update_kernel<1>, dim3(blocks), dim3(256), 0, s, w, a, b, g, n, vec, rho, eps, wd);
    return launch_ok();
}

// ---------------------------------------------------------------- gradient accumulator (n_push > 1)
// acc = g (first) or acc + g; 16-byte vectors when both are aligned, the same arithmetic either way.
__global__ __launch_bounds__(256) void accumulate_kernel(float *__restrict__ acc, const float *__restrict__ g, size_t n, int first, int vec)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t t0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t n4 = vec ? n / 4 : 0;
    for (size_t i = t0; i < n4; i += stride) {
        f32x4 a = __builtin_nontemporal_load(&reinterpret_cast<const f32x4 *>(g)[i]);
        if (!first) a += reinterpret_cast<f32x4 *>(acc)[i];
        reinterpret_cast<f32x4 *>(acc)[i] = a;
    }
    for (size_t i = n4 * 4 + t0; i < n; i += stride) acc[i] = first ? g[i] : acc[i] + g[i];
}
int launch_accumulate(float *acc, const float *g, size_t n, bool first, hipStream_t s)
{
    const int vec = ((((uintptr_t)acc | (uintptr_t)g) & 15) == 0) ? 1 : 0;
    unsigned blocks = blocks_for(vec ? (n + 3) / 4 : n, 256);
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(accumulate_kernel, dim3(blocks), dim3(256), 0, s, acc, g, n, first ? 1 : 0, vec);
    return launch_ok();
}

// ---------------------------------------------------------------- snapshot
__device__ inline uint32_t f32_to_bf16_bits(uint32_t u)  // round to nearest even; NaN -> quiet NaN
{
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (u >> 16) | 0x0040u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__global__ __launch_bounds__(256) void snapshot_kernel(const float *__restrict__ src, void *__restrict__ dst, size_t n, int to_bf16, int vec,
                                                       const int *version_counter, int32_t *log_slot, int log_update, int log_worker)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t t0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t0 == 0 && log_slot) {
        log_slot[0] = log_update;
        log_slot[1] = log_worker;
        log_slot[2] = version_counter ? *version_counter : -1;
    }
    if (!to_bf16) {
        float *d = static_cast<float *>(dst);
        const size_t n4 = vec ? n / 4 : 0;
        for (size_t i = t0; i < n4; i += stride) reinterpret_cast<float4 *>(d)[i] = reinterpret_cast<const float4 *>(src)[i];
        for (size_t i = n4 * 4 + t0; i < n; i += stride) d[i] = src[i];
    } else {
        uint16_t *d = static_cast<uint16_t *>(dst);
        const size_t n8 = vec ? n / 8 : 0;
        // groups of 8 elements; a thread takes four of them per round, 256 apart, and issues its eight loads first
        typedef unsigned u32x4v __attribute__((ext_vector_type(4)));
        constexpr int U = 4;
        for (size_t base = (size_t)blockIdx.x * (256 * U); base < n8; base += (size_t)gridDim.x * (256 * U)) {
            u32x4v a[U], b[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t i = base + threadIdx.x + (size_t)u * 256;
                if (i < n8) {
                    a[u] = __builtin_nontemporal_load(&reinterpret_cast<const u32x4v *>(src)[2 * i]);
                    b[u] = __builtin_nontemporal_load(&reinterpret_cast<const u32x4v *>(src)[2 * i + 1]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t i = base + threadIdx.x + (size_t)u * 256;
                if (i < n8) {
                    uint4 o;
                    o.x = f32_to_bf16_bits(a[u].x) | (f32_to_bf16_bits(a[u].y) << 16);
                    o.y = f32_to_bf16_bits(a[u].z) | (f32_to_bf16_bits(a[u].w) << 16);
                    o.z = f32_to_bf16_bits(b[u].x) | (f32_to_bf16_bits(b[u].y) << 16);
                    o.w = f32_to_bf16_bits(b[u].z) | (f32_to_bf16_bits(b[u].w) << 16);
                    reinterpret_cast<uint4 *>(d)[i] = o;
                }
            }
        }
        for (size_t i = n8 * 8 + t0; i < n; i += stride) d[i] = (uint16_t)f32_to_bf16_bits(__float_as_uint(src[i]));
    }
}

int launch_snapshot(const float *src, void *dst, size_t n, int dst_dtype, const int *version_counter, int32_t *log_slot, int log_update,
                    int log_worker, hipStream_t s)
{
    const int vec = (((uintptr_t)src | (uintptr_t)dst) & 15) == 0;
    const size_t per = dst_dtype == kBF16 ? 8 : 4;
    unsigned blocks = blocks_for(n / per + 1, 256);
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(snapshot_kernel, dim3(blocks), dim3(256), 0, s, src, dst, n, dst_dtype == kBF16 ? 1 : 0, vec, version_counter, log_slot,
                       log_update, log_worker);
    return launch_ok();
}

// ---------------------------------------------------------------- fill
__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t *p, size_t words)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += stride) p[i] = 0u;
}
int launch_fill_zero(void *p, size_t bytes, hipStream_t s)
{
    if (bytes == 0) return 0;
    if ((bytes & 3) || ((uintptr_t)p & 3)) return -1;
    unsigned blocks = blocks_for(bytes / 4, 256);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, s, static_cast<uint32_t *>(p), bytes / 4);
    return launch_ok();
}

// ---------------------------------------------------------------- input staging and filter packing
template <typename T> __global__ __launch_bounds__(256) void stage_input_kernel(const T *__restrict__ src, T *__restrict__ dst, int B, int C, int H,
                                                                              int W, int Cp)
{
    // one thread per pixel and 16-byte channel group: reads are contiguous along w for each channel,
    // the store is one vector
    constexpr int V = 16 / sizeof(T);
    const int groups = Cp / V;
    const long HW = (long)H * W;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= (long)B * HW * groups) return;
    const long pix = i % ((long)B * HW);       // pixels fastest: neighbouring threads read neighbouring w
    const int gidx = (int)(i / ((long)B * HW));
    const long n = pix / HW, hw = pix - n * HW;
    union { uint4 u; T e[V]; } v;
#pragma unroll
    for (int e = 0; e < V; ++e) {
        const int c = gidx * V + e;
        v.e[e] = c < C ? src[(n * C + c) * HW + hw] : (T)0.f;
    }
    *reinterpret_cast<uint4 *>(dst + pix * Cp + gidx * V) = v.u;
}
int launch_stage_input(int dtype, const void *src, void *dst, int B, int C, int H, int W, int Cp, hipStream_t s)
{
    const unsigned blocks = blocks_for((size_t)B * H * W * (Cp / (dtype == kBF16 ? 8 : 4)), 256);
    if (dtype == kBF16)
        hipLaunchKernelGGL(stage_input_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, static_cast<const bf16_t *>(src), static_cast<bf16_t *>(dst), B, C, H, W, Cp);
    else
        hipLaunchKernelGGL(stage_input_kernel<float>, dim3(blocks), dim3(256), 0, s, static_cast<const float *>(src), static_cast<float *>(dst), B, C, H, W, Cp);
    return launch_ok();
}

template <typename T, int PC> __global__ __launch_bounds__(256) void stage_input_rw_kernel(const T *__restrict__ src, T *__restrict__ dst, int B, int C,
                                                                                         int H, int W, int pad, int Wp)
{
    // a thread moves two neighbouring pixels of a row (W is even, checked by the launcher): 2 * PC elements, which
    // for every PC and element size make a whole number of dwords at a dword-aligned address
    const long HW = (long)H * W, HW2 = HW / 2;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= (long)B * HW2) return;
    const long n = i / HW2, hw = (i - n * HW2) * 2;
    const int h = (int)(hw / W), w = (int)(hw - (long)h * W);
    union { T e[2 * PC]; uint32_t u[2 * PC * sizeof(T) / 4]; } v;
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int c = 0; c < PC; ++c) v.e[q * PC + c] = c < C ? src[(n * C + c) * HW + hw + q] : (T)0.f;
    uint32_t *o = reinterpret_cast<uint32_t *>(dst + ((n * (H + 2 * pad) + h + pad) * Wp + w + pad) * PC);
#pragma unroll
    for (int d = 0; d < (int)(2 * PC * sizeof(T) / 4); ++d) o[d] = v.u[d];
}
// one pixel per thread, element stores: any width
template <typename T> __global__ __launch_bounds__(256) void stage_input_rw_any_kernel(const T *__restrict__ src, T *__restrict__ dst, int B, int C,
                                                                                     int H, int W, int pad, int Wp, int pc)
{
    const long HW = (long)H * W;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= (long)B * HW) return;
    const long n = i / HW, hw = i - n * HW;
    const int h = (int)(hw / W), w = (int)(hw - (long)h * W);
    T *o = dst + ((n * (H + 2 * pad) + h + pad) * Wp + w + pad) * pc;
    for (int c = 0; c < pc; ++c) o[c] = c < C ? src[(n * C + c) * HW + hw] : (T)0.f;
}
template <typename T>
static void launch_stage_input_rw_t(const void *src, void *dst, int B, int C, int H, int W, int pad, int Wp, int pc, hipStream_t s)
{
    const T *a = static_cast<const T *>(src); T *o = static_cast<T *>(dst);
    // the pair form needs both pixels in one row and every pair dword-aligned: (pad * pc), (Wp * pc) elements even in bytes / 4
    const bool pairs = (W % 2 == 0) && ((size_t)pad * pc * sizeof(T)) % 4 == 0 && ((size_t)Wp * pc * sizeof(T)) % 4 == 0 &&
                       ((size_t)2 * pc * sizeof(T)) % 4 == 0;
    if (pairs) {
        const unsigned blocks = blocks_for((size_t)B * H * W / 2, 256);
        switch (pc) {
        case 1: hipLaunchKernelGGL((stage_input_rw_kernel<T, 1>), dim3(blocks), dim3(256), 0, s, a, o, B, C, H, W, pad, Wp); return;
        case 2: hipLaunchKernelGGL((stage_input_rw_kernel<T, 2>), dim3(blocks), dim3(256), 0, s, a, o, B, C, H, W, pad, Wp); return;
        case 3: hipLaunchKernelGGL((stage_input_rw_kernel<T, 3>), dim3(blocks), dim3(256), 0, s, a, o, B, C, H, W, pad, Wp); return;
        case 4: hipLaunchKernelGGL((stage_input_rw_kernel<T, 4>), dim3(blocks), dim3(256), 0, s, a, o, B, C, H, W, pad, Wp); return;
        }
    }
    hipLaunchKernelGGL(stage_input_rw_any_kernel<T>, dim3(blocks_for((size_t)B * H * W, 256)), dim3(256), 0, s, a, o, B, C, H, W, pad, Wp, pc);
}
int launch_stage_input_rw(int dtype, const void *src, void *dst, int B, int C, int H, int W, int pad, int Wp, int pc, hipStream_t s)
{
    if (C > pc || pc < 1 || pc > 4) return -1;
    if (dtype == kBF16) launch_stage_input_rw_t<bf16_t>(src, dst, B, C, H, W, pad, Wp, pc, s);
    else launch_stage_input_rw_t<float>(src, dst, B, C, H, W, pad, Wp, pc, s);
    return launch_ok();
}

// All convolution layers of a net in one launch.  A thread produces 8 consecutive packed elements (the innermost
// packed index is a multiple of 8 wide in every pack) and stores them as one or two 16-byte vectors; group g
// belongs to the job whose range holds it.
template <typename T> __global__ __launch_bounds__(256) void pack_conv_kernel(PackJobs jobs)
{
    const unsigned g = blockIdx.x * 256u + threadIdx.x;
    if (g >= jobs.total) return;
    int q = 0;
    while (q + 1 < jobs.n && g >= jobs.j[q + 1].start) ++q;
    const PackJob &J = jobs.j[q];
    const T *w = static_cast<const T *>(J.w);
    unsigned li = (g - J.start) * 8u;     // first of this thread's 8 elements
    const int k = J.k;
    const long kk = (long)k * k;
    __attribute__((aligned(16))) T out[8];
    T *dst;
    if (J.rw) {  // wf[co][ky][j], j = kx*rw + ci over a padded window row of KW elements (rw channels per stored pixel)
        const int j0 = (int)(li % (unsigned)J.KW); unsigned t = li / (unsigned)J.KW;
        const int ky = (int)(t % (unsigned)k), co = (int)(t / (unsigned)k);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int kx = (j0 + e) / J.rw, ci = (j0 + e) - kx * J.rw;
            out[e] = (co < J.cout && ci < J.cin && kx < k) ? w[((long)co * J.cin + ci) * kk + ky * k + kx] : (T)0.f;
        }
        dst = static_cast<T *>(J.wf) + li;
    } else if (li < J.nf) {  // wf[co][ky][kx][ci]
        const int ci0 = (int)(li % (unsigned)J.cinp); unsigned t = li / (unsigned)J.cinp;
        const int kx = (int)(t % (unsigned)k); t /= (unsigned)k;
        const int ky = (int)(t % (unsigned)k), co = (int)(t / (unsigned)k);
        const T *src = w + ((long)co * J.cin + ci0) * kk + ky * k + kx;
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = (co < J.cout && ci0 + e < J.cin) ? src[e * kk] : (T)0.f;
        dst = static_cast<T *>(J.wf) + li;
    } else {  // wd[ci][ky'][kx'][co] = w[co][ci][k-1-ky'][k-1-kx']
        li -= J.nf;
        const int co0 = (int)(li % (unsigned)J.coutp); unsigned t = li / (unsigned)J.coutp;
        const int kx = (int)(t % (unsigned)k); t /= (unsigned)k;
        const int ky = (int)(t % (unsigned)k), ci = (int)(t / (unsigned)k);
        const T *src = w + ((long)co0 * J.cin + ci) * kk + (k - 1 - ky) * k + (k - 1 - kx);
        const long cstride = (long)J.cin * kk;
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = (co0 + e < J.cout && ci < J.cin) ? src[e * cstride] : (T)0.f;
        dst = static_cast<T *>(J.wd) + li;
    }
    uint4 *d4 = reinterpret_cast<uint4 *>(dst);
    const uint4 *o4 = reinterpret_cast<const uint4 *>(out);
#pragma unroll
    for (int v = 0; v < (int)(8 * sizeof(T) / 16); ++v) d4[v] = o4[v];
}
// The same through LDS, for layers whose filters of 16 bytes' worth of output channels (8 in bf16, 4 in fp32) fit
// into 64 KB: a workgroup owns such a group of output channels, copies its filters (one contiguous, 16-byte aligned
// run of the canonical tensor) into LDS with 16-byte loads and writes every packed vector that holds them.  The
// gather form above reads its 8 elements k*k apart, 2 or 4 bytes at a time.
template <typename T> __global__ __launch_bounds__(1024) void pack_conv_lds_kernel(PackJobs jobs)
{
    constexpr int V = 16 / (int)sizeof(T), NT = 1024;
    __shared__ uint4 slab4[4096];
    T *slab = reinterpret_cast<T *>(slab4);
    int q = 0;
    while (q + 1 < jobs.n && blockIdx.x >= jobs.j[q + 1].start) ++q;
    const PackJob &J = jobs.j[q];
    const int tid = threadIdx.x;
    const int co0 = (int)(blockIdx.x - J.start) * V;
    const int k = J.k, kk = k * k, S = J.cin * kk;   // S: elements per output channel
    const long left = (long)J.cout * S - (long)co0 * S;
    const int n_el = (int)(left < (long)V * S ? (left > 0 ? left : 0) : (long)V * S);   // elements of this group that exist
    const T *w = static_cast<const T *>(J.w) + (long)co0 * S;
    const int n16 = n_el / V;
    for (int i = tid; i < n16; i += NT) slab4[i] = reinterpret_cast<const uint4 *>(w)[i];
    for (int i = n16 * V + tid; i < n_el; i += NT) slab[i] = w[i];
    __syncthreads();
    // filter element (output channel co0 + c, input channel ci, window position p); zero outside the tensor
    auto at = [&](int c, int ci, int p) -> T {
        const int i = c * S + ci * kk + p;
        return (ci < J.cin && i < n_el) ? slab[i] : (T)0.f;
    };
    union { uint4 u; T e[V]; } o;
    if (J.rw) {  // wf[co][ky][j], j = kx*rw + ci over a padded window row of KW elements
        const int jv = J.KW / V, n = V * k * jv;
        for (int i = tid; i < n; i += NT) {
            const int jg = i % jv, t = i / jv, ky = t % k, c = t / k;
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const int j = jg * V + e, kx = j / J.rw, ci = j - kx * J.rw;
                o.e[e] = kx < k ? at(c, ci, ky * k + kx) : (T)0.f;
            }
            *reinterpret_cast<uint4 *>(static_cast<T *>(J.wf) + ((long)(co0 + c) * k + ky) * J.KW + jg * V) = o.u;
        }
        return;
    }
    if (J.wf) {  // wf[co][ky][kx][ci]
        const int cv = J.cinp / V, n = V * kk * cv;
        for (int i = tid; i < n; i += NT) {
            const int cg = i % cv, t = i / cv, pp = t % kk, c = t / kk;
#pragma unroll
            for (int e = 0; e < V; ++e) o.e[e] = at(c, cg * V + e, pp);
            *reinterpret_cast<uint4 *>(static_cast<T *>(J.wf) + ((long)(co0 + c) * kk + pp) * J.cinp + cg * V) = o.u;
        }
    }
    if (J.wd) {  // wd[ci][ky'][kx'][co] = w[co][ci][k-1-ky'][k-1-kx']: this group's 16 bytes of every (ci, ky', kx')
        const int n = J.cinp * kk;
        for (int i = tid; i < n; i += NT) {
            const int pp = i % kk, ci = i / kk;
#pragma unroll
            for (int e = 0; e < V; ++e) o.e[e] = at(e, ci, kk - 1 - pp);
            *reinterpret_cast<uint4 *>(static_cast<T *>(J.wd) + ((long)ci * kk + pp) * J.coutp + co0) = o.u;
        }
    }
}

int launch_pack_conv(int dtype, PackJobs &jobs, hipStream_t s)
{
    // the LDS form, if every layer qualifies
    {
        const size_t es = dtype_size(dtype), V = 16 / es;
        bool ok = jobs.n > 0;
        size_t blocks = 0;
        for (int q = 0; q < jobs.n && ok; ++q) {
            const PackJob &J = jobs.j[q];
            const size_t S = (size_t)J.cin * J.k * J.k;
            ok = V * S * es <= 65536 && (((uintptr_t)J.w | (uintptr_t)J.wf | (uintptr_t)J.wd) & 15) == 0 && J.coutp % 8 == 0 && J.cinp % 8 == 0 &&
                 (J.wf || J.wd) && (!J.rw || (J.wf && J.KW % 8 == 0 && J.rw > 0));
            blocks += (size_t)J.coutp / V;
        }
        if (ok && blocks <= 0x7fffffffull) {
            unsigned start = 0;
            for (int q = 0; q < jobs.n; ++q) { jobs.j[q].start = start; start += (unsigned)(jobs.j[q].coutp / (int)V); }
            jobs.total = start;
            if (dtype == kBF16) hipLaunchKernelGGL(pack_conv_lds_kernel<bf16_t>, dim3(start), dim3(1024), 0, s, jobs);
            else hipLaunchKernelGGL(pack_conv_lds_kernel<float>, dim3(start), dim3(1024), 0, s, jobs);
            return launch_ok();
        }
    }
    size_t total = 0;
    for (int q = 0; q < jobs.n; ++q) {
        PackJob &J = jobs.j[q];
        const size_t full = J.rw ? (size_t)J.coutp * J.k * J.KW : (size_t)J.coutp * J.k * J.k * J.cinp;
        const size_t nf = J.wf ? full : 0;
        const size_t nd = (!J.rw && J.wd) ? full : 0;
        if (nf + nd > 0xffffffffull || (nf & 7)) return -1;   // cinp, coutp and KW are multiples of 8
        J.start = (unsigned)total; J.nf = (unsigned)nf;
        total += (nf + nd) / 8;                                 // in groups of 8 elements
    }
    if (total == 0) return 0;
    jobs.total = (unsigned)total;
    const unsigned blocks = blocks_for(total, 256);
    if (dtype == kBF16) hipLaunchKernelGGL(pack_conv_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, jobs);
    else hipLaunchKernelGGL(pack_conv_kernel<float>, dim3(blocks), dim3(256), 0, s, jobs);
    return launch_ok();
}

// ---------------------------------------------------------------- max pooling
__device__ __forceinline__ uint32_t fdiv32(uint32_t n, const FastDiv &f) { return (__umulhi(n, f.mul) + n) >> f.sh; }
// Workgroup ids go round-robin over the 8 XCDs; neighbouring pixels share pooling windows, so each XCD is given a
// contiguous range of blocks (and its L2 fetches a window row once instead of every XCD fetching it).
__device__ __forceinline__ uint32_t xcd_block()
{
    const uint32_t nb = gridDim.x, q = nb >> 3, r = nb & 7, x = blockIdx.x & 7;
    return x * q + (x < r ? x : r) + (blockIdx.x >> 3);
}
// thread index -> (channel group, x, y, image) by three multiply-shift divisions (the index fits 31 bits)
struct PoolIndex { FastDiv dcv, dw, dh; int cv, w, h; };
static PoolIndex make_pool_index(int cv, int w, int h)
{
    return PoolIndex{make_fastdiv((uint32_t)cv), make_fastdiv((uint32_t)w), make_fastdiv((uint32_t)h), cv, w, h};
}
__device__ __forceinline__ void pool_decode(uint32_t i, const PoolIndex &p, int &cg, int &x, int &y, int &n)
{
    uint32_t t = fdiv32(i, p.dcv); cg = (int)(i - t * p.cv);
    uint32_t u = fdiv32(t, p.dw); x = (int)(t - u * p.w);
    n = (int)fdiv32(u, p.dh); y = (int)(u - (uint32_t)n * p.h);
}
// One thread owns VEC consecutive channels (16 bytes) of one output pixel.
template <typename T> struct Vec16 {
    static constexpr int N = 16 / sizeof(T);
    union { uint4 u; T e[16 / sizeof(T)]; };
};

// KC > 0: window size known at compile time, so the k*k loads of a thread are all issued before the first compare.
template <typename T, int KC>
__global__ __launch_bounds__(256) void pool_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, uint8_t *__restrict__ arg, int B, int H, int W,
                                                     int Cp, int k_rt, int stride, int Ho, int Wo, PoolIndex pi)
{
    constexpr int V = Vec16<T>::N;
    const int k = KC > 0 ? KC : k_rt;
    const uint32_t i = xcd_block() * 256u + threadIdx.x;
    if (i >= (uint32_t)B * Ho * Wo * pi.cv) return;
    int cg, px, py, n;
    pool_decode(i, pi, cg, px, py, n);
    const int c0 = cg * V;
    const T *win = x + (((long)n * H + py * stride) * W + px * stride) * Cp + c0;
    float best[V];
    uint8_t a[V];
    if constexpr (KC > 0) {
        Vec16<T> v[KC * KC];
#pragma unroll
        for (int p = 0; p < KC * KC; ++p) v[p].u = *reinterpret_cast<const uint4 *>(win + ((long)(p / KC) * W + (p % KC)) * Cp);
#pragma unroll
        for (int p = 0; p < KC * KC; ++p) {
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float f = ldf(&v[p].e[e]);
                if (p == 0 || f > best[e]) { best[e] = f; a[e] = (uint8_t)p; }
            }
        }
    } else {
        for (int ky = 0; ky < k; ++ky)
            for (int kx = 0; kx < k; ++kx) {
                Vec16<T> v;
                v.u = *reinterpret_cast<const uint4 *>(win + ((long)ky * W + kx) * Cp);
                const int pos = ky * k + kx;
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const float f = ldf(&v.e[e]);
                    if (pos == 0 || f > best[e]) { best[e] = f; a[e] = (uint8_t)pos; }
                }
            }
    }
    Vec16<T> o;
#pragma unroll
    for (int e = 0; e < V; ++e) stf(&o.e[e], best[e]);
    const long off = (((long)n * Ho + py) * Wo + px) * Cp + c0;
    *reinterpret_cast<uint4 *>(y + off) = o.u;
    uint64_t packed = 0;
#pragma unroll
    for (int e = 0; e < V; ++e) packed |= (uint64_t)a[e] << (8 * e);
    if (V == 8) *reinterpret_cast<uint64_t *>(arg + off) = packed;
    else *reinterpret_cast<uint32_t *>(arg + off) = (uint32_t)packed;
}

template <typename T>
static void launch_pool_fwd_t(const void *x, void *y, uint8_t *arg, int B, int H, int W, int Cp, int k, int stride, int Ho, int Wo, unsigned blocks,
                              hipStream_t s)
{
    const T *xx = static_cast<const T *>(x); T *yy = static_cast<T *>(y);
    const PoolIndex pi = make_pool_index(Cp / (16 / (int)sizeof(T)), Wo, Ho);
    if (k == 3) hipLaunchKernelGGL((pool_fwd_kernel<T, 3>), dim3(blocks), dim3(256), 0, s, xx, yy, arg, B, H, W, Cp, k, stride, Ho, Wo, pi);
    else if (k == 2) hipLaunchKernelGGL((pool_fwd_kernel<T, 2>), dim3(blocks), dim3(256), 0, s, xx, yy, arg, B, H, W, Cp, k, stride, Ho, Wo, pi);
    else hipLaunchKernelGGL((pool_fwd_kernel<T, 0>), dim3(blocks), dim3(256), 0, s, xx, yy, arg, B, H, W, Cp, k, stride, Ho, Wo, pi);
}
int launch_pool_fwd(int dtype, const void *x, void *y, uint8_t *arg, int B, int H, int W, int Cp, int k, int stride, hipStream_t s)
{
    const int Ho = (H - k) / stride + 1, Wo = (W - k) / stride + 1;
    const int V = dtype == kBF16 ? 8 : 4;
    if ((size_t)B * Ho * Wo * (Cp / V) > 0x7fffffffu) return -1;
    const unsigned blocks = blocks_for((size_t)B * Ho * Wo * (Cp / V), 256);
    if (dtype == kBF16) launch_pool_fwd_t<bf16_t>(x, y, arg, B, H, W, Cp, k, stride, Ho, Wo, blocks, s);
    else launch_pool_fwd_t<float>(x, y, arg, B, H, W, Cp, k, stride, Ho, Wo, blocks, s);
    return launch_ok();
}

// Gather form: an input pixel sums, in (py, px) order, the gradients of the
// windows whose recorded maximum it is; then, if asked, the ReLU mask of the layer below.
// TWO: at most two windows per axis cover a pixel (k <= 2*stride); the four candidate windows are then
// fetched up front, with the out-of-range ones masked, instead of in a loop whose loads wait for each other.
template <typename T, bool TWO>
__global__ __launch_bounds__(256) void pool_bwd_kernel(const T *__restrict__ dy, const uint8_t *__restrict__ arg, const T *__restrict__ x, int relu,
                                                     T *__restrict__ dx, int B, int H, int W, int Cp, int k, int stride, int Ho, int Wo,
                                                     PoolIndex pi, FastDiv dstride)
{
    constexpr int V = Vec16<T>::N;
    const uint32_t i = xcd_block() * 256u + threadIdx.x;
    if (i >= (uint32_t)B * H * W * pi.cv) return;
    int cg, ix, iy, n;
    pool_decode(i, pi, cg, ix, iy, n);
    const int c0 = cg * V;
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
    int py0 = iy - k + 1; py0 = py0 <= 0 ? 0 : (int)fdiv32((uint32_t)(py0 + stride - 1), dstride);
    int px0 = ix - k + 1; px0 = px0 <= 0 ? 0 : (int)fdiv32((uint32_t)(px0 + stride - 1), dstride);
    const int py1 = min((int)fdiv32((uint32_t)iy, dstride), Ho - 1), px1 = min((int)fdiv32((uint32_t)ix, dstride), Wo - 1);
    auto add = [&](const Vec16<T> &g, uint64_t a8, int pos, bool ok) {
#pragma unroll
        for (int e = 0; e < V; ++e)
            if (ok && (int)((a8 >> (8 * e)) & 0xff) == pos) acc[e] += ldf(&g.e[e]);
    };
    if constexpr (TWO) {
        Vec16<T> g[4];
        uint64_t a8[4];
        int pos[4];
        bool ok[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {   // (py0, px0), (py0, px0+1), (py0+1, px0), (py0+1, px0+1)
            const int py = py0 + (q >> 1), px = px0 + (q & 1);
            ok[q] = py <= py1 && px <= px1;
            pos[q] = (iy - py * stride) * k + (ix - px * stride);
            const long off = (((long)n * Ho + py) * Wo + px) * Cp + c0;
            // windows that do not cover the pixel (more than half of the candidates for 3/2 pooling) are not fetched:
            // the kernel is bound by what it pulls out of L2, not by HBM
            g[q].u = make_uint4(0u, 0u, 0u, 0u);
            a8[q] = 0;
            if (ok[q]) {
                g[q].u = *reinterpret_cast<const uint4 *>(dy + off);
                if (V == 8) a8[q] = *reinterpret_cast<const uint64_t *>(arg + off);
                else a8[q] = *reinterpret_cast<const uint32_t *>(arg + off);
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) add(g[q], a8[q], pos[q], ok[q]);
    } else {
        for (int py = py0; py <= py1; ++py)
            for (int px = px0; px <= px1; ++px) {
                const long off = (((long)n * Ho + py) * Wo + px) * Cp + c0;
                Vec16<T> g;
                g.u = *reinterpret_cast<const uint4 *>(dy + off);
                uint64_t a8;   // the V recorded positions of this window, one byte each
                if (V == 8) a8 = *reinterpret_cast<const uint64_t *>(arg + off);
                else a8 = *reinterpret_cast<const uint32_t *>(arg + off);
                add(g, a8, (iy - py * stride) * k + (ix - px * stride), true);
            }
    }
    const long off = (((long)n * H + iy) * W + ix) * Cp + c0;
    Vec16<T> o;
    if (relu) {
        Vec16<T> xv;
        xv.u = *reinterpret_cast<const uint4 *>(x + off);
#pragma unroll
        for (int e = 0; e < V; ++e) stf(&o.e[e], ldf(&xv.e[e]) > 0.f ? acc[e] : 0.f);
    } else {
#pragma unroll
        for (int e = 0; e < V; ++e) stf(&o.e[e], acc[e]);
    }
    *reinterpret_cast<uint4 *>(dx + off) = o.u;
}

// Stride 2, windows of 2 or 3: a thread owns a 2 x 2 block of input pixels (rows 2*jy, 2*jy+1, columns 2*jx,
// 2*jx+1).  Exactly the four windows (jy-1 .. jy) x (jx-1 .. jx) can cover it: window (jy, jx) covers all four
// pixels, the two neighbours above / to the left cover the pixels of the block's first row / column (3 x 3
// only), the diagonal one its first pixel.  The four windows are fetched once for the four pixels (the
// pixel-per-thread form fetches 2.25 windows per pixel) and each recorded position is decoded once.  The sums
// run over the windows in the same order as in the general kernel, so the results are the same bit for bit.
// If bands is given, the block also leaves the column sums of what it stored (the gradient at the output of the
// convolution below, whose bias gradient they are part of) in bands[column][block]: the values as stored (rounded
// to the element type), added per thread over its pixels, then over the block's threads in thread order.
template <typename T, int K>
__global__ __launch_bounds__(256) void pool_bwd_s2_kernel(const T *__restrict__ dy, const uint8_t *__restrict__ arg, const T *__restrict__ x, int relu,
                                                        T *__restrict__ dx, int B, int H, int W, int Cp, int Ho, int Wo, PoolIndex pi,
                                                        float *__restrict__ bands)
{
    constexpr int V = Vec16<T>::N;
    __shared__ float part[256 * V];
    const uint32_t blk = xcd_block();
    const uint32_t i = blk * 256u + threadIdx.x;
    const bool live = i < (uint32_t)B * pi.h * pi.w * pi.cv;
    if (!live && bands == nullptr) return;
    int cg, jx, jy, n;
    pool_decode(live ? i : 0u, pi, cg, jx, jy, n);
    if (!live) { jy = -4; jx = -4; }   // no window, no pixel: contributes zeros to the band sums
    const int c0 = cg * V;
    Vec16<T> g[4];
    uint64_t a8[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {   // windows (jy-1, jx-1), (jy-1, jx), (jy, jx-1), (jy, jx)
        const int py = jy - 1 + (q >> 1), px = jx - 1 + (q & 1);
        g[q].u = make_uint4(0u, 0u, 0u, 0u);
        a8[q] = ~0ull;   // no position matches
        if (py >= 0 && py < Ho && px >= 0 && px < Wo) {
            const long off = (((long)n * Ho + py) * Wo + px) * Cp + c0;
            g[q].u = *reinterpret_cast<const uint4 *>(dy + off);
            if (V == 8) a8[q] = *reinterpret_cast<const uint64_t *>(arg + off);
            else a8[q] = *reinterpret_cast<const uint32_t *>(arg + off) | 0xffffffff00000000ull;
        }
    }
    float acc[4][V];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int e = 0; e < V; ++e) acc[b][e] = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const int pos = (int)((a8[q] >> (8 * e)) & 0xff);
            const float ge = ldf(&g[q].e[e]);
#pragma unroll
            for (int b = 0; b < 4; ++b) {   // pixel (by, bx) of the block sits at (by + 2*(1 - wy), bx + 2*(1 - wx)) in window q
                constexpr int dummy = 0; (void)dummy;
                const int wy = q >> 1, wx = q & 1, by = b >> 1, bx = b & 1;
                const int ry = by + 2 * (1 - wy), rx = bx + 2 * (1 - wx);
                if (ry < K && rx < K) acc[b][e] += pos == ry * K + rx ? ge : 0.f;
            }
        }
    }
    float colsum[V];
#pragma unroll
    for (int e = 0; e < V; ++e) colsum[e] = 0.f;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int iy = 2 * jy + (b >> 1), ix = 2 * jx + (b & 1);
        if (iy >= 0 && iy < H && ix >= 0 && ix < W) {
            const long off = (((long)n * H + iy) * W + ix) * Cp + c0;
            Vec16<T> o;
            if (relu) {
                Vec16<T> xv;
                xv.u = *reinterpret_cast<const uint4 *>(x + off);
#pragma unroll
                for (int e = 0; e < V; ++e) stf(&o.e[e], ldf(&xv.e[e]) > 0.f ? acc[b][e] : 0.f);
            } else {
#pragma unroll
                for (int e = 0; e < V; ++e) stf(&o.e[e], acc[b][e]);
            }
            *reinterpret_cast<uint4 *>(dx + off) = o.u;
#pragma unroll
            for (int e = 0; e < V; ++e) colsum[e] += ldf(&o.e[e]);
        }
    }
    if (bands == nullptr) return;
    // thread t of the block holds channel group (blk * 256 + t) % cv: column c adds the threads of its group in order
#pragma unroll
    for (int e = 0; e < V; ++e) part[threadIdx.x * V + e] = colsum[e];
    __syncthreads();
    const int cv = pi.cv;
    const int g0 = (int)((blk * 256u) % (uint32_t)cv);   // group of thread 0
    for (int c = threadIdx.x; c < Cp; c += 256) {
        const int gc = c / V, e = c - gc * V;
        float t = 0.f;
        for (int j = (gc - g0 + cv) % cv; j < 256; j += cv) t += part[j * V + e];
        bands[(long)c * gridDim.x + blk] = t;
    }
}

template <typename T>
static void launch_pool_bwd_t(const void *dy, const uint8_t *arg, const void *x, int relu, void *dx, int B, int H, int W, int Cp, int k, int stride,
                              int Ho, int Wo, unsigned blocks, float *bands, hipStream_t s)
{
    const T *d = static_cast<const T *>(dy), *xx = static_cast<const T *>(x); T *o = static_cast<T *>(dx);
    if (stride == 2 && (k == 2 || k == 3)) {
        const int Hb = (H + 1) / 2, Wb = (W + 1) / 2, cv = Cp / (16 / (int)sizeof(T));
        const PoolIndex pb = make_pool_index(cv, Wb, Hb);
        const unsigned nb = blocks_for((size_t)B * Hb * Wb * cv, 256);
        if (k == 3) hipLaunchKernelGGL((pool_bwd_s2_kernel<T, 3>), dim3(nb), dim3(256), 0, s, d, arg, xx, relu, o, B, H, W, Cp, Ho, Wo, pb, bands);
        else hipLaunchKernelGGL((pool_bwd_s2_kernel<T, 2>), dim3(nb), dim3(256), 0, s, d, arg, xx, relu, o, B, H, W, Cp, Ho, Wo, pb, bands);
        return;
    }
    const PoolIndex pi = make_pool_index(Cp / (16 / (int)sizeof(T)), W, H);
    const FastDiv ds = make_fastdiv((uint32_t)stride);
    if (k <= 2 * stride) hipLaunchKernelGGL((pool_bwd_kernel<T, true>), dim3(blocks), dim3(256), 0, s, d, arg, xx, relu, o, B, H, W, Cp, k, stride, Ho, Wo, pi, ds);
    else hipLaunchKernelGGL((pool_bwd_kernel<T, false>), dim3(blocks), dim3(256), 0, s, d, arg, xx, relu, o, B, H, W, Cp, k, stride, Ho, Wo, pi, ds);
}
// Number of column-sum bands the pooling backward pass can leave behind (0: this shape runs a kernel that cannot).
long pool_bwd_bands(int dtype, int B, int H, int W, int Cp, int k, int stride)
{
    if (!(stride == 2 && (k == 2 || k == 3))) return 0;
    const int V = dtype == kBF16 ? 8 : 4;
    return (long)blocks_for((size_t)B * ((H + 1) / 2) * ((W + 1) / 2) * (Cp / V), 256);
}
int launch_pool_bwd(int dtype, const void *dy, const uint8_t *arg, const void *x, int relu, void *dx, int B, int H, int W, int Cp, int k, int stride,
                    float *bands, hipStream_t s)
{
    const int Ho = (H - k) / stride + 1, Wo = (W - k) / stride + 1;
    const int V = dtype == kBF16 ? 8 : 4;
    if ((size_t)B * H * W * (Cp / V) > 0x7fffffffu) return -1;
    if (bands && pool_bwd_bands(dtype, B, H, W, Cp, k, stride) == 0) return -1;
    const unsigned blocks = blocks_for((size_t)B * H * W * (Cp / V), 256);
    if (dtype == kBF16) launch_pool_bwd_t<bf16_t>(dy, arg, x, relu, dx, B, H, W, Cp, k, stride, Ho, Wo, blocks, bands, s);
    else launch_pool_bwd_t<float>(dy, arg, x, relu, dx, B, H, W, Cp, k, stride, Ho, Wo, blocks, bands, s);
    return launch_ok();
}

// ---------------------------------------------------------------- local response normalisation (across channels)
// One thread owns V consecutive channels (16 bytes) of one pixel and reads the channels up to 8 to either side
// (padding channels hold zeros, channels outside the tensor count as zeros), so windows of up to 9 channels fit
// the forward pass and the backward pass, which needs the window sums of the neighbours' windows.
template <typename T> struct LrnWindow {
    static constexpr int V = 16 / sizeof(T), R = 8, N = V + 2 * R;
    float f[N];   // f[R + e] is channel c0 + e
    __device__ __forceinline__ void load(const T *pix, int c0, int Cp)
    {
#pragma unroll
        for (int q = -(R / V); q <= R / V; ++q) {
            const int c = c0 + q * V;
            Vec16<T> v;
            if (c >= 0 && c < Cp) v.u = *reinterpret_cast<const uint4 *>(pix + c);
            else v.u = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (int e = 0; e < V; ++e) f[R + q * V + e] = ldf(&v.e[e]);
        }
    }
};
// s^(-e) for s >= bias > 0, far from the denormal range on both sides: the bare hardware log2 and exp2 (about one
// ulp each) without the range fix-ups of the library routines
__device__ __forceinline__ float pow_neg(float s, float e) { return __builtin_amdgcn_exp2f(-e * __builtin_amdgcn_logf(s)); }

template <typename T, int half>   // half = size / 2, a compile-time constant so that the windows stay in registers
__global__ __launch_bounds__(256) void lrn_fwd_kernel(const T *__restrict__ a, T *__restrict__ y, size_t groups, int Cp, float alpha, float beta,
                                                    float bias)
{
    constexpr int V = LrnWindow<T>::V, R = LrnWindow<T>::R;
    const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= groups) return;
    const int cv = Cp / V;
    const size_t pix = g / cv;
    const int c0 = (int)(g - pix * cv) * V;
    LrnWindow<T> w;
    w.load(a + pix * Cp, c0, Cp);
    Vec16<T> o;
#pragma unroll
    for (int e = 0; e < V; ++e) {
        float sum = 0.f;
#pragma unroll
        for (int j = -half; j <= half; ++j) sum += w.f[R + e + j] * w.f[R + e + j];
        stf(&o.e[e], w.f[R + e] * pow_neg(bias + alpha * sum, beta));
    }
    *reinterpret_cast<uint4 *>(y + pix * Cp + c0) = o.u;
}

template <typename T, int half>
__global__ __launch_bounds__(256) void lrn_bwd_kernel(const T *__restrict__ a, const T *__restrict__ dy, int relu, T *__restrict__ da, size_t groups,
                                                    int Cp, float alpha, float beta, float bias)
{
    constexpr int V = LrnWindow<T>::V, R = LrnWindow<T>::R;
    const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= groups) return;
    const int cv = Cp / V;
    const size_t pix = g / cv;
    const int c0 = (int)(g - pix * cv) * V;
    LrnWindow<T> wa, wd;
    wa.load(a + pix * Cp, c0, Cp);
    wd.load(dy + pix * Cp, c0, Cp);
    // for every channel j within `half` of this thread's channels: s_j, and t_j = dy_j * a_j * s_j^(-beta-1)
    float t[V + 8], pown[V];   // pown: s^(-beta) of the thread's own channels
#pragma unroll
    for (int q = 0; q < V + 8; ++q) {
        const int j = q - 4;                    // channel c0 + j, j in [-4, V+3] covers half <= 4
        t[q] = 0.f;
        if (j >= -half && j < V + half) {       // decided at compile time
            float sum = 0.f;
#pragma unroll
            for (int r = -half; r <= half; ++r) sum += wa.f[R + j + r] * wa.f[R + j + r];
            const float sj = bias + alpha * sum;
            float pj1;                          // s^(-beta-1)
            if (j >= 0 && j < V) {              // own channel: s^(-beta) is needed too, one reciprocal gives the other
                pown[j] = pow_neg(sj, beta);
                pj1 = pown[j] * __builtin_amdgcn_rcpf(sj);
            } else {
                pj1 = pow_neg(sj, beta + 1.f);
            }
            t[q] = wd.f[R + j] * wa.f[R + j] * pj1;
        }
    }
    Vec16<T> o;
#pragma unroll
    for (int e = 0; e < V; ++e) {
        float acc = 0.f;
#pragma unroll
        for (int r = -half; r <= half; ++r) acc += t[e + 4 + r];
        float v = wd.f[R + e] * pown[e] - 2.f * alpha * beta * wa.f[R + e] * acc;
        if (relu && !(wa.f[R + e] > 0.f)) v = 0.f;
        stf(&o.e[e], v);
    }
    *reinterpret_cast<uint4 *>(da + pix * Cp + c0) = o.u;
}

template <typename T, int HALF>
static void launch_lrn_t(const void *a, const void *dy, int relu, void *out, size_t groups, int Cp, float alpha, float beta, float bias, bool bwd,
                         hipStream_t s)
{
    const unsigned blocks = blocks_for(groups, 256);
    if (bwd)
        hipLaunchKernelGGL((lrn_bwd_kernel<T, HALF>), dim3(blocks), dim3(256), 0, s, static_cast<const T *>(a), static_cast<const T *>(dy), relu,
                           static_cast<T *>(out), groups, Cp, alpha, beta, bias);
    else
        hipLaunchKernelGGL((lrn_fwd_kernel<T, HALF>), dim3(blocks), dim3(256), 0, s, static_cast<const T *>(a), static_cast<T *>(out), groups, Cp, alpha,
                           beta, bias);
}
template <typename T>
static int launch_lrn_any(const void *a, const void *dy, int relu, void *out, size_t pixels, int Cp, int size, float alpha, float beta, float bias,
                          bool bwd, hipStream_t s)
{
    if (size < 1 || size > 9 || !(size & 1) || !(bias > 0.f)) return -1;
    const size_t groups = pixels * (size_t)(Cp / (16 / (int)sizeof(T)));
    switch (size / 2) {
    case 0: launch_lrn_t<T, 0>(a, dy, relu, out, groups, Cp, alpha, beta, bias, bwd, s); break;
    case 1: launch_lrn_t<T, 1>(a, dy, relu, out, groups, Cp, alpha, beta, bias, bwd, s); break;
    case 2: launch_lrn_t<T, 2>(a, dy, relu, out, groups, Cp, alpha, beta, bias, bwd, s); break;
    case 3: launch_lrn_t<T, 3>(a, dy, relu, out, groups, Cp, alpha, beta, bias, bwd, s); break;
    default: launch_lrn_t<T, 4>(a, dy, relu, out, groups, Cp, alpha, beta, bias, bwd, s); break;
    }
    return launch_ok();
}
int launch_lrn_fwd(int dtype, const void *a, void *y, size_t pixels, int Cp, int size, float alpha, float beta, float bias, hipStream_t s)
{
    return dtype == kBF16 ? launch_lrn_any<bf16_t>(a, nullptr, 0, y, pixels, Cp, size, alpha, beta, bias, false, s)
                          : launch_lrn_any<float>(a, nullptr, 0, y, pixels, Cp, size, alpha, beta, bias, false, s);
}
int launch_lrn_bwd(int dtype, const void *a, const void *dy, int relu, void *da, size_t pixels, int Cp, int size, float alpha, float beta,
                   float bias, hipStream_t s)
{
    return dtype == kBF16 ? launch_lrn_any<bf16_t>(a, dy, relu, da, pixels, Cp, size, alpha, beta, bias, true, s)
                          : launch_lrn_any<float>(a, dy, relu, da, pixels, Cp, size, alpha, beta, bias, true, s);
}

// ---------------------------------------------------------------- flatten / unflatten
template <typename T>
__global__ __launch_bounds__(256) void flatten_kernel(const T *__restrict__ x, T *__restrict__ flat, int B, int H, int W, int C, int Cp)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;  // (b, c, h, w)
    if (i >= (long)B * C * H * W) return;
    const int w = (int)(i % W); long t = i / W;
    const int h = (int)(t % H); t /= H;
    const int c = (int)(t % C);
    const int b = (int)(t / C);
    flat[i] = x[(((long)b * H + h) * W + w) * Cp + c];
}
int launch_flatten(int dtype, const void *x, void *flat, int B, int H, int W, int C, int Cp, hipStream_t s)
{
    const unsigned blocks = blocks_for((size_t)B * C * H * W, 256);
    if (dtype == kBF16)
        hipLaunchKernelGGL(flatten_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, static_cast<const bf16_t *>(x), static_cast<bf16_t *>(flat), B, H, W, C, Cp);
    else
        hipLaunchKernelGGL(flatten_kernel<float>, dim3(blocks), dim3(256), 0, s, static_cast<const float *>(x), static_cast<float *>(flat), B, H, W, C, Cp);
    return launch_ok();
}

template <typename T>
__global__ __launch_bounds__(256) void unflatten_kernel(const T *__restrict__ dflat, const T *__restrict__ x, int relu, T *__restrict__ dx, int B, int H,
                                                      int W, int C, int Cp)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;  // (b, h, w, cp)
    if (i >= (long)B * H * W * Cp) return;
    const int c = (int)(i % Cp); long t = i / Cp;
    const int w = (int)(t % W); t /= W;
    const int h = (int)(t % H);
    const int b = (int)(t / H);
    float v = 0.f;
    if (c < C) {
        v = ldf(&dflat[(((long)b * C + c) * H + h) * W + w]);
        if (relu && !(ldf(&x[i]) > 0.f)) v = 0.f;
    }
    stf(&dx[i], v);
}
int launch_unflatten(int dtype, const void *dflat, const void *x, int relu, void *dx, int B, int H, int W, int C, int Cp, hipStream_t s)
{
    const unsigned blocks = blocks_for((size_t)B * H * W * Cp, 256);
    if (dtype == kBF16)
        hipLaunchKernelGGL(unflatten_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, static_cast<const bf16_t *>(dflat), static_cast<const bf16_t *>(x), relu,
                           static_cast<bf16_t *>(dx), B, H, W, C, Cp);
    else
        hipLaunchKernelGGL(unflatten_kernel<float>, dim3(blocks), dim3(256), 0, s, static_cast<const float *>(dflat), static_cast<const float *>(x), relu,
                           static_cast<float *>(dx), B, H, W, C, Cp);
    return launch_ok();
}

// ---------------------------------------------------------------- bias gradient (column sums)
// Stage 1: a block owns a band of rows and up to 256 column chunks of 16 bytes;
// thread (c, r) adds rows r, r+RL, ... of chunk c, the RL row lanes are then
// added in lane order.  Stage 2 adds the bands in order.  No atomics, so the
// result does not depend on scheduling.
// Stage 1 for several tensors in one launch: a block finds its job and its (column group, band) in it.
template <typename T>
__global__ __launch_bounds__(256) void colsum_stage1(ColsumS1Jobs jobs)
{
    constexpr int V = 16 / sizeof(T);
    __shared__ float part[256 * V];
    int q = 0;
    while (q + 1 < jobs.n && blockIdx.x >= jobs.j[q + 1].start_block) ++q;
    const ColsumS1Job &J = jobs.j[q];
    const unsigned lb = blockIdx.x - J.start_block, bx = lb % (unsigned)J.gx, by = lb / (unsigned)J.gx;
    const T *dy = static_cast<const T *>(J.dy);
    const long ld = J.ld, M = J.M, rows_per_block = J.rows_per_block;
    const int chunks = J.chunks, cpb = J.cpb, rl = J.rl;
    const int c = threadIdx.x % cpb, r = threadIdx.x / cpb;
    const int gc = (int)bx * cpb + c;
    const long m0 = (long)by * rows_per_block, m1 = min(M, m0 + rows_per_block);
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
    if (r < rl && gc < chunks) {
        for (long m = m0 + r; m < m1; m += rl) {
            union { uint4 u; T e[V]; } v;
            v.u = *reinterpret_cast<const uint4 *>(dy + m * ld + (long)gc * V);
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] += ldf(&v.e[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < V; ++e) part[threadIdx.x * V + e] = acc[e];
    __syncthreads();
    if (r == 0 && gc < chunks) {
#pragma unroll
        for (int e = 0; e < V; ++e) {
            float t = 0.f;
            for (int j = 0; j < rl; ++j) t += part[(j * cpb + c) * V + e];
            J.ws[(long)by * ld + (long)gc * V + e] = t;
        }
    }
}
// Stage 2 for several layers in one launch: a block owns 8 columns of one job.
__global__ __launch_bounds__(256) void colsum_stage2(ColsumJobs jobs)
{
    // Band-major jobs (ws[band][ld], from colsum_stage1): 8 columns per block, 32 lanes per column.  Column-major
    // jobs (ws[column][nblk], from the pooling backward pass, thousands of bands): 4 columns per block, one
    // wavefront per column reading consecutive bands.  A lane adds bands lane, lane + L, ... (eight loads in
    // flight), then the lanes are added in order.
    __shared__ float part[256];
    int q = 0;
    while (q + 1 < jobs.n && blockIdx.x >= jobs.j[q + 1].start_block) ++q;
    const ColsumJob &J = jobs.j[q];
    const float *ws = J.ws;
    const int nblk = J.nblk, N = J.N, cm = J.colmajor, cpb = cm ? 4 : 8, L = 256 / cpb;
    const int tx = cm ? threadIdx.x / L : threadIdx.x % cpb, ty = cm ? threadIdx.x % L : threadIdx.x / cpb;
    const int n = (int)(blockIdx.x - J.start_block) * cpb + tx;
    const long sb = cm ? 1 : J.ld, sn = cm ? nblk : 1;   // strides of the band and of the column index
    float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (n < N) {
        const float *col = ws + (long)n * sn;
        int b = ty;
        for (; b + 7 * L < nblk; b += 8 * L) {
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] += col[(long)(b + u * L) * sb];
        }
        for (; b < nblk; b += L) a[0] += col[(long)b * sb];
    }
    part[ty * cpb + tx] = ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
    __syncthreads();
    if (ty == 0 && n < N) {
        float t = 0.f;
        for (int j = 0; j < L; ++j) t += part[j * cpb + tx];
        J.db[n] = t;
    }
}
static void colsum_geometry(int dtype, long ld, long M, int &chunks, int &cpb, int &rl, long &rows_per_block, int &nblk)
{
    const int V = dtype == kBF16 ? 8 : 4;
    chunks = (int)(ld / V);
    cpb = chunks < 256 ? chunks : 256;
    rl = 256 / cpb;
    rows_per_block = (M + 511) / 512;
    if (rows_per_block < 4L * rl) rows_per_block = 4L * rl;
    rows_per_block = (rows_per_block + rl - 1) / rl * rl;
    nblk = (int)((M + rows_per_block - 1) / rows_per_block);
}
size_t colsum_ws_floats(int dtype, long M, long ld)
{
    int chunks, cpb, rl, nblk; long rpb;
    colsum_geometry(dtype, ld, M, chunks, cpb, rl, rpb, nblk);
    return (size_t)nblk * (size_t)ld;
}
// dy is [M][ld] with ld a multiple of 8 and columns N..ld-1 zero or ignorable.  Stage 1 leaves the band sums in
// ws (colsum_ws_floats) and appends the job that finishes them; launch_colsum_finish runs all appended jobs.
int colsum_partial_defer(int dtype, const void *dy, long ld, long M, int N, float *db, float *ws, ColsumS1Jobs &s1, ColsumJobs &jobs)
{
    if (jobs.n >= 12 || s1.n >= 12 || (ld & 7) || M <= 0) return -1;
    int chunks, cpb, rl, nblk; long rpb;
    colsum_geometry(dtype, ld, M, chunks, cpb, rl, rpb, nblk);
    ColsumS1Job &S = s1.j[s1.n++];
    S.dy = dy; S.ws = ws; S.ld = ld; S.M = M; S.rows_per_block = rpb; S.chunks = chunks; S.cpb = cpb; S.rl = rl;
    S.gx = (chunks + cpb - 1) / cpb; S.gy = nblk; S.start_block = 0;
    ColsumJob &J = jobs.j[jobs.n++];
    J.ws = ws; J.nblk = nblk; J.ld = ld; J.N = N; J.db = db; J.start_block = 0; J.colmajor = 0;
    return 0;
}
int launch_colsum_stage1(int dtype, ColsumS1Jobs &s1, hipStream_t s)
{
    if (s1.n == 0) return 0;
    unsigned long blocks = 0;
    for (int q = 0; q < s1.n; ++q) { s1.j[q].start_block = (unsigned)blocks; blocks += (unsigned long)s1.j[q].gx * (unsigned long)s1.j[q].gy; }
    if (blocks > 0x7fffffffu) return -1;
    if (dtype == kBF16) hipLaunchKernelGGL(colsum_stage1<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, s, s1);
    else hipLaunchKernelGGL(colsum_stage1<float>, dim3((unsigned)blocks), dim3(256), 0, s, s1);
    s1.n = 0;
    return launch_ok();
}
int launch_colsum_partial(int dtype, const void *dy, long ld, long M, int N, float *db, float *ws, ColsumJobs &jobs, hipStream_t s)
{
    ColsumS1Jobs s1; s1.n = 0;
    if (colsum_partial_defer(dtype, dy, ld, M, N, db, ws, s1, jobs) != 0) return -1;
    return launch_colsum_stage1(dtype, s1, s);
}
int launch_colsum_finish(ColsumJobs &jobs, hipStream_t s)
{
    if (jobs.n == 0) return 0;
    unsigned blocks = 0;
    for (int q = 0; q < jobs.n; ++q) {
        ColsumJob &J = jobs.j[q];
        const int cpb = J.colmajor ? 4 : 8;
        J.start_block = blocks;
        blocks += (unsigned)((J.N + cpb - 1) / cpb);
    }
    hipLaunchKernelGGL(colsum_stage2, dim3(blocks), dim3(256), 0, s, jobs);
    jobs.n = 0;
    return launch_ok();
}

// ---------------------------------------------------------------- softmax cross-entropy
// One workgroup per row: lse = max + log(sum exp(z - max)); the row's loss is
// lse - z[label]; dz = (exp(z - lse) - [c == label]) / B.
__device__ inline float wave_max(float v)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline float wave_sum(float v)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
// One workgroup per row: the four wavefronts each reduce their part, the four results meet in LDS.
__device__ inline float block_max(float v, float *sh)
{
    v = wave_max(v);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    v = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
    __syncthreads();
    return v;
}
__device__ inline float block_sum(float v, float *sh)
{
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    v = (sh[0] + sh[1]) + (sh[2] + sh[3]);
    __syncthreads();
    return v;
}
template <typename T>
__global__ __launch_bounds__(256) void softmax_ce_kernel(const float *__restrict__ z, long ld, const int32_t *__restrict__ labels, int B, int C,
                                                       T *__restrict__ dz, float *__restrict__ row_loss)
{
    __shared__ float sh[4];
    const int row = blockIdx.x, t = threadIdx.x;
    const float *zr = z + (long)row * ld;
    // the first four strides of the row stay in registers (all of it up to 1024 classes)
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = t + u * 256 < C ? zr[t + u * 256] : -INFINITY;
    float m = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
    for (int c = t + 1024; c < C; c += 256) m = fmaxf(m, zr[c]);
    m = block_max(m, sh);
    float sum = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) sum += t + u * 256 < C ? expf(v[u] - m) : 0.f;
    for (int c = t + 1024; c < C; c += 256) sum += expf(zr[c] - m);
    sum = block_sum(sum, sh);
    const float lse = m + logf(sum);
    const int label = labels[row];
    // a label outside [0, C) addresses nothing: the row's loss (and with it the mean) becomes NaN, and dz is
    // the plain softmax / B, since no class compares equal to it below
    const bool label_ok = (unsigned)label < (unsigned)C;
    if (t == 0) row_loss[row] = label_ok ? lse - zr[label] : __builtin_nanf("");
    const float inv_b = 1.f / (float)B;
    T *dr = dz + (long)row * ld;
    for (int c = t; c < (int)ld; c += 256) {
        float g = 0.f;
        if (c < C) {
            g = (expf(zr[c] - lse) - (c == label ? 1.f : 0.f)) * inv_b;
        }
        stf(&dr[c], g);
    }
}
__global__ __launch_bounds__(256) void loss_reduce_kernel(const float *__restrict__ row_loss, int B, float *__restrict__ loss)
{
    __shared__ float part[256];
    float acc = 0.f;
    for (int i = threadIdx.x; i < B; i += 256) acc += row_loss[i];
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[0] = part[0] / (float)B;
}
int launch_softmax_ce(int dtype, const float *z, long ld, const int32_t *labels, int B, int C, void *dz, float *loss, float *row_loss, hipStream_t s)
{
    const unsigned blocks = (unsigned)B;
    if (dtype == kBF16) hipLaunchKernelGGL(softmax_ce_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, z, ld, labels, B, C, static_cast<bf16_t *>(dz), row_loss);
    else hipLaunchKernelGGL(softmax_ce_kernel<float>, dim3(blocks), dim3(256), 0, s, z, ld, labels, B, C, static_cast<float *>(dz), row_loss);
    hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(256), 0, s, row_loss, B, loss);
    return launch_ok();
}

// ---------------------------------------------------------------- debug exports
template <typename T>
__global__ __launch_bounds__(256) void export_nhwc_kernel(const T *__restrict__ x, float *__restrict__ dst, int B, int H, int W, int C, int Cp)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;  // (b, c, h, w)
    if (i >= (long)B * C * H * W) return;
    const int w = (int)(i % W); long t = i / W;
    const int h = (int)(t % H); t /= H;
    const int c = (int)(t % C);
    const int b = (int)(t / C);
    dst[i] = ldf(&x[(((long)b * H + h) * W + w) * Cp + c]);
}
int launch_export_nhwc(int dtype, const void *x, float *dst, int B, int H, int W, int C, int Cp, hipStream_t s)
{
    const unsigned blocks = blocks_for((size_t)B * C * H * W, 256);
    if (dtype == kBF16) hipLaunchKernelGGL(export_nhwc_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, static_cast<const bf16_t *>(x), dst, B, H, W, C, Cp);
    else hipLaunchKernelGGL(export_nhwc_kernel<float>, dim3(blocks), dim3(256), 0, s, static_cast<const float *>(x), dst, B, H, W, C, Cp);
    return launch_ok();
}
template <typename T> __global__ __launch_bounds__(256) void export_rows_kernel(const T *__restrict__ x, long ld, float *__restrict__ dst, int B, int F)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= (long)B * F) return;
    const long b = i / F, f = i - b * F;
    dst[i] = ldf(&x[b * ld + f]);
}
int launch_export_rows(int dtype, int src_f32, const void *x, long ld, float *dst, int B, int F, hipStream_t s)
{
    const unsigned blocks = blocks_for((size_t)B * F, 256);
    if (dtype == kBF16 && !src_f32) hipLaunchKernelGGL(export_rows_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, static_cast<const bf16_t *>(x), ld, dst, B, F);
    else hipLaunchKernelGGL(export_rows_kernel<float>, dim3(blocks), dim3(256), 0, s, static_cast<const float *>(x), ld, dst, B, F);
    return launch_ok();
}
__global__ __launch_bounds__(256) void export_argmax_kernel(const uint8_t *__restrict__ arg, uint8_t *__restrict__ dst, int B, int H, int W, int C, int Cp)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;  // (b, c, h, w)
    if (i >= (long)B * C * H * W) return;
    const int w = (int)(i % W); long t = i / W;
    const int h = (int)(t % H); t /= H;
    const int c = (int)(t % C);
    const int b = (int)(t / C);
    dst[i] = arg[(((long)b * H + h) * W + w) * Cp + c];
}
int launch_export_argmax(const uint8_t *arg, uint8_t *dst, int B, int H, int W, int C, int Cp, hipStream_t s)
{
    hipLaunchKernelGGL(export_argmax_kernel, dim3(blocks_for((size_t)B * C * H * W, 256)), dim3(256), 0, s, arg, dst, B, H, W, C, Cp);
    return launch_ok();
}
__global__ __launch_bounds__(256) void dropout_mask_kernel(uint8_t *dst, size_t count, uint64_t key, uint32_t thr)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    const uint32_t u = (uint32_t)(mix64(key + 0x9E3779B97F4A7C15ull * (uint64_t)(i + 1)) >> 32);
    dst[i] = u >= thr ? 1 : 0;
}
int launch_dropout_mask(uint8_t *dst, size_t count, uint64_t key, uint32_t thr, hipStream_t s)
{
    hipLaunchKernelGGL(dropout_mask_kernel, dim3(blocks_for(count, 256)), dim3(256), 0, s, dst, count, key, thr);
    return launch_ok();
}

}  // namespace asgd
