// MFMA GEMM engine for gfx950: one kernel template serves the convolutions
// (forward, data gradient, filter gradient, all as implicit GEMMs) and the fully
// connected layers.  C[M][N] = sum_k A[m][k] * B[n][k], fp32 accumulation.
//
// Geometry (identical in bytes for both element types): a workgroup of 256
// threads (4 wave64) owns a 128x128 tile of C; one K tile is 128 bytes per row
// (64 bf16 or 32 fp32).  Both operand tiles sit in LDS with K contiguous, as
// 128 rows x 8 slots of 16 bytes, the slot index XOR-swizzled with the row so
// that the 16-byte reads of the MFMA fragments, the direct stores and the
// transposed stores are all spread over the banks.  Operands whose memory
// layout has the reduction index strided (filter gradients, FC data gradient)
// are transposed in registers between the global load and the LDS store.
// Each wave computes 64x64 as 2x2 MFMA 32x32 blocks; the MFMA is issued with the
// B-matrix fragment as its first operand so that a lane ends up with four
// consecutive n for one m and can store them as one vector.
#include <hip/hip_runtime.h>

#include "asgd_internal.h"

namespace asgd {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16_t;

template <typename T> struct Geo;
template <> struct Geo<bf16_t> { enum { CH = 8, BK = 64, KSTEPS = 4 }; };
template <> struct Geo<float> { enum { CH = 4, BK = 32, KSTEPS = 2 }; };

constexpr int BM = 128, BN = 128, NT = 256;

FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.d = d;
    uint32_t sh = 0;
    while ((1ull << sh) < d) ++sh;
    f.sh = sh;
    f.mul = (uint32_t)((((1ull << 32) * ((1ull << sh) - d)) / d) + 1);
    if (d == 1) { f.mul = 0; f.sh = 0; }
    return f;
}

__device__ inline uint32_t fdiv(uint32_t n, const FastDiv &f) { return (__umulhi(n, f.mul) + n) >> f.sh; }
__device__ inline uint4 ld16(const void *p) { return *reinterpret_cast<const uint4 *>(p); }
__device__ inline uint4 zero16() { return make_uint4(0u, 0u, 0u, 0u); }
__device__ inline int swz(int row) { return (row ^ (row >> 3)) & 7; }

__device__ inline float to_f32(float v) { return v; }
__device__ inline float to_f32(bf16_t v) { return (float)v; }

// ------------------------------------------------------------------ loaders
// Direct loaders hand out 16-byte pieces of a row that are contiguous in K.
template <typename T> struct PlainK {
    static constexpr bool kTrans = false;
    const T *base; long ld; int rows; int K;
    struct Row { const T *p; };
    struct KPos { int k; };
    __device__ Row row(int r) const { return Row{r < rows ? base + (long)r * ld : nullptr}; }
    __device__ KPos kpos(int k) const { return KPos{k}; }
    __device__ void advance(KPos &kp, int dk) const { kp.k += dk; }
    __device__ uint4 load(const Row &r, const KPos &kp) const
    {
        return (r.p != nullptr && kp.k < K) ? ld16(r.p + kp.k) : zero16();
    }
};

template <typename T> struct GatherK {
    static constexpr bool kTrans = false;
    const T *x; int H, W, C, Ho, Wo, kh, kw, sm, ds, pad, M;
    FastDiv dWo, dHoWo, dC, dkw;
    struct Row { int pix0, y0, x0; };  // pix0 < 0: row out of range
    struct KPos { int ky, kx, c; };
    __device__ Row row(int m) const
    {
        if (m >= M) return Row{-1, 0, 0};
        const int n = (int)fdiv((uint32_t)m, dHoWo);
        const int rem = m - n * (Ho * Wo);
        const int oy = (int)fdiv((uint32_t)rem, dWo);
        const int ox = rem - oy * Wo;
        return Row{n * H * W, oy * sm - pad, ox * sm - pad};
    }
    __device__ KPos kpos(int k) const
    {
        const int t = (int)fdiv((uint32_t)k, dC);
        const int ky = (int)fdiv((uint32_t)t, dkw);
        return KPos{ky, t - ky * kw, k - t * C};
    }
    __device__ void advance(KPos &kp, int dk) const
    {
        kp.c += dk;
        while (kp.c >= C) {
            kp.c -= C;
            if (++kp.kx == kw) { kp.kx = 0; ++kp.ky; }
        }
    }
    __device__ uint4 load(const Row &r, const KPos &kp) const
    {
        if (r.pix0 < 0 || kp.ky >= kh) return zero16();
        int y = r.y0 + kp.ky, xx = r.x0 + kp.kx;
        if (y < 0 || xx < 0) return zero16();
        if (ds > 1) {
            if ((y % ds) != 0 || (xx % ds) != 0) return zero16();
            y /= ds; xx /= ds;
        }
        if (y >= H || xx >= W) return zero16();
        return ld16(x + ((long)(r.pix0 + y * W + xx) * C + kp.c));
    }
};

// Transposing loaders: memory has the GEMM row index contiguous and the
// reduction index strided.  A unit is CH consecutive rows x CH consecutive
// reduction indices, fetched as CH 16-byte loads.
template <typename T> struct PlainT {
    static constexpr bool kTrans = true;
    static constexpr int CH = Geo<T>::CH;
    const T *base; long ld; int rows; int K;
    struct Unit { int row0; };
    __device__ Unit unit(int row0) const { return Unit{row0}; }
    __device__ void load(const Unit &u, int k, uint4 (&out)[CH]) const
    {
#pragma unroll
        for (int j = 0; j < CH; ++j)
            out[j] = (u.row0 < rows && k + j < K) ? ld16(base + (long)(k + j) * ld + u.row0) : zero16();
    }
};

template <typename T> struct GatherT {
    static constexpr bool kTrans = true;
    static constexpr int CH = Geo<T>::CH;
    const T *x; int H, W, C, Ho, Wo, kh, kw, sm, pad, M, Krows;
    FastDiv dWo, dHoWo, dC, dkw;
    struct Unit { int ky, kx, c; };  // ky < 0: rows out of range
    __device__ Unit unit(int row0) const
    {
        if (row0 >= Krows) return Unit{-1, 0, 0};
        const int t = (int)fdiv((uint32_t)row0, dC);
        const int ky = (int)fdiv((uint32_t)t, dkw);
        return Unit{ky, t - ky * kw, row0 - t * C};
    }
    __device__ void load(const Unit &u, int m0, uint4 (&out)[CH]) const
    {
        int n = 0, oy = 0, ox = 0;
        if (m0 < M) {
            n = (int)fdiv((uint32_t)m0, dHoWo);
            const int rem = m0 - n * (Ho * Wo);
            oy = (int)fdiv((uint32_t)rem, dWo);
            ox = rem - oy * Wo;
        }
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            uint4 v = zero16();
            if (u.ky >= 0 && m0 + j < M) {
                const int y = oy * sm + u.ky - pad, xx = ox * sm + u.kx - pad;
                if (y >= 0 && y < H && xx >= 0 && xx < W) v = ld16(x + ((long)((n * H + y) * W + xx) * C + u.c));
            }
            out[j] = v;
            if (++ox == Wo) { ox = 0; if (++oy == Ho) { oy = 0; ++n; } }
        }
    }
};

// ------------------------------------------------------------------ staging
template <typename T, class L, bool kTrans = L::kTrans> struct Stage;

template <typename T, class L> struct Stage<T, L, false> {
    static constexpr int SLOTS = BM * 8 / NT;
    typename L::Row rows[SLOTS];
    typename L::KPos kp;
    uint4 r[SLOTS];
    __device__ void init(const L &l, int row0, int k0, int tid, int)
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) rows[s] = l.row(row0 + (tid >> 3) + s * (NT / 8));
        kp = l.kpos(k0 + (tid & 7) * Geo<T>::CH);
    }
    __device__ void load(const L &l)
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) r[s] = l.load(rows[s], kp);
    }
    __device__ void next(const L &l) { l.advance(kp, Geo<T>::BK); }
    __device__ void store(uint4 *sm, int tid) const
    {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const int row = (tid >> 3) + s * (NT / 8);
            sm[row * 8 + ((tid & 7) ^ swz(row))] = r[s];
        }
    }
};

__device__ inline void transpose_unit(const uint4 (&r)[4], uint4 (&o)[4])  // fp32: 4 k x 4 rows
{
    o[0] = make_uint4(r[0].x, r[1].x, r[2].x, r[3].x);
    o[1] = make_uint4(r[0].y, r[1].y, r[2].y, r[3].y);
    o[2] = make_uint4(r[0].z, r[1].z, r[2].z, r[3].z);
    o[3] = make_uint4(r[0].w, r[1].w, r[2].w, r[3].w);
}

__device__ inline uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ inline uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

__device__ inline void transpose_unit(const uint4 (&r)[8], uint4 (&o)[8])  // bf16: 8 k x 8 rows
{
    o[0] = make_uint4(pack_lo(r[0].x, r[1].x), pack_lo(r[2].x, r[3].x), pack_lo(r[4].x, r[5].x), pack_lo(r[6].x, r[7].x));
    o[1] = make_uint4(pack_hi(r[0].x, r[1].x), pack_hi(r[2].x, r[3].x), pack_hi(r[4].x, r[5].x), pack_hi(r[6].x, r[7].x));
    o[2] = make_uint4(pack_lo(r[0].y, r[1].y), pack_lo(r[2].y, r[3].y), pack_lo(r[4].y, r[5].y), pack_lo(r[6].y, r[7].y));
    o[3] = make_uint4(pack_hi(r[0].y, r[1].y), pack_hi(r[2].y, r[3].y), pack_hi(r[4].y, r[5].y), pack_hi(r[6].y, r[7].y));
    o[4] = make_uint4(pack_lo(r[0].z, r[1].z), pack_lo(r[2].z, r[3].z), pack_lo(r[4].z, r[5].z), pack_lo(r[6].z, r[7].z));
    o[5] = make_uint4(pack_hi(r[0].z, r[1].z), pack_hi(r[2].z, r[3].z), pack_hi(r[4].z, r[5].z), pack_hi(r[6].z, r[7].z));
    o[6] = make_uint4(pack_lo(r[0].w, r[1].w), pack_lo(r[2].w, r[3].w), pack_lo(r[4].w, r[5].w), pack_lo(r[6].w, r[7].w));
    o[7] = make_uint4(pack_hi(r[0].w, r[1].w), pack_hi(r[2].w, r[3].w), pack_hi(r[4].w, r[5].w), pack_hi(r[6].w, r[7].w));
}

template <typename T, class L> struct Stage<T, L, true> {
    static constexpr int CH = Geo<T>::CH;
    static constexpr int RCH = BM / CH;              // row chunks per tile
    static constexpr int NUNITS = RCH * 8;           // x 8 slots along K
    typename L::Unit un;
    int rowchunk, kq, k;
    bool active;
    uint4 r[CH];
    __device__ void init(const L &l, int row0, int k0, int tid, int shift)
    {
        const int vt = (tid + shift) & (NT - 1);     // spreads the two operands over different waves
        active = vt < NUNITS;
        rowchunk = vt % RCH;
        kq = vt / RCH;
        un = l.unit(row0 + rowchunk * CH);
        k = k0 + kq * CH;
    }
    __device__ void load(const L &l)
    {
        if (active) l.load(un, k, r);
    }
    __device__ void next(const L &) { k += Geo<T>::BK; }
    __device__ void store(uint4 *sm, int) const
    {
        if (!active) return;
        uint4 o[CH];
        transpose_unit(r, o);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int row = rowchunk * CH + i;
            sm[row * 8 + (kq ^ swz(row))] = o[i];
        }
    }
};

// ------------------------------------------------------------------ MFMA step
template <typename T> struct Frag;
template <> struct Frag<bf16_t> {
    uint4 v;
    __device__ void read(const uint4 *sm, int row, int ks, int half) { v = sm[row * 8 + ((ks * 2 + half) ^ swz(row))]; }
};
template <> struct Frag<float> {
    uint4 v[2];
    __device__ void read(const uint4 *sm, int row, int ks, int half)
    {
        const int q = ks * 4 + half * 2, z = swz(row);
        v[0] = sm[row * 8 + (q ^ z)];
        v[1] = sm[row * 8 + ((q + 1) ^ z)];
    }
};

__device__ inline void mma(f32x16 &acc, const Frag<bf16_t> &first, const Frag<bf16_t> &second)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, first.v), __builtin_bit_cast(bf16x8, second.v),
                                                  acc, 0, 0, 0);
}
__device__ inline void mma(f32x16 &acc, const Frag<float> &first, const Frag<float> &second)
{
    const uint32_t a[8] = {first.v[0].x, first.v[0].y, first.v[0].z, first.v[0].w, first.v[1].x, first.v[1].y, first.v[1].z, first.v[1].w};
    const uint32_t b[8] = {second.v[0].x, second.v[0].y, second.v[0].z, second.v[0].w, second.v[1].x, second.v[1].y, second.v[1].z, second.v[1].w};
#pragma unroll
    for (int e = 0; e < 8; ++e)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[e]), __uint_as_float(b[e]), acc, 0, 0, 0);
}

// ------------------------------------------------------------------ epilogue
__device__ inline uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

template <typename T> __device__ inline void store4(T *p, const float (&v)[4]);
template <> __device__ inline void store4<float>(float *p, const float (&v)[4])
{
    if ((reinterpret_cast<uintptr_t>(p) & 15) == 0) *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    else { p[0] = v[0]; p[1] = v[1]; p[2] = v[2]; p[3] = v[3]; }
}
template <> __device__ inline void store4<bf16_t>(bf16_t *p, const float (&v)[4])
{
    union { bf16_t h[4]; uint2 u; } t;
    t.h[0] = (bf16_t)v[0]; t.h[1] = (bf16_t)v[1]; t.h[2] = (bf16_t)v[2]; t.h[3] = (bf16_t)v[3];
    if ((reinterpret_cast<uintptr_t>(p) & 7) == 0) *reinterpret_cast<uint2 *>(p) = t.u;
    else { p[0] = t.h[0]; p[1] = t.h[1]; p[2] = t.h[2]; p[3] = t.h[3]; }
}

// Four consecutive columns n0..n0+3 of row m (n0 a multiple of 4, all in range).
template <typename T> __device__ inline void epilogue4(const Epilogue &ep, int m, int n0, float (&v)[4])
{
    if (ep.mode == 1) {  // conv filter gradient: (cout, (ky,kx,ci_padded)) -> canonical [cout][cin][kh][kw]
        if (m >= ep.cw_cout) return;
        const int t = n0 / ep.cw_cinp, ci0 = n0 - t * ep.cw_cinp;
        const int ky = t / ep.cw_kw, kx = t - ky * ep.cw_kw;
        float *o = static_cast<float *>(ep.out);
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (ci0 + r < ep.cw_cin) o[(((long)m * ep.cw_cin + ci0 + r) * ep.cw_kh + ky) * ep.cw_kw + kx] = v[r];
        return;
    }
    if (ep.bias) {
        const T *b = static_cast<const T *>(ep.bias);
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (n0 + r < ep.bias_n) v[r] += to_f32(b[n0 + r]);
    }
    if (ep.relu) {
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = v[r] > 0.f ? v[r] : 0.f;
    }
    if (ep.drop) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint64_t idx = (uint64_t)m * (uint64_t)ep.drop_F + (uint64_t)(n0 + r);
            const uint32_t u = (uint32_t)(mix64(ep.drop_key + 0x9E3779B97F4A7C15ull * (idx + 1)) >> 32);
            v[r] = (u >= ep.drop_thr) ? v[r] * ep.drop_scale : 0.f;
        }
    }
    if (ep.mask_src) {
        const T *ms = static_cast<const T *>(ep.mask_src) + (long)m * ep.mask_ld + n0;
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = to_f32(ms[r]) > 0.f ? v[r] * ep.mask_scale : 0.f;
    }
    if (ep.out_f32) store4<float>(static_cast<float *>(ep.out) + (long)m * ep.ld + n0, v);
    else store4<T>(static_cast<T *>(ep.out) + (long)m * ep.ld + n0, v);
}

// ------------------------------------------------------------------ kernel
template <typename T, class LA, class LB>
__global__ __launch_bounds__(NT) void gemm_kernel(LA la, LB lb, Epilogue ep, int M, int N, int nkt, int kt_per_split,
                                                  int tiles_m, int tiles_n, float *ws)
{
    constexpr int BK = Geo<T>::BK;
    __shared__ uint4 sA[BM * 8];
    __shared__ uint4 sB[BN * 8];
    const int tid = threadIdx.x;
    int bid = blockIdx.x;
    const int tn = bid % tiles_n; bid /= tiles_n;
    const int tm = bid % tiles_m;
    const int split = bid / tiles_m;
    const int kt0 = split * kt_per_split;
    const int kt1 = min(nkt, kt0 + kt_per_split);

    Stage<T, LA> stA;
    Stage<T, LB> stB;
    stA.init(la, tm * BM, kt0 * BK, tid, 0);
    stB.init(lb, tn * BN, kt0 * BK, tid, NT / 2);

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave & 1) * 64, wn = (wave >> 1) * 64;
    const int lrow = lane & 31, half = lane >> 5;

    if (kt0 < kt1) { stA.load(la); stB.load(lb); }
    for (int kt = kt0; kt < kt1; ++kt) {
        stA.store(sA, tid);
        stB.store(sB, tid);
        __syncthreads();
        if (kt + 1 < kt1) {
            stA.next(la); stB.next(lb);
            stA.load(la); stB.load(lb);
        }
#pragma unroll
        for (int ks = 0; ks < Geo<T>::KSTEPS; ++ks) {
            Frag<T> fa[2], fb[2];
            fa[0].read(sA, wm + lrow, ks, half);
            fa[1].read(sA, wm + 32 + lrow, ks, half);
            fb[0].read(sB, wn + lrow, ks, half);
            fb[1].read(sB, wn + 32 + lrow, ks, half);
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) mma(acc[nb][mb], fb[nb], fa[mb]);
        }
        __syncthreads();
    }

    // acc[nb][mb][v]: m = wm + mb*32 + lrow, n = wn + nb*32 + 8*(v/4) + 4*half + v%4
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
        const int m = tm * BM + wm + mb * 32 + lrow;
        if (m >= M) continue;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n0 = tn * BN + wn + nb * 32 + 8 * g + 4 * half;
                if (n0 >= N) continue;
                float v[4] = {acc[nb][mb][4 * g], acc[nb][mb][4 * g + 1], acc[nb][mb][4 * g + 2], acc[nb][mb][4 * g + 3]};
                if (ws) store4<float>(ws + ((long)split * M + m) * N + n0, v);
                else epilogue4<T>(ep, m, n0, v);
            }
    }
}

template <typename T> __global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *ws, int splits, Epilogue ep, int M, int N)
{
    const long g = (long)blockIdx.x * 256 + threadIdx.x;
    const int n4 = N / 4;
    if (g >= (long)M * n4) return;
    const int m = (int)(g / n4), n0 = (int)(g - (long)m * n4) * 4;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < splits; ++s) {
        const float4 p = *reinterpret_cast<const float4 *>(ws + ((long)s * M + m) * N + n0);
        v[0] += p.x; v[1] += p.y; v[2] += p.z; v[3] += p.w;
    }
    epilogue4<T>(ep, m, n0, v);
}

// ------------------------------------------------------------------ host side
GemmPlan plan_gemm(long M, long N, long K, int dtype, int max_splits)
{
    const int BK = dtype == kBF16 ? (int)Geo<bf16_t>::BK : (int)Geo<float>::BK;
    const long tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    const long nkt = (K + BK - 1) / BK;
    long splits = 1;
    if (max_splits > 1 && tiles < 512) {
        splits = (512 + tiles - 1) / tiles;
        if (splits > nkt / 4) splits = nkt / 4;   // at least four K tiles per split
        if (splits > max_splits) splits = max_splits;
        if (splits < 1) splits = 1;
    }
    if (splits > 1) {  // no empty split
        const long per = (nkt + splits - 1) / splits;
        splits = (nkt + per - 1) / per;
    }
    GemmPlan p;
    p.splits = (int)splits;
    p.ws_floats = splits > 1 ? (size_t)splits * (size_t)M * (size_t)N : 0;
    return p;
}

template <typename T, class LA, class LB>
static int run(const LA &la, const LB &lb, int M, int N, int K, const Epilogue &ep, const GemmPlan &plan, float *ws, hipStream_t s)
{
    if (M <= 0 || N <= 0 || K <= 0 || (N & 3)) return -1;
    constexpr int BK = Geo<T>::BK;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int nkt = (K + BK - 1) / BK;
    int splits = plan.splits;
    if (splits > 1 && ws == nullptr) return -1;
    const int per = (nkt + splits - 1) / splits;
    splits = (nkt + per - 1) / per;
    const long blocks = (long)tiles_m * tiles_n * splits;
    if (blocks > 0x7fffffffL) return -1;
    hipLaunchKernelGGL((gemm_kernel<T, LA, LB>), dim3((unsigned)blocks), dim3(NT), 0, s, la, lb, ep, M, N, nkt, per, tiles_m,
                       tiles_n, splits > 1 ? ws : nullptr);
    if (splits > 1) {
        const long groups = (long)M * (N / 4);
        hipLaunchKernelGGL((splitk_reduce_kernel<T>), dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, s, ws, splits, ep, M, N);
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <typename T> static GatherK<T> make_gather_k(const Gather &g)
{
    GatherK<T> l;
    l.x = static_cast<const T *>(g.x);
    l.H = g.H; l.W = g.W; l.C = g.C; l.Ho = g.Ho; l.Wo = g.Wo; l.kh = g.kh; l.kw = g.kw;
    l.sm = g.sm; l.ds = g.ds; l.pad = g.pad; l.M = g.N * g.Ho * g.Wo;
    l.dWo = make_fastdiv(g.Wo); l.dHoWo = make_fastdiv(g.Ho * g.Wo); l.dC = make_fastdiv(g.C); l.dkw = make_fastdiv(g.kw);
    return l;
}
template <typename T> static GatherT<T> make_gather_t(const Gather &g)
{
    GatherT<T> l;
    l.x = static_cast<const T *>(g.x);
    l.H = g.H; l.W = g.W; l.C = g.C; l.Ho = g.Ho; l.Wo = g.Wo; l.kh = g.kh; l.kw = g.kw;
    l.sm = g.sm; l.pad = g.pad; l.M = g.N * g.Ho * g.Wo; l.Krows = g.kh * g.kw * g.C;
    l.dWo = make_fastdiv(g.Wo); l.dHoWo = make_fastdiv(g.Ho * g.Wo); l.dC = make_fastdiv(g.C); l.dkw = make_fastdiv(g.kw);
    return l;
}
template <typename T> static PlainK<T> make_plain_k(const void *p, long ld, int rows, int K)
{
    return PlainK<T>{static_cast<const T *>(p), ld, rows, K};
}
template <typename T> static PlainT<T> make_plain_t(const void *p, long ld, int rows, int K)
{
    return PlainT<T>{static_cast<const T *>(p), ld, rows, K};
}

template <typename T>
static int gather_plain_t(const Gather &a, const void *b, long ldb, int N, const Epilogue &ep, const GemmPlan &plan, float *ws, hipStream_t s)
{
    const int K = a.kh * a.kw * a.C;
    return run<T>(make_gather_k<T>(a), make_plain_k<T>(b, ldb, N, K), a.N * a.Ho * a.Wo, N, K, ep, plan, ws, s);
}
int gemm_gather_plain(int dtype, const Gather &a, const void *b, long ldb, int N, const Epilogue &ep, const GemmPlan &plan, float *ws,
                      hipStream_t s)
{
    if (a.ds != 1 && a.sm != 1) return -1;
    return dtype == kBF16 ? gather_plain_t<bf16_t>(a, b, ldb, N, ep, plan, ws, s) : gather_plain_t<float>(a, b, ldb, N, ep, plan, ws, s);
}

int gemm_plain_plain(int dtype, const void *a, long lda, int M, const void *b, long ldb, int N, int b_rows, int K, const Epilogue &ep,
                     const GemmPlan &plan, float *ws, hipStream_t s)
{
    if (b_rows > N) return -1;
    if (dtype == kBF16) return run<bf16_t>(make_plain_k<bf16_t>(a, lda, M, K), make_plain_k<bf16_t>(b, ldb, b_rows, K), M, N, K, ep, plan, ws, s);
    return run<float>(make_plain_k<float>(a, lda, M, K), make_plain_k<float>(b, ldb, b_rows, K), M, N, K, ep, plan, ws, s);
}

int gemm_plain_trans(int dtype, const void *a, long lda, int M, const void *bt, long ldb, int N, int K, const Epilogue &ep,
                     const GemmPlan &plan, float *ws, hipStream_t s)
{
    if (dtype == kBF16) return run<bf16_t>(make_plain_k<bf16_t>(a, lda, M, K), make_plain_t<bf16_t>(bt, ldb, N, K), M, N, K, ep, plan, ws, s);
    return run<float>(make_plain_k<float>(a, lda, M, K), make_plain_t<float>(bt, ldb, N, K), M, N, K, ep, plan, ws, s);
}

int gemm_trans_trans(int dtype, const void *at, long lda, int M, const void *bt, long ldb, int N, int K, const Epilogue &ep,
                     const GemmPlan &plan, float *ws, hipStream_t s)
{
    if (dtype == kBF16) return run<bf16_t>(make_plain_t<bf16_t>(at, lda, M, K), make_plain_t<bf16_t>(bt, ldb, N, K), M, N, K, ep, plan, ws, s);
    return run<float>(make_plain_t<float>(at, lda, M, K), make_plain_t<float>(bt, ldb, N, K), M, N, K, ep, plan, ws, s);
}

int gemm_trans_gather(int dtype, const void *at, long lda, int M, const Gather &b, const Epilogue &ep, const GemmPlan &plan, float *ws,
                      hipStream_t s)
{
    if (b.ds != 1) return -1;
    const int K = b.N * b.Ho * b.Wo, N = b.kh * b.kw * b.C;
    if (dtype == kBF16) return run<bf16_t>(make_plain_t<bf16_t>(at, lda, M, K), make_gather_t<bf16_t>(b), M, N, K, ep, plan, ws, s);
    return run<float>(make_plain_t<float>(at, lda, M, K), make_gather_t<float>(b), M, N, K, ep, plan, ws, s);
}

}  // namespace asgd
