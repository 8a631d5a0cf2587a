// MFMA GEMM engine for gfx950: one kernel template serves the convolutions
// (forward, data gradient, filter gradient, all as implicit GEMMs) and the fully
// connected layers.  C[M][N] = sum_k A[m][k] * B[n][k], fp32 accumulation.
//
// Geometry (identical in bytes for both element types): a workgroup owns a
// 128 x 128 tile of C; one K tile is 128 bytes per row (64 bf16 or 32 fp32).
// Two workgroups share a CU.  The GEMMs run 8 wave64 per workgroup (wave tile
// 64 x 32, four waves per SIMD), except the fp32 convolution filter gradient,
// which runs 4 (wave tile 64 x 64).  Operands arrive through range-checked 16-byte
// buffer loads (out-of-range pieces read as zeros), two K tiles ahead, into
// registers, and go from there to one of two LDS stages, so that one barrier per
// K tile suffices.  An operand whose memory has K contiguous sits in LDS as rows
// x 8 slots of 16 bytes, the slot index XOR-swizzled with the row so that
// fragment reads and stores are spread over the banks.  An operand whose memory
// has the GEMM row contiguous and K strided (both operands of the filter
// gradients, the weights in the FC data gradient) is copied to LDS in that
// orientation and transposed by the LDS read itself (ds_read_b64_tr_b16).  The
// MFMA is issued with the B-matrix fragment as its first operand so that a lane
// ends up with four consecutive n for one m.  The output goes through LDS once
// more, so that a lane owns 8 consecutive columns of a row and a wave stores
// whole row segments as 16-byte vectors.  Workgroup ids are remapped so that each
// of the 8 XCDs (which receive ids round-robin) works on a contiguous range of
// tiles and its L2 sees neighbouring tiles' shared operand rows.  A wave runs at
// raised priority while it multiplies a tile, and a wave whose part of the tile
// lies outside C does not multiply at all.
//
// Stride-1 convolutions whose output grid equals their input grid have a second
// kernel (conv_patch_kernel, further down): the run of input pixels that the 128
// output pixels of a tile need is staged in LDS once per 128 bytes of channels
// and serves every window position from there.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <type_traits>

#include "asgd_internal.h"

namespace asgd {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16_t;

template <typename T> struct Geo;
template <> struct Geo<bf16_t> { enum { CH = 8, BK = 64, KSTEPS = 4 }; };
template <> struct Geo<float> { enum { CH = 4, BK = 32, KSTEPS = 2 }; };

// Tile configuration: block tile BM x BN, WAVES_M x WAVES_N wave64s, DEPTH K tiles in flight in registers,
// MINB workgroups per CU the register budget is sized for.
template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int DEPTH_, int MINB_> struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, DEPTH = DEPTH_, MINB = MINB_;
    static constexpr int NT = 64 * WAVES_M_ * WAVES_N_;
    static constexpr int MB = BM_ / WAVES_M_ / 32, NB = BN_ / WAVES_N_ / 32;   // MFMA 32x32 blocks per wave
    static_assert((BM_ / WAVES_M_) % 64 == 0 && (BN_ / WAVES_N_) % 32 == 0, "wave tiles: rows in 64s, columns in 32s");
};
using Cfg128 = TileCfg<128, 128, 2, 2, 2, 2>;   // 256 threads (wave tile 64x64), two workgroups per CU: two waves per SIMD
using Cfg128w8 = TileCfg<128, 128, 2, 4, 2, 2>; // 512 threads (wave tile 64x32), two workgroups per CU: four waves per SIMD
using Cfg64n = TileCfg<128, 64, 2, 2, 2, 4>;     // 256 threads (wave tile 64x32), four workgroups per CU: four waves per SIMD
#define ASGD_INLINE __attribute__((always_inline))

// Compile-time loop: indices reach the body as constants, so register arrays are never addressed dynamically.
template <int I, int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}


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

__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv &f) { return (__umulhi(n, f.mul) + n) >> f.sh; }
__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }

// ------------------------------------------------------------------ loaders
// All operand fetches are 16-byte buffer loads: the operand tensor is described to the hardware as a byte range,
// a lane passes a 32-bit byte offset, and an offset outside the range returns zeros.  A loader therefore never
// builds a 64-bit address and never branches: pieces that must read as zero (rows or K positions past the end,
// window positions outside the image) get an offset with the top two bits set.  Offsets of valid pieces stay
// below 1 GiB (checked on the host), so the sum of a valid and an invalid part is still out of range.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
constexpr unsigned kInv = 0xC0000000u;
constexpr unsigned kMaxOperandBytes = 0x40000000u;

struct Operand {
    const void *base; unsigned bytes;
    __device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc() const
    {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
    }
};
__device__ __forceinline__ uint4 buf_ld16(__amdgpu_buffer_rsrc_t rs, unsigned off)
{
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}
// value of lane S of the caller's quad (4 consecutive lanes)
template <int S> __device__ __forceinline__ unsigned quad_bcast(unsigned v)
{
    return (unsigned)__builtin_amdgcn_mov_dpp((int)v, S * 0x55, 0xF, 0xF, true);
}

// Direct loaders hand out 16-byte pieces of a row that are contiguous in K.
template <typename T> struct PlainK {
    static constexpr bool kTrans = false;
    Operand op; unsigned ldb; int rows, K;   // ldb: bytes from one row to the next
    struct Row { unsigned off; };
    struct KPos { int k; unsigned koff; };
    __device__ __forceinline__ Row row(int r) const { return Row{r < rows ? (unsigned)r * ldb : kInv}; }
    __device__ __forceinline__ KPos kpos(int k) const { return KPos{k, k < K ? (unsigned)k * (unsigned)sizeof(T) : kInv}; }
    __device__ __forceinline__ void advance(KPos &kp, int dk) const
    {
        kp.k += dk;
        kp.koff = kp.k < K ? (unsigned)kp.k * (unsigned)sizeof(T) : kInv;
    }
    __device__ __forceinline__ unsigned voff(const Row &r, const KPos &kp) const { return r.off + kp.koff; }
};

// Implicit-GEMM gather, unit divisor (forward convolution, stride-1 data gradient).
// All per-row work is done once: a row keeps the byte offset of its window origin
// and a bit mask saying which window positions (ky, kx) fall inside the image; a K
// position keeps the byte offset of (ky, kx, c) relative to a window origin and
// the bit of its window position.  Fetching a piece is then one mask test, one add
// and one select.  WIDE = windows of more than 32 positions (two 16-bit masks, one per axis).
template <typename T, bool WIDE> struct GatherK {
    static constexpr bool kTrans = false;
    Operand op;
    unsigned rowb, pix;  // bytes from one image row / one pixel to the next
    int H, W, C, Ho, Wo, kh, kw, sm, pad, M;
    int adv_px, adv_c;   // one K tile = adv_px whole pixels + adv_c channels
    FastDiv dWo, dHoWo, dC, dkw;
    struct Row { unsigned off, mask; };
    struct KPos { int ky, kx, c; unsigned delta, bit; };
    __device__ __forceinline__ Row row(int m) const
    {
        if (m >= M) return Row{0u, 0u};
        const int n = (int)fdiv((uint32_t)m, dHoWo);
        const int rem = m - n * (Ho * Wo);
        const int oy = (int)fdiv((uint32_t)rem, dWo);
        const int ox = rem - oy * Wo;
        const int y0 = oy * sm - pad, x0 = ox * sm - pad;
        // ky is inside for max(0,-y0) <= ky < min(kh, H-y0); the same along x
        const int ylo = max(0, -y0), yhi = max(ylo, min(kh, H - y0));
        const int xlo = max(0, -x0), xhi = max(xlo, min(kw, W - x0));
        const unsigned ym = ((1u << yhi) - 1u) & ~((1u << ylo) - 1u), xm = ((1u << xhi) - 1u) & ~((1u << xlo) - 1u);
        unsigned mask = 0;
        if (WIDE) {
            mask = ym | (xm << 16);
        } else {
            for (int a = 0; a < kh; ++a)
                if ((ym >> a) & 1u) mask |= xm << (a * kw);
        }
        return Row{(unsigned)(n * H + y0) * rowb + (unsigned)x0 * pix, mask};
    }
    __device__ __forceinline__ unsigned bit_of(int ky, int kx) const
    {
        const unsigned b = WIDE ? ((1u << (ky & 15)) | (1u << (16 + kx))) : (1u << ((ky * kw + kx) & 31));
        return ky < kh ? b : 0u;
    }
    __device__ __forceinline__ KPos kpos(int k) const
    {
        const int t = (int)fdiv((uint32_t)k, dC);
        const int ky = (int)fdiv((uint32_t)t, dkw);
        const int kx = t - ky * kw, c = k - t * C;
        return KPos{ky, kx, c, (unsigned)ky * rowb + (unsigned)kx * pix + (unsigned)c * (unsigned)sizeof(T), bit_of(ky, kx)};
    }
    // branch-free: no divergent control flow between the loads of a pipeline step
    __device__ __forceinline__ void advance(KPos &kp, int) const
    {
        kp.c += adv_c;
        const int wrap = kp.c >= C ? 1 : 0;
        kp.c -= wrap * C;
        kp.kx += adv_px + wrap;
        const int up = (int)fdiv((uint32_t)kp.kx, dkw);
        kp.kx -= up * kw;
        kp.ky += up;
        kp.delta = (unsigned)kp.ky * rowb + (unsigned)kp.kx * pix + (unsigned)kp.c * (unsigned)sizeof(T);
        kp.bit = bit_of(kp.ky, kp.kx);
    }
    __device__ __forceinline__ unsigned voff(const Row &r, const KPos &kp) const
    {
        const bool ok = WIDE ? (kp.bit != 0u && (r.mask & kp.bit) == kp.bit) : ((r.mask & kp.bit) != 0u);
        return ok ? r.off + kp.delta : kInv;
    }
};

// The same gather with a divisor (data gradient of a strided convolution): positions
// that are not multiples of the stride contribute nothing.  Rare, kept simple.
template <typename T> struct GatherKS {
    static constexpr bool kTrans = false;
    Operand op; unsigned pix;   // bytes from one pixel to the next
    int H, W, C, Ho, Wo, kh, kw, sm, ds, pad, M;
    FastDiv dWo, dHoWo, dC, dkw;
    struct Row { int pix0, y0, x0; };  // pix0 < 0: row out of range
    struct KPos { int ky, kx, c; };
    __device__ __forceinline__ Row row(int m) const
    {
        if (m >= M) return Row{-1, 0, 0};
        const int n = (int)fdiv((uint32_t)m, dHoWo);
        const int rem = m - n * (Ho * Wo);
        const int oy = (int)fdiv((uint32_t)rem, dWo);
        const int ox = rem - oy * Wo;
        return Row{n * H * W, oy * sm - pad, ox * sm - pad};
    }
    __device__ __forceinline__ KPos kpos(int k) const
    {
        const int t = (int)fdiv((uint32_t)k, dC);
        const int ky = (int)fdiv((uint32_t)t, dkw);
        return KPos{ky, t - ky * kw, k - t * C};
    }
    __device__ __forceinline__ void advance(KPos &kp, int dk) const
    {
        kp.c += dk;
        while (kp.c >= C) {
            kp.c -= C;
            if (++kp.kx == kw) { kp.kx = 0; ++kp.ky; }
        }
    }
    __device__ __forceinline__ unsigned voff(const Row &r, const KPos &kp) const
    {
        if (r.pix0 < 0 || kp.ky >= kh) return kInv;
        int y = r.y0 + kp.ky, xx = r.x0 + kp.kx;
        if (y < 0 || xx < 0) return kInv;
        if ((y % ds) != 0 || (xx % ds) != 0) return kInv;
        y /= ds; xx /= ds;
        if (y >= H || xx >= W) return kInv;
        return (unsigned)(r.pix0 + y * W + xx) * pix + (unsigned)kp.c * (unsigned)sizeof(T);
    }
};

// Row-contiguous loaders: memory has the GEMM row index contiguous and the
// reduction index strided ([k][rows]).  The tile is copied to LDS in that same
// orientation, 16 bytes (8 or 4 consecutive rows) at a time; the transposition
// the MFMA needs happens in the LDS read (ds_read_b64_tr_b16 for 16-bit data).
// A thread keeps one column of 16-byte pieces (Col) and walks down the K axis.
template <typename T> struct PlainT {
    static constexpr bool kTrans = true, kShared = false;
    Operand op; unsigned ldb; int rows, K;
    struct Col { unsigned off; };
    struct KState { int k; unsigned koff; };
    __device__ __forceinline__ Col col(int row0) const { return Col{row0 < rows ? (unsigned)row0 * (unsigned)sizeof(T) : kInv}; }
    __device__ __forceinline__ KState kstate(int k) const { return KState{k, k < K ? (unsigned)k * ldb : kInv}; }
    __device__ __forceinline__ void advance(KState &ks, int dk) const
    {
        ks.k += dk;
        ks.koff = ks.k < K ? ks.koff + (unsigned)dk * ldb : kInv;   // once past K it stays past K
    }
    __device__ __forceinline__ unsigned voff(const Col &c, const KState &ks) const { return c.off + ks.koff; }
};

// Filter-gradient gather: rows enumerate (ky, kx, c) (fixed per column of pieces), the reduction index
// enumerates output pixels m = (n, oy, ox).  What depends on the pixel alone (the byte offset of its window
// origin and the mask of window positions that fall inside the image) is computed once per pixel and K tile:
// the four lanes of a quad copy the same column for four different pixels, each works out one pixel and the
// quad exchanges the results with DPP moves.  A column keeps its offset inside the window and the mask bits of
// its (ky, kx); a piece is fetched iff the pixel's mask has both bits.
template <typename T> struct GatherT {
    static constexpr bool kTrans = true, kShared = true;
    Operand op;
    unsigned rowb, pix;  // bytes from one image row / one pixel to the next
    int H, W, C, Ho, Wo, kh, kw, sm, pad, M, Krows;
    FastDiv dWo, dHo, dHoWo, dC, dkw;
    struct Col { unsigned off, bits; };   // out-of-range columns: bits no pixel mask can have
    struct KState { int m, n, oy, ox; };
    struct Pixel { unsigned base, mask; };
    __device__ __forceinline__ Col col(int row0) const
    {
        if (row0 >= Krows) return Col{0u, 0xFFFFFFFFu};
        const int t = (int)fdiv((uint32_t)row0, dC);
        const int ky = (int)fdiv((uint32_t)t, dkw);
        const int kx = t - ky * kw, c = row0 - t * C;
        return Col{(unsigned)(ky - pad) * rowb + (unsigned)(kx - pad) * pix + (unsigned)c * (unsigned)sizeof(T),
                   (1u << ky) | (1u << (16 + kx))};
    }
    __device__ __forceinline__ KState kstate(int m) const
    {
        const int n = (int)fdiv((uint32_t)m, dHoWo);
        const int rem = m - n * (Ho * Wo);
        const int oy = (int)fdiv((uint32_t)rem, dWo);
        return KState{m, n, oy, rem - oy * Wo};
    }
    __device__ __forceinline__ void advance(KState &ks, int dk) const
    {
        ks.m += dk;
        ks.ox += dk;
        const int q = (int)fdiv((uint32_t)ks.ox, dWo);
        ks.ox -= q * Wo;
        ks.oy += q;
        const int q2 = (int)fdiv((uint32_t)ks.oy, dHo);
        ks.oy -= q2 * Ho;
        ks.n += q2;
    }
    __device__ __forceinline__ Pixel pixel(const KState &ks) const
    {
        const int y0 = ks.oy * sm - pad, x0 = ks.ox * sm - pad;
        const int ylo = max(0, -y0), yhi = max(ylo, min(kh, H - y0));
        const int xlo = max(0, -x0), xhi = max(xlo, min(kw, W - x0));
        const unsigned ym = ((1u << yhi) - 1u) & ~((1u << ylo) - 1u), xm = ((1u << xhi) - 1u) & ~((1u << xlo) - 1u);
        return Pixel{(unsigned)(ks.n * H + ks.oy * sm) * rowb + (unsigned)(ks.ox * sm) * pix, ks.m < M ? (ym | (xm << 16)) : 0u};
    }
    __device__ __forceinline__ unsigned voff(const Col &c, unsigned base, unsigned mask) const
    {
        return (mask & c.bits) == c.bits ? c.off + base : kInv;
    }
};

// ------------------------------------------------------------------ staging
template <typename T, class L, int ROWS, int NT, int DEPTH, bool kTrans = L::kTrans> struct Stage;

template <typename T, class L, int ROWS, int NT, int DEPTH> struct Stage<T, L, ROWS, NT, DEPTH, false> {
    static constexpr int SLOTS = ROWS * 8 / NT;
    typename L::Row rows[SLOTS];
    typename L::KPos kp;
    uint4 r[DEPTH][SLOTS];   // DEPTH K tiles in flight
    unsigned wo[2];      // LDS byte offset of slot 0 / slot 1; slot s sits s/2 * 64 rows further
    __device__ __forceinline__ void init(const L &l, int row0, int k0, int tid, int)
    {
        static_for<0, 2>([&](auto par) ASGD_INLINE {
            const int row = (tid >> 3) + par * (NT / 8);
            wo[par] = (unsigned)(row * 8 + ((tid & 7) ^ swz(row))) * 16u;
        });
        static_for<0, SLOTS>([&](auto s) ASGD_INLINE { rows[s] = l.row(row0 + (tid >> 3) + s * (NT / 8)); });
        kp = l.kpos(k0 + (tid & 7) * Geo<T>::CH);
    }
    // fetch the K tile at the cursor into register set RB and advance the cursor
    template <int RB> __device__ __forceinline__ void load(const L &l)
    {
        const __amdgpu_buffer_rsrc_t rs = l.op.rsrc();
        static_for<0, SLOTS>([&](auto s) ASGD_INLINE { r[RB][s] = buf_ld16(rs, l.voff(rows[s], kp)); });
        l.advance(kp, Geo<T>::BK);
    }
    template <int RB> __device__ __forceinline__ void store(uint4 *sm, int tid) const
    {
        // rows 64 apart share the swizzle, so the offset of slot s is that of slot s%2 plus a constant
        char *base = reinterpret_cast<char *>(sm);
        static_for<0, SLOTS>([&](auto s) ASGD_INLINE {
            *reinterpret_cast<uint4 *>(base + wo[s % 2] + (s / 2) * (2 * (NT / 8) * 128)) = r[RB][s];
        });
    }
};

// LDS tile of a row-contiguous operand: BK lines of ROWS elements.  A transposing read makes half a wave touch
// 4 K lines x 64 bytes; with lines 64 bytes (mod 256) apart those eight 32-byte groups cover all banks once.
template <typename T, int ROWS> struct TransTile {
    static constexpr int LINE = ROWS * (int)sizeof(T) + (sizeof(T) == 2 ? 64 : 32);   // bytes
    static constexpr int BYTES = Geo<T>::BK * LINE;
};

template <typename T, class L, int ROWS, int NT, int DEPTH> struct Stage<T, L, ROWS, NT, DEPTH, true> {
    static constexpr int CPL = ROWS * (int)sizeof(T) / 16;   // 16-byte pieces per K line
    static constexpr int LPP = NT / CPL;                     // K lines covered by one pass of the workgroup
    static constexpr int SLOTS = Geo<T>::BK / LPP;
    static constexpr int NKS = L::kShared ? 1 : SLOTS;
    static_assert(NT % CPL == 0 && Geo<T>::BK % LPP == 0, "tile / thread-count mismatch");
    static_assert(!L::kShared || ((SLOTS == 4 || SLOTS == 2) && CPL % 4 == 0), "a quad shares one column and owns its K lines");
    typename L::Col c;
    typename L::KState ks[NKS];   // shared form: the K line of slot (tid & 3) only
    uint4 r[DEPTH][SLOTS];
    unsigned wo;   // LDS byte offset of slot 0
    __device__ __forceinline__ void init(const L &l, int row0, int k0, int tid, int)
    {
        const int cc = tid % CPL, line = tid / CPL;
        c = l.col(row0 + cc * (16 / (int)sizeof(T)));
        if constexpr (L::kShared) ks[0] = l.kstate(k0 + line + (tid & (SLOTS - 1)) * LPP);
        else static_for<0, SLOTS>([&](auto s) ASGD_INLINE { ks[s] = l.kstate(k0 + line + s * LPP); });
        wo = (unsigned)(line * TransTile<T, ROWS>::LINE + cc * 16);
    }
    template <int RB> __device__ __forceinline__ void load(const L &l)
    {
        const __amdgpu_buffer_rsrc_t rs = l.op.rsrc();
        if constexpr (L::kShared) {
            const auto px = l.pixel(ks[0]);
            l.advance(ks[0], Geo<T>::BK);
            static_for<0, SLOTS>([&](auto s) ASGD_INLINE {
                r[RB][s] = buf_ld16(rs, l.voff(c, quad_bcast<s>(px.base), quad_bcast<s>(px.mask)));
            });
        } else {
            static_for<0, SLOTS>([&](auto s) ASGD_INLINE {
                r[RB][s] = buf_ld16(rs, l.voff(c, ks[s]));
                l.advance(ks[s], Geo<T>::BK);
            });
        }
    }
    template <int RB> __device__ __forceinline__ void store(uint4 *sm, int) const
    {
        char *base = reinterpret_cast<char *>(sm);
        static_for<0, SLOTS>([&](auto s) ASGD_INLINE {
            *reinterpret_cast<uint4 *>(base + wo + s * (LPP * TransTile<T, ROWS>::LINE)) = r[RB][s];
        });
    }
};

// ------------------------------------------------------------------ MFMA step
// A fragment is the 8 consecutive K elements of one row that a lane feeds to the
// MFMA.  FragOff holds, per K step, the LDS byte offset of that piece for the
// lane's row in row block 0 and in row block 1 (blocks 64 rows apart share it), so
// the inner loop issues its LDS reads with no address arithmetic.
template <typename T> struct Frag;
template <typename T, bool TRANS, int ROWS> struct FragOff;
template <int ROWS> struct FragOff<bf16_t, false, ROWS> {
    unsigned o[Geo<bf16_t>::KSTEPS][2];
    __device__ __forceinline__ void init(int row0, int lane)
    {
        const int lrow = lane & 31, half = lane >> 5;
        static_for<0, Geo<bf16_t>::KSTEPS>([&](auto ks) ASGD_INLINE {
            static_for<0, 2>([&](auto par) ASGD_INLINE {
                const int row = row0 + par * 32 + lrow;
                o[ks][par] = (unsigned)(row * 8 + ((ks * 2 + half) ^ swz(row))) * 16u;
            });
        });
    }
};
template <int ROWS> struct FragOff<float, false, ROWS> {
    unsigned o[Geo<float>::KSTEPS][2][2];
    __device__ __forceinline__ void init(int row0, int lane)
    {
        const int lrow = lane & 31, half = lane >> 5;
        static_for<0, Geo<float>::KSTEPS>([&](auto ks) ASGD_INLINE {
            static_for<0, 2>([&](auto par) ASGD_INLINE {
                const int row = row0 + par * 32 + lrow, q = ks * 4 + half * 2, z = swz(row);
                o[ks][par][0] = (unsigned)(row * 8 + (q ^ z)) * 16u;
                o[ks][par][1] = (unsigned)(row * 8 + ((q + 1) ^ z)) * 16u;
            });
        });
    }
};
// Row-contiguous tiles.  16-bit data: ds_read_b64_tr_b16 works on blocks of 16 lanes; when lane j of a block
// points at K line (j >> 2) and row piece (j & 3) of a 4 x 16 patch, lane i receives row i of the patch for the
// four K lines in order.  Lane L = 16*b + i of the wave wants row 16*(b & 1) + i and K lines 8*(b >> 1) + 0..7
// of the K step, i.e. two such reads.  32-bit data needs no hardware help: eight 4-byte reads down the K axis.
template <int ROWS> struct FragOff<bf16_t, true, ROWS> {
    unsigned base;
    __device__ __forceinline__ void init(int row0, int lane)
    {
        const int b = lane >> 4, i = lane & 15;
        base = (unsigned)((8 * (b >> 1) + (i >> 2)) * TransTile<bf16_t, ROWS>::LINE + (row0 + 16 * (b & 1) + 4 * (i & 3)) * 2);
    }
};
template <int ROWS> struct FragOff<float, true, ROWS> {
    unsigned base;
    __device__ __forceinline__ void init(int row0, int lane)
    {
        base = (unsigned)(8 * (lane >> 5) * TransTile<float, ROWS>::LINE + (row0 + (lane & 31)) * 4);
    }
};
// Fragment offsets into an activation patch (see conv_patch_kernel): the byte address of the lane's pixel for
// row block 0 / 1, K-half included, at each of the PPT window positions of the K tile; the K steps of one
// position are 32 (bf16) or 64 (fp32) bytes apart.
template <int PPT> struct PatchOff { unsigned a[2][PPT]; };
typedef short short4v __attribute__((ext_vector_type(4)));
template <> struct Frag<bf16_t> {
    uint4 v;
    template <int KS, int BLK, int PPT> __device__ __forceinline__ void read(const char *sm, const PatchOff<PPT> &fo)
    {
        constexpr int SPP = Geo<bf16_t>::KSTEPS / PPT;   // K steps per window position
        v = *reinterpret_cast<const uint4 *>(sm + fo.a[BLK][KS / SPP] + (KS % SPP) * 32);
    }
    template <int KS, int BLK, int ROWS> __device__ __forceinline__ void read(const char *sm, const FragOff<bf16_t, false, ROWS> &fo)
    {
        v = *reinterpret_cast<const uint4 *>(sm + fo.o[KS][BLK % 2] + (BLK / 2) * (64 * 128));
    }
    template <int KS, int BLK, int ROWS> __device__ __forceinline__ void read(const char *sm, const FragOff<bf16_t, true, ROWS> &fo)
    {
        constexpr int LINE = TransTile<bf16_t, ROWS>::LINE;
        typedef __attribute__((address_space(3))) short4v lds_s4;
        const char *p = sm + fo.base + KS * 16 * LINE + BLK * 64;
        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4 *)(p));
        const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4 *)(p + 4 * LINE));
        const uint2 a = __builtin_bit_cast(uint2, lo), b = __builtin_bit_cast(uint2, hi);
        v = make_uint4(a.x, a.y, b.x, b.y);
    }
};
template <> struct Frag<float> {
    uint4 v[2];
    template <int KS, int BLK, int PPT> __device__ __forceinline__ void read(const char *sm, const PatchOff<PPT> &fo)
    {
        constexpr int SPP = Geo<float>::KSTEPS / PPT;
        v[0] = *reinterpret_cast<const uint4 *>(sm + fo.a[BLK][KS / SPP] + (KS % SPP) * 64);
        v[1] = *reinterpret_cast<const uint4 *>(sm + fo.a[BLK][KS / SPP] + (KS % SPP) * 64 + 16);
    }
    template <int KS, int BLK, int ROWS> __device__ __forceinline__ void read(const char *sm, const FragOff<float, false, ROWS> &fo)
    {
        v[0] = *reinterpret_cast<const uint4 *>(sm + fo.o[KS][BLK % 2][0] + (BLK / 2) * (64 * 128));
        v[1] = *reinterpret_cast<const uint4 *>(sm + fo.o[KS][BLK % 2][1] + (BLK / 2) * (64 * 128));
    }
    template <int KS, int BLK, int ROWS> __device__ __forceinline__ void read(const char *sm, const FragOff<float, true, ROWS> &fo)
    {
        constexpr int LINE = TransTile<float, ROWS>::LINE;
        const char *p = sm + fo.base + KS * 16 * LINE + BLK * 128;
        uint32_t e[8];
        static_for<0, 8>([&](auto j) ASGD_INLINE { e[j] = *reinterpret_cast<const uint32_t *>(p + j * LINE); });
        v[0] = make_uint4(e[0], e[1], e[2], e[3]);
        v[1] = make_uint4(e[4], e[5], e[6], e[7]);
    }
};

__device__ __forceinline__ void mma(f32x16 &acc, const Frag<bf16_t> &first, const Frag<bf16_t> &second)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, first.v), __builtin_bit_cast(bf16x8, second.v),
                                                  acc, 0, 0, 0);
}
__device__ __forceinline__ void mma(f32x16 &acc, const Frag<float> &first, const Frag<float> &second)
{
    const uint32_t a[8] = {first.v[0].x, first.v[0].y, first.v[0].z, first.v[0].w, first.v[1].x, first.v[1].y, first.v[1].z, first.v[1].w};
    const uint32_t b[8] = {second.v[0].x, second.v[0].y, second.v[0].z, second.v[0].w, second.v[1].x, second.v[1].y, second.v[1].z, second.v[1].w};
#pragma unroll
    for (int e = 0; e < 8; ++e)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[e]), __uint_as_float(b[e]), acc, 0, 0, 0);
}

// ------------------------------------------------------------------ epilogue
__device__ __forceinline__ uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

// Store of 8 consecutive output elements (32 bytes fp32 / 16 bytes bf16) as 16-byte vectors: every output
// row starts 16-byte aligned and has a multiple of 8 elements (checked on the host).
typedef float f32x4 __attribute__((ext_vector_type(4)));
template <typename T> __device__ __forceinline__ void store8(T *p, const float (&v)[8]);
template <> __device__ __forceinline__ void store8<float>(float *p, const float (&v)[8])
{
    f32x4 *q = reinterpret_cast<f32x4 *>(__builtin_assume_aligned(p, 16));
    q[0] = f32x4{v[0], v[1], v[2], v[3]};
    q[1] = f32x4{v[4], v[5], v[6], v[7]};
}
template <> __device__ __forceinline__ void store8<bf16_t>(bf16_t *p, const float (&v)[8])
{
    union { bf16_t h[8]; u32x4 u; } t;
#pragma unroll
    for (int r = 0; r < 8; ++r) t.h[r] = (bf16_t)v[r];
    *reinterpret_cast<u32x4 *>(__builtin_assume_aligned(p, 16)) = t.u;
}

template <typename T> struct Vec8;
template <> struct Vec8<float> { union { float4 u[2]; float e[8]; }; };
template <> struct Vec8<bf16_t> { union { uint4 u[1]; bf16_t e[8]; }; };

// Eight consecutive columns n0..n0+7 of row m (n0 a multiple of 8, all in range).
// The bias of these 8 columns, as fp32 (zeros past bias_n or without a bias).
template <typename T> __device__ __forceinline__ void load_bias8(const Epilogue &ep, int n0, float (&b8)[8])
{
#pragma unroll
    for (int r = 0; r < 8; ++r) b8[r] = 0.f;
    if (ep.bias) {
        const T *b = static_cast<const T *>(ep.bias);
#pragma unroll
        for (int r = 0; r < 8; ++r)
            if (n0 + r < ep.bias_n) b8[r] = to_f32(b[n0 + r]);
    }
}

template <typename T> __device__ __forceinline__ void epilogue8(const Epilogue &ep, int m, int n0, float (&v)[8], const float (&b8)[8])
{
    if (ep.mode == 1) {  // conv filter gradient: (cout, (ky,kx,ci_padded)) -> canonical [cout][cin][kh][kw]
        if (m >= ep.cw_cout) return;
        const int t = n0 / ep.cw_cinp, ci0 = n0 - t * ep.cw_cinp;
        const int ky = t / ep.cw_kw, kx = t - ky * ep.cw_kw;
        float *o = static_cast<float *>(ep.out);
#pragma unroll
        for (int r = 0; r < 8; ++r)
            if (ci0 + r < ep.cw_cin) o[(((long)m * ep.cw_cin + ci0 + r) * ep.cw_kh + ky) * ep.cw_kw + kx] = v[r];
        return;
    }
    if (ep.mode == 2) {  // the same for window rows: columns are (ky, j), j = kx*cw_rwc + ci over a padded row of cw_cinp elements
        if (m >= ep.cw_cout) return;
        const int ky = n0 / ep.cw_cinp, j0 = n0 - ky * ep.cw_cinp;
        float *o = static_cast<float *>(ep.out);
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int kx = (j0 + r) / ep.cw_rwc, ci = (j0 + r) - kx * ep.cw_rwc;
            if (ci < ep.cw_cin && kx < ep.cw_kw) o[(((long)m * ep.cw_cin + ci) * ep.cw_kh + ky) * ep.cw_kw + kx] = v[r];
        }
        return;
    }
    if (ep.bias) {
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] += b8[r];
    }
    if (ep.relu) {
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = v[r] > 0.f ? v[r] : 0.f;
    }
    if (ep.drop) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint64_t idx = (uint64_t)m * (uint64_t)ep.drop_F + (uint64_t)(n0 + r);
            const uint32_t u = (uint32_t)(mix64(ep.drop_key + 0x9E3779B97F4A7C15ull * (idx + 1)) >> 32);
            v[r] = (u >= ep.drop_thr) ? v[r] * ep.drop_scale : 0.f;
        }
    }
    if (ep.mask_src) {
        Vec8<T> ms;   // the mask tensor is a workspace tensor: rows and column groups are 16-byte aligned
        const T *mp = static_cast<const T *>(ep.mask_src) + (long)m * ep.mask_ld + n0;
        static_for<0, sizeof(ms.u) / 16>([&](auto i) ASGD_INLINE { ms.u[i] = reinterpret_cast<const std::remove_reference_t<decltype(ms.u[0])> *>(mp)[i]; });
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = to_f32(ms.e[r]) > 0.f ? v[r] * ep.mask_scale : 0.f;
    }
    if (ep.out_f32) {
        // fp32 output = a parameter gradient: read again only by the update, long after it has left every cache
        f32x4 *q = reinterpret_cast<f32x4 *>(__builtin_assume_aligned(static_cast<float *>(ep.out) + (long)m * ep.ld + n0, 16));
        __builtin_nontemporal_store(f32x4{v[0], v[1], v[2], v[3]}, q);
        __builtin_nontemporal_store(f32x4{v[4], v[5], v[6], v[7]}, q + 1);
    }
    else store8<T>(static_cast<T *>(ep.out) + (long)m * ep.ld + n0, v);
}

// ------------------------------------------------------------------ kernel
// One K tile out of LDS.  The fragments of K step ks+1 are requested before the
// MFMAs of step ks are issued, so the LDS latency hides behind the matrix pipe.
template <typename T, int MB, int NB, class FOA, class FOB>
__device__ __forceinline__ void compute_tile(const uint4 *sA, const uint4 *sB, f32x16 (&acc)[NB][MB], const FOA &foA, const FOB &foB)
{
    constexpr int KS = Geo<T>::KSTEPS;
    const char *pa = reinterpret_cast<const char *>(sA), *pb = reinterpret_cast<const char *>(sB);
    Frag<T> fa[2][MB], fb[2][NB];
    static_for<0, MB>([&](auto mb) ASGD_INLINE { fa[0][mb].template read<0, mb>(pa, foA); });
    static_for<0, NB>([&](auto nb) ASGD_INLINE { fb[0][nb].template read<0, nb>(pb, foB); });
    static_for<0, KS>([&](auto ks) ASGD_INLINE {
        constexpr int cur = ks % 2, nxt = (ks + 1) % 2;
        if constexpr (ks + 1 < KS) {
            static_for<0, MB>([&](auto mb) ASGD_INLINE { fa[nxt][mb].template read<ks + 1, mb>(pa, foA); });
            static_for<0, NB>([&](auto nb) ASGD_INLINE { fb[nxt][nb].template read<ks + 1, nb>(pb, foB); });
        }
        static_for<0, NB>([&](auto nb) ASGD_INLINE { static_for<0, MB>([&](auto mb) ASGD_INLINE { mma(acc[nb][mb], fb[cur][nb], fa[cur][mb]); }); });
    });
}

// Output of a block tile: the accumulators go through LDS so that every lane ends up with 8 consecutive columns
// of one row and a wave stores whole row segments (the MFMA layout gives a lane 4 columns of one row and its
// neighbours other rows).  The whole tile is staged at once, BM rows of BN floats without padding: the 16-byte
// chunk index is XOR-ed with the row, so that the 16 lanes of a write (16 rows, one chunk column) and the 16
// lanes of a read (one row, 16 chunks) each touch every bank once.
// acc[nb][mb][v]: m = wm + mb*32 + lrow, n = wn + nb*32 + 8*(v/4) + 4*half + v%4
// Second half of the output phase: NTALL threads take the staged tile out of LDS, eight columns of a row each.
template <typename T, class Cfg, int NTALL>
__device__ __forceinline__ void emit_tile(const uint4 *smem, const Epilogue &ep, int tm, int tn, int split, int M, int N, float *ws,
                                          const float (&bias8)[8], int tid)
{
    constexpr int BM = Cfg::BM, BN = Cfg::BN;
    constexpr int CPR = BN / 4;                       // 16-byte chunks per row
    const float4 *stg = reinterpret_cast<const float4 *>(smem);
    constexpr int LPR = BN / 8, RPR = NTALL / LPR;   // lanes per row, rows per round
    static_for<0, BM / RPR>([&](auto r) ASGD_INLINE {
        const int row = r * RPR + tid / LPR, chunk = (tid % LPR) * 2;
        const int m = tm * BM + row, n0 = tn * BN + chunk * 4;
        if (m < M && n0 < N) {
            const float4 lo = stg[row * CPR + (chunk ^ (row & (CPR - 1)))];
            const float4 hi = stg[row * CPR + ((chunk + 1) ^ (row & (CPR - 1)))];
            float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
            if (ws) store8<float>(ws + ((long)split * M + m) * N + n0, v);
            else epilogue8<T>(ep, m, n0, v, bias8);
        }
    });
}

// The push of a parameter gradient done in place of storing it (Epilogue::upd_w): the staged tile is the gradient of
// a BM x BN block of parameters.  A thread asks for the parameters and momenta of all its rows before the barrier
// that completes the staging, so that the whole block (2 x 64 KB) is in flight at once; the arithmetic is that of
// the streaming update kernel, contraction for contraction, and the worker copy is rounded as the snapshot rounds.
__device__ __forceinline__ uint32_t bf16_bits_rne(uint32_t u)
{
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (u >> 16) | 0x0040u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
template <typename T, class Cfg, int NTALL>
__device__ __forceinline__ void update_tile(const uint4 *smem, const Epilogue &ep, int tm, int tn, int M, int N, int tid)
{
    // a lane owns 4 consecutive columns, so that the 16-byte pieces of one store instruction are consecutive in
    // memory (32 lanes = 512 bytes of a row): whole lines leave the CU at once
    constexpr int BM = Cfg::BM, BN = Cfg::BN, CPR = BN / 4, RPR = NTALL / CPR, R = BM / RPR;
    const float4 *stg = reinterpret_cast<const float4 *>(smem);
    const int chunk = tid % CPR, n0 = tn * BN + chunk * 4;
    f32x4 w[R], mo[R];
    static_for<0, R>([&](auto r) ASGD_INLINE {
        const int m = tm * BM + r * RPR + tid / CPR;
        if (m < M && n0 < N) {
            const long p = (long)m * ep.ld + n0;
            w[r] = *reinterpret_cast<const f32x4 *>(__builtin_assume_aligned(ep.upd_w + p, 16));
            mo[r] = *reinterpret_cast<const f32x4 *>(__builtin_assume_aligned(ep.upd_v + p, 16));
        }
    });
    __syncthreads();
    static_for<0, R>([&](auto r) ASGD_INLINE {
        const int row = r * RPR + tid / CPR, m = tm * BM + row;
        if (m < M && n0 < N) {
            const float4 g4 = stg[row * CPR + (chunk ^ (row & (CPR - 1)))];
            const float g[4] = {g4.x, g4.y, g4.z, g4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float wo = w[r][e], vo = mo[r][e];
                const float t = __builtin_fmaf(ep.upd_wd, wo, g[e]);
                const float vn = __builtin_fmaf(ep.upd_mu, vo, -(ep.upd_lr * t));
                mo[r][e] = vn;
                w[r][e] = wo + vn;
            }
            const long p = (long)m * ep.ld + n0;
            __builtin_nontemporal_store(w[r], reinterpret_cast<f32x4 *>(__builtin_assume_aligned(ep.upd_w + p, 16)));
            __builtin_nontemporal_store(mo[r], reinterpret_cast<f32x4 *>(__builtin_assume_aligned(ep.upd_v + p, 16)));
            if constexpr (sizeof(T) == 4) {
                *reinterpret_cast<f32x4 *>(__builtin_assume_aligned(static_cast<float *>(ep.upd_copy) + p, 16)) = w[r];
            } else {
                typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
                u32x2 o;
                o.x = bf16_bits_rne(__float_as_uint(w[r][0])) | (bf16_bits_rne(__float_as_uint(w[r][1])) << 16);
                o.y = bf16_bits_rne(__float_as_uint(w[r][2])) | (bf16_bits_rne(__float_as_uint(w[r][3])) << 16);
                *reinterpret_cast<u32x2 *>(__builtin_assume_aligned(static_cast<bf16_t *>(ep.upd_copy) + p, 8)) = o;
            }
        }
    });
}

// The output phase of the Cfg::NT threads that hold accumulators; NTALL >= Cfg::NT threads of the workgroup take part in
// its second half (the others pass the two barriers and call emit_tile themselves).
template <typename T, class Cfg, int SMEM_BYTES, int NTALL = Cfg::NT, bool PUSH = false>
__device__ __forceinline__ void output_tile(uint4 *smem, f32x16 (&acc)[Cfg::NB][Cfg::MB], const Epilogue &ep, int tm, int tn, int split, int M,
                                            int N, float *ws, const float (&bias8)[8], int tid, int wm, int wn)
{
    constexpr int BM = Cfg::BM, BN = Cfg::BN, MB = Cfg::MB, NB = Cfg::NB;
    constexpr int CPR = BN / 4;                   // 16-byte chunks per row
    static_assert(BM * BN * 4 <= SMEM_BYTES, "staging area");
    float4 *stg = reinterpret_cast<float4 *>(smem);
    const int lane = tid & 63, lrow = lane & 31, half = lane >> 5;
    __syncthreads();
    static_for<0, MB>([&](auto mb) ASGD_INLINE {
        const int row = wm + mb * 32 + lrow;
        static_for<0, NB>([&](auto nb) ASGD_INLINE {
            static_for<0, 4>([&](auto g) ASGD_INLINE {
                const int chunk = (wn + nb * 32 + 8 * g + 4 * half) / 4;
                stg[row * CPR + (chunk ^ (row & (CPR - 1)))] =
                    make_float4(acc[nb][mb][4 * g], acc[nb][mb][4 * g + 1], acc[nb][mb][4 * g + 2], acc[nb][mb][4 * g + 3]);
            });
        });
    });
    if constexpr (PUSH) {   // only the kernel instance that serves the fully-connected weight gradient carries this path
        static_assert(NTALL == Cfg::NT, "every thread of the workgroup takes part in the push");
        if (ep.upd_w) { update_tile<T, Cfg, NTALL>(smem, ep, tm, tn, M, N, tid); return; }
    }
    __syncthreads();
    emit_tile<T, Cfg, NTALL>(smem, ep, tm, tn, split, M, N, ws, bias8, tid);
}

// Software pipeline.  LDS holds two stages so that one barrier per K tile
// suffices; DEPTH K tiles are in flight in registers while another is being
// multiplied out of LDS.  At the top of step t, LDS stage t%2 holds tile t and
// the register sets hold tiles t+1 .. t+DEPTH-1 (possibly still arriving).
template <typename T, class Cfg, class LA, class LB>
__global__ __launch_bounds__(Cfg::NT, Cfg::MINB) void gemm_kernel(LA la, LB lb, Epilogue ep, int M, int N, int nkt, int kt_per_split,
                                                                int tiles_m, int tiles_n, float *ws)
{
    constexpr int BK = Geo<T>::BK, BM = Cfg::BM, BN = Cfg::BN, NT = Cfg::NT, MB = Cfg::MB, NB = Cfg::NB, DEPTH = Cfg::DEPTH;
    constexpr int TA = LA::kTrans ? TransTile<T, BM>::BYTES : BM * 128, TB = LB::kTrans ? TransTile<T, BN>::BYTES : BN * 128;
    __shared__ uint4 smem[2 * (TA + TB) / 16];   // two stages of A and B tiles; reused to stage the output
    uint4 (*sA)[TA / 16] = reinterpret_cast<uint4 (*)[TA / 16]>(smem);
    uint4 (*sB)[TB / 16] = reinterpret_cast<uint4 (*)[TB / 16]>(smem + 2 * TA / 16);
    const int tid = threadIdx.x;
    // XCD-aware remap: ids congruent mod 8 run on one XCD; give that XCD a contiguous range of tiles
    int bid;
    {
        const int nb = gridDim.x, q = nb >> 3, r = nb & 7, x = blockIdx.x & 7;
        bid = x * q + (x < r ? x : r) + (blockIdx.x >> 3);
    }
    const int tn = bid % tiles_n; bid /= tiles_n;
    const int tm = bid % tiles_m;
    const int split = bid / tiles_m;
    const int kt0 = split * kt_per_split;
    const int nt = min(nkt, kt0 + kt_per_split) - kt0;   // K tiles of this workgroup (>= 1)

    Stage<T, LA, BM, NT, DEPTH> stA;
    Stage<T, LB, BN, NT, DEPTH> stB;
    stA.init(la, tm * BM, kt0 * BK, tid, 0);
    stB.init(lb, tn * BN, kt0 * BK, tid, NT / 2);

    f32x16 acc[NB][MB];
    static_for<0, NB>([&](auto i) ASGD_INLINE { static_for<0, MB>([&](auto j) ASGD_INLINE { acc[i][j] = f32x16{}; }); });

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave % Cfg::WAVES_M) * (BM / Cfg::WAVES_M), wn = (wave / Cfg::WAVES_M) * (BN / Cfg::WAVES_N);
    FragOff<T, LA::kTrans, BM> foA;
    FragOff<T, LB::kTrans, BN> foB;
    foA.init(wm, lane);
    foB.init(wn, lane);
    // a wave whose whole tile lies outside C (96 output columns in a tile of 128: a quarter of the waves) only helps
    // to move the operands; wave-uniform
    const bool busy = __builtin_amdgcn_readfirstlane((tm * BM + wm < M && tn * BN + wn < N) ? 1 : 0) != 0;

    // register set that receives tile j is j % DEPTH (tile 0 goes through set 0 straight into LDS stage 0)
    stA.template load<0>(la); stB.template load<0>(lb);
    if constexpr (DEPTH == 2) { stA.template load<1>(la); stB.template load<1>(lb); }
    // every output row this thread writes has the same 8 columns: their bias is asked for behind the first tiles,
    // so that tile 0 does not wait for it (the parameters are cold in every cache, the tiles mostly are not)
    float bias8[8];
    load_bias8<T>(ep, tn * BN + (tid % (BN / 8)) * 8, bias8);
    stA.template store<0>(sA[0], tid); stB.template store<0>(sB[0], tid);
    // The loop body is two whole steps without a condition in it, so that the compiler knows exactly which fetches are
    // in flight at its head (with a conditional store it has to assume that those of two steps ago may be, and
    // waits for everything before it issues the next ones).  The store at the end of the last pair moves a tile that
    // exists only if the number of tiles is odd; otherwise it moves zeros that nobody reads.
    for (int i = nt >> 1; i > 0; --i) {
        // step t (even): multiply out of LDS stage 0, fetch tile t+DEPTH, then move tile t+1 into stage 1
        __syncthreads();
        stA.template load<0>(la); stB.template load<0>(lb);   // past the last tile this fetches zeros
        __builtin_amdgcn_s_setprio(1);   // the waves that multiply go first; those of the other workgroup are fetching or waiting
        if (busy) compute_tile<T, MB, NB>(sA[0], sB[0], acc, foA, foB);
        __builtin_amdgcn_s_setprio(0);
        stA.template store<DEPTH - 1>(sA[1], tid); stB.template store<DEPTH - 1>(sB[1], tid);
        // step t+1 (odd): multiply out of LDS stage 1, fetch tile t+1+DEPTH, then move tile t+2 into stage 0
        __syncthreads();
        stA.template load<DEPTH - 1>(la); stB.template load<DEPTH - 1>(lb);
        __builtin_amdgcn_s_setprio(1);
        if (busy) compute_tile<T, MB, NB>(sA[1], sB[1], acc, foA, foB);
        __builtin_amdgcn_s_setprio(0);
        stA.template store<0>(sA[0], tid); stB.template store<0>(sB[0], tid);
    }
    if (nt & 1) {
        __syncthreads();
        if (busy) compute_tile<T, MB, NB>(sA[0], sB[0], acc, foA, foB);
    }

    output_tile<T, Cfg, (int)sizeof(smem), Cfg::NT, LA::kTrans && LB::kTrans>(smem, acc, ep, tm, tn, split, M, N, ws, bias8, tid, wm, wn);
}

// gemm_kernel with the waves of a workgroup in two roles, as in conv_patch_ws_kernel further down: Cfg::NT / 64 waves read
// fragments and multiply (wave tiles of 64 x 64), four more fetch both operands and move them into LDS.  Step t of
// a fetching wave: after the barrier, tile t+1 (fetched two steps ago) goes from its register set into the LDS stage
// that was multiplied in step t-1, and the set is refilled with tile t+3.
constexpr int kFetchThreads = 256;
template <typename T, class Cfg, class LA, class LB>
__global__ __launch_bounds__(Cfg::NT + kFetchThreads, 2) void gemm_ws_kernel(LA la, LB lb, Epilogue ep, int M, int N, int nkt, int kt_per_split,
                                                                           int tiles_m, int tiles_n, float *ws)
{
    constexpr int BK = Geo<T>::BK, BM = Cfg::BM, BN = Cfg::BN, NT = Cfg::NT, MB = Cfg::MB, NB = Cfg::NB, NP = kFetchThreads;
    constexpr int TA = LA::kTrans ? TransTile<T, BM>::BYTES : BM * 128, TB = LB::kTrans ? TransTile<T, BN>::BYTES : BN * 128;
    __shared__ uint4 smem[2 * (TA + TB) / 16];   // two stages of A and B tiles; reused to stage the output
    uint4 (*sA)[TA / 16] = reinterpret_cast<uint4 (*)[TA / 16]>(smem);
    uint4 (*sB)[TB / 16] = reinterpret_cast<uint4 (*)[TB / 16]>(smem + 2 * TA / 16);
    const int tid = threadIdx.x;
    int bid;
    {
        const int nb = gridDim.x, q = nb >> 3, r = nb & 7, x = blockIdx.x & 7;
        bid = x * q + (x < r ? x : r) + (blockIdx.x >> 3);
    }
    const int tn = bid % tiles_n; bid /= tiles_n;
    const int tm = bid % tiles_m;
    const int split = bid / tiles_m;
    const int kt0 = split * kt_per_split;
    const int nt = min(nkt, kt0 + kt_per_split) - kt0;   // K tiles of this workgroup (>= 1)

    if (tid >= NT) {
        const int ptid = tid - NT;
        Stage<T, LA, BM, NP, 2> stA;
        Stage<T, LB, BN, NP, 2> stB;
        stA.init(la, tm * BM, kt0 * BK, ptid, 0);
        stB.init(lb, tn * BN, kt0 * BK, ptid, NP / 2);
        stA.template load<0>(la); stB.template load<0>(lb);
        stA.template load<1>(la); stB.template load<1>(lb);
        stA.template store<0>(sA[0], ptid); stB.template store<0>(sB[0], ptid);
        stA.template load<0>(la); stB.template load<0>(lb);
        for (int t = 0; t < nt; t += 2) {
            __syncthreads();
            if (t + 1 < nt) { stA.template store<1>(sA[1], ptid); stB.template store<1>(sB[1], ptid); }
            stA.template load<1>(la); stB.template load<1>(lb);   // past the last tile this fetches zeros
            if (t + 1 < nt) {
                __syncthreads();
                if (t + 2 < nt) { stA.template store<0>(sA[0], ptid); stB.template store<0>(sB[0], ptid); }
                stA.template load<0>(la); stB.template load<0>(lb);
            }
        }
        // A wave that has ended no longer counts at the barriers of the output phase.  (Letting these waves help to take
        // the tile out of LDS, as in the patch kernel, makes the filter gradient 3.5 % slower.)
        return;
    }

    f32x16 acc[NB][MB];
    static_for<0, NB>([&](auto i) ASGD_INLINE { static_for<0, MB>([&](auto j) ASGD_INLINE { acc[i][j] = f32x16{}; }); });
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave % Cfg::WAVES_M) * (BM / Cfg::WAVES_M), wn = (wave / Cfg::WAVES_M) * (BN / Cfg::WAVES_N);
    FragOff<T, LA::kTrans, BM> foA;
    FragOff<T, LB::kTrans, BN> foB;
    foA.init(wm, lane);
    foB.init(wn, lane);
    const bool busy = __builtin_amdgcn_readfirstlane((tm * BM + wm < M && tn * BN + wn < N) ? 1 : 0) != 0;
    float bias8[8];
    load_bias8<T>(ep, tn * BN + (tid % (BN / 8)) * 8, bias8);
    for (int t = 0; t < nt; t += 2) {
        __syncthreads();
        if (busy) compute_tile<T, MB, NB>(sA[0], sB[0], acc, foA, foB);
        if (t + 1 < nt) {
            __syncthreads();
            if (busy) compute_tile<T, MB, NB>(sA[1], sB[1], acc, foA, foB);
        }
    }
    output_tile<T, Cfg, (int)sizeof(smem)>(smem, acc, ep, tm, tn, split, M, N, ws, bias8, tid, wm, wn);
}

// ------------------------------------------------------------------ patch convolution
// Stride-1 convolutions whose output grid equals the input grid (and their data gradients, which have the
// same form).  With channel-last storage the input pixel that output pixel m needs at window position
// (ky, kx) is pixel m + (ky - pad) * W + (kx - pad) of the flattened tensor, whenever it is inside the image.
// So the 128 output pixels of a block tile need, for ALL window positions, one contiguous run of
// 128 + (kh-1) * W + (kw-1) input pixels.  The K loop therefore runs channel chunk by channel chunk (one
// chunk = one K tile = 128 bytes of channels): the run of pixels of the chunk (the patch) is brought into LDS
// once and serves the kh * kw K tiles of the chunk, the A fragment of a window position being the same LDS
// read at a shifted address.  Only the weights are fetched and written to LDS per K tile, which about halves
// what a workgroup pulls through the L2-to-CU path and takes a quarter off its LDS traffic compared with the
// im2col-style gather.  Window positions outside the image (zero padding, and rows past M) are handled per
// lane: its fragment address is redirected to a pixel of zeros kept behind the patch.  Pixels sit 144 bytes
// apart in LDS: 16 consecutive pixels' 16-byte pieces then fall into 16 different groups of four banks,
// whatever pixel the run starts at.
// A chunk is a whole K tile of channels (PPT = 1) or half a K tile (PPT = 2: a K tile then holds two window
// positions of the half-wide chunk, pixels sit 80 bytes apart).  Channel counts of 1.5, 2.5, ... K tiles
// (96 channels in 16-bit data) lose nothing in the second form, where the first would multiply a third more K
// tiles than there are.
template <int PPT> constexpr int kPatchPitch = PPT == 1 ? 144 : 80;

// The weights [rows][npos][C] as the B operand when K tiles enumerate (chunk, group of PPT window positions).
template <typename T, int PPT> struct ChunkK {
    static constexpr bool kTrans = false;
    static constexpr int CW = Geo<T>::BK / PPT;   // channels of a chunk
    Operand op; unsigned ldb, posb; int rows, C, npos, ntc;   // posb: bytes from one window position to the next; ntc: K tiles of a chunk
    FastDiv dntc;
    struct Row { unsigned off; };
    struct KPos { int pos, c; unsigned koff; };   // window position and channel of this thread's piece
    __device__ __forceinline__ Row row(int r) const { return Row{r < rows ? (unsigned)r * ldb : kInv}; }
    __device__ __forceinline__ unsigned off_of(int pos, int c) const
    {
        return (c < C && pos < npos) ? (unsigned)pos * posb + (unsigned)c * (unsigned)sizeof(T) : kInv;
    }
    // k = K tile * BK + element inside the tile
    __device__ __forceinline__ KPos kpos(int k) const
    {
        const int t = k / (int)Geo<T>::BK, e = k % (int)Geo<T>::BK;
        const int ch = (int)fdiv((uint32_t)t, dntc), pos = (t - ch * ntc) * PPT + e / CW, c = ch * CW + e % CW;
        return KPos{pos, c, off_of(pos, c)};
    }
    __device__ __forceinline__ void advance(KPos &kp, int) const
    {
        const bool wrap = kp.pos + PPT >= ntc * PPT;
        kp.pos = wrap ? kp.pos + PPT - ntc * PPT : kp.pos + PPT;
        kp.c += wrap ? CW : 0;
        kp.koff = off_of(kp.pos, kp.c);
    }
    __device__ __forceinline__ unsigned voff(const Row &r, const KPos &kp) const { return r.off + kp.koff; }
};

template <typename T> struct PatchSrc {
    Operand op; unsigned pix;              // bytes from one pixel to the next
    int H, W, C, kh, kw, pad, npos, ntc, M;   // ntc: K tiles of a chunk; M: pixels of the tensor = GEMM rows
    FastDiv dW, dHW, dkw, dntc;
};

template <typename T, int NPL, class Cfg, int PPT>
__global__ __launch_bounds__(Cfg::NT, Cfg::MINB) void conv_patch_kernel(PatchSrc<T> pa, ChunkK<T, PPT> lb, Epilogue ep, int M, int N, int nkt,
                                                                    int kt_per_split, int tiles_m, int tiles_n, float *ws)
{
    constexpr int BK = Geo<T>::BK, BM = Cfg::BM, BN = Cfg::BN, NT = Cfg::NT, MB = Cfg::MB, NB = Cfg::NB;
    constexpr int TB = BN * 128;
    constexpr int PIECES = 8 / PPT;                       // 16-byte pieces of a pixel's chunk
    constexpr int PITCH = kPatchPitch<PPT>;
    constexpr int CW = Geo<T>::BK / PPT;                  // channels of a chunk
    constexpr int PPMAX = NPL * NT / PIECES;              // pixels the patch buffer holds
    constexpr int ZBYTES = 256 + 128;                     // zeros behind them: one 16-byte piece per group of four banks, and the reach of a K tile's fragment offsets
    constexpr int PBYTES = PPMAX * PITCH + ZBYTES;
    static_assert((PPMAX * PITCH) % 256 == 0 && (2 * TB) % 256 == 0, "the zeros start at bank 0");
    static_assert(MB == 2 && BM == 128, "two row blocks per wave");
    constexpr int SMEM = (2 * TB + PBYTES) > BM * BN * 4 ? (2 * TB + PBYTES) : BM * BN * 4;
    __shared__ uint4 smem[SMEM / 16];        // two stages of B tiles, the patch; reused to stage the whole output tile
    uint4 (*sB)[TB / 16] = reinterpret_cast<uint4 (*)[TB / 16]>(smem);
    char *sP = reinterpret_cast<char *>(smem + 2 * TB / 16);
    const int tid = threadIdx.x;
    int bid;
    {
        const int nb = gridDim.x, q = nb >> 3, r = nb & 7, x = blockIdx.x & 7;
        bid = x * q + (x < r ? x : r) + (blockIdx.x >> 3);
    }
    const int tn = bid % tiles_n; bid /= tiles_n;
    const int tm = bid % tiles_m;
    const int split = bid / tiles_m;
    const int kt0 = split * kt_per_split;
    const int nt = min(nkt, kt0 + kt_per_split) - kt0;

    Stage<T, ChunkK<T, PPT>, BN, NT, 2> stB;
    stB.init(lb, tn * BN, kt0 * BK, tid, NT / 2);

    // chunk, first window position and its place in the window for the first K tile (all uniform)
    int ch = (int)fdiv((uint32_t)kt0, pa.dntc);
    int pos = (kt0 - ch * pa.ntc) * PPT;
    int ky = (int)fdiv((uint32_t)pos, pa.dkw), kx = pos - ky * pa.kw;

    // patch pieces of this thread: piece q = tid + j * NT is slot q % PIECES (= tid % PIECES) of patch pixel q / PIECES
    const __amdgpu_buffer_rsrc_t prs = pa.op.rsrc();
    const int slot = tid & (PIECES - 1);
    const int gp0 = tm * BM - pa.pad * pa.W - pa.pad + tid / PIECES;   // tensor pixel of piece 0
    unsigned poff[NPL];
    static_for<0, NPL>([&](auto j) ASGD_INLINE {
        const int gp = gp0 + j * (NT / PIECES);
        poff[j] = (gp >= 0 && gp < pa.M) ? (unsigned)gp * pa.pix + (unsigned)slot * 16u : kInv;
    });
    const unsigned pwo = (unsigned)((tid / PIECES) * PITCH + slot * 16);
    uint4 pr[NPL];
    auto patch_load = [&](int chunk) ASGD_INLINE {
        const unsigned coff = (chunk * CW + slot * (int)Geo<T>::CH < pa.C) ? (unsigned)chunk * (128u / PPT) : kInv;
        static_for<0, NPL>([&](auto j) ASGD_INLINE { pr[j] = buf_ld16(prs, poff[j] + coff); });
    };
    auto patch_store = [&]() ASGD_INLINE {
        static_for<0, NPL>([&](auto j) ASGD_INLINE {
            *reinterpret_cast<uint4 *>(sP + pwo + j * (NT / PIECES) * PITCH) = pr[j];
        });
    };

    f32x16 acc[NB][MB];
    static_for<0, NB>([&](auto i) ASGD_INLINE { static_for<0, MB>([&](auto j) ASGD_INLINE { acc[i][j] = f32x16{}; }); });

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave % Cfg::WAVES_M) * (BM / Cfg::WAVES_M), wn = (wave / Cfg::WAVES_M) * (BN / Cfg::WAVES_N);
    const int lrow = lane & 31, half = lane >> 5;
    FragOff<T, false, BN> foB;
    foB.init(wn, lane);
    // a wave whose whole tile lies outside C (96 output columns in a tile of 128: a quarter of the waves) only helps
    // to move the operands; wave-uniform
    const bool busy = __builtin_amdgcn_readfirstlane((tm * BM + wm < M && tn * BN + wn < N) ? 1 : 0) != 0;
    // the two fragment rows of this lane: patch address at window position (0, 0) and the mask of positions inside the image
    constexpr unsigned kHalfBytes = 8 * (unsigned)sizeof(T);
    // A lane whose window position lies outside the image reads zeros instead, at the address behind the patch
    // that falls into the same banks as the pixel it would have read: the lanes that read together hit different
    // banks among the pixels, and a single shared pixel of zeros would collide with one of them.
    constexpr unsigned zero_base = (unsigned)(PPMAX * PITCH);
    unsigned abase[2], amask[2];
    static_for<0, 2>([&](auto mb) ASGD_INLINE {
        const int rr = wm + mb * 32 + lrow, m = tm * BM + rr;
        abase[mb] = (unsigned)(rr * PITCH) + (unsigned)half * kHalfBytes;
        unsigned mask = 0;
        if (m < M) {
            const int n = (int)fdiv((uint32_t)m, pa.dHW);
            const int rem = m - n * (pa.H * pa.W);
            const int y = (int)fdiv((uint32_t)rem, pa.dW);
            const int y0 = y - pa.pad, x0 = rem - y * pa.W - pa.pad;
            const int ylo = max(0, -y0), yhi = max(ylo, min(pa.kh, pa.H - y0));
            const int xlo = max(0, -x0), xhi = max(xlo, min(pa.kw, pa.W - x0));
            const unsigned xm = ((1u << xhi) - 1u) & ~((1u << xlo) - 1u);
            for (int a = ylo; a < yhi; ++a) mask |= xm << (a * pa.kw);
        }
        amask[mb] = mask;
    });

    if (tid < ZBYTES / 16) *reinterpret_cast<uint4 *>(sP + PPMAX * PITCH + tid * 16) = make_uint4(0u, 0u, 0u, 0u);
    patch_load(ch);
    stB.template load<0>(lb);
    stB.template load<1>(lb);
    float bias8[8];   // asked for behind the first tiles, which therefore do not wait for it
    load_bias8<T>(ep, tn * BN + (tid % (BN / 8)) * 8, bias8);
    patch_store();
    stB.template store<0>(sB[0], tid);
    patch_load(ch + 1);

    // One K tile: the B pipeline is that of gemm_kernel; when a tile opens a new chunk, the patch fetched during
    // the previous chunk replaces the old one between two barriers and the fetch of the next one is issued.
    auto step = [&](auto par, bool first, bool more) ASGD_INLINE {
        __syncthreads();
        if (pos == 0 && !first) {
            patch_store();
            __syncthreads();
            ++ch;
            patch_load(ch + 1);
        }
        stB.template load<par>(lb);
        PatchOff<PPT> foA;
        static_for<0, PPT>([&](auto h) ASGD_INLINE {
            // a position past the last one (odd window sizes with two positions per tile) has no mask bit and no weights
            const unsigned sh = (unsigned)((ky * pa.W + kx) * PITCH);
            const unsigned a0 = abase[0] + sh, a1 = abase[1] + sh;
            foA.a[0][h] = ((amask[0] >> pos) & 1u) ? a0 : zero_base + (a0 & 0xF0u);
            foA.a[1][h] = ((amask[1] >> pos) & 1u) ? a1 : zero_base + (a1 & 0xF0u);
            ++pos; ++kx;
            if (kx == pa.kw) { kx = 0; ++ky; }
        });
        __builtin_amdgcn_s_setprio(1);
        if (busy) compute_tile<T, MB, NB>(reinterpret_cast<const uint4 *>(sP), sB[par], acc, foA, foB);
        __builtin_amdgcn_s_setprio(0);
        if (pos >= pa.npos) { pos = 0; ky = 0; kx = 0; }
        if (more) stB.template store<1 - par>(sB[1 - par], tid);
    };
    for (int t = 0; t < nt; t += 2) {
        step(std::integral_constant<int, 0>{}, t == 0, t + 1 < nt);
        if (t + 1 < nt) step(std::integral_constant<int, 1>{}, false, t + 2 < nt);
    }

    output_tile<T, Cfg, (int)sizeof(smem)>(smem, acc, ep, tm, tn, split, M, N, ws, bias8, tid, wm, wn);
}

// The same convolution with the waves of a workgroup in two roles: the first Cfg::NT / 64 waves read fragments and
// multiply, four more fetch the weights and the patch and move them into LDS.  The multiplying waves hold no
// staging registers and no fetch addresses, which leaves room for wave tiles of 64 x 64 (four multiplying waves
// on a 128 x 128 tile) at four waves per SIMD: a third fewer fragment reads from LDS than with 64 x 32, and the
// K loop gets 3-7 % faster.  Both kinds of wave go through the same barriers; the fetching waves end after the
// K loop and then help to take the output tile out of LDS.
//
// NSTG = 3: the weights do not pass through registers.  A fetching wave asks for its pieces with buffer loads that
// write LDS directly (lane l of the instruction fills bytes [16 l, 16 l + 16) behind a wave-uniform LDS address, so
// one instruction fills eight rows of a tile and the XOR swizzle is applied on the global side: the lane fetches the
// K piece that belongs into its slot).  Tile t lives in stage t % 3 and is asked for two steps ahead, right after the
// barrier that retires the stage's previous tile; before the barrier of step t the wave waits until at most the
// pieces of tile t + 1 are outstanding (the counter retires in order).  Against register staging this takes the
// fetched bytes off the return path into the register file and removes the LDS store instructions: in a loop of
// nothing but fragment reads, MFMAs and the fetch of a 16 KB tile per step, 0.60 instead of 0.81 us per step.
constexpr int kProducers = 256;
typedef __attribute__((address_space(3))) void lds_void;
// The barrier of a wave that has such loads in flight: its own LDS stores are waited for, the buffer loads are not
// (__syncthreads carries a release fence, for which the compiler drains every load that writes LDS); the "memory"
// clobber keeps the compiler from moving LDS accesses across it.
__device__ __forceinline__ void barrier_keep_loads() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
template <typename T, int NPL, class Cfg, int PPT, int NSTG>
__global__ __launch_bounds__(Cfg::NT + kProducers, 2) void conv_patch_ws_kernel(PatchSrc<T> pa, ChunkK<T, PPT> lb, Epilogue ep, int M, int N, int nkt,
                                                                              int kt_per_split, int tiles_m, int tiles_n, float *ws)
{
    constexpr int BK = Geo<T>::BK, BM = Cfg::BM, BN = Cfg::BN, NT = Cfg::NT, MB = Cfg::MB, NB = Cfg::NB, NP = kProducers;
    constexpr int TB = BN * 128;
    constexpr int PIECES = 8 / PPT;
    constexpr int PITCH = kPatchPitch<PPT>;
    constexpr int CW = Geo<T>::BK / PPT;
    constexpr int PPMAX = NPL * NP / PIECES;
    constexpr int ZBYTES = 256 + 128;
    constexpr int PBYTES = PPMAX * PITCH + ZBYTES;
    static_assert(NSTG == 2 || NSTG == 3, "B stages");
    static_assert((PPMAX * PITCH) % 256 == 0 && (NSTG * TB) % 256 == 0, "the zeros start at bank 0");
    static_assert(MB == 2 && BM == 128, "two row blocks per wave");
    constexpr int SMEM = (NSTG * TB + PBYTES) > BM * BN * 4 ? (NSTG * TB + PBYTES) : BM * BN * 4;
    static_assert(SMEM <= 81920, "two workgroups per CU");
    __shared__ uint4 smem[SMEM / 16];
    uint4 (*sB)[TB / 16] = reinterpret_cast<uint4 (*)[TB / 16]>(smem);
    char *sP = reinterpret_cast<char *>(smem + NSTG * TB / 16);
    const int tid = threadIdx.x;
    int bid;
    {
        const int nb = gridDim.x, q = nb >> 3, r = nb & 7, x = blockIdx.x & 7;
        bid = x * q + (x < r ? x : r) + (blockIdx.x >> 3);
    }
    const int tn = bid % tiles_n; bid /= tiles_n;
    const int tm = bid % tiles_m;
    const int split = bid / tiles_m;
    const int kt0 = split * kt_per_split;
    const int nt = min(nkt, kt0 + kt_per_split) - kt0;
    int ch = (int)fdiv((uint32_t)kt0, pa.dntc);
    int pos = (kt0 - ch * pa.ntc) * PPT;

    if (tid >= NT) {
        // ---- fetching waves.  Step t: after the barrier, tile t+1 (fetched two steps ago) goes from its register set
        // into the LDS stage that was multiplied in step t-1, and the set is refilled with tile t+3.
        const int ptid = tid - NT;
        Stage<T, ChunkK<T, PPT>, BN, NP, 2> stB;
        if constexpr (NSTG == 2) stB.init(lb, tn * BN, kt0 * BK, ptid, NP / 2);
        // NSTG == 3: instruction i = s * 4 + fw of a tile fills rows 8 i .. 8 i + 7 (lane l: row 8 i + l / 8, slot l % 8); the
        // slot holds K piece slot ^ swz(row), and swz(row) = (l / 8 ^ i) & 7 is the same for all s of one parity
        constexpr int SL = BN * 8 / NP;
        static_assert(NP == 256 && SL == 4, "four instructions per wave and tile");
        const int fw = __builtin_amdgcn_readfirstlane(ptid >> 6), fl = ptid & 63;
        typename ChunkK<T, PPT>::Row brow[SL];
        typename ChunkK<T, PPT>::KPos bkp[2];
        const __amdgpu_buffer_rsrc_t brs = lb.op.rsrc();
        if constexpr (NSTG == 3) {
            static_for<0, SL>([&](auto sl) ASGD_INLINE { brow[sl] = lb.row(tn * BN + (sl * 4 + fw) * 8 + (fl >> 3)); });
            const int piece = (fl & 7) ^ (((fl >> 3) ^ fw) & 7);
            bkp[0] = lb.kpos(kt0 * BK + piece * (int)Geo<T>::CH);
            bkp[1] = lb.kpos(kt0 * BK + (piece ^ 4) * (int)Geo<T>::CH);
        }
        auto issue = [&](auto stage) ASGD_INLINE {   // the tile at the cursor into LDS stage `stage`; advances the cursor
            static_for<0, SL>([&](auto sl) ASGD_INLINE {
                __builtin_amdgcn_raw_ptr_buffer_load_lds(brs, (lds_void *)(reinterpret_cast<char *>(smem) + stage * TB + (sl * 4 + fw) * 1024), 16,
                                                         (int)lb.voff(brow[sl], bkp[sl & 1]), 0, 0, 0);
            });
            lb.advance(bkp[0], BK); lb.advance(bkp[1], BK);
        };
        const __amdgpu_buffer_rsrc_t prs = pa.op.rsrc();
        const int slot = ptid & (PIECES - 1);
        const int gp0 = tm * BM - pa.pad * pa.W - pa.pad + ptid / PIECES;
        unsigned poff[NPL];
        static_for<0, NPL>([&](auto j) ASGD_INLINE {
            const int gp = gp0 + j * (NP / PIECES);
            poff[j] = (gp >= 0 && gp < pa.M) ? (unsigned)gp * pa.pix + (unsigned)slot * 16u : kInv;
        });
        const unsigned pwo = (unsigned)((ptid / PIECES) * PITCH + slot * 16);
        uint4 pr[NPL];
        auto patch_load = [&](int chunk) ASGD_INLINE {
            const unsigned coff = (chunk * CW + slot * (int)Geo<T>::CH < pa.C) ? (unsigned)chunk * (128u / PPT) : kInv;
            static_for<0, NPL>([&](auto j) ASGD_INLINE { pr[j] = buf_ld16(prs, poff[j] + coff); });
        };
        auto patch_store = [&]() ASGD_INLINE {
            static_for<0, NPL>([&](auto j) ASGD_INLINE {
                *reinterpret_cast<uint4 *>(sP + pwo + j * (NP / PIECES) * PITCH) = pr[j];
            });
        };
        if constexpr (NSTG == 3) {
            patch_load(ch);
            issue(std::integral_constant<int, 0>{});
            if (nt > 1) issue(std::integral_constant<int, 1>{});
            patch_store();
            patch_load(ch + 1);
            // step t: tile t must have landed (whatever was asked for after tile t + 1's pieces, i.e. nothing, may be
            // outstanding with them; a patch asked for in step t - 1 precedes them and is waited for too); after the
            // barrier the stage of tile t - 1 is free and takes tile t + 2
            auto step = [&](auto stage, int t) ASGD_INLINE {
                if (t + 1 < nt) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                barrier_keep_loads();
                if (pos == 0 && t != 0) {
                    patch_store();
                    barrier_keep_loads();
                    ++ch;
                    patch_load(ch + 1);
                }
                pos += PPT;
                if (pos >= pa.npos) pos = 0;
                if (t + 2 < nt) issue(std::integral_constant<int, (stage + 2) % 3>{});
            };
            for (int t = 0; t < nt; t += 3) {
                step(std::integral_constant<int, 0>{}, t);
                if (t + 1 < nt) step(std::integral_constant<int, 1>{}, t + 1);
                if (t + 2 < nt) step(std::integral_constant<int, 2>{}, t + 2);
            }
        } else {
        patch_load(ch);
        stB.template load<0>(lb);
        stB.template load<1>(lb);
        patch_store();
        stB.template store<0>(sB[0], ptid);
        stB.template load<0>(lb);
        patch_load(ch + 1);
        auto step = [&](auto par, bool first, bool more) ASGD_INLINE {
            __syncthreads();
            if (pos == 0 && !first) {
                patch_store();
                __syncthreads();
                ++ch;
                patch_load(ch + 1);
            }
            pos += PPT;
            if (pos >= pa.npos) pos = 0;
            if (more) stB.template store<1 - par>(sB[1 - par], ptid);
            stB.template load<1 - par>(lb);
        };
        for (int t = 0; t < nt; t += 2) {
            step(std::integral_constant<int, 0>{}, t == 0, t + 1 < nt);
            if (t + 1 < nt) step(std::integral_constant<int, 1>{}, false, t + 2 < nt);
        }
        }
            // the fetching waves help to take the output tile out of LDS
        float bias8[8];
        load_bias8<T>(ep, tn * BN + (tid % (BN / 8)) * 8, bias8);
        __syncthreads();
        __syncthreads();
        emit_tile<T, Cfg, NT + NP>(smem, ep, tm, tn, split, M, N, ws, bias8, tid);
        return;
    }

    // ---- multiplying waves
    int ky = (int)fdiv((uint32_t)pos, pa.dkw), kx = pos - ky * pa.kw;
    f32x16 acc[NB][MB];
    static_for<0, NB>([&](auto i) ASGD_INLINE { static_for<0, MB>([&](auto j) ASGD_INLINE { acc[i][j] = f32x16{}; }); });
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = (wave % Cfg::WAVES_M) * (BM / Cfg::WAVES_M), wn = (wave / Cfg::WAVES_M) * (BN / Cfg::WAVES_N);
    const int lrow = lane & 31, half = lane >> 5;
    FragOff<T, false, BN> foB;
    foB.init(wn, lane);
    const bool busy = __builtin_amdgcn_readfirstlane((tm * BM + wm < M && tn * BN + wn < N) ? 1 : 0) != 0;
    constexpr unsigned kHalfBytes = 8 * (unsigned)sizeof(T);
    constexpr unsigned zero_base = (unsigned)(PPMAX * PITCH);
    unsigned abase[2], amask[2];
    static_for<0, 2>([&](auto mb) ASGD_INLINE {
        const int rr = wm + mb * 32 + lrow, m = tm * BM + rr;
        abase[mb] = (unsigned)(rr * PITCH) + (unsigned)half * kHalfBytes;
        unsigned mask = 0;
        if (m < M) {
            const int n = (int)fdiv((uint32_t)m, pa.dHW);
            const int rem = m - n * (pa.H * pa.W);
            const int y = (int)fdiv((uint32_t)rem, pa.dW);
            const int y0 = y - pa.pad, x0 = rem - y * pa.W - pa.pad;
            const int ylo = max(0, -y0), yhi = max(ylo, min(pa.kh, pa.H - y0));
            const int xlo = max(0, -x0), xhi = max(xlo, min(pa.kw, pa.W - x0));
            const unsigned xm = ((1u << xhi) - 1u) & ~((1u << xlo) - 1u);
            for (int a = ylo; a < yhi; ++a) mask |= xm << (a * pa.kw);
        }
        amask[mb] = mask;
    });
    if (tid < ZBYTES / 16) *reinterpret_cast<uint4 *>(sP + PPMAX * PITCH + tid * 16) = make_uint4(0u, 0u, 0u, 0u);
    float bias8[8];
    load_bias8<T>(ep, tn * BN + (tid % (BN / 8)) * 8, bias8);
    auto step = [&](auto par, bool first) ASGD_INLINE {
        __syncthreads();
        if (pos == 0 && !first) __syncthreads();   // the fetching waves replace the patch between these two
        PatchOff<PPT> foA;
        static_for<0, PPT>([&](auto h) ASGD_INLINE {
            const unsigned sh = (unsigned)((ky * pa.W + kx) * PITCH);
            const unsigned a0 = abase[0] + sh, a1 = abase[1] + sh;
            foA.a[0][h] = ((amask[0] >> pos) & 1u) ? a0 : zero_base + (a0 & 0xF0u);
            foA.a[1][h] = ((amask[1] >> pos) & 1u) ? a1 : zero_base + (a1 & 0xF0u);
            ++pos; ++kx;
            if (kx == pa.kw) { kx = 0; ++ky; }
        });
        if (busy) compute_tile<T, MB, NB>(reinterpret_cast<const uint4 *>(sP), sB[par], acc, foA, foB);
        if (pos >= pa.npos) { pos = 0; ky = 0; kx = 0; }
    };
    if constexpr (NSTG == 3) {
        for (int t = 0; t < nt; t += 3) {
            step(std::integral_constant<int, 0>{}, t == 0);
            if (t + 1 < nt) step(std::integral_constant<int, 1>{}, false);
            if (t + 2 < nt) step(std::integral_constant<int, 2>{}, false);
        }
    } else {
        for (int t = 0; t < nt; t += 2) {
            step(std::integral_constant<int, 0>{}, t == 0);
            if (t + 1 < nt) step(std::integral_constant<int, 1>{}, false);
        }
    }
    output_tile<T, Cfg, (int)sizeof(smem), NT + NP>(smem, acc, ep, tm, tn, split, M, N, ws, bias8, tid, wm, wn);
}

// ------------------------------------------------------------------ first-layer convolution from staged image rows
// The window-row form of a first convolution (few input channels: a window row (kx, c) is one contiguous run of the
// bordered, channel-last image; K = (ky, j) with j over the padded run) has a short reduction (440 for 11 x 11 x 3)
// and a huge number of rows, so the tile engine above spends most of its time outside its seven-step K loop: every
// one of its 3025 workgroups fetches the same filters again, gathers an im2col tile that repeats every input element
// 7.6 times, and pays a head and an output phase.  This kernel keeps the whole filter bank in LDS for the lifetime
// of a workgroup (one per CU), walks over tiles of 128 output pixels of one image, and takes the A fragments
// straight from the image rows the tile needs (a contiguous block of the staged image, copied to LDS as it is): a
// lane's 8 consecutive K elements are 16 contiguous bytes of a window row, at byte offset
// (oy * stride + ky) * row_bytes + ox * stride * pixel_bytes + 2 j of the block.  There is no barrier inside the K
// loop.  Waves 0-3 multiply 64 x 32 blocks of the 128 x 96 tile, waves 4-7 32 x 32 blocks, which gives every SIMD
// three MFMA blocks.  The block of the next tile is fetched during the K loop of the current one; the output goes
// through LDS (the finished tile's block) so that a pixel's channels leave as 16-byte pieces.
struct RowsConv {
    Operand x; unsigned rowb, imgb;        // staged image: bytes per row (a multiple of 16) and per image
    unsigned pixstep;                      // bytes between the window origins of neighbouring output pixels (a multiple of 8)
    int Ho, Wo, stride, kh, KW, K;         // K = kh * KW; KW a multiple of 8
    int tiles_per_image, total, npix;      // npix = Ho * Wo
    Operand w; unsigned ldw;               // filters [N][K], bytes per row
    FastDiv dWo, dtpi, dKW;
};
constexpr int kRowsBM = 128, kRowsBN = 96, kRowsChunks = 7, kRowsPatchBytes = 32256, kRowsOutPitch = 208;

__global__ __launch_bounds__(512, 2) void conv_rows_kernel(RowsConv a, Epilogue ep, int N)
{
    typedef bf16_t T;
    constexpr int BM = kRowsBM, BN = kRowsBN, KC = kRowsChunks, PB = kRowsPatchBytes;
    constexpr int WBYTES = KC * BN * 128;                    // filters: [chunk][row][8 slots of 16 bytes], slots swizzled with the row
    __shared__ uint4 smem[(WBYTES + 2 * PB + 256) / 16];
    char *sW = reinterpret_cast<char *>(smem);
    char *sP = sW + WBYTES;                                  // two blocks of image rows
    constexpr unsigned kZero = (unsigned)(2 * PB);           // 256 bytes of zeros behind them (relative to sP)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lrow = lane & 31, half = lane >> 5;

    // ---- filters into LDS, once
    {
        const __amdgpu_buffer_rsrc_t rs = a.w.rsrc();
        for (int p = tid; p < KC * BN * 8; p += 512) {
            const int slot = p & 7, row = (p >> 3) % BN, chunk = (p >> 3) / BN;
            const int k = chunk * 64 + slot * 8;
            const unsigned off = (row < N && k < a.K) ? (unsigned)row * a.ldw + (unsigned)k * 2u : kInv;
            *reinterpret_cast<uint4 *>(sW + (chunk * BN + row) * 128 + ((slot ^ swz(row)) * 16)) = buf_ld16(rs, off);
        }
        if (tid < 16) *reinterpret_cast<uint4 *>(sP + kZero + tid * 16) = make_uint4(0u, 0u, 0u, 0u);
    }
    // ---- this wave's part of the tile
    const bool big = wave < 4;                               // 64 x 32 (two row blocks) or 32 x 32
    const int wm = big ? (wave & 1) * 64 : (wave - 4) * 32, wn = big ? (wave >> 1) * 32 : 64;
    FragOff<T, false, BN> foB;
    foB.init(wn, lane);
    // bias of this lane's 16 output columns: n = wn + 8 g + 4 half + j
    float bias[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int n = wn + 8 * (q >> 2) + 4 * half + (q & 3);
        bias[q] = (ep.bias && n < ep.bias_n) ? to_f32(static_cast<const T *>(ep.bias)[n]) : 0.f;
    }
    const __amdgpu_buffer_rsrc_t xrs = a.x.rsrc();
    // tile v of this workgroup -> (image, first pixel, first output row), and the block of image rows it needs
    auto decode = [&](int v, int &img, int &p0, int &oy0) ASGD_INLINE {
        const int q = a.total >> 3, r = a.total & 7, xx = v & 7;
        const int t = xx * q + (xx < r ? xx : r) + (v >> 3);     // each XCD gets a contiguous range of tiles
        img = (int)fdiv((uint32_t)t, a.dtpi);
        p0 = (t - img * a.tiles_per_image) * BM;
        oy0 = (int)fdiv((uint32_t)p0, a.dWo);
    };
    uint4 pr[4];                                             // the next tile's block on its way: 4 pieces of 16 bytes per thread
    auto block_load = [&](int v) ASGD_INLINE {
        int img, p0, oy0;
        decode(v, img, p0, oy0);
        const int p1 = min(p0 + BM, a.npix) - 1;
        const int rows = ((int)fdiv((uint32_t)p1, a.dWo) - oy0) * a.stride + a.kh;
        const unsigned src = (unsigned)img * a.imgb + (unsigned)(oy0 * a.stride) * a.rowb, bytes = (unsigned)rows * a.rowb;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned o = (unsigned)(tid + j * 512) * 16u;
            pr[j] = buf_ld16(xrs, o < bytes ? src + o : kInv);
        }
    };
    auto block_store = [&](int buf) ASGD_INLINE {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if ((tid + j * 512) * 16 < PB) *reinterpret_cast<uint4 *>(sP + buf * PB + (tid + j * 512) * 16) = pr[j];
    };

    int v = blockIdx.x;
    block_load(v);
    block_store(0);
    __syncthreads();
    for (int it = 0; v < a.total; ++it, v += gridDim.x) {
        const int buf = it & 1;
        const bool more = v + (int)gridDim.x < a.total;
        if (more) block_load(v + gridDim.x);                 // arrives during the K loop
        int img, p0, oy0;
        decode(v, img, p0, oy0);
        // the lane's rows of A: byte offset of the window origin inside the block, or nothing for rows past the image
        unsigned abase[2];
        bool aval[2];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            const int p = p0 + wm + mb * 32 + lrow;
            aval[mb] = p < a.npix && (mb == 0 || big);
            const int oy = (int)fdiv((uint32_t)min(p, a.npix - 1), a.dWo), ox = min(p, a.npix - 1) - oy * a.Wo;
            abase[mb] = (unsigned)(buf * PB) + (unsigned)((oy - oy0) * a.stride) * a.rowb + (unsigned)ox * a.pixstep;
        }
        f32x16 acc[2];
        acc[0] = f32x16{}; acc[1] = f32x16{};
        // K position of this lane's 8-element piece: (ky, j), advancing by 16 elements per K step.  The fragments of
        // K step s + 2 are asked for before the MFMAs of step s (three sets of fragment registers): a wave has only
        // one or two MFMAs per step, too few to hide the LDS latency of the step after it.
        int ky = 0, j = half * 8;
        if (j >= a.KW) { j -= a.KW; ky = 1; }
        Frag<T> fb[3], fa[3][2];
        auto issue = [&](auto sidx) ASGD_INLINE {
            constexpr int S = decltype(sidx)::value, SET = S % 3;
            const bool kval = ky < a.kh;
            const unsigned koff = (unsigned)ky * a.rowb + (unsigned)j * 2u;
            fb[SET].v = *reinterpret_cast<const uint4 *>(sW + (S / 4) * (BN * 128) + foB.o[S % 4][0]);
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                if (mb == 0 || big) {
                    const unsigned ad = (kval && aval[mb]) ? abase[mb] + koff : kZero;
                    const uint2 lo = *reinterpret_cast<const uint2 *>(sP + ad), hi = *reinterpret_cast<const uint2 *>(sP + ad + 8);
                    fa[SET][mb].v = make_uint4(lo.x, lo.y, hi.x, hi.y);
                }
            }
            j += 16;
            if (j >= a.KW) { j -= a.KW; ++ky; }
            if (j >= a.KW) { j -= a.KW; ++ky; }               // KW >= 8: at most two window rows per step
        };
        issue(std::integral_constant<int, 0>{});
        issue(std::integral_constant<int, 1>{});
        static_for<0, KC * 4>([&](auto sidx) ASGD_INLINE {
            constexpr int S = decltype(sidx)::value, SET = S % 3;
            if constexpr (S + 2 < KC * 4) issue(std::integral_constant<int, S + 2>{});
            mma(acc[0], fb[SET], fa[SET][0]);
            if (big) mma(acc[1], fb[SET], fa[SET][1]);
        });
        __syncthreads();                                     // every wave has read its fragments: the block becomes the output stage
        char *so = sP + buf * PB;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            if (mb == 0 || big) {
                const int row = wm + mb * 32 + lrow;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    union { bf16_t h[4]; uint2 u; } o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float x = acc[mb][4 * g + e] + bias[4 * g + e];
                        if (ep.relu) x = x > 0.f ? x : 0.f;
                        o.h[e] = (bf16_t)x;
                    }
                    *reinterpret_cast<uint2 *>(so + row * kRowsOutPitch + (wn + 8 * g + 4 * half) * 2) = o.u;
                }
            }
        }
        __syncthreads();
        {   // a pixel's N channels leave as 16-byte pieces: 12 pieces per row of the 96 columns
            const long pix0 = (long)img * a.npix + p0;
            const int valid = min(BM, a.npix - p0), pieces = N / 8;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const int e = tid + r * 512, row = e / 12, piece = e - row * 12;
                if (row < valid && piece < pieces)
                    *reinterpret_cast<uint4 *>(static_cast<char *>(ep.out) + ((pix0 + row) * ep.ld + piece * 8) * 2) =
                        *reinterpret_cast<const uint4 *>(so + row * kRowsOutPitch + piece * 16);
            }
        }
        if (more) block_store(buf ^ 1);                      // the other block: its tile's output left an iteration ago
        __syncthreads();
    }
}


// ------------------------------------------------------------------ first-layer filter gradient from staged image rows
// dW[cout][(ky, j)] = sum over output pixels of dY[pixel][cout] * window row element (ky, j) of that pixel: the
// reduction runs over the pixels, of which there are hundreds of thousands, and the result is tiny (96 x 440).  The
// tile engine splits it 128 ways, multiplies a quarter of its 128 x 512 padded tiles for nothing and gathers the
// im2col operand from memory again for every column tile.  Here a persistent workgroup (one per CU) walks over tiles
// of whole output rows of one image (up to 112 pixels) and keeps the whole 96 x 448 result in the accumulators of six waves (two
// or three blocks of 32 K columns each, all three blocks of output channels: 96 or 144 accumulator registers).  Both operands
// are read with transposing LDS reads, in which every lane supplies its own address: the dY tile is stored pixel by
// pixel (256-byte lines, the 64-byte group index XOR-ed with the line so that the four lines of a read fall into
// different banks), and the window-row elements come straight out of the block of image rows the tile touches,
// copied to LDS as it is (lane's K line = pixel: the byte offset of its window origin; lane's row piece = four
// consecutive K columns: ky * row_bytes + 2 j).  Two more waves do nothing but bring in the image rows and the dY tiles
// of the tiles to come with buffer loads that write LDS directly, three buffers each and two tiles ahead (with one tile of
// lead the period of a tile was the issue time of its 64 loads plus their latency, 3.2 us against 1.3 us of MFMAs),
// one barrier per tile.  Every workgroup leaves one partial result; the ordered split-K reduction adds them and
// scatters to canonical order.
constexpr int kRowsWgBN = 448, kRowsWgTP = 112, kRowsWgIB = 22528, kRowsWgDB = kRowsWgTP * 256, kRowsWgGrid = 256;

// rpt: output rows per tile (rpt * Wo <= kRowsWgTP pixels); a.tiles_per_image = ceil(Ho / rpt)
__global__ __launch_bounds__(512, 2) void conv_rows_wgrad_kernel(RowsConv a, int rpt, Operand dy, unsigned ldyb, int M, float *ws)
{
    typedef bf16_t T;
    constexpr int TP = kRowsWgTP, IB = kRowsWgIB, DB = kRowsWgDB, NI = IB / 1024, ND = DB / 1024;
    static_assert(NI <= 31 && ND <= 31, "two tiles of one wave's loads fit the six-bit in-order wait counter");
    __shared__ uint4 smem[(3 * IB + 3 * DB) / 16];
    char *sP = reinterpret_cast<char *>(smem);          // three blocks of image rows
    char *sD = sP + 3 * IB;                             // three dY tiles: TP lines of 256 bytes
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    auto decode = [&](int v, int &img, int &r0) ASGD_INLINE {
        const int q = a.total >> 3, r = a.total & 7, xx = v & 7;
        const int t = xx * q + (xx < r ? xx : r) + (v >> 3);     // each XCD gets a contiguous range of tiles
        img = (int)fdiv((uint32_t)t, a.dtpi);
        r0 = (t - img * a.tiles_per_image) * rpt;                // first output row of the tile
    };

    if (wave >= 6) {
        // ---- the two fetching waves (wave 6: image rows, wave 7: dY): tile `it` goes to buffers it % 3, two tiles ahead of
        // the multiplying waves.  One wave can have 63 loads (63 KB) in flight, less than a tile period needs.
        const __amdgpu_buffer_rsrc_t xrs = a.x.rsrc(), drs = dy.rsrc();
        // dY: instruction i fills lines 4 i .. 4 i + 3; lane l: line 4 i + l / 16, physical 16-byte slot l % 16, which holds
        // logical slot ((l % 16 / 4) ^ (line & 3)) * 4 + l % 4 of the pixel's row (line & 3 = l / 16)
        const int dline = lane >> 4, dslot = ((((lane & 15) >> 2) ^ dline) << 2) | (lane & 3);
        const bool dcol = dslot * 8 < M;
        const bool rows_wave = wave == 6;
        auto issue = [&](int v, int buf) ASGD_INLINE {   // always NI (or ND) instructions: the wait below counts them
            int img, r0;
            decode(v, img, r0);
            const int rows_out = min(rpt, a.Ho - r0);
            if (rows_wave) {
                const unsigned src = (unsigned)img * a.imgb + (unsigned)(r0 * a.stride) * a.rowb;
                const unsigned bytes = (unsigned)((rows_out - 1) * a.stride + a.kh) * a.rowb;
#pragma unroll 2
                for (int i = 0; i < NI; ++i) {
                    const unsigned o = (unsigned)(i * 64 + lane) * 16u;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(xrs, (lds_void *)(sP + buf * IB + i * 1024), 16, (int)(o < bytes ? src + o : kInv), 0, 0, 0);
                }
            } else {
                const int valid = rows_out * a.Wo;
                const unsigned dsrc = (unsigned)(img * a.npix + r0 * a.Wo) * ldyb + (unsigned)dslot * 16u;
#pragma unroll 2
                for (int i = 0; i < ND; ++i) {
                    const int line = i * 4 + dline;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(drs, (lds_void *)(sD + buf * DB + i * 1024), 16,
                                                             (int)((dcol && line < valid) ? dsrc + (unsigned)line * ldyb : kInv), 0, 0, 0);
                }
            }
        };
        int v = blockIdx.x;
        const int g = (int)gridDim.x;
        issue(v, 0);
        if (v + g < a.total) issue(v + g, 1);
        int buf2 = 2;                                        // buffer of tile it + 2
        for (int it = 0; v < a.total; ++it, v += g) {
            // tile `it` has landed when at most the next tile's instructions are outstanding (the counter retires in order)
            if (v + g >= a.total) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            else if (rows_wave) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NI) : "memory");
            else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(ND) : "memory");
            barrier_keep_loads();                            // ... and the buffers of tile it - 1 have been read to the end
            if (v + 2 * g < a.total) issue(v + 2 * g, buf2);
            buf2 = buf2 == 2 ? 0 : buf2 + 1;
        }
        return;
    }

    // ---- multiplying waves, all three blocks of output channels each.  Waves 0, 1, 4, 5 (two to a SIMD) own two blocks of
    // 32 K columns, waves 2 and 3 (which share their SIMDs with the fetching waves) three: 12 / 12 / 9 / 9 MFMAs per
    // K step on the four SIMDs.
    const int b4 = lane >> 4, i16 = lane & 15, lrow = lane & 31, half = lane >> 5;
    // A (dY tile): lane supplies K line 8 (b4 / 2) + i16 / 4 (+ 4) of the K step, channels mb * 32 + 16 (b4 & 1) + 4 (i16 & 3) ..+3
    unsigned aoff[3];
    static_for<0, 3>([&](auto mb) ASGD_INLINE {
        aoff[mb] = (unsigned)((8 * (b4 >> 1) + (i16 >> 2)) * 256 + ((mb ^ (i16 >> 2)) << 6) + 32 * (b4 & 1) + 8 * (i16 & 3));
    });
    // B (image rows): lane supplies the pixel of the same K line and K columns n .. n + 3.  The window origins of the
    // tile's pixels relative to its block of rows are the same for every tile (a tile is whole output rows).
    const int tp = rpt * a.Wo;                           // pixels of a full tile
    unsigned org[TP / 16][2];
    static_for<0, TP / 16>([&](auto ks) ASGD_INLINE {
        static_for<0, 2>([&](auto h) ASGD_INLINE {
            const int p = min(ks * 16 + 8 * (b4 >> 1) + (i16 >> 2) + 4 * h, tp - 1);   // lines past the tile hold zeros in dY
            const int oy = (int)fdiv((uint32_t)p, a.dWo), ox = p - oy * a.Wo;
            org[ks][h] = (unsigned)(oy * a.stride) * a.rowb + (unsigned)ox * a.pixstep;
        });
    });
    typedef __attribute__((address_space(3))) short4v lds_s4;
    auto tr_read = [&](const char *p0, const char *p1) ASGD_INLINE -> Frag<T> {
        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4 *)(p0));
        const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4 *)(p1));
        const uint2 x = __builtin_bit_cast(uint2, lo), y = __builtin_bit_cast(uint2, hi);
        Frag<T> f;
        f.v = make_uint4(x.x, x.y, y.x, y.y);
        return f;
    };
    auto body = [&](auto nbw, int nb0) ASGD_INLINE {     // this wave's NBW blocks of K columns start at block nb0
        constexpr int NBW = decltype(nbw)::value;
        unsigned coff[NBW];
        static_for<0, NBW>([&](auto nb) ASGD_INLINE {
            int n = (nb0 + nb) * 32 + 16 * (b4 & 1) + 4 * (i16 & 3);
            n = min(n, a.K - 4);                         // columns past K: any valid address (their sums are not stored)
            const int ky = (int)fdiv((uint32_t)n, a.dKW);
            coff[nb] = (unsigned)ky * a.rowb + (unsigned)(n - ky * a.KW) * 2u;
        });
        f32x16 acc[NBW][3];
        static_for<0, NBW>([&](auto i) ASGD_INLINE { static_for<0, 3>([&](auto j) ASGD_INLINE { acc[i][j] = f32x16{}; }); });
        int buf = 0;
        for (int v = blockIdx.x; v < a.total; v += gridDim.x) {
            __syncthreads();
            const char *pa = sD + buf * DB, *pb = sP + buf * IB;
            // all TP / 16 K steps, whatever the tile holds (lines past its pixels are zeros in dY); the fragments of step
            // ks + 1 are asked for before the MFMAs of step ks
            Frag<T> fa[2][3], fb[2][NBW];
            auto frags = [&](auto ks) ASGD_INLINE {
                constexpr int S = decltype(ks)::value, SET = S & 1;
                static_for<0, 3>([&](auto mb) ASGD_INLINE { fa[SET][mb] = tr_read(pa + aoff[mb] + S * 16 * 256, pa + aoff[mb] + S * 16 * 256 + 4 * 256); });
                static_for<0, NBW>([&](auto nb) ASGD_INLINE { fb[SET][nb] = tr_read(pb + org[S][0] + coff[nb], pb + org[S][1] + coff[nb]); });
            };
            frags(std::integral_constant<int, 0>{});
            static_for<0, TP / 16>([&](auto ks) ASGD_INLINE {
                constexpr int S = decltype(ks)::value, SET = S & 1;
                if constexpr (S + 1 < TP / 16) frags(std::integral_constant<int, S + 1>{});
                static_for<0, NBW>([&](auto nb) ASGD_INLINE { static_for<0, 3>([&](auto mb) ASGD_INLINE { mma(acc[nb][mb], fb[SET][nb], fa[SET][mb]); }); });
            });
            buf = buf == 2 ? 0 : buf + 1;
        }
        // this workgroup's partial result: ws[block][m][n], n < K
        float *o = ws + (size_t)blockIdx.x * (size_t)M * (size_t)a.K;
        static_for<0, NBW>([&](auto nb) ASGD_INLINE {
            static_for<0, 3>([&](auto mb) ASGD_INLINE {
                const int m = mb * 32 + lrow;
                static_for<0, 4>([&](auto g) ASGD_INLINE {
                    const int n = (nb0 + nb) * 32 + 8 * g + 4 * half;
                    if (m < M && n < a.K)
                        *reinterpret_cast<f32x4 *>(o + (size_t)m * a.K + n) = f32x4{acc[nb][mb][4 * g], acc[nb][mb][4 * g + 1], acc[nb][mb][4 * g + 2], acc[nb][mb][4 * g + 3]};
                });
            });
        });
    };
    if (wave == 2 || wave == 3) body(std::integral_constant<int, 3>{}, 8 + (wave - 2) * 3);
    else body(std::integral_constant<int, 2>{}, (wave < 2 ? wave : wave - 2) * 2);
}

template <typename T> __global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *ws, int splits, Epilogue ep, int M, int N)
{
    const long g = (long)blockIdx.x * 256 + threadIdx.x;
    const int n8 = N / 8;
    if (g >= (long)M * n8) return;
    const int m = (int)(g / n8), n0 = (int)(g - (long)m * n8) * 8;
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const long stride = (long)M * N;
    const float *p0 = ws + (long)m * N + n0;
    int s = 0;
    for (; s + 4 <= splits; s += 4) {   // four partials in flight; added in split order all the same
        float4 a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float4 *p = reinterpret_cast<const float4 *>(p0 + (s + u) * stride);
            a[u] = p[0]; b[u] = p[1];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            v[0] += a[u].x; v[1] += a[u].y; v[2] += a[u].z; v[3] += a[u].w;
            v[4] += b[u].x; v[5] += b[u].y; v[6] += b[u].z; v[7] += b[u].w;
        }
    }
    for (; s < splits; ++s) {
        const float4 *p = reinterpret_cast<const float4 *>(p0 + s * stride);
        const float4 a = p[0], b = p[1];
        v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w;
        v[4] += b.x; v[5] += b.y; v[6] += b.z; v[7] += b.w;
    }
    float b8[8];
    load_bias8<T>(ep, n0, b8);
    epilogue8<T>(ep, m, n0, v, b8);
}

// The same for few outputs and many partial sums (the first layer's filter gradient: 5280 groups of 8 outputs, up
// to 256 partials each): L = 8 or 32 neighbouring lanes share a group, lane l adds partials l, l+L, ... in that order, and
// the L sums are combined in a fixed butterfly, so the result does not depend on anything but the inputs.
template <typename T, int L> __global__ __launch_bounds__(256) void splitk_reduce_wide_kernel(const float *ws, int splits, Epilogue ep, int M, int N)
{
    static_assert(L == 8 || L == 32, "lanes per group of outputs");
    constexpr int SH = L == 8 ? 3 : 5;
    const long g = ((long)blockIdx.x * 256 + threadIdx.x) >> SH;
    const int l = threadIdx.x & (L - 1);
    const int n8 = N / 8;
    const bool live = g < (long)M * n8;   // whole groups of L lanes are live or not; all lanes take part in the shuffles
    const long gg = live ? g : 0;
    const int m = (int)(gg / n8), n0 = (int)(gg - (long)m * n8) * 8;
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const long stride = (long)M * N;
    const float *p0 = ws + (long)m * N + n0;
    int s = l;
    for (; s + 3 * L < splits; s += 4 * L) {   // four partials in flight
        float4 a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float4 *p = reinterpret_cast<const float4 *>(p0 + (s + L * u) * stride);
            a[u] = p[0]; b[u] = p[1];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            v[0] += a[u].x; v[1] += a[u].y; v[2] += a[u].z; v[3] += a[u].w;
            v[4] += b[u].x; v[5] += b[u].y; v[6] += b[u].z; v[7] += b[u].w;
        }
    }
    for (; s < splits; s += L) {
        const float4 *p = reinterpret_cast<const float4 *>(p0 + s * stride);
        const float4 a = p[0], b = p[1];
        v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w;
        v[4] += b.x; v[5] += b.y; v[6] += b.z; v[7] += b.w;
    }
#pragma unroll
    for (int d = 1; d < L; d <<= 1) {
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] += __shfl_xor(v[r], d, L);
    }
    if (!live || l != 0) return;
    float b8[8];
    load_bias8<T>(ep, n0, b8);
    epilogue8<T>(ep, m, n0, v, b8);
}

// the reduction that follows a split GEMM
template <typename T> static void launch_splitk_reduce(const float *ws, int splits, const Epilogue &ep, int M, int N, hipStream_t s)
{
    const long groups = (long)M * (N / 8);
    if (splits >= 192 && groups < 8192)      // one partial per CU (the first-layer filter gradient): 32 lanes share a group, two rounds of reads each
        hipLaunchKernelGGL((splitk_reduce_wide_kernel<T, 32>), dim3((unsigned)((groups * 32 + 255) / 256)), dim3(256), 0, s, ws, splits, ep, M, N);
    else if (splits >= 16 && groups < 32768)
        hipLaunchKernelGGL((splitk_reduce_wide_kernel<T, 8>), dim3((unsigned)((groups * 8 + 255) / 256)), dim3(256), 0, s, ws, splits, ep, M, N);
    else
        hipLaunchKernelGGL((splitk_reduce_kernel<T>), dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, s, ws, splits, ep, M, N);
}

// ------------------------------------------------------------------ host side
GemmPlan plan_gemm(long M, long N, long K, int dtype, int max_splits)
{
    const int BK = dtype == kBF16 ? (int)Geo<bf16_t>::BK : (int)Geo<float>::BK;
    const int BM = Cfg128::BM, BN = Cfg128::BN;
    const long tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    const long nkt = (K + BK - 1) / BK;
    // A single row of tiles with a moderate K (the FC layers at batch <= 128) is bound by the partial sums it
    // writes and re-reads: one workgroup per CU with a deeper K range each beats two with half of it.
    const long target = (M <= BM && nkt <= 256) ? 256 : 512;
    long splits = 1;
    if (max_splits > 1 && tiles < target) {
        splits = target / tiles;                  // never more workgroups than run at once: a second, nearly empty round would double the time
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

template <typename T, class Cfg, class LA, class LB>
static int run_tile(const LA &la, const LB &lb, int M, int N, int K, const Epilogue &ep, const GemmPlan &plan, float *ws, hipStream_t s)
{
    constexpr int BK = Geo<T>::BK, BM = Cfg::BM, BN = Cfg::BN;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int nkt = (K + BK - 1) / BK;
    int splits = plan.splits;
    if (splits > 1 && ws == nullptr) return -1;
    const int per = (nkt + splits - 1) / splits;
    splits = (nkt + per - 1) / per;
    const long blocks = (long)tiles_m * tiles_n * splits;
    if (blocks > 0x7fffffffL) return -1;
    // The convolution filter gradient runs with fetching and multiplying waves (gemm_ws_kernel: -2.6 % in bf16, -4 % in
    // fp32 for the class); the im2col forward gather of the first layer is 12 % slower that way (seven K tiles: the
    // head of a workgroup weighs more than its loop) and stays as it is.
    if constexpr (std::is_same<LB, GatherT<T>>::value)
        hipLaunchKernelGGL((gemm_ws_kernel<T, Cfg128, LA, LB>), dim3((unsigned)blocks), dim3(Cfg128::NT + kFetchThreads), 0, s, la, lb, ep, M, N, nkt,
                           per, tiles_m, tiles_n, splits > 1 ? ws : nullptr);
    else
        hipLaunchKernelGGL((gemm_kernel<T, Cfg, LA, LB>), dim3((unsigned)blocks), dim3(Cfg::NT), 0, s, la, lb, ep, M, N, nkt, per, tiles_m,
                           tiles_n, splits > 1 ? ws : nullptr);
    if (splits > 1) launch_splitk_reduce<T>(ws, splits, ep, M, N, s);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <typename T, class LA, class LB>
static int run(const LA &la, const LB &lb, int M, int N, int K, const Epilogue &ep, const GemmPlan &plan, float *ws, hipStream_t s)
{
    if (M <= 0 || N <= 0 || K <= 0 || (N & 7)) return -1;
    if (la.op.bytes == 0 || lb.op.bytes == 0) return -1;   // an operand beyond the 1 GiB the 32-bit offsets cover
    // Measured on the AlexNet-style shapes: the 8-wave form (four waves per SIMD hide more latency) wins everywhere
    // except the fp32 convolution filter gradient, whose two transposing operands cost eight 4-byte LDS reads per
    // fragment: the wider wave tile of the 4-wave form needs a third fewer of them.  (In bf16 the 4-wave form was
    // ahead there too until the multiplying waves got their raised priority.)
    if constexpr (std::is_same<LB, GatherT<T>>::value && sizeof(T) == 4) return run_tile<T, Cfg128>(la, lb, M, N, K, ep, plan, ws, s);
    else return run_tile<T, Cfg128w8>(la, lb, M, N, K, ep, plan, ws, s);
}

static Operand operand(const void *p, size_t bytes) { return Operand{p, bytes <= kMaxOperandBytes ? (unsigned)bytes : 0u}; }

template <typename T, bool WIDE> static GatherK<T, WIDE> make_gather_k(const Gather &g)
{
    GatherK<T, WIDE> l;
    l.op = operand(g.x, g.bytes);
    l.pix = g.pix ? (unsigned)g.pix : (unsigned)(g.C * sizeof(T)); l.rowb = g.rowb ? (unsigned)g.rowb : (unsigned)(g.W * g.C * sizeof(T));
    l.H = g.H; l.W = g.W; l.C = g.C; l.Ho = g.Ho; l.Wo = g.Wo; l.kh = g.kh; l.kw = g.kw;
    l.sm = g.sm; l.pad = g.pad; l.M = g.N * g.Ho * g.Wo;
    l.adv_px = (int)Geo<T>::BK / g.C; l.adv_c = (int)Geo<T>::BK % g.C;
    l.dWo = make_fastdiv(g.Wo); l.dHoWo = make_fastdiv(g.Ho * g.Wo); l.dC = make_fastdiv(g.C); l.dkw = make_fastdiv(g.kw);
    return l;
}
template <typename T> static GatherKS<T> make_gather_ks(const Gather &g)
{
    GatherKS<T> l;
    l.op = operand(g.x, g.bytes);
    l.pix = g.pix ? (unsigned)g.pix : (unsigned)(g.C * sizeof(T));
    l.H = g.H; l.W = g.W; l.C = g.C; l.Ho = g.Ho; l.Wo = g.Wo; l.kh = g.kh; l.kw = g.kw;
    l.sm = g.sm; l.ds = g.ds; l.pad = g.pad; l.M = g.N * g.Ho * g.Wo;
    l.dWo = make_fastdiv(g.Wo); l.dHoWo = make_fastdiv(g.Ho * g.Wo); l.dC = make_fastdiv(g.C); l.dkw = make_fastdiv(g.kw);
    return l;
}
template <typename T> static GatherT<T> make_gather_t(const Gather &g)
{
    GatherT<T> l;
    l.op = operand(g.x, g.bytes);
    l.pix = g.pix ? (unsigned)g.pix : (unsigned)(g.C * sizeof(T)); l.rowb = g.rowb ? (unsigned)g.rowb : (unsigned)(g.W * g.C * sizeof(T));
    l.H = g.H; l.W = g.W; l.C = g.C; l.Ho = g.Ho; l.Wo = g.Wo; l.kh = g.kh; l.kw = g.kw;
    l.sm = g.sm; l.pad = g.pad; l.M = g.N * g.Ho * g.Wo; l.Krows = g.kh * g.kw * g.C;
    l.dWo = make_fastdiv(g.Wo); l.dHo = make_fastdiv(g.Ho); l.dHoWo = make_fastdiv(g.Ho * g.Wo); l.dC = make_fastdiv(g.C); l.dkw = make_fastdiv(g.kw);
    return l;
}
// [rows][ld] with K contiguous / [K][ld] with the rows contiguous; the byte range ends with the last element used
template <typename T> static PlainK<T> make_plain_k(const void *p, long ld, int rows, int K)
{
    return PlainK<T>{operand(p, ((size_t)(rows - 1) * ld + K) * sizeof(T)), (unsigned)(ld * sizeof(T)), rows, K};
}
template <typename T> static PlainT<T> make_plain_t(const void *p, long ld, int rows, int K)
{
    return PlainT<T>{operand(p, ((size_t)(K - 1) * ld + rows) * sizeof(T)), (unsigned)(ld * sizeof(T)), rows, K};
}

// The patch form applies to stride-1 convolutions with equal input and output grids over a dense tensor whose
// run of pixels per block tile fits the patch buffer.  Returns the window positions per K tile to run it with
// (1 or 2), or 0 where the im2col gather is the better choice.
template <typename T> static int patch_applies(const Gather &a, long ldb)
{
    const size_t pixb = a.pix ? a.pix : (size_t)a.C * sizeof(T);
    const int npos = a.kh * a.kw;
    if (!(a.sm == 1 && a.ds == 1 && a.Ho == a.H && a.Wo == a.W && npos > 1 && npos <= 32 && 2 * a.pad == a.kh - 1 &&
                 2 * a.pad == a.kw - 1 && (a.rowb == 0 || a.rowb == (size_t)a.W * pixb) && pixb % 16 == 0 && a.C % (int)Geo<T>::CH == 0 &&
                 ((uintptr_t)a.x & 15) == 0 && ldb == (long)npos * a.C && 128 + (a.kh - 1) * a.W + a.kw - 1 <= 256))
        return 0;
    // A chunk is a whole K tile of channels, or half of one with two window positions per K tile.  Where the
    // channel count is not a multiple of the chunk the patch form multiplies more K tiles than the gather, which
    // packs K densely; beyond 15 % more it loses.  (96 channels in 16-bit data, 5 x 5: 38 K tiles dense, 50 with
    // whole-tile chunks, 39 with half-tile chunks.)
    const int BK = (int)Geo<T>::BK;
    const long nkt_gather = ((long)npos * a.C + BK - 1) / BK;
    const long nkt1 = (long)((a.C + BK - 1) / BK) * npos, nkt2 = (long)((a.C + BK / 2 - 1) / (BK / 2)) * ((npos + 1) / 2);
    const int ppt = nkt2 < nkt1 ? 2 : 1;
    return (ppt == 1 ? nkt1 : nkt2) * 100 <= nkt_gather * 115 ? ppt : 0;
}

template <typename T, class Cfg, int PPT>
static int run_patch_cfg(const Gather &a, const void *b, long ldb, int N, const Epilogue &ep, const GemmPlan &plan, float *ws, hipStream_t s);
template <typename T, int PPT>
static int run_patch(const Gather &a, const void *b, long ldb, int N, const Epilogue &ep, const GemmPlan &plan, float *ws, hipStream_t s)
{
    // Both shapes run wave tiles of 64 x 32 at four waves per SIMD and take the same time per tile; the narrow one
    // fills the chip better when the wide one would leave more than an eighth of the 512 workgroup slots empty
    // (conv5 at batch 128: 338 workgroups against 676).
    // The narrow one holds runs of up to 160 pixels (more pieces per thread cost it its fourth wave per SIMD).
    const long wide = (long)((a.N * a.H * a.W + 127) / 128) * ((N + 127) / 128) * plan.splits;
    const int pp = 128 + (a.kh - 1) * a.W + a.kw - 1;
    if (N > 64 && wide < 448 && pp <= 5 * Cfg64n::NT / 8) return run_patch_cfg<T, Cfg64n, PPT>(a, b, ldb, N, ep, plan, ws, s);
    return run_patch_cfg<T, Cfg128w8, PPT>(a, b, ldb, N, ep, plan, ws, s);
}
template <typename T, class Cfg, int PPT>
static int run_patch_cfg(const Gather &a, const void *b, long ldb, int N, const Epilogue &ep, const GemmPlan &plan, float *ws, hipStream_t s)
{
    constexpr int BK = Geo<T>::BK;
    const int M = a.N * a.H * a.W, npos = a.kh * a.kw, K = npos * a.C;
    if (M <= 0 || N <= 0 || (N & 7)) return -1;
    PatchSrc<T> pa;
    pa.op = operand(a.x, a.bytes);
    pa.pix = a.pix ? (unsigned)a.pix : (unsigned)(a.C * sizeof(T));
    constexpr int CW = BK / PPT;                 // channels of a chunk
    const int ntc = (npos + PPT - 1) / PPT;      // K tiles of a chunk
    pa.H = a.H; pa.W = a.W; pa.C = a.C; pa.kh = a.kh; pa.kw = a.kw; pa.pad = a.pad; pa.npos = npos; pa.ntc = ntc; pa.M = M;
    pa.dW = make_fastdiv(a.W); pa.dHW = make_fastdiv(a.H * a.W); pa.dkw = make_fastdiv(a.kw); pa.dntc = make_fastdiv(ntc);
    ChunkK<T, PPT> lb;
    lb.op = operand(b, ((size_t)(N - 1) * ldb + K) * sizeof(T));
    lb.ldb = (unsigned)(ldb * sizeof(T)); lb.posb = (unsigned)(a.C * sizeof(T)); lb.rows = N; lb.C = a.C; lb.npos = npos; lb.ntc = ntc;
    lb.dntc = pa.dntc;
    if (pa.op.bytes == 0 || lb.op.bytes == 0) return -1;
    const int tiles_m = (M + Cfg::BM - 1) / Cfg::BM, tiles_n = (N + Cfg::BN - 1) / Cfg::BN;
    const int nkt = ((a.C + CW - 1) / CW) * ntc;
    int splits = plan.splits;
    if (splits > 1 && ws == nullptr) return -1;
    const int per = (nkt + splits - 1) / splits;
    splits = (nkt + per - 1) / per;
    const long blocks = (long)tiles_m * tiles_n * splits;
    if (blocks > 0x7fffffffL) return -1;
    const int pp = 128 + (a.kh - 1) * a.W + a.kw - 1;   // pixels a block tile needs
    // The wide shape runs with the two kinds of waves (see conv_patch_ws_kernel).
    if constexpr (Cfg::NT == 512) {
        if (pp > 256) return -1;
        if constexpr (PPT == 2)
            hipLaunchKernelGGL((conv_patch_ws_kernel<T, 4, Cfg128, 2, 3>), dim3((unsigned)blocks), dim3(Cfg128::NT + kProducers), 0, s, pa, lb, ep, M, N, nkt, per,
                               tiles_m, tiles_n, splits > 1 ? ws : nullptr);
        else if (pp <= 192)
            hipLaunchKernelGGL((conv_patch_ws_kernel<T, 6, Cfg128, 1, 3>), dim3((unsigned)blocks), dim3(Cfg128::NT + kProducers), 0, s, pa, lb, ep, M, N, nkt, per,
                               tiles_m, tiles_n, splits > 1 ? ws : nullptr);
        else
            hipLaunchKernelGGL((conv_patch_ws_kernel<T, 8, Cfg128, 1, 2>), dim3((unsigned)blocks), dim3(Cfg128::NT + kProducers), 0, s, pa, lb, ep, M, N, nkt, per,
                               tiles_m, tiles_n, splits > 1 ? ws : nullptr);
    } else if constexpr (PPT == 2) {
        // the narrow shape, half-wide chunks: four pieces per pixel, three per thread hold 192 pixels with 256 threads
        constexpr int NPL = 3;
        if (pp > NPL * Cfg::NT / 4) return -1;
        hipLaunchKernelGGL((conv_patch_kernel<T, NPL, Cfg, 2>), dim3((unsigned)blocks), dim3(Cfg::NT), 0, s, pa, lb, ep, M, N, nkt, per, tiles_m,
                           tiles_n, splits > 1 ? ws : nullptr);
    } else {
        // the narrow shape, whole-tile chunks: five pieces per thread hold runs of up to 160 pixels with 256 threads
        constexpr int NPL_S = 5;
        if (pp > NPL_S * Cfg::NT / 8) return -1;
        hipLaunchKernelGGL((conv_patch_kernel<T, NPL_S, Cfg, 1>), dim3((unsigned)blocks), dim3(Cfg::NT), 0, s, pa, lb, ep, M, N, nkt, per, tiles_m,
                           tiles_n, splits > 1 ? ws : nullptr);
    }
    if (splits > 1) launch_splitk_reduce<T>(ws, splits, ep, M, N, s);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// The window-row form of a first convolution in 16-bit data with up to 96 output columns runs conv_rows_kernel when
// the filter bank and the image rows of a tile fit its LDS layout; everything else takes the tile engine.
static bool rows_applies(const Gather &a, long ldb, int N, const Epilogue &ep, const GemmPlan &plan)
{
    const long K = (long)a.kh * a.C;
    if (!(a.kw == 1 && a.pad == 0 && a.ds == 1 && a.pix != 0 && a.rowb != 0 && a.C % 8 == 0 && ldb == K && K <= 64 * kRowsChunks)) return false;
    if (!(N > 64 && N <= kRowsBN && N % 8 == 0 && plan.splits == 1)) return false;
    if (!(a.rowb % 16 == 0 && ((size_t)a.sm * a.pix) % 8 == 0 && ((uintptr_t)a.x & 15) == 0 && a.bytes <= kMaxOperandBytes)) return false;
    if (!(ep.mode == 0 && !ep.drop && !ep.mask_src && !ep.out_f32 && ep.ld % 8 == 0 && ((uintptr_t)ep.out & 15) == 0)) return false;
    const long out_rows = std::min<long>(a.Ho, (kRowsBM + a.Wo - 1) / a.Wo + 1);      // output rows a run of 128 pixels can touch
    const long block = ((out_rows - 1) * a.sm + a.kh) * (long)a.rowb;
    return block <= kRowsPatchBytes && a.H >= (a.Ho - 1) * a.sm + a.kh;
}
static int run_rows(const Gather &a, const void *b, long ldb, int N, const Epilogue &ep, hipStream_t s)
{
    RowsConv r;
    r.x = operand(a.x, a.bytes);
    r.rowb = (unsigned)a.rowb; r.imgb = (unsigned)((size_t)a.H * a.rowb); r.pixstep = (unsigned)((size_t)a.sm * a.pix);
    r.Ho = a.Ho; r.Wo = a.Wo; r.stride = a.sm; r.kh = a.kh; r.KW = a.C; r.K = a.kh * a.C;
    r.npix = a.Ho * a.Wo;
    r.tiles_per_image = (r.npix + kRowsBM - 1) / kRowsBM;
    const long total = (long)a.N * r.tiles_per_image;
    if (total <= 0 || total > 0x7fffffffL) return -1;
    r.total = (int)total;
    r.w = operand(b, (size_t)N * ldb * sizeof(bf16_t)); r.ldw = (unsigned)(ldb * sizeof(bf16_t));
    r.dWo = make_fastdiv((uint32_t)a.Wo); r.dtpi = make_fastdiv((uint32_t)r.tiles_per_image); r.dKW = make_fastdiv((uint32_t)a.C);
    if (r.x.bytes == 0 || r.w.bytes == 0) return -1;
    // one workgroup per CU (its LDS holds the filter bank and two blocks of image rows); a multiple of 8 so that every
    // workgroup's tiles stay on its XCD's contiguous range
    const long grid = total < 256 ? total : 256;
    hipLaunchKernelGGL(conv_rows_kernel, dim3((unsigned)grid), dim3(512), 0, s, r, ep, N);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <typename T>
static int gather_plain_t(const Gather &a, const void *b, long ldb, int N, const Epilogue &ep, const GemmPlan &plan, float *ws, hipStream_t s)
{
    const int K = a.kh * a.kw * a.C;
    if constexpr (sizeof(T) == 2) {
        if (rows_applies(a, ldb, N, ep, plan)) return run_rows(a, b, ldb, N, ep, s);
    }
    const int ppt = patch_applies<T>(a, ldb);
    if (ppt == 1) return run_patch<T, 1>(a, b, ldb, N, ep, plan, ws, s);
    if (ppt == 2) return run_patch<T, 2>(a, b, ldb, N, ep, plan, ws, s);
    if (a.ds == 1 && a.kh * a.kw <= 32)
        return run<T>(make_gather_k<T, false>(a), make_plain_k<T>(b, ldb, N, K), a.N * a.Ho * a.Wo, N, K, ep, plan, ws, s);
    if (a.ds == 1)
        return run<T>(make_gather_k<T, true>(a), make_plain_k<T>(b, ldb, N, K), a.N * a.Ho * a.Wo, N, K, ep, plan, ws, s);
    return run<T>(make_gather_ks<T>(a), make_plain_k<T>(b, ldb, N, K), a.N * a.Ho * a.Wo, N, K, ep, plan, ws, s);
}
int gemm_gather_plain(int dtype, const Gather &a, const void *b, long ldb, int N, const Epilogue &ep, const GemmPlan &plan, float *ws, hipStream_t s)
{
    if (a.ds != 1 && a.sm != 1) return -1;
    if (a.kh > 15 || a.kw > 15) return -1;
    return dtype == kBF16 ? gather_plain_t<bf16_t>(a, b, ldb, N, ep, plan, ws, s) : gather_plain_t<float>(a, b, ldb, N, ep, plan, ws, s);
}

int gemm_plain_plain(int dtype, const void *a, long lda, int M, const void *b, long ldb, int N, int b_rows, int K, const Epilogue &ep,
                     const GemmPlan &plan, float *ws, hipStream_t s)
{
    if (b_rows > N) return -1;
    if (dtype == kBF16)
        return run<bf16_t>(make_plain_k<bf16_t>(a, lda, M, K), make_plain_k<bf16_t>(b, ldb, b_rows, K), M, N, K, ep, plan, ws, s);
    return run<float>(make_plain_k<float>(a, lda, M, K), make_plain_k<float>(b, ldb, b_rows, K), M, N, K, ep, plan, ws, s);
}

int gemm_plain_trans(int dtype, const void *a, long lda, int M, const void *bt, long ldb, int N, int K, const Epilogue &ep,
                     const GemmPlan &plan, float *ws, hipStream_t s)
{
    if (dtype == kBF16)
        return run<bf16_t>(make_plain_k<bf16_t>(a, lda, M, K), make_plain_t<bf16_t>(bt, ldb, N, K), M, N, K, ep, plan, ws, s);
    return run<float>(make_plain_k<float>(a, lda, M, K), make_plain_t<float>(bt, ldb, N, K), M, N, K, ep, plan, ws, s);
}

int gemm_trans_trans(int dtype, const void *at, long lda, int M, const void *bt, long ldb, int N, int K, const Epilogue &ep,
                     const GemmPlan &plan, float *ws, hipStream_t s)
{
    if (ep.upd_w) {   // push inside the kernel (gemm_kernel over two transposed plain operands carries that path):
                      // whole sums only, 16-byte rows and column groups in all three buffers
        const uintptr_t al = (uintptr_t)ep.upd_w | (uintptr_t)ep.upd_v | (uintptr_t)ep.upd_copy;
        if (plan.splits != 1 || ep.mode != 0 || !ep.upd_v || !ep.upd_copy || (al & 15) || (ep.ld & 7)) return -1;
    }
    if (dtype == kBF16)
        return run<bf16_t>(make_plain_t<bf16_t>(at, lda, M, K), make_plain_t<bf16_t>(bt, ldb, N, K), M, N, K, ep, plan, ws, s);
    return run<float>(make_plain_t<float>(at, lda, M, K), make_plain_t<float>(bt, ldb, N, K), M, N, K, ep, plan, ws, s);
}

// The filter gradient of a first convolution in window-row form (16-bit data, up to 96 output channels, up to 448 K
// columns) runs conv_rows_wgrad_kernel when the image rows of a tile fit its LDS layout and the plan has the scratch
// for one partial result per workgroup.
static int rows_wgrad_rpt(const Gather &b) { return b.Wo > 0 && b.Wo <= kRowsWgTP ? std::min(b.Ho, kRowsWgTP / b.Wo) : 0; }   // output rows per tile
static long rows_wgrad_tiles(const Gather &b)
{
    const int rpt = rows_wgrad_rpt(b);
    return rpt > 0 ? (long)b.N * ((b.Ho + rpt - 1) / rpt) : 0;
}
size_t rows_wgrad_ws_floats(int dtype, int M, const Gather &b)
{
    const long K = (long)b.kh * b.C, tiles = rows_wgrad_tiles(b);
    if (dtype != kBF16 || b.kw != 1 || b.pad != 0 || b.ds != 1 || M > 96 || K > kRowsWgBN || tiles <= 0) return 0;
    return (size_t)std::min<long>(tiles, kRowsWgGrid) * (size_t)M * (size_t)K;
}
static bool rows_wgrad_applies(const void *at, long lda, int M, const Gather &b, const Epilogue &ep, const GemmPlan &plan, const float *ws)
{
    const long K = (long)b.kh * b.C;
    const int rpt = rows_wgrad_rpt(b);
    if (rpt <= 0) return false;
    if (!(b.kw == 1 && b.pad == 0 && b.ds == 1 && b.pix != 0 && b.rowb != 0 && b.C % 8 == 0 && K <= kRowsWgBN && K % 8 == 0)) return false;
    if (!(M > 0 && M <= 96 && M % 8 == 0 && lda >= M && (lda * 2) % 16 == 0 && ((uintptr_t)at & 15) == 0)) return false;
    if (!(b.rowb % 16 == 0 && ((size_t)b.sm * b.pix) % 8 == 0 && ((uintptr_t)b.x & 15) == 0 && b.bytes <= kMaxOperandBytes)) return false;
    if (!(ep.mode == 2 && ep.out_f32 && ws != nullptr && ((uintptr_t)ws & 15) == 0 && plan.ws_floats >= rows_wgrad_ws_floats(kBF16, M, b))) return false;
    if ((size_t)b.N * b.Ho * b.Wo * lda * 2 > kMaxOperandBytes) return false;
    const long block = ((long)(rpt - 1) * b.sm + b.kh) * (long)b.rowb;   // image rows of a tile
    return block <= kRowsWgIB && b.H >= (b.Ho - 1) * b.sm + b.kh && rows_wgrad_tiles(b) <= 0x7fffffffL;
}
static int run_rows_wgrad(const void *at, long lda, int M, const Gather &b, const Epilogue &ep, float *ws, hipStream_t s)
{
    RowsConv r;
    const int rpt = rows_wgrad_rpt(b);
    r.x = operand(b.x, b.bytes);
    r.rowb = (unsigned)b.rowb; r.imgb = (unsigned)((size_t)b.H * b.rowb); r.pixstep = (unsigned)((size_t)b.sm * b.pix);
    r.Ho = b.Ho; r.Wo = b.Wo; r.stride = b.sm; r.kh = b.kh; r.KW = b.C; r.K = b.kh * b.C;
    r.npix = b.Ho * b.Wo;
    r.tiles_per_image = (b.Ho + rpt - 1) / rpt;
    r.total = (int)rows_wgrad_tiles(b);
    r.w = Operand{nullptr, 0u}; r.ldw = 0;
    r.dWo = make_fastdiv((uint32_t)b.Wo); r.dtpi = make_fastdiv((uint32_t)r.tiles_per_image); r.dKW = make_fastdiv((uint32_t)b.C);
    const Operand dy = operand(at, (size_t)b.N * r.npix * lda * sizeof(bf16_t));
    if (r.x.bytes == 0 || dy.bytes == 0) return -1;
    const int grid = r.total < kRowsWgGrid ? r.total : kRowsWgGrid;
    hipLaunchKernelGGL(conv_rows_wgrad_kernel, dim3((unsigned)grid), dim3(512), 0, s, r, rpt, dy, (unsigned)(lda * sizeof(bf16_t)), M, ws);
    launch_splitk_reduce<bf16_t>(ws, grid, ep, M, r.K, s);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int gemm_trans_gather(int dtype, const void *at, long lda, int M, const Gather &b, const Epilogue &ep, const GemmPlan &plan, float *ws,
                      hipStream_t s)
{
    if (b.ds != 1 || b.kh > 15 || b.kw > 15) return -1;
    if (dtype == kBF16 && rows_wgrad_applies(at, lda, M, b, ep, plan, ws)) return run_rows_wgrad(at, lda, M, b, ep, ws, s);
    const int K = b.N * b.Ho * b.Wo, N = b.kh * b.kw * b.C;
    if (dtype == kBF16) return run<bf16_t>(make_plain_t<bf16_t>(at, lda, M, K), make_gather_t<bf16_t>(b), M, N, K, ep, plan, ws, s);
    return run<float>(make_plain_t<float>(at, lda, M, K), make_gather_t<float>(b), M, N, K, ep, plan, ws, s);
}

}  // namespace asgd
