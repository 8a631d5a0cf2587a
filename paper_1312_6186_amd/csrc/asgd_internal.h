// Internal declarations shared by the host orchestration (api.cpp) and the
// kernel files.  Activations live channel-last, [B][H][W][Cp] with the channel
// count rounded up to a multiple of 8 (padding channels hold zeros); FC-side
// activations are [B][ld] row-major.  The input of a first convolution over at
// most 4 channels is instead kept with 4 channels per pixel and its zero border
// (see Gather).  All kernels target gfx950 only.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

namespace asgd {

enum DType { kF32 = 0, kBF16 = 1 };
inline size_t dtype_size(int dt) { return dt == kBF16 ? 2 : 4; }

// n / d for 0 <= n < 2^31 by multiply-high and shift.
struct FastDiv {
    uint32_t d, mul, sh;
};
FastDiv make_fastdiv(uint32_t d);

// What happens to one accumulator element C[m][n] on its way to memory.
// The same routine serves the GEMM kernels and the split-K reduction.
struct Epilogue {
    void *out = nullptr;   // OutT [M][ld] (mode 0) or fp32 canonical conv filter gradient (mode 1)
    long ld = 0;
    int out_f32 = 0;       // 1: out is fp32 whatever the compute type
    const void *bias = nullptr;  // compute type, [bias_n]; added first to columns n < bias_n
    int bias_n = 0;
    int relu = 0;
    int drop = 0;          // dropout after ReLU: keep iff hash(m*drop_F+n) >= drop_thr
    uint64_t drop_key = 0;
    uint32_t drop_thr = 0;
    int drop_F = 0;
    float drop_scale = 1.f;
    const void *mask_src = nullptr;  // compute type, [M][mask_ld]: v = mask_src > 0 ? v*mask_scale : 0
    long mask_ld = 0;
    float mask_scale = 1.f;
    int mode = 0;          // 1: rows are cout, columns are (ky,kx,ci_padded) -> [cout][cin][kh][kw]
                           // 2: columns are (ky, kx*cw_rwc+ci) over window rows of cw_cinp elements -> the same
    int cw_cout = 0, cw_cin = 0, cw_cinp = 0, cw_kh = 0, cw_kw = 0;
    int cw_rwc = 4;        // mode 2: channels per stored pixel (column j of a window row is kx * cw_rwc + ci)
    // Push inside the gradient kernel (mode 0, no split-K): C[m][n] is the gradient of parameter upd_w[m*ld + n] and is
    // not stored; the kernel applies t = g + wd*w, v = mu*v - lr*t, w += v to upd_w / upd_v and writes the new
    // parameters to upd_copy in the compute type (all [M][ld], rows and column groups of 8 aligned to 16 bytes).
    float *upd_w = nullptr, *upd_v = nullptr;
    void *upd_copy = nullptr;
    float upd_lr = 0.f, upd_mu = 0.f, upd_wd = 0.f;
};

// Gather description for an implicit-GEMM operand taken from a channel-last
// tensor x[N][H][W][C].  GEMM rows (direct form) enumerate (n, oy, ox) on a
// grid Ho x Wo; the K index enumerates (ky, kx, c).  The element is
// x[n][(oy*sm + ky - pad)/ds][(ox*sm + kx - pad)/ds][c] when both divisions
// are exact and in range, else 0.  Forward conv: sm = stride, ds = 1.
// Data gradient: sm = 1, ds = stride, pad = k-1-pad with a flipped filter.
struct Gather {
    const void *x = nullptr;
    int N = 0, H = 0, W = 0, C = 0;
    int Ho = 0, Wo = 0;
    int kh = 0, kw = 0, sm = 1, ds = 1, pad = 0;
    size_t bytes = 0;      // size of the tensor in bytes (at most 1 GiB); pieces outside it read as zeros
    // Byte strides between image rows and between pixels; 0 = dense (W*C and C elements).  Window-row form of a
    // convolution over few input channels: the tensor is stored with its zero border, 4 channels per pixel, and
    // described as kw = 1, pad = 0, C = one padded window row (kw*4 elements rounded up to 16 bytes), so that
    // the K index is (ky, kx*4 + c) and a whole window row is one contiguous run.
    size_t rowb = 0, pix = 0;
};

struct GemmPlan {
    int splits = 1;          // split-K factor
    size_t ws_floats = 0;    // fp32 scratch needed when splits > 1
};

// Every operand must fit in 1 GiB.
// C[M][N] = A[M][K] * B[N][K]^T; A gathered (direct), B plain K-contiguous.
GemmPlan plan_gemm(long M, long N, long K, int dtype, int max_splits);
int gemm_gather_plain(int dtype, const Gather &a, const void *b, long ldb, int N, const Epilogue &ep,
                      const GemmPlan &plan, float *ws, hipStream_t s);
// A plain [M][lda], B plain [b_rows][ldb], both K-contiguous; columns n >= b_rows of C are computed as zeros.
int gemm_plain_plain(int dtype, const void *a, long lda, int M, const void *b, long ldb, int N, int b_rows, int K,
                     const Epilogue &ep, const GemmPlan &plan, float *ws, hipStream_t s);
// A plain [M][lda] K-contiguous; B stored [K][ldb] (rows n contiguous).
int gemm_plain_trans(int dtype, const void *a, long lda, int M, const void *bt, long ldb, int N, int K,
                     const Epilogue &ep, const GemmPlan &plan, float *ws, hipStream_t s);
// A stored [K][lda] (rows m contiguous), B stored [K][ldb].
int gemm_trans_trans(int dtype, const void *at, long lda, int M, const void *bt, long ldb, int N, int K,
                     const Epilogue &ep, const GemmPlan &plan, float *ws, hipStream_t s);
// Filter gradient: A stored [K = B*Ho*Wo][lda] (rows = cout), B gathered with the
// reduction index enumerating (n, oy, ox) and rows enumerating (ky, kx, c).
int gemm_trans_gather(int dtype, const void *at, long lda, int M, const Gather &b, const Epilogue &ep,
                      const GemmPlan &plan, float *ws, hipStream_t s);
// fp32 scratch (in floats) the filter gradient of a first convolution in window-row form wants in plan.ws_floats to
// run as one persistent kernel with a partial result per workgroup; 0 where that kernel does not apply
size_t rows_wgrad_ws_floats(int dtype, int M, const Gather &b);

// ---- streaming kernels (kernels_stream.hip) --------------------------------
int launch_update(float *w, float *v, const float *g, size_t n, float lr, float mu, float wd,
                  int *version_counter, hipStream_t s);
// the update, and the updated parameters written to `copy` (fp32 or bf16) in the same pass
int launch_update_snapshot(float *w, float *v, const float *g, size_t n, float lr, float mu, float wd, void *copy,
                           int dst_dtype, hipStream_t s);
// the same over up to 8 ranges [off, off + cnt) of the parameter vector in one launch (w, v, g, copy: 16-byte aligned bases)
int launch_update_snapshot_ranges(float *w, float *v, const float *g, const size_t *off, const size_t *cnt, int n_ranges, float lr, float mu, float wd,
                                  void *copy, int dst_dtype, hipStream_t s);
// Adagrad / Adadelta server updates (one pass, in place)
int launch_adagrad(float *w, float *h, const float *g, size_t n, float lr, float eps, float wd, hipStream_t s);
int launch_adadelta(float *w, float *a, float *b, const float *g, size_t n, float rho, float eps, float wd, hipStream_t s);
// acc = g (first) or acc + g
int launch_accumulate(float *acc, const float *g, size_t n, bool first, hipStream_t s);
int launch_snapshot(const float *src, void *dst, size_t n, int dst_dtype, const int *version_counter,
                    int32_t *log_slot, int log_update, int log_worker, hipStream_t s);
// images [B][C][H][W] (compute type) -> channel-last [B][H][W][Cp], zero padding channels
int launch_stage_input(int dtype, const void *src, void *dst, int B, int C, int H, int W, int Cp, hipStream_t s);
// the same into the interior of a bordered [B][H+2*pad][Wp][4] tensor (C <= 4; the border is not written)
int launch_stage_input_rw(int dtype, const void *src, void *dst, int B, int C, int H, int W, int pad, int Wp, int pc, hipStream_t s);
// Filter packing for all convolution layers of a net in one launch.  Per layer: canonical filters
// [cout][cin][k][k] -> forward pack wf [coutp][k][k][cinp] and, if wd is given, the flipped data-gradient pack
// wd [cinp][k][k][coutp]; or (rw = channels per stored pixel > 0) the window-row pack wf [coutp][k][KW], element (ky, kx*rw + ci), zeros elsewhere.
struct PackJob {
    const void *w; void *wf; void *wd;
    int cout, cin, k, coutp, cinp, rw, KW;
    unsigned start, nf;   // filled by launch_pack_conv
};
struct PackJobs { PackJob j[12]; int n; unsigned total; };
int launch_pack_conv(int dtype, PackJobs &jobs, hipStream_t s);
int launch_pool_fwd(int dtype, const void *x, void *y, uint8_t *arg, int B, int H, int W, int Cp, int k, int stride,
                    hipStream_t s);
// dx[pixel] = sum of dy over the windows whose recorded maximum is this pixel; times [x > 0] if relu
int launch_pool_bwd(int dtype, const void *dy, const uint8_t *arg, const void *x, int relu, void *dx, int B, int H,
                    int W, int Cp, int k, int stride, float *bands, hipStream_t s);
// bands != nullptr: the kernel also leaves the column sums of dx in bands[Cp][pool_bwd_bands(...)] (stage 1 of a
// bias gradient); only for shapes where pool_bwd_bands is not 0
long pool_bwd_bands(int dtype, int B, int H, int W, int Cp, int k, int stride);
// cross-channel response normalisation on channel-last tensors: y = a * (bias + alpha * window sum of a^2)^(-beta);
// backward writes da (times [a > 0], the ReLU of the convolution below, if relu) from a and dy; size odd, <= 9
int launch_lrn_fwd(int dtype, const void *a, void *y, size_t pixels, int Cp, int size, float alpha, float beta, float bias, hipStream_t s);
int launch_lrn_bwd(int dtype, const void *a, const void *dy, int relu, void *da, size_t pixels, int Cp, int size, float alpha, float beta,
                   float bias, hipStream_t s);
// channel-last [B][H][W][Cp] -> [B][C*H*W] in (c,h,w) order, and back (zero padding channels; optional ReLU mask)
int launch_flatten(int dtype, const void *x, void *flat, int B, int H, int W, int C, int Cp, hipStream_t s);
int launch_unflatten(int dtype, const void *dflat, const void *x_for_mask, int relu, void *dx, int B, int H, int W,
                     int C, int Cp, hipStream_t s);
// db[n] = sum_m dy[m][n], n < N, fp32, fixed summation order, in two stages: launch_colsum_partial sums bands of
// rows into ws (colsum_ws_floats floats, not shared with another pending job) and appends a job;
// launch_colsum_finish adds the bands of all pending jobs (up to 12) in one launch.
struct ColsumJob { const float *ws; float *db; long ld; int nblk, N; unsigned start_block; int colmajor; };   // ws[band][ld], or ws[column][nblk] if colmajor
struct ColsumJobs { ColsumJob j[12]; int n; };
int launch_colsum_partial(int dtype, const void *dy, long ld, long M, int N, float *db, float *ws, ColsumJobs &jobs, hipStream_t s);
// the same with the first stage put off: colsum_partial_defer appends the tensor to s1 (and its second stage to jobs),
// launch_colsum_stage1 sums the bands of all appended tensors (up to 12) in one launch
struct ColsumS1Job { const void *dy; float *ws; long ld, M, rows_per_block; int chunks, cpb, rl, gx, gy; unsigned start_block; };
struct ColsumS1Jobs { ColsumS1Job j[12]; int n; };
int colsum_partial_defer(int dtype, const void *dy, long ld, long M, int N, float *db, float *ws, ColsumS1Jobs &s1, ColsumJobs &jobs);
int launch_colsum_stage1(int dtype, ColsumS1Jobs &s1, hipStream_t s);
int launch_colsum_finish(ColsumJobs &jobs, hipStream_t s);
size_t colsum_ws_floats(int dtype, long M, long ld);
// softmax cross-entropy over fp32 logits [B][ld]: loss (mean) and dz (compute type, [B][ld], zero padding columns)
int launch_softmax_ce(int dtype, const float *z, long ld, const int32_t *labels, int B, int C, void *dz, float *loss,
                      float *row_loss, hipStream_t s);
int launch_fill_zero(void *p, size_t bytes, hipStream_t s);
// debug exports (canonical layouts)
int launch_export_nhwc(int dtype, const void *x, float *dst, int B, int H, int W, int C, int Cp, hipStream_t s);
int launch_export_rows(int dtype, int src_f32, const void *x, long ld, float *dst, int B, int F, hipStream_t s);
int launch_export_argmax(const uint8_t *arg, uint8_t *dst, int B, int H, int W, int C, int Cp, hipStream_t s);
int launch_dropout_mask(uint8_t *dst, size_t count, uint64_t key, uint32_t thr, hipStream_t s);

// host-side key of the dropout generator for one (seed, step, worker, layer)
uint64_t dropout_key(uint64_t seed, uint64_t step, uint32_t worker, uint32_t layer);

}  // namespace asgd
