/*
 * CPU oracle for the GPU A-SGD hot path (arXiv 1312.6186).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of every
 * operation on the hot path, in double precision, canonical NCHW / row-major
 * storage.  It shares no code with the HIP library and must never be called
 * from it: only the test-suite, the smoke check and the benchmark's
 * cpu_baseline leg load it.
 *
 * The paper (Section 2, "Training neural networks") states the work unit:
 * the gradient of the objective over a minibatch, followed by a parameter
 * update.  Section 1 fixes the model family by citation: a Krizhevsky-2012
 * style convnet with ReLU units, dropout and a 1000-way softmax objective.
 * Section 2.3 ("Our contribution: GPU A-SGD") states the protocol: model
 * replicas fetch parameters from, and push gradients to, a central parameter
 * server.  The paper prints no formulas; each function below writes out the
 * textbook definition of the operation named there.
 *
 * Loop nests follow the definitions directly.  The only liberty taken is the
 * order of independent loops (so that OpenMP can split the outer one); the
 * order in which terms enter any single sum is the one written in the comment
 * of that function.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int out_extent(int in, int k, int stride, int pad)
{
    /* floor rule; the caller guarantees in + 2*pad >= k */
    return (in + 2 * pad - k) / stride + 1;
}

/* ---------------------------------------------------------------------------
 * Convolution layer (Section 3: "same architecture as" the cited convnet).
 *   y[n,co,oy,ox] = b[co] + sum_{ci,ky,kx} x[n,ci,oy*s+ky-p,ox*s+kx-p] * w[co,ci,ky,kx]
 * Cross-correlation (no kernel flip); x is zero outside the image.
 * Terms are added in (ci, ky, kx) lexicographic order, after the bias.
 * ------------------------------------------------------------------------ */
void oracle_conv_fwd(const double *x, const double *w, const double *b, double *y,
                     int N, int Cin, int H, int W, int Cout, int k, int s, int p)
{
    const int Ho = out_extent(H, k, s, p), Wo = out_extent(W, k, s, p);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Cout; ++co) {
            double *yp = y + ((size_t)n * Cout + co) * Ho * Wo;
            for (int i = 0; i < Ho * Wo; ++i) yp[i] = b[co];
            for (int ci = 0; ci < Cin; ++ci) {
                const double *xp = x + ((size_t)n * Cin + ci) * H * W;
                for (int ky = 0; ky < k; ++ky)
                    for (int kx = 0; kx < k; ++kx) {
                        const double wv = w[(((size_t)co * Cin + ci) * k + ky) * k + kx];
                        for (int oy = 0; oy < Ho; ++oy) {
                            const int iy = oy * s + ky - p;
                            if (iy < 0 || iy >= H) continue;
                            for (int ox = 0; ox < Wo; ++ox) {
                                const int ix = ox * s + kx - p;
                                if (ix < 0 || ix >= W) continue;
                                yp[oy * Wo + ox] += xp[iy * W + ix] * wv;
                            }
                        }
                    }
            }
        }
}

/* Gradient of the loss with respect to the convolution input:
 *   dx[n,ci,iy,ix] = sum over all (co,ky,kx,oy,ox) with oy*s+ky-p == iy and
 *                    ox*s+kx-p == ix of dy[n,co,oy,ox] * w[co,ci,ky,kx]
 * i.e. every forward product term sends its dy*w back to the x it read. */
void oracle_conv_bwd_data(const double *dy, const double *w, double *dx,
                          int N, int Cin, int H, int W, int Cout, int k, int s, int p)
{
    const int Ho = out_extent(H, k, s, p), Wo = out_extent(W, k, s, p);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int ci = 0; ci < Cin; ++ci) {
            double *dxp = dx + ((size_t)n * Cin + ci) * H * W;
            for (int i = 0; i < H * W; ++i) dxp[i] = 0.0;
            for (int co = 0; co < Cout; ++co) {
                const double *dyp = dy + ((size_t)n * Cout + co) * Ho * Wo;
                for (int ky = 0; ky < k; ++ky)
                    for (int kx = 0; kx < k; ++kx) {
                        const double wv = w[(((size_t)co * Cin + ci) * k + ky) * k + kx];
                        for (int oy = 0; oy < Ho; ++oy) {
                            const int iy = oy * s + ky - p;
                            if (iy < 0 || iy >= H) continue;
                            for (int ox = 0; ox < Wo; ++ox) {
                                const int ix = ox * s + kx - p;
                                if (ix < 0 || ix >= W) continue;
                                dxp[iy * W + ix] += dyp[oy * Wo + ox] * wv;
                            }
                        }
                    }
            }
        }
}

/* Gradient with respect to the filters and the bias:
 *   dw[co,ci,ky,kx] = sum_{n,oy,ox} dy[n,co,oy,ox] * x[n,ci,oy*s+ky-p,ox*s+kx-p]
 *   db[co]          = sum_{n,oy,ox} dy[n,co,oy,ox]
 * Terms are added in (n, oy, ox) lexicographic order. */
void oracle_conv_bwd_weight(const double *x, const double *dy, double *dw, double *db,
                            int N, int Cin, int H, int W, int Cout, int k, int s, int p)
{
    const int Ho = out_extent(H, k, s, p), Wo = out_extent(W, k, s, p);
#pragma omp parallel for collapse(2) schedule(static)
    for (int co = 0; co < Cout; ++co)
        for (int ci = 0; ci < Cin; ++ci)
            for (int ky = 0; ky < k; ++ky)
                for (int kx = 0; kx < k; ++kx) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n) {
                        const double *xp = x + ((size_t)n * Cin + ci) * H * W;
                        const double *dyp = dy + ((size_t)n * Cout + co) * Ho * Wo;
                        for (int oy = 0; oy < Ho; ++oy) {
                            const int iy = oy * s + ky - p;
                            if (iy < 0 || iy >= H) continue;
                            for (int ox = 0; ox < Wo; ++ox) {
                                const int ix = ox * s + kx - p;
                                if (ix < 0 || ix >= W) continue;
                                acc += dyp[oy * Wo + ox] * xp[iy * W + ix];
                            }
                        }
                    }
                    dw[(((size_t)co * Cin + ci) * k + ky) * k + kx] = acc;
                }
#pragma omp parallel for schedule(static)
    for (int co = 0; co < Cout; ++co) {
        double acc = 0.0;
        for (int n = 0; n < N; ++n) {
            const double *dyp = dy + ((size_t)n * Cout + co) * Ho * Wo;
            for (int i = 0; i < Ho * Wo; ++i) acc += dyp[i];
        }
        db[co] = acc;
    }
}

/* ---------------------------------------------------------------------------
 * Rectified linear unit (Section 1: "relu neurons").
 *   r = max(y, 0);   dy = dr where y > 0, else 0  (derivative taken as 0 at 0)
 * ------------------------------------------------------------------------ */
void oracle_relu_fwd(const double *y, double *r, size_t count)
{
    for (size_t i = 0; i < count; ++i) r[i] = y[i] > 0.0 ? y[i] : 0.0;
}

void oracle_relu_bwd(const double *y, const double *dr, double *dy, size_t count)
{
    for (size_t i = 0; i < count; ++i) dy[i] = y[i] > 0.0 ? dr[i] : 0.0;
}

/* ---------------------------------------------------------------------------
 * Max pooling, unpadded, floor rule (part of the cited architecture).
 *   p[n,c,py,px] = max_{ky,kx<k} r[n,c,py*s+ky,px*s+kx]
 * The recorded position is idx = ky*k + kx of the FIRST maximum met in a
 * row-major scan of the window (an element replaces the running maximum only
 * if strictly greater).
 * ------------------------------------------------------------------------ */
void oracle_maxpool_fwd(const double *r, double *p, uint8_t *idx,
                        int N, int C, int H, int W, int k, int s)
{
    const int Ho = out_extent(H, k, s, 0), Wo = out_extent(W, k, s, 0);
#pragma omp parallel for schedule(static)
    for (int nc = 0; nc < N * C; ++nc) {
        const double *rp = r + (size_t)nc * H * W;
        for (int py = 0; py < Ho; ++py)
            for (int px = 0; px < Wo; ++px) {
                double best = rp[(py * s) * W + px * s];
                int arg = 0;
                for (int ky = 0; ky < k; ++ky)
                    for (int kx = 0; kx < k; ++kx) {
                        const double v = rp[(py * s + ky) * W + px * s + kx];
                        if (v > best) { best = v; arg = ky * k + kx; }
                    }
                p[((size_t)nc * Ho + py) * Wo + px] = best;
                idx[((size_t)nc * Ho + py) * Wo + px] = (uint8_t)arg;
            }
    }
}

/* Pooling with the positions given instead of searched: p = r at position idx of
 * each window.  Used when a near-tie between two window elements may legitimately
 * be decided either way (values equal up to rounding) and the rest of the
 * computation is to be followed for one particular valid choice. */
void oracle_maxpool_gather(const double *r, const uint8_t *idx, double *p,
                           int N, int C, int H, int W, int k, int s)
{
    const int Ho = out_extent(H, k, s, 0), Wo = out_extent(W, k, s, 0);
    for (int nc = 0; nc < N * C; ++nc)
        for (int py = 0; py < Ho; ++py)
            for (int px = 0; px < Wo; ++px) {
                const int a = idx[((size_t)nc * Ho + py) * Wo + px];
                p[((size_t)nc * Ho + py) * Wo + px] = r[(size_t)nc * H * W + (py * s + a / k) * W + px * s + a % k];
            }
}

/* Each pooled gradient goes to the recorded position of its window
 * (windows may overlap, so positions accumulate):  dr[argmax] += dp. */
void oracle_maxpool_bwd(const double *dp, const uint8_t *idx, double *dr,
                        int N, int C, int H, int W, int k, int s)
{
    const int Ho = out_extent(H, k, s, 0), Wo = out_extent(W, k, s, 0);
#pragma omp parallel for schedule(static)
    for (int nc = 0; nc < N * C; ++nc) {
        double *drp = dr + (size_t)nc * H * W;
        for (int i = 0; i < H * W; ++i) drp[i] = 0.0;
        for (int py = 0; py < Ho; ++py)
            for (int px = 0; px < Wo; ++px) {
                const int a = idx[((size_t)nc * Ho + py) * Wo + px];
                const int ky = a / k, kx = a % k;
                drp[(py * s + ky) * W + px * s + kx] += dp[((size_t)nc * Ho + py) * Wo + px];
            }
    }
}

/* ---------------------------------------------------------------------------
 * Local response normalisation across channels (part of the cited architecture,
 * Section 3: "the same architecture as described in" Krizhevsky et al. 2012,
 * whose Section 3.3 defines it):
 *   s[n,c,h,w] = k + alpha * sum_{c' = max(0, c - size/2)}^{min(C-1, c + size/2)} a[n,c',h,w]^2
 *   b = a * s^(-beta)
 *   da[i] = db[i] * s[i]^(-beta) - 2*alpha*beta * a[i] * sum_{j : |i-j| <= size/2} db[j] * a[j] * s[j]^(-beta-1)
 * ------------------------------------------------------------------------ */
void oracle_lrn_fwd(const double *a, double *b, int N, int C, int H, int W, int size, double alpha, double beta, double k)
{
    const int half = size / 2;
    const size_t HW = (size_t)H * W;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (size_t p = 0; p < HW; ++p) {
                double sum = 0.0;
                for (int j = c - half; j <= c + half; ++j)
                    if (j >= 0 && j < C) { const double v = a[((size_t)n * C + j) * HW + p]; sum += v * v; }
                b[((size_t)n * C + c) * HW + p] = a[((size_t)n * C + c) * HW + p] * pow(k + alpha * sum, -beta);
            }
}

void oracle_lrn_bwd(const double *a, const double *db, double *da, int N, int C, int H, int W, int size, double alpha, double beta,
                    double k)
{
    const int half = size / 2;
    const size_t HW = (size_t)H * W;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (size_t p = 0; p < HW; ++p) {
            for (int i = 0; i < C; ++i) {
                double acc = 0.0, s_i = 0.0;
                for (int j = i - half; j <= i + half; ++j) {
                    if (j < 0 || j >= C) continue;
                    double s_j = 0.0;
                    for (int q = j - half; q <= j + half; ++q)
                        if (q >= 0 && q < C) { const double v = a[((size_t)n * C + q) * HW + p]; s_j += v * v; }
                    s_j = k + alpha * s_j;
                    if (j == i) s_i = s_j;
                    acc += db[((size_t)n * C + j) * HW + p] * a[((size_t)n * C + j) * HW + p] * pow(s_j, -beta - 1.0);
                }
                const size_t o = ((size_t)n * C + i) * HW + p;
                da[o] = db[o] * pow(s_i, -beta) - 2.0 * alpha * beta * a[o] * acc;
            }
        }
}

/* ---------------------------------------------------------------------------
 * Fully connected layer.   y[n,o] = b[o] + sum_i x[n,i] * w[o,i]
 *   dx[n,i] = sum_o dy[n,o] * w[o,i]
 *   dw[o,i] = sum_n dy[n,o] * x[n,i]        db[o] = sum_n dy[n,o]
 * ------------------------------------------------------------------------ */
void oracle_fc_fwd(const double *x, const double *w, const double *b, double *y,
                   int N, int in, int out)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < out; ++o) {
            double acc = b[o];
            for (int i = 0; i < in; ++i) acc += x[(size_t)n * in + i] * w[(size_t)o * in + i];
            y[(size_t)n * out + o] = acc;
        }
}

void oracle_fc_bwd(const double *x, const double *w, const double *dy,
                   double *dx, double *dw, double *db, int N, int in, int out)
{
    if (dx) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < in; ++i) {
                double acc = 0.0;
                for (int o = 0; o < out; ++o) acc += dy[(size_t)n * out + o] * w[(size_t)o * in + i];
                dx[(size_t)n * in + i] = acc;
            }
    }
#pragma omp parallel for schedule(static)
    for (int o = 0; o < out; ++o) {
        double accb = 0.0;
        for (int n = 0; n < N; ++n) accb += dy[(size_t)n * out + o];
        db[o] = accb;
        for (int i = 0; i < in; ++i) {
            double acc = 0.0;
            for (int n = 0; n < N; ++n) acc += dy[(size_t)n * out + o] * x[(size_t)n * in + i];
            dw[(size_t)o * in + i] = acc;
        }
    }
}

/* ---------------------------------------------------------------------------
 * Dropout (Section 1 cites Hinton et al. 2012).  A unit is kept with
 * probability 1-p; kept activations are multiplied by `scale` (1 in the cited
 * form), dropped ones are zero.  The mask comes from a stateless counter-based
 * integer generator so that two independent implementations agree bit for bit:
 *
 *   mix(z): z ^= z>>30; z *= 0xBF58476D1CE4E5B9; z ^= z>>27;
 *           z *= 0x94D049BB133111EB; z ^= z>>31          (SplitMix64 finaliser)
 *   key  = mix( mix( mix(seed) + step ) + (worker<<32 | layer) )    (mod 2^64)
 *   u(i) = top 32 bits of mix( key + 0x9E3779B97F4A7C15 * (i+1) )
 *   keep(i) <=> u(i) >= threshold,   threshold = floor(p * 2^32)
 *
 * i is the logical element index n*F + f of the layer output.
 * ------------------------------------------------------------------------ */
static uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

uint32_t oracle_dropout_threshold(double p)
{
    return (uint32_t)floor(p * 4294967296.0);
}

void oracle_dropout_mask(uint8_t *mask, size_t count, uint64_t seed, uint64_t step,
                         uint32_t worker, uint32_t layer, uint32_t threshold)
{
    const uint64_t key = mix64(mix64(mix64(seed) + step) + (((uint64_t)worker << 32) | layer));
    for (size_t i = 0; i < count; ++i) {
        const uint32_t u = (uint32_t)(mix64(key + 0x9E3779B97F4A7C15ull * (uint64_t)(i + 1)) >> 32);
        mask[i] = u >= threshold ? 1 : 0;
    }
}

void oracle_dropout_apply(const double *r, const uint8_t *mask, double scale, double *h, size_t count)
{
    for (size_t i = 0; i < count; ++i) h[i] = mask[i] ? r[i] * scale : 0.0;
}

/* ---------------------------------------------------------------------------
 * Softmax + cross-entropy over a minibatch (Section 1: 1000 classes), mean
 * over the batch:
 *   lse_n = m_n + log sum_c exp(z[n,c] - m_n),  m_n = max_c z[n,c]
 *   loss  = (1/N) sum_n ( lse_n - z[n,label_n] )
 *   dz[n,c] = ( exp(z[n,c] - lse_n) - [c == label_n] ) / N
 * ------------------------------------------------------------------------ */
double oracle_softmax_ce(const double *z, const int32_t *labels, double *dz, int N, int C)
{
    double loss = 0.0;
    for (int n = 0; n < N; ++n) {
        const double *zn = z + (size_t)n * C;
        double m = zn[0];
        for (int c = 1; c < C; ++c) if (zn[c] > m) m = zn[c];
        double sum = 0.0;
        for (int c = 0; c < C; ++c) sum += exp(zn[c] - m);
        const double lse = m + log(sum);
        loss += lse - zn[labels[n]];
        if (dz)
            for (int c = 0; c < C; ++c)
                dz[(size_t)n * C + c] = (exp(zn[c] - lse) - (c == labels[n] ? 1.0 : 0.0)) / N;
    }
    return loss / N;
}

/* ---------------------------------------------------------------------------
 * Parameter-server update (Section 3.1: "the same settings we used in the
 * single GPU cases", i.e. the momentum SGD with weight decay of the cited
 * pipeline), applied to the whole flat parameter buffer:
 *   t = g + wd*w;   v = mu*v - lr*t;   w = w + v
 * ------------------------------------------------------------------------ */
void oracle_apply_update(double *w, double *v, const double *g, size_t count,
                         double lr, double mu, double wd)
{
    for (size_t i = 0; i < count; ++i) {
        const double t = g[i] + wd * w[i];
        v[i] = mu * v[i] - lr * t;
        w[i] = w[i] + v[i];
    }
}

/* ---------------------------------------------------------------------------
 * The two server updates the paper names as the next thing to try (Section 4,
 * "Future directions": Adagrad and Adadelta), with the same weight-decay
 * convention as above (t = g + wd*w).
 *   Adagrad  (Duchi et al. 2011):  h = h + t*t;   w = w - lr * t / (sqrt(h) + eps)
 *   Adadelta (Zeiler 2012, Algorithm 1):
 *       a = rho*a + (1-rho)*t*t;   d = -sqrt(b + eps) / sqrt(a + eps) * t;
 *       b = rho*b + (1-rho)*d*d;   w = w + d
 * ------------------------------------------------------------------------ */
void oracle_apply_adagrad(double *w, double *h, const double *g, size_t count, double lr, double eps, double wd)
{
    for (size_t i = 0; i < count; ++i) {
        const double t = g[i] + wd * w[i];
        h[i] = h[i] + t * t;
        w[i] = w[i] - lr * t / (sqrt(h[i]) + eps);
    }
}

void oracle_apply_adadelta(double *w, double *a, double *b, const double *g, size_t count, double rho, double eps, double wd)
{
    for (size_t i = 0; i < count; ++i) {
        const double t = g[i] + wd * w[i];
        a[i] = rho * a[i] + (1.0 - rho) * t * t;
        const double d = -sqrt(b[i] + eps) / sqrt(a[i] + eps) * t;
        b[i] = rho * b[i] + (1.0 - rho) * d * d;
        w[i] = w[i] + d;
    }
}

/* ---------------------------------------------------------------------------
 * Worker copy of the server's parameters (Section 2.3: a replica "requests
 * updated parameters").  fp32 -> bf16 by round-to-nearest-even on the bit
 * pattern; NaN stays a quiet NaN with its sign.
 * ------------------------------------------------------------------------ */
void oracle_snapshot_bf16(const float *params, uint16_t *copy, size_t count)
{
    for (size_t i = 0; i < count; ++i) {
        uint32_t u;
        memcpy(&u, &params[i], 4);
        if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) {
            copy[i] = (uint16_t)((u >> 16) | 0x0040u);
        } else {
            const uint32_t lsb = (u >> 16) & 1u;
            copy[i] = (uint16_t)((u + 0x7FFFu + lsb) >> 16);
        }
    }
}

/* Rounding of a stored activation to bf16 (round to nearest even of the fp32
 * value), for networks whose activations are kept in bf16 between layers: the
 * integer decisions that follow (pooling position, ReLU mask) are then taken on
 * the same values as in the implementation under test. */
void oracle_round_bf16(double *a, size_t count)
{
    for (size_t i = 0; i < count; ++i) {
        const float f = (float)a[i];
        uint16_t b;
        oracle_snapshot_bf16(&f, &b, 1);
        const uint32_t u = (uint32_t)b << 16;
        float r;
        memcpy(&r, &u, 4);
        a[i] = (double)r;
    }
}

/* ---------------------------------------------------------------------------
 * Staleness schedule for the A-SGD replay (Section 3.3 attributes artefacts
 * of the learning curves to stale updates).  Update a (0-based) is pushed by
 * worker a mod n_workers and was computed on parameter version
 * a - s_a, with s_a = min(a, top32(mix(mix(seed)+a)) mod (max_stale+1)).
 * ------------------------------------------------------------------------ */
void oracle_schedule(int32_t *worker, int32_t *read_version, int T, uint64_t seed,
                     int n_workers, int max_stale)
{
    for (int a = 0; a < T; ++a) {
        const uint32_t h = (uint32_t)(mix64(mix64(seed) + (uint64_t)a) >> 32);
        int s = (int)(h % (uint32_t)(max_stale + 1));
        if (s > a) s = a;
        worker[a] = a % n_workers;
        read_version[a] = a - s;
    }
}
