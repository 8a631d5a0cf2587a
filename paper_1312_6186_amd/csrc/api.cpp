// Host side of the C ABI declared in include/asgd.h: network planning, workspace
// management and the order in which the kernels of one minibatch gradient are
// enqueued.  No arithmetic of the method happens on the host.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/asgd.h"
#include "asgd_internal.h"

using namespace asgd;

namespace {

thread_local std::string g_err;

int fail(int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

int hip_fail(hipError_t e, const char *what) { return fail(ASGD_EHIP, "%s: %s", what, hipGetErrorString(e)); }

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

enum StageKind { ST_CONV = 1, ST_POOL = 2, ST_FC = 3, ST_LRN = 4 };

struct Stage {
    int kind = 0;
    int first_layer = 0, last_layer = 0;
    // spatial stages: channel-last tensors [B][H][W][Cp]
    int inC = 0, inCp = 0, inH = 0, inW = 0;
    int outC = 0, outCp = 0, outH = 0, outW = 0;
    // fc stages: [B][ld]
    int in_f = 0, out_f = 0, out_ld = 0;
    bool in_is_spatial = false;  // an fc fed by a conv / pool stage (flatten boundary)
    bool last = false;           // produces the fp32 logits
    int k = 0, stride = 1, pad = 0;
    int groups = 1;   // convolution channel groups
    // window-row form (first stage, <= 4 input channels): bordered input [B][rwHp][rwWp][rwC], K = k * rwKW
    int rw = 0, rwC = 0, rwKW = 0, rwHp = 0, rwWp = 0;
    int relu = 0, drop = 0, drop_layer = -1;
    float lrn_alpha = 0.f, lrn_beta = 0.f, lrn_bias = 0.f;   // ST_LRN (window size in k)
    bool has_params() const { return kind == ST_CONV || kind == ST_FC; }
    float drop_p = 0.f, drop_scale = 1.f;
    uint32_t drop_thr = 0;
    size_t w_off = 0, w_cnt = 0, b_off = 0, b_cnt = 0;
    // workspace
    void *out = nullptr, *dout = nullptr;
    uint8_t *argmax = nullptr;
    void *wf = nullptr, *wd = nullptr;
    void *flat_in = nullptr, *dflat_in = nullptr;
    float *colsum_ws = nullptr; size_t colsum_floats = 0;   // band sums of the bias gradient
    long pool_bands = 0;       // CONV directly under a pool whose backward kernel leaves those band sums: their number
    bool bands_ready = false;  // ... and whether the pool's backward pass of this call has left them
    GemmPlan p_fwd, p_dgrad, p_wgrad;
    size_t out_elems() const { return kind == ST_FC ? (size_t)out_ld : (size_t)outH * outW * outCp; }
};

}  // namespace

struct asgd_net {
    std::vector<asgd_layer_desc_t> layers;
    std::vector<int> layer_stage;         // descriptor index -> stage index (-1 for softmax)
    std::vector<int32_t> layer_shape;     // 3 per layer
    std::vector<Stage> stages;
    std::vector<asgd_tensor_info_t> tensors;
    int batch = 0, in_c = 0, in_cp = 0, in_h = 0, in_w = 0, dtype = 0, classes = 0;
    size_t param_count = 0;
    size_t ws_bytes = 0;
    // device workspace
    void *arena = nullptr;
    int device = -1;
    void *act0 = nullptr;      // staged input
    float *scratch = nullptr;       // split-K partials of the kernels on the caller's stream
    float *scratch_side = nullptr;  // split-K and column-sum partials of the parameter-gradient kernels (side stream)
    // The parameter gradients of a layer (and the filter packing of the forward pass) do not feed the next
    // layer: they run on an internal stream beside the caller's, forked and joined with events.
    hipStream_t side = nullptr;
    bool in_replay = false;   // replicas of a replay already run beside each other: no side stream then (measured slower)
    bool serial = false;      // every kernel on the caller's stream (asgd_net_set_serial, or ASGD_SERIAL=1 at creation)
    // Streams and events of the A-SGD replay, kept by the plan of worker 0 from one replay to the next (created on
    // first use, released with the plan), so that a replay only enqueues.
    std::vector<hipStream_t> replay_streams;   // one per worker, then the server's
    std::vector<hipEvent_t> replay_events;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr, ev_bias = nullptr;
    std::vector<hipEvent_t> ev_pack, ev_dy, ev_dg;   // per stage: filters packed, output gradient ready, data gradient issued
    float *row_loss = nullptr;
    int *version_counter = nullptr;  // device-side count of applied updates (A-SGD replay)
    size_t scratch_floats = 0, scratch_side_floats = 0;
    // key of the last forward pass (for the dropout mask export)
    uint64_t last_seed = 0, last_step = 0;
    uint32_t last_worker = 0;
    bool ran = false;
    // per-class event timing (asgd_profile_begin / asgd_profile_end)
    bool prof_on = false;
    std::vector<hipEvent_t> prof_ev;    // start, stop pairs
    std::vector<int> prof_cls;
    double prof_flops[ASGD_K_COUNT] = {0}, prof_bytes[ASGD_K_COUNT] = {0};
};

namespace {

struct Carver {
    size_t off = 0;
    size_t take(size_t bytes)
    {
        const size_t o = off;
        off += (bytes + 255) / 256 * 256;
        return o;
    }
};

// Lays the workspace out; with base == nullptr only the total size is computed.
size_t carve(asgd_net &n, char *base)
{
    Carver c;
    const size_t es = dtype_size(n.dtype);
    const size_t B = (size_t)n.batch;
    auto at = [&](size_t bytes) -> void * {
        const size_t o = c.take(bytes);
        return base ? base + o : nullptr;
    };
    // the arena is cleared once when it is allocated: the zero border of a bordered input is never written
    // afterwards; tensors are spaced by 256 spare bytes
    const Stage *s0 = n.stages.empty() ? nullptr : &n.stages[0];
    n.act0 = at((s0 && s0->rw ? B * s0->rwHp * s0->rwWp * s0->rwC : B * n.in_h * n.in_w * n.in_cp) * es + 256);
    for (size_t i = 0; i < n.stages.size(); ++i) {
        Stage &s = n.stages[i];
        const size_t oe = B * s.out_elems();
        s.out = at(oe * (s.last ? 4 : es) + 256);
        s.dout = at(oe * es + 256);
        if (s.kind == ST_POOL) s.argmax = static_cast<uint8_t *>(at(oe));
        if (s.kind == ST_CONV) {
            s.wf = at((size_t)s.outCp * s.k * (s.rw ? s.rwKW : s.k * s.inCp) * es);
            s.wd = i > 0 ? at((size_t)s.inCp * s.k * s.k * s.outCp * es) : nullptr;
        }
        if (s.has_params()) s.colsum_ws = static_cast<float *>(at(s.colsum_floats * 4));
        if (s.kind == ST_FC && s.in_is_spatial) {
            s.flat_in = at(B * s.in_f * es);
            s.dflat_in = at(B * s.in_f * es);
        }
    }
    n.row_loss = static_cast<float *>(at(B * 4));
    n.version_counter = static_cast<int *>(at(256));
    n.scratch = static_cast<float *>(at(n.scratch_floats * 4));
    n.scratch_side = static_cast<float *>(at(n.scratch_side_floats * 4));
    return c.off;
}

Gather conv_gather(const Stage &s, const void *x, int B, int dt, int group = 0);

int plan_net(asgd_net &n)
{
    const int L = (int)n.layers.size();
    n.layer_stage.assign(L, -1);
    n.layer_shape.assign(3 * L, 0);
    n.in_cp = round_up(n.in_c, 8);
    int C = n.in_c, H = n.in_h, W = n.in_w;
    long F = 0;  // > 0 once on the fc side
    size_t off = 0;
    int i = 0;
    while (i < L) {
        const asgd_layer_desc_t &l = n.layers[i];
        Stage s;
        s.first_layer = i;
        if (l.kind == ASGD_LAYER_CONV) {
            if (F > 0) return fail(ASGD_ESHAPE, "layer %d: CONV after FC", i);
            if (l.out <= 0 || l.k <= 0 || l.k > 15 || l.stride <= 0 || l.pad < 0) return fail(ASGD_ESHAPE, "layer %d: bad CONV parameters (filter size 1..15)", i);
            if (H + 2 * l.pad < l.k || W + 2 * l.pad < l.k) return fail(ASGD_ESHAPE, "layer %d: filter larger than padded input", i);
            s.kind = ST_CONV;
            s.groups = l.groups > 1 ? l.groups : 1;
            if (s.groups > 1 && (C % s.groups || l.out % s.groups || (C / s.groups) % 8 || (l.out / s.groups) % 8))
                return fail(ASGD_ESHAPE, "layer %d: a grouped CONV needs input and output channels per group in multiples of 8", i);
            s.inC = C; s.inCp = round_up(C, 8); s.inH = H; s.inW = W;
            s.k = l.k; s.stride = l.stride; s.pad = l.pad;
            s.outC = l.out; s.outCp = round_up(l.out, 8);
            s.outH = (H + 2 * l.pad - l.k) / l.stride + 1;
            s.outW = (W + 2 * l.pad - l.k) / l.stride + 1;
            // First layer over <= 4 channels: padding them to 8 would make most of the reduction zeros.  Keep the
            // pixels narrow and merge (kx, c) into one contiguous run per window row instead.  Pixels of exactly C
            // channels if the window origins (stride * C elements apart) stay dword-aligned, which is all a 16-byte
            // buffer load needs; else 4 channels per pixel if that keeps them 16-byte aligned; else the general form.
            const int es0 = (int)dtype_size(n.dtype);
            int rwC = 0;
            if (n.stages.empty() && C <= 4 && s.groups == 1) {
                if ((l.stride * C * es0) % 4 == 0) rwC = C;
                else if ((l.stride * 4 * es0) % 16 == 0) rwC = 4;
            }
            if (rwC) {
                s.rw = 1; s.rwC = rwC;
                s.rwKW = round_up(l.k * rwC, 8);   // the filter-gradient GEMM wants its column count in eights
                s.rwHp = H + 2 * l.pad;
                // a row holds the border and the padded run of the last window; its width is rounded up until a row is a
                // whole number of 16-byte pieces (rows then start 16-byte aligned, which the row-block copy of the
                // first-layer kernel and its 8-byte fragment reads rely on)
                s.rwWp = std::max(W + 2 * l.pad, (s.outW - 1) * l.stride + (s.rwKW + rwC - 1) / rwC);
                while (((size_t)s.rwWp * rwC * es0) % 16 != 0) ++s.rwWp;
            }
            s.w_off = off; s.w_cnt = (size_t)l.out * (C / s.groups) * l.k * l.k; s.b_off = off + s.w_cnt; s.b_cnt = l.out;
            off += s.w_cnt + s.b_cnt;
            C = l.out; H = s.outH; W = s.outW;
            n.layer_shape[3 * i] = C; n.layer_shape[3 * i + 1] = H; n.layer_shape[3 * i + 2] = W;
            if (i + 1 < L && n.layers[i + 1].kind == ASGD_LAYER_RELU) {
                s.relu = 1; ++i;
                n.layer_shape[3 * i] = C; n.layer_shape[3 * i + 1] = H; n.layer_shape[3 * i + 2] = W;
            }
        } else if (l.kind == ASGD_LAYER_MAXPOOL) {
            if (F > 0) return fail(ASGD_ESHAPE, "layer %d: MAXPOOL after FC", i);
            if (l.k <= 0 || l.k > 15 || l.stride <= 0 || H < l.k || W < l.k) return fail(ASGD_ESHAPE, "layer %d: bad MAXPOOL window", i);
            s.kind = ST_POOL;
            s.inC = s.outC = C; s.inCp = s.outCp = round_up(C, 8); s.inH = H; s.inW = W;
            s.k = l.k; s.stride = l.stride;
            s.outH = (H - l.k) / l.stride + 1; s.outW = (W - l.k) / l.stride + 1;
            H = s.outH; W = s.outW;
            n.layer_shape[3 * i] = C; n.layer_shape[3 * i + 1] = H; n.layer_shape[3 * i + 2] = W;
        } else if (l.kind == ASGD_LAYER_LRN) {
            if (n.stages.empty() || n.stages.back().kind != ST_CONV || !n.stages.back().relu)
                return fail(ASGD_ESHAPE, "layer %d: LRN must directly follow CONV + RELU", i);
            if (l.k < 1 || l.k > 9 || !(l.k & 1)) return fail(ASGD_ESHAPE, "layer %d: LRN window must be odd and at most 9", i);
            if (!(l.bias > 0.f) || !(l.p >= 0.f) || !(l.scale >= 0.f)) return fail(ASGD_ESHAPE, "layer %d: LRN needs bias > 0, alpha >= 0, beta >= 0", i);
            s.kind = ST_LRN;
            s.inC = s.outC = C; s.inCp = s.outCp = round_up(C, 8); s.inH = s.outH = H; s.inW = s.outW = W;
            s.k = l.k; s.lrn_alpha = l.p; s.lrn_beta = l.scale; s.lrn_bias = l.bias;
            n.layer_shape[3 * i] = C; n.layer_shape[3 * i + 1] = H; n.layer_shape[3 * i + 2] = W;
        } else if (l.kind == ASGD_LAYER_FC) {
            if (l.out <= 0) return fail(ASGD_ESHAPE, "layer %d: bad FC size", i);
            s.kind = ST_FC;
            s.in_is_spatial = F == 0;
            const long fin = F > 0 ? F : (long)C * H * W;
            if (fin % 8 != 0) return fail(ASGD_ESHAPE, "layer %d: FC fan-in %ld is not a multiple of 8", i, fin);
            if (fin > 0x7fffffffL / 4) return fail(ASGD_ESHAPE, "layer %d: FC fan-in too large", i);
            if (s.in_is_spatial) { s.inC = C; s.inCp = round_up(C, 8); s.inH = H; s.inW = W; }
            s.in_f = (int)fin; s.out_f = l.out; s.out_ld = round_up(l.out, 8);
            s.w_off = off; s.w_cnt = (size_t)l.out * fin; s.b_off = off + s.w_cnt; s.b_cnt = l.out;
            if (s.w_off % 8 != 0) return fail(ASGD_ESHAPE, "layer %d: FC weights start at element %zu, not a multiple of 8", i, s.w_off);
            off += s.w_cnt + s.b_cnt;
            F = l.out;
            n.layer_shape[3 * i] = (int)F; n.layer_shape[3 * i + 1] = 1; n.layer_shape[3 * i + 2] = 1;
            if (i + 1 < L && n.layers[i + 1].kind == ASGD_LAYER_RELU) {
                s.relu = 1; ++i;
                n.layer_shape[3 * i] = (int)F; n.layer_shape[3 * i + 1] = 1; n.layer_shape[3 * i + 2] = 1;
                if (i + 1 < L && n.layers[i + 1].kind == ASGD_LAYER_DROPOUT) {
                    ++i;
                    const asgd_layer_desc_t &d = n.layers[i];
                    if (!(d.p >= 0.f && d.p < 1.f)) return fail(ASGD_ESHAPE, "layer %d: dropout p must be in [0,1)", i);
                    if (d.scale < 0.f) return fail(ASGD_ESHAPE, "layer %d: dropout scale must be positive", i);
                    s.drop = 1; s.drop_layer = i; s.drop_p = d.p; s.drop_scale = d.scale == 0.f ? 1.f : d.scale;
                    s.drop_thr = (uint32_t)std::floor((double)d.p * 4294967296.0);
                    n.layer_shape[3 * i] = (int)F; n.layer_shape[3 * i + 1] = 1; n.layer_shape[3 * i + 2] = 1;
                }
            }
        } else if (l.kind == ASGD_LAYER_SOFTMAX_CE) {
            if (i != L - 1) return fail(ASGD_ESHAPE, "layer %d: SOFTMAX_CE must be last", i);
            if (n.stages.empty() || n.stages.back().kind != ST_FC || n.stages.back().relu)
                return fail(ASGD_ESHAPE, "layer %d: SOFTMAX_CE must directly follow an FC", i);
            n.stages.back().last = true;
            n.classes = (int)F;
            n.layer_shape[3 * i] = (int)F; n.layer_shape[3 * i + 1] = 1; n.layer_shape[3 * i + 2] = 1;
            ++i;
            break;
        } else if (l.kind == ASGD_LAYER_RELU) {
            return fail(ASGD_ESHAPE, "layer %d: RELU must directly follow a CONV or an FC", i);
        } else if (l.kind == ASGD_LAYER_DROPOUT) {
            return fail(ASGD_ESHAPE, "layer %d: DROPOUT must directly follow FC + RELU", i);
        } else {
            return fail(ASGD_EINVAL, "layer %d: unknown kind %d", i, l.kind);
        }
        s.last_layer = i;
        for (int j = s.first_layer; j <= s.last_layer; ++j) n.layer_stage[j] = (int)n.stages.size();
        if ((s.kind == ST_CONV || s.kind == ST_FC)) {
            asgd_tensor_info_t t;
            memset(&t, 0, sizeof t);
            t.layer = s.first_layer; t.kind = s.kind == ST_CONV ? ASGD_LAYER_CONV : ASGD_LAYER_FC;
            t.w_offset = s.w_off; t.w_count = s.w_cnt; t.b_offset = s.b_off; t.b_count = s.b_cnt;
            if (s.kind == ST_CONV) { t.w_shape[0] = s.outC; t.w_shape[1] = s.inC / s.groups; t.w_shape[2] = s.k; t.w_shape[3] = s.k; }
            else { t.w_shape[0] = s.out_f; t.w_shape[1] = s.in_f; t.w_shape[2] = 1; t.w_shape[3] = 1; }
            n.tensors.push_back(t);
        }
        n.stages.push_back(s);
        ++i;
    }
    if (n.classes == 0 || n.stages.empty() || !n.stages.back().last) return fail(ASGD_ESHAPE, "the layer list must end with FC, SOFTMAX_CE");
    n.param_count = off;

    // sizes, GEMM plans, scratch
    const long B = n.batch;
    size_t scratch = 0, scratch_side = 0;
    for (size_t si = 0; si < n.stages.size(); ++si) {
        Stage &s = n.stages[si];
        if (s.kind == ST_CONV) {
            const long M = B * s.outH * s.outW, Min = B * s.inH * s.inW;
            const long K = s.rw ? (long)s.k * s.rwKW : (long)s.k * s.k * s.inCp;
            if (s.rw && (long)B * s.rwHp * s.rwWp * s.rwC * 4 > 0x7fffffffL) return fail(ASGD_ESHAPE, "layer %d: tensor too large", s.first_layer);
            if (M > 0x7fffffffL / 2 || Min > 0x7fffffffL / 2 || M * s.outCp * 4 > 0x7fffffffL || Min * s.inCp * 4 > 0x7fffffffL) return fail(ASGD_ESHAPE, "layer %d: tensor too large", s.first_layer);
            if (s.groups > 1) {   // one GEMM per group, on that group's channel slices
                const long Cg = s.inC / s.groups, Og = s.outC / s.groups, Kg = (long)s.k * s.k * Cg;
                s.p_fwd = plan_gemm(M, Og, Kg, n.dtype, 1);
                s.p_dgrad = plan_gemm(Min, Cg, (long)s.k * s.k * Og, n.dtype, 1);
                s.p_wgrad = plan_gemm(Og, Kg, M, n.dtype, 128);
            } else {
                s.p_fwd = plan_gemm(M, s.outCp, K, n.dtype, 1);
                s.p_dgrad = plan_gemm(Min, s.inCp, (long)s.k * s.k * s.outCp, n.dtype, 1);
                s.p_wgrad = plan_gemm(s.outCp, K, M, n.dtype, 128);
                // the first layer's filter gradient as one persistent kernel wants a partial result per workgroup
                if (s.rw) s.p_wgrad.ws_floats = std::max(s.p_wgrad.ws_floats, rows_wgrad_ws_floats(n.dtype, s.outCp, conv_gather(s, nullptr, (int)B, n.dtype)));
            }
            scratch_side = std::max(scratch_side, s.p_wgrad.ws_floats);
            s.colsum_floats = colsum_ws_floats(n.dtype, M, s.outCp);
            if (si + 1 < n.stages.size() && n.stages[si + 1].kind == ST_POOL) {
                const Stage &pl = n.stages[si + 1];
                s.pool_bands = pool_bwd_bands(n.dtype, B, s.outH, s.outW, s.outCp, pl.k, pl.stride);
                s.colsum_floats = std::max(s.colsum_floats, (size_t)s.pool_bands * s.outCp);
            }
        } else if (s.kind == ST_FC) {
            s.p_fwd = plan_gemm(B, s.out_ld, s.in_f, n.dtype, 32);
            s.p_dgrad = plan_gemm(B, s.in_f, s.out_f, n.dtype, 32);
            s.p_wgrad = plan_gemm(s.out_f, s.in_f, B, n.dtype, 1);
            scratch = std::max(scratch, std::max(s.p_fwd.ws_floats, s.p_dgrad.ws_floats));
            s.colsum_floats = colsum_ws_floats(n.dtype, B, s.out_ld);
        }
    }
    n.scratch_floats = scratch + 64;
    n.scratch_side_floats = scratch_side + 64;
    n.ws_bytes = carve(n, nullptr);
    return ASGD_OK;
}

// Frees what ensure_prepared made (after waiting for the internal stream).
int release_device(asgd_net *n)
{
    int rc = ASGD_OK;
    if (n->side) { (void)hipStreamSynchronize(n->side); (void)hipStreamDestroy(n->side); n->side = nullptr; }
    for (hipStream_t st : n->replay_streams) if (st) { (void)hipStreamSynchronize(st); (void)hipStreamDestroy(st); }
    for (hipEvent_t e : n->replay_events) if (e) (void)hipEventDestroy(e);
    n->replay_streams.clear(); n->replay_events.clear();
    if (n->ev_fork) { (void)hipEventDestroy(n->ev_fork); n->ev_fork = nullptr; }
    if (n->ev_join) { (void)hipEventDestroy(n->ev_join); n->ev_join = nullptr; }
    if (n->ev_bias) { (void)hipEventDestroy(n->ev_bias); n->ev_bias = nullptr; }
    for (hipEvent_t e : n->ev_pack) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : n->ev_dy) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : n->ev_dg) if (e) (void)hipEventDestroy(e);
    n->ev_pack.clear(); n->ev_dy.clear(); n->ev_dg.clear();
    if (n->arena) {
        const hipError_t e = hipFree(n->arena);
        n->arena = nullptr;
        if (e != hipSuccess) rc = hip_fail(e, "hipFree");
    }
    return rc;
}

int ensure_prepared(asgd_net *n)
{
    if (n->arena) return ASGD_OK;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    e = hipMalloc(&n->arena, n->ws_bytes);
    if (e != hipSuccess) { n->arena = nullptr; (void)hipGetLastError(); return fail(ASGD_ENOMEM, "hipMalloc of %zu workspace bytes: %s", n->ws_bytes, hipGetErrorString(e)); }
    e = hipMemset(n->arena, 0, n->ws_bytes);
    if (e != hipSuccess) { (void)hipFree(n->arena); n->arena = nullptr; return hip_fail(e, "hipMemset"); }
    n->device = dev;
    carve(*n, static_cast<char *>(n->arena));
    e = hipStreamCreateWithFlags(&n->side, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&n->ev_fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&n->ev_join, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&n->ev_bias, hipEventDisableTiming);
    n->ev_pack.assign(n->stages.size(), nullptr);
    n->ev_dy.assign(n->stages.size(), nullptr);
    n->ev_dg.assign(n->stages.size(), nullptr);
    for (size_t i = 0; i < n->stages.size() && e == hipSuccess; ++i) {
        e = hipEventCreateWithFlags(&n->ev_pack[i], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&n->ev_dy[i], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&n->ev_dg[i], hipEventDisableTiming);
    }
    if (e != hipSuccess) { release_device(n); return hip_fail(e, "creating the internal stream and events"); }
    return ASGD_OK;
}

#define CHECK_HIP(expr, what)                                   \
    do {                                                        \
        const hipError_t e_ = (expr);                           \
        if (e_ != hipSuccess) return hip_fail(e_, what);        \
    } while (0)

#define CHECK_LAUNCH(expr, what)                                                             \
    do {                                                                                     \
        if ((expr) != 0) {                                                                   \
            const hipError_t e_ = hipGetLastError();                                         \
            return fail(ASGD_EHIP, "%s: %s", what, e_ == hipSuccess ? "bad launch arguments" : hipGetErrorString(e_)); \
        }                                                                                    \
    } while (0)

// Brackets one operation with a pair of events when profiling is on.
struct ProfScope {
    asgd_net *n; hipStream_t st; hipEvent_t stop = nullptr;
    ProfScope(asgd_net *net, hipStream_t s, int cls, double flops, double bytes) : n(net), st(s)
    {
        if (!n->prof_on) return;
        hipEvent_t a = nullptr, b = nullptr;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { if (a) (void)hipEventDestroy(a); return; }
        (void)hipEventRecord(a, st);
        n->prof_ev.push_back(a); n->prof_ev.push_back(b); n->prof_cls.push_back(cls);
        n->prof_flops[cls] += flops; n->prof_bytes[cls] += bytes;
        stop = b;
    }
    ~ProfScope() { if (stop) (void)hipEventRecord(stop, st); }
};

// ASGD_SERIAL=1 in the environment makes new plans keep every kernel on the caller's stream (no internal side
// stream), so that a profiler sees each kernel running alone; asgd_net_set_serial switches one plan.  The results
// are the same bit for bit either way (every kernel is deterministic and the two streams share no output).
bool serial_default()
{
    static const bool on = getenv("ASGD_SERIAL") && getenv("ASGD_SERIAL")[0] == '1';
    return on;
}

// ReLU commutes with max pooling, and the pooled value is the value at the recorded maximum: where a pooling
// stage sits on a CONV+RELU, the ReLU mask of that convolution is applied to the gradient at the pool's OUTPUT
// (mask = pooled activation > 0) by whoever produces that gradient, and the pooling backward pass then has
// nothing to read but the gradient and the positions.
bool relu_under_pool(const std::vector<Stage> &st, int pool_idx)
{
    return pool_idx > 0 && st[pool_idx].kind == ST_POOL && st[pool_idx - 1].kind == ST_CONV && st[pool_idx - 1].relu;
}

// The input side of a convolution stage as a gather over its (possibly bordered) input tensor x.
Gather conv_gather(const Stage &s, const void *x, int B, int dt, int group)
{
    const size_t es = dtype_size(dt);
    Gather g;
    g.x = x; g.N = B; g.Ho = s.outH; g.Wo = s.outW; g.sm = s.stride; g.ds = 1;
    if (s.groups > 1) {   // the group's channels of every pixel: pixels keep the full tensor's strides
        const int Cg = s.inC / s.groups;
        g.x = static_cast<const char *>(x) + (size_t)group * Cg * es;
        g.H = s.inH; g.W = s.inW; g.C = Cg; g.kh = g.kw = s.k; g.pad = s.pad;
        g.pix = (size_t)s.inCp * es; g.rowb = (size_t)s.inW * s.inCp * es;
        g.bytes = (size_t)B * s.inH * s.inW * s.inCp * es - (size_t)group * Cg * es;
        return g;
    }
    if (s.rw) {
        g.H = s.rwHp; g.W = s.rwWp; g.C = s.rwKW; g.kh = s.k; g.kw = 1; g.pad = 0;
        g.pix = (size_t)s.rwC * es; g.rowb = (size_t)s.rwWp * s.rwC * es;
        g.bytes = (size_t)B * s.rwHp * s.rwWp * s.rwC * es;
    } else {
        g.H = s.inH; g.W = s.inW; g.C = s.inCp; g.kh = g.kw = s.k; g.pad = s.pad;
        g.bytes = (size_t)B * s.inH * s.inW * s.inCp * es;
    }
    return g;
}

const char *param_ptr(const asgd_net *n, const void *params, size_t off) { return static_cast<const char *>(params) + off * dtype_size(n->dtype); }

int forward(asgd_net *n, const void *params, const void *images, const int32_t *labels, uint64_t seed, uint64_t step, uint32_t worker,
            float *loss, hipStream_t st)
{
    const int B = n->batch, dt = n->dtype;
    const double es = (double)dtype_size(dt), Bd = (double)B;
    {
        ProfScope ps(n, st, ASGD_K_LAYOUT, 0, 2 * Bd * n->in_c * n->in_h * n->in_w * es);
        const Stage &s0 = n->stages[0];
        if (s0.rw) CHECK_LAUNCH(launch_stage_input_rw(dt, images, n->act0, B, n->in_c, n->in_h, n->in_w, s0.pad, s0.rwWp, s0.rwC, st), "stage_input");
        else CHECK_LAUNCH(launch_stage_input(dt, images, n->act0, B, n->in_c, n->in_h, n->in_w, n->in_cp, st), "stage_input");
    }
    // filter packing: beside the input staging and the first layers (in line when profiling, to be timed alone)
    const bool fork = !n->prof_on && !n->in_replay && !n->serial;
    hipStream_t sd = fork ? n->side : st;
    if (fork) {
        CHECK_HIP(hipEventRecord(n->ev_fork, st), "hipEventRecord");
        CHECK_HIP(hipStreamWaitEvent(sd, n->ev_fork, 0), "hipStreamWaitEvent");
    }
    {   // all layers' filters in one launch (twelve layers per launch at most)
        PackJobs jobs; jobs.n = 0; jobs.total = 0;
        double bytes = 0;
        auto flush = [&]() -> int {
            if (jobs.n == 0) return ASGD_OK;
            ProfScope ps(n, sd, ASGD_K_LAYOUT, 0, bytes);
            CHECK_LAUNCH(launch_pack_conv(dt, jobs, sd), "pack_conv");
            jobs.n = 0; bytes = 0;
            return ASGD_OK;
        };
        for (size_t si = 0; si < n->stages.size(); ++si) {
            Stage &s = n->stages[si];
            if (s.kind != ST_CONV) continue;
            if (s.groups > 1) {
                // forward pack of all groups at once (rows are output channels, each over its group's Cg inputs);
                // one flipped data-gradient pack per group
                const int Cg = s.inC / s.groups, Og = s.outC / s.groups;
                const size_t gw = (size_t)Og * Cg * s.k * s.k;          // canonical filters / packed elements of one group
                {
                    PackJob &J = jobs.j[jobs.n++];
                    J.w = param_ptr(n, params, s.w_off); J.wf = s.wf; J.wd = nullptr;
                    J.cout = s.outC; J.cin = Cg; J.k = s.k; J.coutp = s.outC; J.cinp = Cg; J.rw = 0; J.KW = 0;
                    bytes += (double)s.w_cnt * es * 2;
                    if (jobs.n == 12) { const int rc = flush(); if (rc != ASGD_OK) return rc; }
                }
                for (int g = 0; g < s.groups && s.wd; ++g) {
                    PackJob &J = jobs.j[jobs.n++];
                    J.w = param_ptr(n, params, s.w_off + g * gw); J.wf = nullptr; J.wd = static_cast<char *>(s.wd) + g * gw * dtype_size(dt);
                    J.cout = Og; J.cin = Cg; J.k = s.k; J.coutp = Og; J.cinp = Cg; J.rw = 0; J.KW = 0;
                    bytes += (double)gw * es * 2;
                    if (jobs.n == 12) { const int rc = flush(); if (rc != ASGD_OK) return rc; }
                }
                continue;
            }
            PackJob &J = jobs.j[jobs.n++];
            J.w = param_ptr(n, params, s.w_off); J.wf = s.wf; J.wd = s.rw ? nullptr : s.wd;
            J.cout = s.outC; J.cin = s.inC; J.k = s.k; J.coutp = s.outCp; J.cinp = s.inCp; J.rw = s.rw ? s.rwC : 0; J.KW = s.rwKW;
            bytes += (double)s.w_cnt * es * (J.wd ? 3 : 2);
            if (jobs.n == 12) { const int rc = flush(); if (rc != ASGD_OK) return rc; }
        }
        const int rc = flush();
        if (rc != ASGD_OK) return rc;
        if (fork) CHECK_HIP(hipEventRecord(n->ev_pack[0], sd), "hipEventRecord");
    }
    bool packed_seen = false;
    const void *cur = n->act0;
    for (size_t si = 0; si < n->stages.size(); ++si) {
        Stage &s = n->stages[si];
        if (s.kind == ST_CONV) {
            if (fork && !packed_seen) CHECK_HIP(hipStreamWaitEvent(st, n->ev_pack[0], 0), "hipStreamWaitEvent");
            packed_seen = true;
            const double Mo = Bd * s.outH * s.outW;
            ProfScope ps(n, st, ASGD_K_CONV_FWD, 2 * Mo * s.outC * (s.inC / s.groups) * s.k * s.k,
                         (Bd * s.inH * s.inW * s.inC + (double)s.w_cnt + Mo * s.outC) * es);
            if (s.groups > 1) {
                const int Cg = s.inC / s.groups, Og = s.outC / s.groups;
                const long Kg = (long)s.k * s.k * Cg;
                for (int gi = 0; gi < s.groups; ++gi) {
                    const Gather g = conv_gather(s, cur, B, dt, gi);
                    Epilogue ep;
                    ep.out = static_cast<char *>(s.out) + (size_t)gi * Og * dtype_size(dt); ep.ld = s.outCp;
                    ep.bias = param_ptr(n, params, s.b_off + (size_t)gi * Og); ep.bias_n = Og; ep.relu = s.relu;
                    CHECK_LAUNCH(gemm_gather_plain(dt, g, static_cast<const char *>(s.wf) + (size_t)gi * Og * Kg * dtype_size(dt), Kg, Og, ep, s.p_fwd,
                                                   n->scratch, st),
                                 "conv forward");
                }
            } else {
                const Gather g = conv_gather(s, cur, B, dt);
                Epilogue ep;
                ep.out = s.out; ep.ld = s.outCp; ep.bias = param_ptr(n, params, s.b_off); ep.bias_n = s.outC; ep.relu = s.relu;
                CHECK_LAUNCH(gemm_gather_plain(dt, g, s.wf, (long)g.kh * g.kw * g.C, s.outCp, ep, s.p_fwd, n->scratch, st), "conv forward");
            }
        } else if (s.kind == ST_LRN) {
            ProfScope ps(n, st, ASGD_K_LRN, 0, 2 * Bd * s.outC * s.outH * s.outW * es);
            CHECK_LAUNCH(launch_lrn_fwd(dt, cur, s.out, (size_t)B * s.outH * s.outW, s.outCp, s.k, s.lrn_alpha, s.lrn_beta, s.lrn_bias, st), "lrn forward");
        } else if (s.kind == ST_POOL) {
            ProfScope ps(n, st, ASGD_K_POOL_FWD, 0, Bd * s.outC * ((double)s.inH * s.inW * es + (double)s.outH * s.outW * (es + 1)));
            CHECK_LAUNCH(launch_pool_fwd(dt, cur, s.out, s.argmax, B, s.inH, s.inW, s.inCp, s.k, s.stride, st), "pool forward");
        } else {
            const void *x = cur;
            long ldx = si > 0 && n->stages[si - 1].kind == ST_FC ? n->stages[si - 1].out_ld : s.in_f;
            if (s.in_is_spatial) {
                ProfScope ps(n, st, ASGD_K_LAYOUT, 0, 2 * Bd * s.in_f * es);
                CHECK_LAUNCH(launch_flatten(dt, cur, s.flat_in, B, s.inH, s.inW, s.inC, s.inCp, st), "flatten");
                x = s.flat_in;
                ldx = s.in_f;
            }
            Epilogue ep;
            ep.out = s.out; ep.ld = s.out_ld; ep.out_f32 = s.last ? 1 : 0;
            ep.bias = param_ptr(n, params, s.b_off); ep.bias_n = s.out_f; ep.relu = s.relu;
            if (s.drop) {
                ep.drop = 1; ep.drop_key = dropout_key(seed, step, worker, (uint32_t)s.drop_layer);
                ep.drop_thr = s.drop_thr; ep.drop_F = s.out_f; ep.drop_scale = s.drop_scale;
            }
            ProfScope ps(n, st, ASGD_K_FC_FWD, 2 * Bd * s.in_f * s.out_f, (Bd * s.in_f + (double)s.w_cnt) * es + Bd * s.out_f * (s.last ? 4 : es));
            CHECK_LAUNCH(gemm_plain_plain(dt, x, ldx, B, param_ptr(n, params, s.w_off), s.in_f, s.out_ld, s.out_f, s.in_f, ep, s.p_fwd, n->scratch, st),
                         "fc forward");
        }
        cur = s.out;
    }
    Stage &last = n->stages.back();
    ProfScope ps(n, st, ASGD_K_SOFTMAX_CE, 0, Bd * n->classes * (4 + es));
    CHECK_LAUNCH(launch_softmax_ce(dt, static_cast<const float *>(last.out), last.out_ld, labels, B, n->classes, last.dout, loss, n->row_loss, st),
                 "softmax cross-entropy");
    return ASGD_OK;
}

// The server side of a whole training step: where a replica and the server share the GPU, a layer's slice of
// the parameters is updated (and the replica's copy of it refreshed) as soon as that layer's gradient is complete
// and its data gradient, the last reader of the old values, has been issued.
struct ServerArgs {
    float *master, *momentum;
    void *copy;          // the replica's parameters (== params of the step), compute dtype
    float lr, mu, wd;
    bool fuse;           // fully-connected weights: the push happens inside the weight-gradient kernel, which stores no gradient
};

int backward(asgd_net *n, const void *params, float *grads, hipStream_t st, const ServerArgs *srv)
{
    const int B = n->batch, dt = n->dtype;
    const double es = (double)dtype_size(dt), Bd = (double)B;
    const bool fork = !n->prof_on && !n->in_replay && !n->serial;
    hipStream_t sd = fork ? n->side : st;   // parameter gradients go here
    ColsumJobs bias_jobs; bias_jobs.n = 0;  // second stage of the bias gradients: one launch at the end, or per layer when pushing by layer
    ColsumS1Jobs bias_s1; bias_s1.n = 0;    // first stages that wait for that launch too (one launch for all of them)
    double bias_s1_bytes = 0;
    int first_param = -1;
    for (int q = 0; q < (int)n->stages.size() && first_param < 0; ++q) if (n->stages[q].has_params()) first_param = q;
    // Whether a fully-connected layer's weights are pushed by its weight-gradient kernel: whole sums (no split-K) and
    // 16-byte rows in the three parameter-shaped buffers.
    auto fused_fc = [&](const Stage &s) -> bool {
        return srv && srv->fuse && s.kind == ST_FC && s.p_wgrad.splits == 1 && s.in_f % 8 == 0 && s.w_off % 8 == 0;
    };
    // Push by layer (asgd_train_step), or, with fused fully-connected weights, everything else in one pass per
    // contiguous range behind the backward pass.
    const bool by_layer = srv && !srv->fuse;
    // Column sums of dy [M][ld] into db: at once when pushing by layer; otherwise the tensor joins the one first-stage
    // launch that precedes the second stage (the tensors stay where they are until the pass ends).
    auto bias_sums = [&](const void *dy, long ld, long M, int N, float *db, float *ws, double bytes, const char *what) -> int {
        if (by_layer) {
            ProfScope ps(n, sd, ASGD_K_BIAS_GRAD, 0, bytes);
            CHECK_LAUNCH(launch_colsum_partial(dt, dy, ld, M, N, db, ws, bias_jobs, sd), what);
            CHECK_LAUNCH(launch_colsum_finish(bias_jobs, sd), what);
            return ASGD_OK;
        }
        if (bias_s1.n == 12 || bias_jobs.n == 12) {
            ProfScope ps(n, sd, ASGD_K_BIAS_GRAD, 0, bias_s1_bytes);
            CHECK_LAUNCH(launch_colsum_stage1(dt, bias_s1, sd), what);
            CHECK_LAUNCH(launch_colsum_finish(bias_jobs, sd), what);
            bias_s1_bytes = 0;
        }
        if (colsum_partial_defer(dt, dy, ld, M, N, db, ws, bias_s1, bias_jobs) != 0) return fail(ASGD_EINVAL, "%s: bad shape", what);
        bias_s1_bytes += bytes;
        return ASGD_OK;
    };
    auto bias_first_stages = [&]() -> int {   // the pending first stages, on the side stream
        if (bias_s1.n == 0) return ASGD_OK;
        ProfScope ps(n, sd, ASGD_K_BIAS_GRAD, 0, bias_s1_bytes);
        CHECK_LAUNCH(launch_colsum_stage1(dt, bias_s1, sd), "bias gradients");
        bias_s1_bytes = 0;
        return ASGD_OK;
    };
    auto push = [&](int si) -> int {      // after the stage's gradients are queued on sd and its data gradient on st
        Stage &s = n->stages[si];
        if (!by_layer || !s.has_params()) return ASGD_OK;
        if (fork) {
            CHECK_HIP(hipEventRecord(n->ev_dg[si], st), "hipEventRecord");
            CHECK_HIP(hipStreamWaitEvent(sd, n->ev_dg[si], 0), "hipStreamWaitEvent");
        }
        const size_t off = s.w_off, cnt = s.w_cnt + s.b_cnt;   // weights and bias of a layer are adjacent
        ProfScope ps(n, sd, ASGD_K_UPDATE, 0, (double)cnt * (20.0 + es));
        if (launch_update_snapshot(srv->master + off, srv->momentum + off, grads + off, cnt, srv->lr, srv->mu, srv->wd,
                                   static_cast<char *>(srv->copy) + off * dtype_size(dt), dt, sd) != 0)
            return hip_fail(hipGetLastError(), "update kernel");
        return ASGD_OK;
    };
    for (int si = (int)n->stages.size() - 1; si >= 0; --si) {
        Stage &s = n->stages[si];
        Stage *prev = si > 0 ? &n->stages[si - 1] : nullptr;
        const void *xin = prev ? prev->out : n->act0;
        if (fork && s.has_params()) {  // the gradient at this stage's output is complete on the caller's stream
            CHECK_HIP(hipEventRecord(n->ev_dy[si], st), "hipEventRecord");
            CHECK_HIP(hipStreamWaitEvent(sd, n->ev_dy[si], 0), "hipStreamWaitEvent");
        }
        if (s.kind == ST_FC) {
            const void *x = s.in_is_spatial ? s.flat_in : xin;
            const long ldx = s.in_is_spatial ? s.in_f : prev->out_ld;
            const bool fused = fused_fc(s);
            auto param_grads = [&]() -> int {
                Epilogue ew;
                ew.out = grads + s.w_off; ew.ld = s.in_f; ew.out_f32 = 1;
                if (fused) {
                    ew.upd_w = srv->master + s.w_off; ew.upd_v = srv->momentum + s.w_off;
                    ew.upd_copy = static_cast<char *>(srv->copy) + s.w_off * dtype_size(dt);
                    ew.upd_lr = srv->lr; ew.upd_mu = srv->mu; ew.upd_wd = srv->wd;
                }
                {
                    ProfScope ps(n, sd, ASGD_K_FC_WGRAD, 2 * Bd * s.in_f * s.out_f,
                                 Bd * (s.in_f + s.out_f) * es + (double)s.w_cnt * (fused ? 16.0 + es : 4.0));
                    CHECK_LAUNCH(gemm_trans_trans(dt, s.dout, s.out_ld, s.out_f, x, ldx, s.in_f, B, ew, s.p_wgrad, n->scratch_side, sd), "fc weight gradient");
                }
                return bias_sums(s.dout, s.out_ld, B, s.out_f, grads + s.b_off, s.colsum_ws, Bd * s.out_f * es + s.out_f * 4.0, "fc bias gradient");
            };
            auto data_grad = [&]() -> int {
                if (!prev) return ASGD_OK;
                Epilogue ed;
                if (s.in_is_spatial) {
                    ed.out = s.dflat_in; ed.ld = s.in_f;
                } else {
                    ed.out = prev->dout; ed.ld = prev->out_ld;
                    if (prev->relu) { ed.mask_src = prev->out; ed.mask_ld = prev->out_ld; ed.mask_scale = prev->drop ? prev->drop_scale : 1.f; }
                }
                {
                    ProfScope ps(n, st, ASGD_K_FC_DGRAD, 2 * Bd * s.in_f * s.out_f, (Bd * s.out_f + (double)s.w_cnt + Bd * s.in_f * (ed.mask_src ? 2 : 1)) * es);
                    CHECK_LAUNCH(gemm_plain_trans(dt, s.dout, s.out_ld, B, param_ptr(n, params, s.w_off), s.in_f, s.in_f, s.out_f, ed, s.p_dgrad,
                                                  n->scratch, st),
                                 "fc data gradient");
                }
                ProfScope ps(n, st, ASGD_K_LAYOUT, 0, s.in_is_spatial ? 3 * Bd * s.in_f * es : 0);
                if (s.in_is_spatial)
                    CHECK_LAUNCH(launch_unflatten(dt, s.dflat_in, prev->out, (prev->kind == ST_CONV && prev->relu) || relu_under_pool(n->stages, si - 1),
                                                  prev->dout, B, s.inH, s.inW, s.inC, s.inCp, st),
                                 "unflatten");
                return ASGD_OK;
            };
            // A fused layer's weight-gradient kernel rewrites the replica's weights, which the data gradient reads: the
            // data gradient goes first and the other stream waits for it.
            int frc = ASGD_OK;
            if (fused) {
                frc = data_grad();
                if (frc == ASGD_OK && fork) {
                    CHECK_HIP(hipEventRecord(n->ev_dg[si], st), "hipEventRecord");
                    CHECK_HIP(hipStreamWaitEvent(sd, n->ev_dg[si], 0), "hipStreamWaitEvent");
                }
                if (frc == ASGD_OK) frc = param_grads();
            } else {
                frc = param_grads();
                if (frc == ASGD_OK) frc = data_grad();
            }
            if (frc != ASGD_OK) return frc;
        } else if (s.kind == ST_LRN) {
            // prev is the CONV + RELU it normalises: the ReLU mask of that convolution is applied here
            ProfScope ps(n, st, ASGD_K_LRN, 0, 3 * Bd * s.outC * s.outH * s.outW * es);
            CHECK_LAUNCH(launch_lrn_bwd(dt, prev->out, s.dout, 1, prev->dout, (size_t)B * s.outH * s.outW, s.outCp, s.k, s.lrn_alpha, s.lrn_beta,
                                        s.lrn_bias, st),
                         "lrn backward");
        } else if (s.kind == ST_POOL) {
            // prev exists: a pool cannot be first... unless the net starts with a pool, which feeds no parameters
            // a ReLU below has been applied to s.dout already by a CONV or FC above (relu_under_pool); only a pool
            // on top of this pool leaves it to be done here
            const bool masked_above = si + 1 < (int)n->stages.size() && n->stages[si + 1].has_params();
            const bool relu_here = prev && prev->kind == ST_CONV && prev->relu && !masked_above;
            ProfScope ps(n, st, ASGD_K_POOL_BWD, 0,
                         Bd * s.outC * ((double)s.outH * s.outW * (es + 1) + (double)s.inH * s.inW * es * (relu_here ? 2 : 1)));
            if (prev) {
                // what this writes is the output gradient of a convolution directly below: the kernel can leave the
                // first stage of that layer's bias gradient behind, which saves reading the tensor again
                float *bands = nullptr;
                if (prev->kind == ST_CONV && prev->pool_bands > 0) { bands = prev->colsum_ws; prev->bands_ready = true; }
                CHECK_LAUNCH(launch_pool_bwd(dt, s.dout, s.argmax, prev->out, relu_here, prev->dout, B, s.inH, s.inW, s.inCp, s.k, s.stride, bands, st),
                             "pool backward");
            }
        } else {
            const long M = (long)B * s.outH * s.outW;
            const double Mo = (double)M, conv_flops = 2 * Mo * s.outC * (s.inC / s.groups) * s.k * s.k;
            const int Cg = s.inC / s.groups, Og = s.outC / s.groups;   // channels per group (all of them when ungrouped)
            const size_t esz = dtype_size(dt);
            auto bias_part = [&]() -> int {
                if (!s.bands_ready)
                    return bias_sums(s.dout, s.outCp, M, s.outC, grads + s.b_off, s.colsum_ws, Mo * s.outC * es + s.outC * 4.0, "conv bias gradient");
                // the pooling backward pass above has left the band sums
                s.bands_ready = false;
                ProfScope ps(n, sd, ASGD_K_BIAS_GRAD, 0, s.outC * 4.0);
                if (bias_jobs.n == 12) {
                    CHECK_LAUNCH(launch_colsum_stage1(dt, bias_s1, sd), "conv bias gradient");
                    CHECK_LAUNCH(launch_colsum_finish(bias_jobs, sd), "conv bias gradient");
                }
                ColsumJob &J = bias_jobs.j[bias_jobs.n++];
                J.ws = s.colsum_ws; J.nblk = (int)s.pool_bands; J.ld = s.outCp; J.N = s.outC; J.db = grads + s.b_off; J.start_block = 0; J.colmajor = 1;
                if (by_layer) CHECK_LAUNCH(launch_colsum_finish(bias_jobs, sd), "conv bias gradient");
                return ASGD_OK;
            };
            // The last layer of the backward pass: its filter gradient is the tail of the side stream, which ends after
            // the caller's.  The second stage of all bias gradients goes to the caller's stream before it, so that it
            // runs beside that GEMM instead of behind it.
            const bool bias_first = fork && !by_layer && si == first_param;
            if (bias_first) {
                int brc = bias_part();
                if (brc == ASGD_OK) brc = bias_first_stages();
                if (brc != ASGD_OK) return brc;
                CHECK_HIP(hipEventRecord(n->ev_bias, sd), "hipEventRecord");
                CHECK_HIP(hipStreamWaitEvent(st, n->ev_bias, 0), "hipStreamWaitEvent");
                CHECK_LAUNCH(launch_colsum_finish(bias_jobs, st), "bias gradients");
            }
            {
                ProfScope ps(n, sd, ASGD_K_CONV_WGRAD, conv_flops, (Mo * s.outC + Bd * s.inH * s.inW * s.inC) * es + (double)s.w_cnt * 4);
                if (s.groups > 1) {
                    for (int gi = 0; gi < s.groups; ++gi) {
                        const Gather g = conv_gather(s, xin, B, dt, gi);
                        Epilogue ew;
                        ew.out = grads + s.w_off + (size_t)gi * Og * Cg * s.k * s.k; ew.mode = 1; ew.out_f32 = 1;
                        ew.cw_cout = Og; ew.cw_cin = Cg; ew.cw_cinp = Cg; ew.cw_kh = s.k; ew.cw_kw = s.k;
                        CHECK_LAUNCH(gemm_trans_gather(dt, static_cast<const char *>(s.dout) + (size_t)gi * Og * esz, s.outCp, Og, g, ew, s.p_wgrad,
                                                       n->scratch_side, sd),
                                     "conv filter gradient");
                    }
                } else {
                    const Gather g = conv_gather(s, xin, B, dt);
                    Epilogue ew;
                    ew.out = grads + s.w_off; ew.mode = s.rw ? 2 : 1; ew.out_f32 = 1;
                    ew.cw_cout = s.outC; ew.cw_cin = s.inC; ew.cw_cinp = s.rw ? s.rwKW : s.inCp; ew.cw_kh = s.k; ew.cw_kw = s.k; ew.cw_rwc = s.rw ? s.rwC : 4;
                    CHECK_LAUNCH(gemm_trans_gather(dt, s.dout, s.outCp, s.outCp, g, ew, s.p_wgrad, n->scratch_side, sd), "conv filter gradient");
                }
            }
            if (!bias_first) {
                const int brc = bias_part();
                if (brc != ASGD_OK) return brc;
            }
            if (prev) {
                const bool masked = (prev->kind == ST_CONV && prev->relu) || relu_under_pool(n->stages, si - 1);
                ProfScope ps(n, st, ASGD_K_CONV_DGRAD, conv_flops,
                             (Mo * s.outC + (double)s.w_cnt + Bd * s.inH * s.inW * s.inC * (masked ? 2 : 1)) * es);
                for (int gi = 0; gi < s.groups; ++gi) {
                    // the group's slice of the output gradient, gathered with the flipped filters of that group
                    const int Ogp = s.groups > 1 ? Og : s.outCp, Cgp = s.groups > 1 ? Cg : s.inCp;
                    Gather d;
                    d.x = static_cast<const char *>(s.dout) + (size_t)gi * Og * esz; d.N = B; d.H = s.outH; d.W = s.outW; d.C = Ogp;
                    d.Ho = s.inH; d.Wo = s.inW;
                    d.kh = d.kw = s.k; d.sm = 1; d.ds = s.stride; d.pad = s.k - 1 - s.pad;
                    d.pix = (size_t)s.outCp * esz; d.rowb = (size_t)s.outW * s.outCp * esz;
                    d.bytes = (size_t)B * s.outH * s.outW * s.outCp * esz - (size_t)gi * Og * esz;
                    Epilogue ed;
                    ed.out = static_cast<char *>(prev->dout) + (size_t)gi * Cg * esz; ed.ld = s.inCp;
                    if (masked) { ed.mask_src = static_cast<const char *>(prev->out) + (size_t)gi * Cg * esz; ed.mask_ld = s.inCp; ed.mask_scale = 1.f; }
                    const void *wd = static_cast<const char *>(s.wd) + (size_t)gi * Og * Cg * s.k * s.k * esz;
                    CHECK_LAUNCH(gemm_gather_plain(dt, d, wd, (long)s.k * s.k * Ogp, Cgp, ed, s.p_dgrad, n->scratch, st), "conv data gradient");
                }
            }
        }
        const int prc = push(si);
        if (prc != ASGD_OK) return prc;
    }
    {
        const int brc = bias_first_stages();
        if (brc != ASGD_OK) return brc;
        ProfScope ps(n, sd, ASGD_K_BIAS_GRAD, 0, 0);
        CHECK_LAUNCH(launch_colsum_finish(bias_jobs, sd), "bias gradients");
    }
    if (fork) {
        CHECK_HIP(hipEventRecord(n->ev_join, sd), "hipEventRecord");
        CHECK_HIP(hipStreamWaitEvent(st, n->ev_join, 0), "hipStreamWaitEvent");
    }
    if (srv && srv->fuse) {
        // everything the gradient kernels have not pushed themselves: maximal runs of adjacent slices, up to eight runs
        // per launch (for an AlexNet-style net: all convolution layers in one run, then one run per fully-connected bias)
        size_t offs[8], cnts[8];
        int nr = 0;
        auto flush = [&]() -> int {
            if (nr == 0) return ASGD_OK;
            double total = 0;
            for (int q = 0; q < nr; ++q) total += (double)cnts[q];
            ProfScope ps(n, st, ASGD_K_UPDATE, 0, total * (20.0 + es));
            if (launch_update_snapshot_ranges(srv->master, srv->momentum, grads, offs, cnts, nr, srv->lr, srv->mu, srv->wd, srv->copy, dt, st) != 0)
                return hip_fail(hipGetLastError(), "update kernel");
            nr = 0;
            return ASGD_OK;
        };
        auto add = [&](size_t off, size_t cnt) -> int {
            if (cnt == 0) return ASGD_OK;
            if (nr && offs[nr - 1] + cnts[nr - 1] == off) { cnts[nr - 1] += cnt; return ASGD_OK; }
            if (nr == 8) { const int rc = flush(); if (rc != ASGD_OK) return rc; }
            offs[nr] = off; cnts[nr] = cnt; ++nr;
            return ASGD_OK;
        };
        for (const Stage &s : n->stages) {
            if (!s.has_params()) continue;
            int rc = ASGD_OK;
            if (!fused_fc(s)) rc = add(s.w_off, s.w_cnt);
            if (rc == ASGD_OK) rc = add(s.b_off, s.b_cnt);
            if (rc != ASGD_OK) return rc;
        }
        const int rc = flush();
        if (rc != ASGD_OK) return rc;
    }
    return ASGD_OK;
}

}  // namespace

extern "C" {

const char *asgd_last_error(void) { return g_err.c_str(); }

int asgd_net_create(const asgd_layer_desc_t *layers, int n_layers, int batch, int in_c, int in_h, int in_w, int compute_dtype, asgd_net_t **out)
{
    if (!layers || !out) return fail(ASGD_EINVAL, "asgd_net_create: null argument");
    *out = nullptr;
    if (n_layers <= 0 || n_layers > 4096) return fail(ASGD_EINVAL, "asgd_net_create: bad layer count %d", n_layers);
    if (batch <= 0 || in_c <= 0 || in_h <= 0 || in_w <= 0) return fail(ASGD_ESHAPE, "asgd_net_create: batch and image sizes must be positive");
    if ((long)batch * in_c * in_h * in_w > 0x7fffffffL) return fail(ASGD_ESHAPE, "asgd_net_create: input larger than 2^31 elements");
    if (compute_dtype != ASGD_F32 && compute_dtype != ASGD_BF16) return fail(ASGD_EINVAL, "asgd_net_create: unknown dtype %d", compute_dtype);
    asgd_net *n = new (std::nothrow) asgd_net;
    if (!n) return fail(ASGD_ENOMEM, "asgd_net_create: out of host memory");
    try {
        n->layers.assign(layers, layers + n_layers);
        n->batch = batch; n->in_c = in_c; n->in_h = in_h; n->in_w = in_w; n->dtype = compute_dtype;
        n->serial = serial_default();
        const int rc = plan_net(*n);
        if (rc != ASGD_OK) { delete n; return rc; }
    } catch (const std::bad_alloc &) {
        delete n;
        return fail(ASGD_ENOMEM, "asgd_net_create: out of host memory");
    }
    *out = n;
    return ASGD_OK;
}

int asgd_net_prepare(asgd_net_t *net)
{
    if (!net) return fail(ASGD_EINVAL, "asgd_net_prepare: null plan");
    return ensure_prepared(net);
}

int asgd_net_set_serial(asgd_net_t *net, int on)
{
    if (!net) return fail(ASGD_EINVAL, "asgd_net_set_serial: null plan");
    net->serial = on != 0;
    return ASGD_OK;
}

int asgd_net_destroy(asgd_net_t *net)
{
    if (!net) return ASGD_OK;
    int rc = ASGD_OK;
    for (hipEvent_t e : net->prof_ev) (void)hipEventDestroy(e);
    rc = release_device(net);
    delete net;
    return rc;
}

size_t asgd_param_count(const asgd_net_t *net) { return net ? net->param_count : 0; }

int asgd_param_layout(const asgd_net_t *net, asgd_tensor_info_t *info, int cap)
{
    if (!net || (cap > 0 && !info)) return fail(ASGD_EINVAL, "asgd_param_layout: null argument");
    const int cnt = (int)net->tensors.size();
    for (int i = 0; i < cnt && i < cap; ++i) info[i] = net->tensors[i];
    return cnt;
}

int asgd_layer_shape(const asgd_net_t *net, int layer, int32_t chw[3])
{
    if (!net || !chw) return fail(ASGD_EINVAL, "asgd_layer_shape: null argument");
    if (layer < 0 || layer >= (int)net->layers.size()) return fail(ASGD_EINVAL, "asgd_layer_shape: layer %d out of range", layer);
    for (int j = 0; j < 3; ++j) chw[j] = net->layer_shape[3 * layer + j];
    return ASGD_OK;
}

size_t asgd_workspace_bytes(const asgd_net_t *net) { return net ? net->ws_bytes : 0; }

int asgd_fwd_bwd(asgd_net_t *net, const void *params, const void *images, const int32_t *labels, uint64_t dropout_seed, uint64_t step,
                 uint32_t worker, float *loss, float *grads, void *stream)
{
    if (!net || !params || !images || !labels || !loss || !grads) return fail(ASGD_EINVAL, "asgd_fwd_bwd: null argument");
    if (((uintptr_t)params | (uintptr_t)grads | (uintptr_t)images) & 15) return fail(ASGD_EALIGN, "asgd_fwd_bwd: params, images and grads must be 16-byte aligned");
    if (((uintptr_t)labels | (uintptr_t)loss) & 3) return fail(ASGD_EALIGN, "asgd_fwd_bwd: labels and loss must be 4-byte aligned");
    int rc = ensure_prepared(net);
    if (rc != ASGD_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = forward(net, params, images, labels, dropout_seed, step, worker, loss, st);
    if (rc != ASGD_OK) return rc;
    net->last_seed = dropout_seed; net->last_step = step; net->last_worker = worker; net->ran = true;
    return backward(net, params, grads, st, nullptr);
}

// ---- the entry point that allocates nothing
// Workspace for callers that cannot allocate: one array per GPU, held from the moment the library's code is loaded
// on that GPU until the process ends.  Host code never uses the array's name as an address (on the host it is
// only a handle for the runtime): the device address is asked for once per device and kept.
constexpr size_t kStaticWsBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (looked up on the first call per device).
int static_workspace(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(ASGD_EHIP, "device index %d is beyond the %d this library keeps a static workspace for", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(static workspace)");
        if (!p) return fail(ASGD_EHIP, "hipGetSymbolAddress returned no address for the static workspace");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ASGD_OK;
}
}  // namespace

size_t asgd_static_workspace_bytes(void) { return kStaticWsBytes; }

int asgd_fwd_bwd_static(asgd_net_t *net, const void *params, const void *images, const int32_t *labels, uint64_t dropout_seed, uint64_t step,
                        uint32_t worker, float *loss, float *grads, void *stream)
{
    if (!net || !params || !images || !labels || !loss || !grads) return fail(ASGD_EINVAL, "asgd_fwd_bwd_static: null argument");
    if (((uintptr_t)params | (uintptr_t)grads | (uintptr_t)images) & 15) return fail(ASGD_EALIGN, "asgd_fwd_bwd_static: params, images and grads must be 16-byte aligned");
    if (((uintptr_t)labels | (uintptr_t)loss) & 3) return fail(ASGD_EALIGN, "asgd_fwd_bwd_static: labels and loss must be 4-byte aligned");
    if (net->ws_bytes > kStaticWsBytes)
        return fail(ASGD_ENOMEM, "asgd_fwd_bwd_static: this plan needs %zu bytes of workspace, the static workspace holds %zu", net->ws_bytes, kStaticWsBytes);
    if (net->prof_on) return fail(ASGD_EINVAL, "asgd_fwd_bwd_static: not between asgd_profile_begin and asgd_profile_end");
    void *base = nullptr;
    int rc = static_workspace(&base);
    if (rc != ASGD_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // The plan's tensors are laid out in the static array for the duration of this call (the layout is host
    // arithmetic), every kernel goes to the caller's stream (no internal stream, no events), and the part of the
    // array the plan uses is cleared first by a kernel: it holds whatever the previous call on this GPU left, and
    // the zero border of a bordered input is never written by the path itself.
    carve(*net, static_cast<char *>(base));
    const bool was_serial = net->serial;
    net->serial = true;
    if (launch_fill_zero(base, net->ws_bytes, st) != 0) rc = hip_fail(hipGetLastError(), "fill kernel");
    if (rc == ASGD_OK) rc = forward(net, params, images, labels, dropout_seed, step, worker, loss, st);
    if (rc == ASGD_OK) rc = backward(net, params, grads, st, nullptr);
    net->serial = was_serial;
    carve(*net, static_cast<char *>(net->arena));   // back to the plan's own workspace (null pointers if it has none yet)
    net->ran = false;                               // nothing of this call is left where asgd_debug_get looks
    return rc;
}

namespace {
int train_step_impl(const char *name, bool fuse, asgd_net_t *net, float *master, float *momentum, void *worker_copy, const void *images,
                    const int32_t *labels, uint64_t dropout_seed, uint64_t step, uint32_t worker, float *loss, float *grads, float lr, float mu,
                    float wd, void *stream)
{
    if (!net || !master || !momentum || !worker_copy || !images || !labels || !loss || !grads) return fail(ASGD_EINVAL, "%s: null argument", name);
    if (((uintptr_t)master | (uintptr_t)momentum | (uintptr_t)worker_copy | (uintptr_t)grads | (uintptr_t)images) & 15)
        return fail(ASGD_EALIGN, "%s: master, momentum, worker_copy, images and grads must be 16-byte aligned", name);
    if (((uintptr_t)labels | (uintptr_t)loss) & 3) return fail(ASGD_EALIGN, "%s: labels and loss must be 4-byte aligned", name);
    int rc = ensure_prepared(net);
    if (rc != ASGD_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = forward(net, worker_copy, images, labels, dropout_seed, step, worker, loss, st);
    if (rc != ASGD_OK) return rc;
    net->last_seed = dropout_seed; net->last_step = step; net->last_worker = worker; net->ran = true;
    const ServerArgs srv{master, momentum, worker_copy, lr, mu, wd, fuse};
    return backward(net, worker_copy, grads, st, &srv);
}
}  // namespace

int asgd_train_step(asgd_net_t *net, float *master, float *momentum, void *worker_copy, const void *images, const int32_t *labels,
                    uint64_t dropout_seed, uint64_t step, uint32_t worker, float *loss, float *grads, float lr, float mu, float wd, void *stream)
{
    return train_step_impl("asgd_train_step", false, net, master, momentum, worker_copy, images, labels, dropout_seed, step, worker, loss, grads,
                           lr, mu, wd, stream);
}

int asgd_train_step_fused(asgd_net_t *net, float *master, float *momentum, void *worker_copy, const void *images, const int32_t *labels,
                          uint64_t dropout_seed, uint64_t step, uint32_t worker, float *loss, float *grads, float lr, float mu, float wd,
                          void *stream)
{
    return train_step_impl("asgd_train_step_fused", true, net, master, momentum, worker_copy, images, labels, dropout_seed, step, worker, loss,
                           grads, lr, mu, wd, stream);
}

int asgd_apply_update(float *params, float *momentum, const float *grads, size_t n, float lr, float mu, float wd, void *stream)
{
    if (n == 0) return ASGD_OK;
    if (!params || !momentum || !grads) return fail(ASGD_EINVAL, "asgd_apply_update: null argument");
    if (((uintptr_t)params | (uintptr_t)momentum | (uintptr_t)grads) & 3) return fail(ASGD_EALIGN, "asgd_apply_update: buffers must be 4-byte aligned");
    if (launch_update(params, momentum, grads, n, lr, mu, wd, nullptr, static_cast<hipStream_t>(stream)) != 0)
        return hip_fail(hipGetLastError(), "update kernel");
    return ASGD_OK;
}

int asgd_apply_update_snapshot(float *params, float *momentum, const float *grads, size_t n, float lr, float mu, float wd, void *worker_copy,
                               int dst_dtype, void *stream)
{
    if (dst_dtype != ASGD_F32 && dst_dtype != ASGD_BF16) return fail(ASGD_EINVAL, "asgd_apply_update_snapshot: unknown dtype %d", dst_dtype);
    if (n == 0) return ASGD_OK;
    if (!params || !momentum || !grads || !worker_copy) return fail(ASGD_EINVAL, "asgd_apply_update_snapshot: null argument");
    if ((((uintptr_t)params | (uintptr_t)momentum | (uintptr_t)grads) & 3) || ((uintptr_t)worker_copy & (dst_dtype == ASGD_BF16 ? 1 : 3)))
        return fail(ASGD_EALIGN, "asgd_apply_update_snapshot: misaligned buffer");
    if (launch_update_snapshot(params, momentum, grads, n, lr, mu, wd, worker_copy, dst_dtype, static_cast<hipStream_t>(stream)) != 0)
        return hip_fail(hipGetLastError(), "update kernel");
    return ASGD_OK;
}

int asgd_snapshot(const float *params, void *worker_copy, size_t n, int dst_dtype, void *stream)
{
    if (dst_dtype != ASGD_F32 && dst_dtype != ASGD_BF16) return fail(ASGD_EINVAL, "asgd_snapshot: unknown dtype %d", dst_dtype);
    if (n == 0) return ASGD_OK;
    if (!params || !worker_copy) return fail(ASGD_EINVAL, "asgd_snapshot: null argument");
    if (((uintptr_t)params & 3) || ((uintptr_t)worker_copy & (dst_dtype == ASGD_BF16 ? 1 : 3))) return fail(ASGD_EALIGN, "asgd_snapshot: misaligned buffer");
    if (launch_snapshot(params, worker_copy, n, dst_dtype, nullptr, nullptr, 0, 0, static_cast<hipStream_t>(stream)) != 0)
        return hip_fail(hipGetLastError(), "snapshot kernel");
    return ASGD_OK;
}

int asgd_debug_get(asgd_net_t *net, int what, int layer, void *dst, size_t cap_bytes, void *stream)
{
    if (!net || !dst) return fail(ASGD_EINVAL, "asgd_debug_get: null argument");
    if (!net->ran || !net->arena) return fail(ASGD_EINVAL, "asgd_debug_get: no forward pass has run on this plan");
    if (layer < 0 || layer >= (int)net->layers.size() || net->layer_stage[layer] < 0) return fail(ASGD_EINVAL, "asgd_debug_get: layer %d has no output to export", layer);
    Stage &s = net->stages[net->layer_stage[layer]];
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int B = net->batch;
    if (what == ASGD_DEBUG_OUTPUT) {
        if (layer != s.last_layer) return fail(ASGD_EINVAL, "asgd_debug_get: layer %d is fused into the group ending at layer %d", layer, s.last_layer);
        if (s.kind == ST_FC) {
            if (cap_bytes < (size_t)B * s.out_f * 4) return fail(ASGD_EINVAL, "asgd_debug_get: destination too small");
            CHECK_LAUNCH(launch_export_rows(net->dtype, s.last ? 1 : 0, s.out, s.out_ld, static_cast<float *>(dst), B, s.out_f, st), "export");
        } else {
            if (cap_bytes < (size_t)B * s.outC * s.outH * s.outW * 4) return fail(ASGD_EINVAL, "asgd_debug_get: destination too small");
            CHECK_LAUNCH(launch_export_nhwc(net->dtype, s.out, static_cast<float *>(dst), B, s.outH, s.outW, s.outC, s.outCp, st), "export");
        }
        return ASGD_OK;
    }
    if (what == ASGD_DEBUG_ARGMAX) {
        if (s.kind != ST_POOL) return fail(ASGD_EINVAL, "asgd_debug_get: layer %d is not a MAXPOOL", layer);
        if (cap_bytes < (size_t)B * s.outC * s.outH * s.outW) return fail(ASGD_EINVAL, "asgd_debug_get: destination too small");
        CHECK_LAUNCH(launch_export_argmax(s.argmax, static_cast<uint8_t *>(dst), B, s.outH, s.outW, s.outC, s.outCp, st), "export");
        return ASGD_OK;
    }
    if (what == ASGD_DEBUG_MASK) {
        if (s.kind != ST_FC || !s.drop || layer != s.drop_layer) return fail(ASGD_EINVAL, "asgd_debug_get: layer %d is not a DROPOUT", layer);
        if (cap_bytes < (size_t)B * s.out_f) return fail(ASGD_EINVAL, "asgd_debug_get: destination too small");
        CHECK_LAUNCH(launch_dropout_mask(static_cast<uint8_t *>(dst), (size_t)B * s.out_f,
                                         dropout_key(net->last_seed, net->last_step, net->last_worker, (uint32_t)s.drop_layer), s.drop_thr, st),
                     "export");
        return ASGD_OK;
    }
    return fail(ASGD_EINVAL, "asgd_debug_get: unknown selector %d", what);
}

int asgd_profile_begin(asgd_net_t *net)
{
    if (!net) return fail(ASGD_EINVAL, "asgd_profile_begin: null plan");
    for (hipEvent_t e : net->prof_ev) (void)hipEventDestroy(e);
    net->prof_ev.clear(); net->prof_cls.clear();
    for (int c = 0; c < ASGD_K_COUNT; ++c) net->prof_flops[c] = net->prof_bytes[c] = 0;
    net->prof_on = true;
    return ASGD_OK;
}

int asgd_profile_end(asgd_net_t *net, asgd_profile_entry_t *out)
{
    if (!net || !out) return fail(ASGD_EINVAL, "asgd_profile_end: null argument");
    if (!net->prof_on) return fail(ASGD_EINVAL, "asgd_profile_end: profiling was not begun on this plan");
    net->prof_on = false;
    for (int c = 0; c < ASGD_K_COUNT; ++c) { out[c].kclass = c; out[c].launches = 0; out[c].ms = 0; out[c].flops = net->prof_flops[c]; out[c].bytes = net->prof_bytes[c]; }
    int rc = ASGD_OK;
    for (size_t i = 0; i < net->prof_cls.size(); ++i) {
        hipEvent_t a = net->prof_ev[2 * i], b = net->prof_ev[2 * i + 1];
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
        if (e != hipSuccess) { if (rc == ASGD_OK) rc = hip_fail(e, "profile event"); continue; }
        out[net->prof_cls[i]].launches += 1;
        out[net->prof_cls[i]].ms += ms;
    }
    for (hipEvent_t e : net->prof_ev) (void)hipEventDestroy(e);
    net->prof_ev.clear(); net->prof_cls.clear();
    return rc;
}

int asgd_schedule_generate(int32_t *worker, int32_t *read_version, int T, uint64_t seed, int n_workers, int max_stale)
{
    if (T < 0 || (T > 0 && (!worker || !read_version))) return fail(ASGD_EINVAL, "asgd_schedule_generate: null argument");
    if (n_workers <= 0 || max_stale < 0 || max_stale >= n_workers)
        return fail(ASGD_EINVAL, "asgd_schedule_generate: need 0 <= max_stale < n_workers");
    auto mix = [](uint64_t z) {
        z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
        z ^= z >> 27; z *= 0x94D049BB133111EBull;
        z ^= z >> 31;
        return z;
    };
    const uint64_t k = mix(seed);
    for (int a = 0; a < T; ++a) {
        const uint32_t h = (uint32_t)(mix(k + (uint64_t)a) >> 32);
        int st = (int)(h % (uint32_t)(max_stale + 1));
        if (st > a) st = a;
        worker[a] = a % n_workers;
        read_version[a] = a - st;
    }
    return ASGD_OK;
}

// Replica-side state of the n_sync regime: each replica's own fp32 parameters, momentum and gradient accumulator.
struct LocalState {
    int n_sync;
    float *const *params, *const *momentum, *const *accum;
};

static int replay_impl(asgd_net_t *const *nets, int n_workers, float *params, float *momentum, void *const *worker_copy,
                       float *const *worker_grads, const void *images, const int32_t *labels, const int32_t *worker,
                       const int32_t *read_version, int T, float lr, float mu, float wd, uint64_t dropout_seed, float *losses, int32_t *log,
                       void *stream, const LocalState *loc)
{
    if (!nets || !params || !momentum || !worker_copy || !worker_grads || !images || !labels || !worker || !read_version || !losses || !log)
        return fail(ASGD_EINVAL, "asgd_replay_run: null argument");
    if (loc && (loc->n_sync < 1 || !loc->params || !loc->momentum || !loc->accum)) return fail(ASGD_EINVAL, "asgd_replay_nsync_run: bad n_sync or null argument");
    const int n_sync = loc ? loc->n_sync : 1;
    if (n_workers <= 0 || n_workers > 64 || T < 0) return fail(ASGD_EINVAL, "asgd_replay_run: bad worker count or length");
    if (T == 0) return ASGD_OK;
    for (int w = 0; w < n_workers; ++w) {
        if (!nets[w] || !worker_copy[w] || !worker_grads[w]) return fail(ASGD_EINVAL, "asgd_replay_run: null entry for worker %d", w);
        if (loc && (!loc->params[w] || !loc->momentum[w] || !loc->accum[w])) return fail(ASGD_EINVAL, "asgd_replay_nsync_run: null entry for worker %d", w);
        if (nets[w]->param_count != nets[0]->param_count || nets[w]->batch != nets[0]->batch || nets[w]->dtype != nets[0]->dtype)
            return fail(ASGD_EINVAL, "asgd_replay_run: worker %d has a different network", w);
        for (int u = 0; u < w; ++u)
            if (nets[u] == nets[w]) return fail(ASGD_EINVAL, "asgd_replay_run: workers %d and %d share a plan", u, w);
    }
    // the schedule must be causally possible
    std::vector<int> last_push(n_workers, -1);
    for (int a = 0; a < T; ++a) {
        if (worker[a] < 0 || worker[a] >= n_workers) return fail(ASGD_EINVAL, "asgd_replay_run: update %d names worker %d", a, worker[a]);
        if (read_version[a] < 0 || read_version[a] > a) return fail(ASGD_EINVAL, "asgd_replay_run: update %d reads version %d", a, read_version[a]);
        if (read_version[a] <= last_push[worker[a]])
            return fail(ASGD_EINVAL, "asgd_replay_run: update %d reads version %d before its worker's previous push %d was applied", a,
                        read_version[a], last_push[worker[a]]);
        last_push[worker[a]] = a;
    }
    for (int w = 0; w < n_workers; ++w) {
        const int rc = ensure_prepared(nets[w]);
        if (rc != ASGD_OK) return rc;
    }
    for (int w = 0; w < n_workers; ++w) nets[w]->in_replay = n_workers > 1;   // until this call has enqueued its work
    const asgd_net *n0 = nets[0];
    const size_t P = n0->param_count;
    const size_t img_bytes = (size_t)n0->batch * n0->in_c * n0->in_h * n0->in_w * dtype_size(n0->dtype);
    int *counter = nets[0]->version_counter;
    hipStream_t caller = static_cast<hipStream_t>(stream);

    // Streams and events live in the plan of worker 0 and are reused by later replays: recording an event again is
    // safe, because a stream that waits for an event waits for the record that preceded the wait call.
    asgd_net *keeper = nets[0];
    int rc = ASGD_OK;
#define RP(expr)                                                                    \
    do {                                                                            \
        const hipError_t e_ = (expr);                                               \
        if (e_ != hipSuccess && rc == ASGD_OK) rc = hip_fail(e_, #expr);            \
    } while (0)
    while ((int)keeper->replay_streams.size() < n_workers + 1 && rc == ASGD_OK) {
        hipStream_t st = nullptr;
        RP(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
        if (rc == ASGD_OK) keeper->replay_streams.push_back(st);
    }
    const size_t n_events = 3 * (size_t)T + 2;
    while (keeper->replay_events.size() < n_events && rc == ASGD_OK) {
        hipEvent_t e = nullptr;
        RP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        if (rc == ASGD_OK) keeper->replay_events.push_back(e);
    }
    if (rc != ASGD_OK) { for (int w = 0; w < n_workers; ++w) nets[w]->in_replay = false; return rc; }
    hipStream_t *ws = keeper->replay_streams.data();
    hipStream_t server = keeper->replay_streams[n_workers];
    hipEvent_t *ev_upd = keeper->replay_events.data(), *ev_snap = ev_upd + T, *ev_grad = ev_snap + T;
    hipEvent_t ev_start = keeper->replay_events[3 * (size_t)T], ev_reset = keeper->replay_events[3 * (size_t)T + 1];
    // Everything below waits, directly or through the server stream, for the work already on the caller's stream; the
    // internal streams of a previous replay on these plans were joined into the caller's stream of that replay.
    RP(hipEventRecord(ev_start, caller));
    RP(hipStreamWaitEvent(server, ev_start, 0));
    for (int w = 0; w < n_workers; ++w) RP(hipStreamWaitEvent(ws[w], ev_start, 0));
    if (rc == ASGD_OK && launch_fill_zero(counter, 4, server) != 0) rc = hip_fail(hipGetLastError(), "fill kernel");
    RP(hipEventRecord(ev_reset, server));
    // Iteration v enqueues every snapshot that must see exactly v applied updates
    // (and the gradient computed on it), then update v, which waits for them.
    for (int v = 0; v < T && rc == ASGD_OK; ++v) {
        for (int a = v; a < T && rc == ASGD_OK; ++a) {
            if (read_version[a] != v) continue;
            const int w = worker[a];
            RP(hipStreamWaitEvent(ws[w], v > 0 ? ev_upd[v - 1] : ev_reset, 0));
            if (launch_snapshot(params, worker_copy[w], P, n0->dtype, counter, log + 3 * (size_t)a, a, w, ws[w]) != 0 && rc == ASGD_OK)
                rc = hip_fail(hipGetLastError(), "snapshot kernel");
            if (loc && launch_snapshot(params, loc->params[w], P, kF32, nullptr, nullptr, 0, 0, ws[w]) != 0 && rc == ASGD_OK)
                rc = hip_fail(hipGetLastError(), "snapshot kernel");   // the replica's own fp32 parameters
            RP(hipEventRecord(ev_snap[a], ws[w]));
            for (int i = 0; i < n_sync && rc == ASGD_OK; ++i) {
                const size_t b = (size_t)a * n_sync + i;   // minibatch and dropout step of local step i of cycle a
                rc = asgd_fwd_bwd(nets[w], worker_copy[w], static_cast<const char *>(images) + b * img_bytes, labels + b * n0->batch,
                                  dropout_seed, (uint64_t)b, (uint32_t)w, losses + b, worker_grads[w], ws[w]);
                if (loc && rc == ASGD_OK) {
                    // the push is the sum of the cycle's gradients; the replica keeps training on its own parameters
                    if (launch_accumulate(loc->accum[w], worker_grads[w], P, i == 0, ws[w]) != 0) rc = hip_fail(hipGetLastError(), "accumulate kernel");
                    else if (launch_update_snapshot(loc->params[w], loc->momentum[w], worker_grads[w], P, lr, mu, wd, worker_copy[w], n0->dtype,
                                                    ws[w]) != 0)
                        rc = hip_fail(hipGetLastError(), "update kernel");
                }
            }
            RP(hipEventRecord(ev_grad[a], ws[w]));
        }
        for (int a = v; a < T && rc == ASGD_OK; ++a)
            if (read_version[a] == v) RP(hipStreamWaitEvent(server, ev_snap[a], 0));
        RP(hipStreamWaitEvent(server, ev_grad[v], 0));
        if (rc == ASGD_OK && launch_update(params, momentum, loc ? loc->accum[worker[v]] : worker_grads[worker[v]], P, lr, mu, wd, counter, server) != 0)
            rc = hip_fail(hipGetLastError(), "update kernel");
        RP(hipEventRecord(ev_upd[v], server));
    }
    // Update T-1 is behind every snapshot and every gradient of the replay, so the caller's stream, which waits for
    // it, is behind all of the replay's work.  After an error part of the schedule may be enqueued: wait for what is.
    if (rc == ASGD_OK) RP(hipStreamWaitEvent(caller, ev_upd[T - 1], 0));
    else {
        for (int w = 0; w <= n_workers; ++w) (void)hipStreamSynchronize(keeper->replay_streams[w]);
    }
    for (int w = 0; w < n_workers; ++w) nets[w]->in_replay = false;
#undef RP
    return rc;
}

int asgd_replay_run(asgd_net_t *const *nets, int n_workers, float *params, float *momentum, void *const *worker_copy,
                    float *const *worker_grads, const void *images, const int32_t *labels, const int32_t *worker,
                    const int32_t *read_version, int T, float lr, float mu, float wd, uint64_t dropout_seed, float *losses, int32_t *log,
                    void *stream)
{
    return replay_impl(nets, n_workers, params, momentum, worker_copy, worker_grads, images, labels, worker, read_version, T, lr, mu, wd,
                       dropout_seed, losses, log, stream, nullptr);
}

int asgd_replay_nsync_run(asgd_net_t *const *nets, int n_workers, int n_sync, float *params, float *momentum, float *const *worker_params,
                          float *const *worker_momentum, float *const *worker_accum, void *const *worker_copy, float *const *worker_grads,
                          const void *images, const int32_t *labels, const int32_t *worker, const int32_t *read_version, int T, float lr,
                          float mu, float wd, uint64_t dropout_seed, float *losses, int32_t *log, void *stream)
{
    const LocalState loc{n_sync, worker_params, worker_momentum, worker_accum};
    return replay_impl(nets, n_workers, params, momentum, worker_copy, worker_grads, images, labels, worker, read_version, T, lr, mu, wd,
                       dropout_seed, losses, log, stream, &loc);
}

int asgd_apply_update_adagrad(float *params, float *hist, const float *grads, size_t n, float lr, float eps, float wd, void *stream)
{
    if (n == 0) return ASGD_OK;
    if (!params || !hist || !grads) return fail(ASGD_EINVAL, "asgd_apply_update_adagrad: null argument");
    if (((uintptr_t)params | (uintptr_t)hist | (uintptr_t)grads) & 3) return fail(ASGD_EALIGN, "asgd_apply_update_adagrad: buffers must be 4-byte aligned");
    if (launch_adagrad(params, hist, grads, n, lr, eps, wd, static_cast<hipStream_t>(stream)) != 0) return hip_fail(hipGetLastError(), "update kernel");
    return ASGD_OK;
}

int asgd_apply_update_adadelta(float *params, float *avg_sq_grad, float *avg_sq_step, const float *grads, size_t n, float rho, float eps, float wd,
                               void *stream)
{
    if (n == 0) return ASGD_OK;
    if (!params || !avg_sq_grad || !avg_sq_step || !grads) return fail(ASGD_EINVAL, "asgd_apply_update_adadelta: null argument");
    if (((uintptr_t)params | (uintptr_t)avg_sq_grad | (uintptr_t)avg_sq_step | (uintptr_t)grads) & 3)
        return fail(ASGD_EALIGN, "asgd_apply_update_adadelta: buffers must be 4-byte aligned");
    if (launch_adadelta(params, avg_sq_grad, avg_sq_step, grads, n, rho, eps, wd, static_cast<hipStream_t>(stream)) != 0)
        return hip_fail(hipGetLastError(), "update kernel");
    return ASGD_OK;
}

int asgd_accumulate(float *accum, const float *grads, size_t n, int first, void *stream)
{
    if (n == 0) return ASGD_OK;
    if (!accum || !grads) return fail(ASGD_EINVAL, "asgd_accumulate: null argument");
    if (((uintptr_t)accum | (uintptr_t)grads) & 3) return fail(ASGD_EALIGN, "asgd_accumulate: buffers must be 4-byte aligned");
    if (launch_accumulate(accum, grads, n, first != 0, static_cast<hipStream_t>(stream)) != 0) return hip_fail(hipGetLastError(), "accumulate kernel");
    return ASGD_OK;
}

}  // extern "C"
