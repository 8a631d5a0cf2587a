"""Pins for the oracle's layer functions: library routines, closed forms,
adjoint identities and brute force.  No GPU, no HIP library."""
import numpy as np
import pytest
import scipy.signal
import scipy.special
import torch

import oracle
from oracle import ops

RNG = np.random.default_rng(7)


def randn(*shape):
    return RNG.standard_normal(shape)


# ------------------------------------------------------------------ conv forward
def test_conv_fwd_matches_scipy_correlate2d():
    # stride 1: each output plane is the sum over input channels of a 2-D
    # cross-correlation (library routine), plus the bias.
    x, w, b = randn(2, 3, 9, 8), randn(4, 3, 3, 3), randn(4)
    y = ops.conv_fwd(x, w, b, 1, 1)
    xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
    for n in range(2):
        for co in range(4):
            ref = b[co] + sum(scipy.signal.correlate2d(xp[n, ci], w[co, ci], mode="valid") for ci in range(3))
            np.testing.assert_allclose(y[n, co], ref, rtol=0, atol=1e-12)


def test_conv_fwd_no_kernel_flip():
    # a filter with a single 1 at (ky,kx)=(0,2) must shift the image, not mirror it
    x = randn(1, 1, 5, 5)
    w = np.zeros((1, 1, 3, 3)); w[0, 0, 0, 2] = 1.0
    y = ops.conv_fwd(x, w, np.zeros(1), 1, 0)
    np.testing.assert_array_equal(y[0, 0], x[0, 0, 0:3, 2:5])


@pytest.mark.parametrize("k,s,p,H,W", [(11, 4, 2, 35, 31), (5, 1, 2, 7, 9), (3, 2, 0, 8, 8), (3, 1, 1, 6, 5)])
def test_conv_fwd_bwd_match_torch(k, s, p, H, W):
    x, w, b = randn(2, 3, H, W), randn(5, 3, k, k), randn(5)
    tx = torch.tensor(x, requires_grad=True); tw = torch.tensor(w, requires_grad=True)
    tb = torch.tensor(b, requires_grad=True)
    ty = torch.nn.functional.conv2d(tx, tw, tb, stride=s, padding=p)
    y = ops.conv_fwd(x, w, b, s, p)
    assert y.shape == tuple(ty.shape)
    np.testing.assert_allclose(y, ty.detach().numpy(), atol=1e-11)
    dy = randn(*y.shape)
    ty.backward(torch.tensor(dy))
    np.testing.assert_allclose(ops.conv_bwd_data(dy, w, (H, W), s, p), tx.grad.numpy(), atol=1e-11)
    dw, db = ops.conv_bwd_weight(x, dy, k, s, p)
    np.testing.assert_allclose(dw, tw.grad.numpy(), atol=1e-10)
    np.testing.assert_allclose(db, tb.grad.numpy(), atol=1e-10)


def test_conv_1x1_is_matrix_product():
    x, w, b = randn(3, 6, 4, 5), randn(7, 6, 1, 1), randn(7)
    y = ops.conv_fwd(x, w, b, 1, 0)
    ref = np.einsum("nchw,oc->nohw", x, w[:, :, 0, 0]) + b[None, :, None, None]
    np.testing.assert_allclose(y, ref, atol=1e-12)


def test_full_extent_conv_equals_fc():
    # a pad-0 filter as large as the input is a fully connected layer over the
    # C,H,W-flattened input: pins the conv oracle against the FC oracle.
    x, w, b = randn(4, 3, 6, 6), randn(5, 3, 6, 6), randn(5)
    y_conv = ops.conv_fwd(x, w, b, 1, 0).reshape(4, 5)
    y_fc = ops.fc_fwd(x.reshape(4, -1), w.reshape(5, -1), b)
    np.testing.assert_allclose(y_conv, y_fc, atol=1e-12)
    np.testing.assert_allclose(y_fc, x.reshape(4, -1) @ w.reshape(5, -1).T + b, atol=1e-12)


def test_conv_brute_force_against_im2col_matmul():
    k, s, p = 3, 2, 1
    x, w, b = randn(2, 2, 7, 6), randn(3, 2, k, k), randn(3)
    y = ops.conv_fwd(x, w, b, s, p)
    Ho, Wo = y.shape[2:]
    xp = np.pad(x, ((0, 0), (0, 0), (p, p), (p, p)))
    cols = np.stack([xp[:, :, oy * s:oy * s + k, ox * s:ox * s + k].reshape(2, -1)
                     for oy in range(Ho) for ox in range(Wo)], axis=1)  # [N, Ho*Wo, Cin*k*k]
    ref = (cols @ w.reshape(3, -1).T + b).transpose(0, 2, 1).reshape(2, 3, Ho, Wo)
    np.testing.assert_allclose(y, ref, atol=1e-12)


# ------------------------------------------------------------------ adjoints
@pytest.mark.parametrize("k,s,p", [(5, 1, 2), (3, 2, 1), (11, 4, 2), (2, 2, 0)])
def test_conv_adjoint_identities(k, s, p):
    H, W = 23, 19
    x, w = randn(2, 3, H, W), randn(4, 3, k, k)
    y = ops.conv_fwd(x, w, np.zeros(4), s, p)
    dy = randn(*y.shape)
    lhs = np.vdot(y, dy)
    np.testing.assert_allclose(np.vdot(x, ops.conv_bwd_data(dy, w, (H, W), s, p)), lhs, rtol=1e-12)
    dw, db = ops.conv_bwd_weight(x, dy, k, s, p)
    np.testing.assert_allclose(np.vdot(w, dw), lhs, rtol=1e-12)
    np.testing.assert_allclose(db, dy.sum(axis=(0, 2, 3)), rtol=1e-12)


def test_fc_bwd_closed_forms():
    x, w, b = randn(6, 11), randn(4, 11), randn(4)
    dy = randn(6, 4)
    dx, dw, db = ops.fc_bwd(x, w, dy)
    np.testing.assert_allclose(dx, dy @ w, atol=1e-12)
    np.testing.assert_allclose(dw, dy.T @ x, atol=1e-12)
    np.testing.assert_allclose(db, dy.sum(0), atol=1e-12)
    # transposed-operand mistakes fail the adjoint identity
    np.testing.assert_allclose(np.vdot(ops.fc_fwd(x, w, np.zeros(4)), dy), np.vdot(x, dx), rtol=1e-12)


# ------------------------------------------------------------------ relu
def test_relu():
    y = np.array([-2.0, -0.0, 0.0, 1e-300, 3.0])
    np.testing.assert_array_equal(ops.relu_fwd(y), [0, 0, 0, 1e-300, 3.0])
    np.testing.assert_array_equal(ops.relu_bwd(y, np.full(5, 7.0)), [0, 0, 0, 7.0, 7.0])


# ------------------------------------------------------------------ max pool
@pytest.mark.parametrize("k,s,H,W", [(2, 2, 28, 28), (3, 2, 15, 15), (3, 2, 7, 8), (3, 2, 13, 13)])
def test_maxpool_properties(k, s, H, W):
    r = np.maximum(randn(2, 3, H, W), 0)  # post-ReLU: many ties at zero
    p, idx = ops.maxpool_fwd(r, k, s)
    Ho, Wo = (H - k) // s + 1, (W - k) // s + 1
    assert p.shape == (2, 3, Ho, Wo)
    tp = torch.nn.functional.max_pool2d(torch.tensor(r), k, s)
    np.testing.assert_array_equal(p, tp.numpy())  # values against the library routine
    for n in range(2):
        for c in range(3):
            for py in range(Ho):
                for px in range(Wo):
                    win = r[n, c, py * s:py * s + k, px * s:px * s + k].reshape(-1)
                    a = idx[n, c, py, px]
                    assert win[a] == p[n, c, py, px] == win.max()
                    assert a == int(np.argmax(win))  # numpy argmax = first maximum in row-major order
    dp = randn(*p.shape)
    dr = ops.maxpool_bwd(dp, idx, (H, W), k, s)
    np.testing.assert_allclose(dr.sum(), dp.sum(), rtol=1e-12)
    # gather form written independently: each input sums the windows that point at it
    ref = np.zeros_like(r)
    for py in range(Ho):
        for px in range(Wo):
            a = idx[:, :, py, px]
            for n in range(2):
                for c in range(3):
                    ref[n, c, py * s + a[n, c] // k, px * s + a[n, c] % k] += dp[n, c, py, px]
    np.testing.assert_allclose(dr, ref, atol=1e-14)


def test_maxpool_tie_break_first_in_row_major():
    r = np.zeros((1, 1, 5, 5))
    _, idx = ops.maxpool_fwd(r, 3, 2)
    assert (idx == 0).all()
    r[0, 0, 1, 2] = 1.0; r[0, 0, 2, 1] = 1.0  # two equal maxima: (1,2) comes first in the scan
    _, idx = ops.maxpool_fwd(r, 3, 2)
    assert idx[0, 0, 0, 0] == 1 * 3 + 2
    assert idx[0, 0, 0, 1] == 1 * 3 + 0     # window starts at column 2: element (1,2) is (ky,kx)=(1,0)
    r2 = np.full((1, 1, 2, 2), -3.0)
    _, idx = ops.maxpool_fwd(r2, 2, 2)
    assert idx[0, 0, 0, 0] == 0


# ------------------------------------------------------------------ softmax cross-entropy
def test_lrn_special_cases_and_library():
    rng = np.random.default_rng(12)
    a = rng.standard_normal((2, 7, 3, 4))
    # window of one channel: elementwise closed form
    b1 = ops.lrn_fwd(a, 1, 0.3, 0.75, 2.0)
    np.testing.assert_allclose(b1, a / (2.0 + 0.3 * a * a) ** 0.75, rtol=1e-14)
    # window covering every channel from anywhere: one sum per pixel
    b_all = ops.lrn_fwd(a, 13, 0.1, 0.5, 1.0)
    np.testing.assert_allclose(b_all, a / np.sqrt(1.0 + 0.1 * (a * a).sum(1, keepdims=True)), rtol=1e-14)
    # window of 5, written out by hand for one element, edges clipped
    b5 = ops.lrn_fwd(a, 5, 1e-4, 0.75, 2.0)
    assert abs(b5[1, 0, 2, 1] - a[1, 0, 2, 1] / (2.0 + 1e-4 * (a[1, 0:3, 2, 1] ** 2).sum()) ** 0.75) < 1e-15
    assert abs(b5[0, 4, 0, 0] - a[0, 4, 0, 0] / (2.0 + 1e-4 * (a[0, 2:7, 0, 0] ** 2).sum()) ** 0.75) < 1e-15
    # the library routine averages over the window (alpha / size): same thing with alpha * size
    for size, alpha, beta, k in [(5, 1e-4, 0.75, 2.0), (3, 0.2, 0.6, 1.5)]:
        t = torch.tensor(a, requires_grad=True)
        y = torch.nn.functional.local_response_norm(t, size, alpha=alpha * size, beta=beta, k=k)
        np.testing.assert_allclose(ops.lrn_fwd(a, size, alpha, beta, k), y.detach().numpy(), rtol=1e-12)
        db = rng.standard_normal(a.shape)
        y.backward(torch.tensor(db))
        np.testing.assert_allclose(ops.lrn_bwd(a, db, size, alpha, beta, k), t.grad.numpy(), rtol=1e-10, atol=1e-14)


def test_lrn_backward_by_finite_differences():
    rng = np.random.default_rng(13)
    a = rng.standard_normal((1, 6, 2, 2))
    db = rng.standard_normal(a.shape)
    size, alpha, beta, k = 5, 0.4, 0.75, 2.0      # a large alpha, so that the cross terms matter
    da = ops.lrn_bwd(a, db, size, alpha, beta, k)
    h = 1e-6
    for idx in np.ndindex(a.shape):
        ap, am = a.copy(), a.copy()
        ap[idx] += h; am[idx] -= h
        fd = ((ops.lrn_fwd(ap, size, alpha, beta, k) - ops.lrn_fwd(am, size, alpha, beta, k)) * db).sum() / (2 * h)
        assert abs(fd - da[idx]) < 1e-8 * (1 + abs(da[idx]))


def test_softmax_ce_closed_forms():
    for C in (10, 1000):
        N = 4
        labels = np.array([0, 3, C - 1, 5], dtype=np.int32)
        loss, dz = ops.softmax_ce(np.zeros((N, C)), labels)
        assert abs(loss - np.log(C)) < 1e-13
        ref = np.full((N, C), 1.0 / C); ref[np.arange(N), labels] -= 1.0
        np.testing.assert_allclose(dz, ref / N, atol=1e-15)


def test_softmax_ce_against_library_and_invariants():
    N, C = 5, 17
    z = randn(N, C) * 4
    labels = RNG.integers(0, C, N).astype(np.int32)
    loss, dz = ops.softmax_ce(z, labels)
    logp = scipy.special.log_softmax(z, axis=1)
    np.testing.assert_allclose(loss, -logp[np.arange(N), labels].mean(), rtol=1e-13)
    onehot = np.eye(C)[labels]
    np.testing.assert_allclose(dz, (scipy.special.softmax(z, axis=1) - onehot) / N, atol=1e-15)
    np.testing.assert_allclose(dz.sum(axis=1), 0, atol=1e-15)
    loss2, dz2 = ops.softmax_ce(z + 123.0, labels)   # shift invariance
    np.testing.assert_allclose(loss2, loss, rtol=1e-12)
    np.testing.assert_allclose(dz2, dz, atol=1e-14)
    loss3, _ = ops.softmax_ce(z * 1e3, labels)        # max-subtraction keeps it finite
    assert np.isfinite(loss3)


# ------------------------------------------------------------------ dropout
MASK64 = (1 << 64) - 1


def _mix(z):
    z ^= z >> 30; z = (z * 0xBF58476D1CE4E5B9) & MASK64
    z ^= z >> 27; z = (z * 0x94D049BB133111EB) & MASK64
    z ^= z >> 31
    return z


def _mask_bigint(count, seed, step, worker, layer, p):
    thr = int(np.floor(p * 4294967296.0))
    key = _mix((_mix((_mix(seed) + step) & MASK64) + ((worker << 32) | layer)) & MASK64)
    return np.array([1 if (_mix((key + 0x9E3779B97F4A7C15 * (i + 1)) & MASK64) >> 32) >= thr else 0
                     for i in range(count)], dtype=np.uint8)


def test_splitmix_finaliser_reference_values():
    # SplitMix64 seeded with 0 yields these first outputs (published test vector of
    # the generator whose finaliser the mask uses): out_i = mix(i * golden).
    golden = 0x9E3779B97F4A7C15
    assert _mix(golden) == 0xE220A8397B1DCDAF
    assert _mix((2 * golden) & MASK64) == 0x6E789E6AA1B965F4


@pytest.mark.parametrize("seed,step,worker,layer,p", [(0, 0, 0, 0, 0.5), (3002, 7, 2, 9, 0.5),
                                                      (2**63 + 5, 2**40, 3, 17, 0.25),
                                                      (1, 1, 1, 1, 0.9)])
def test_dropout_mask_matches_bigint_reimplementation(seed, step, worker, layer, p):
    m = ops.dropout_mask(300, seed, step, worker, layer, p)
    np.testing.assert_array_equal(m, _mask_bigint(300, seed, step, worker, layer, p))


def test_dropout_mask_golden_vectors():
    import json, os
    with open(os.path.join(os.path.dirname(__file__), "golden", "dropout_mask_vectors.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        m = _mask_bigint(len(c["mask"]), c["seed"], c["step"], c["worker"], c["layer"], c["p"])
        assert "".join(map(str, m)) == c["mask"]


def test_dropout_statistics_and_keys():
    n = 200000
    for p in (0.5, 0.2):
        m = ops.dropout_mask(n, 11, 0, 0, 0, p)
        assert abs(m.mean() - (1 - p)) < 4 * np.sqrt(p * (1 - p) / n)
    assert ops.dropout_mask(64, 1, 2, 3, 4, 0.0).all()
    assert ops.dropout_threshold(0.5) == 1 << 31
    base = ops.dropout_mask(4096, 1, 2, 3, 4, 0.5)
    for other in [(2, 2, 3, 4), (1, 3, 3, 4), (1, 2, 0, 4), (1, 2, 3, 5)]:
        assert (ops.dropout_mask(4096, *other, 0.5) != base).mean() > 0.4   # every key field matters
    r = randn(64)
    h = ops.dropout_apply(r, base[:64], 2.0)
    np.testing.assert_array_equal(h, np.where(base[:64] == 1, r * 2.0, 0.0))


# ------------------------------------------------------------------ update
def test_update_closed_forms():
    n = 50
    w0, g = randn(n), randn(n)
    # mu = 0, wd = 0: plain gradient step
    w, v = w0.copy(), np.zeros(n)
    ops.apply_update(w, v, g, 0.1, 0.0, 0.0)
    np.testing.assert_allclose(w, w0 - 0.1 * g, rtol=1e-15)
    # constant gradient, wd = 0: v_t = -lr*g*(1-mu^t)/(1-mu)
    w, v = w0.copy(), np.zeros(n)
    lr, mu, T = 0.01, 0.9, 25
    for _ in range(T):
        ops.apply_update(w, v, g, lr, mu, 0.0)
    np.testing.assert_allclose(v, -lr * g * (1 - mu**T) / (1 - mu), rtol=1e-12)
    np.testing.assert_allclose(w, w0 - lr * g * (T - mu * (1 - mu**T) / (1 - mu)) / (1 - mu), rtol=1e-11)
    # g = 0, mu = 0: geometric weight decay
    w, v = w0.copy(), np.zeros(n)
    for _ in range(10):
        ops.apply_update(w, v, np.zeros(n), 0.1, 0.0, 0.05)
    np.testing.assert_allclose(w, w0 * (1 - 0.1 * 0.05) ** 10, rtol=1e-13)
    # one general step, written out
    w, v = w0.copy(), randn(n); v0 = v.copy()
    ops.apply_update(w, v, g, 0.02, 0.8, 5e-4)
    np.testing.assert_allclose(v, 0.8 * v0 - 0.02 * (g + 5e-4 * w0), rtol=1e-14)
    np.testing.assert_allclose(w, w0 + v, rtol=1e-14)


def test_adagrad_and_adadelta_closed_forms_and_library():
    n = 40
    w0, g = randn(n), randn(n)
    # Adagrad, constant gradient, no decay, eps = 0: step t moves by lr * sign(g) / sqrt(t)
    w, h = w0.copy(), np.zeros(n)
    T, lr = 12, 0.3
    for _ in range(T):
        ops.apply_adagrad(w, h, g, lr, 0.0, 0.0)
    np.testing.assert_allclose(h, T * g * g, rtol=1e-13)
    np.testing.assert_allclose(w, w0 - lr * np.sign(g) * sum(1 / np.sqrt(t) for t in range(1, T + 1)), rtol=1e-12)
    # Adadelta, first step from zero state: d = -sqrt(eps) / sqrt((1-rho) g^2 + eps) * g
    w, a, b = w0.copy(), np.zeros(n), np.zeros(n)
    rho, eps = 0.95, 1e-6
    ops.apply_adadelta(w, a, b, g, rho, eps, 0.0)
    d = -np.sqrt(eps) / np.sqrt((1 - rho) * g * g + eps) * g
    np.testing.assert_allclose(w - w0, d, rtol=1e-9)
    np.testing.assert_allclose(a, (1 - rho) * g * g, rtol=1e-14)
    np.testing.assert_allclose(b, (1 - rho) * d * d, rtol=1e-9)
    # both against the library optimisers in float64, several steps with weight decay and fresh gradients
    gs = [randn(n) for _ in range(6)]
    for name in ("adagrad", "adadelta"):
        p = torch.tensor(w0.copy(), requires_grad=True)
        if name == "adagrad":
            opt = torch.optim.Adagrad([p], lr=0.05, eps=1e-7, weight_decay=1e-3)
            w, h = w0.copy(), np.zeros(n)
        else:
            opt = torch.optim.Adadelta([p], lr=1.0, rho=0.9, eps=1e-6, weight_decay=1e-3)
            w, a, b = w0.copy(), np.zeros(n), np.zeros(n)
        for gi in gs:
            p.grad = torch.tensor(gi)
            opt.step()
            if name == "adagrad":
                ops.apply_adagrad(w, h, gi, 0.05, 1e-7, 1e-3)
            else:
                ops.apply_adadelta(w, a, b, gi, 0.9, 1e-6, 1e-3)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-11, atol=1e-15)


# ------------------------------------------------------------------ snapshot
def test_snapshot_bf16_matches_library_cast_and_hand_cases():
    a = np.concatenate([RNG.standard_normal(5000).astype(np.float32) * np.float32(10.0) ** RNG.integers(-30, 30, 5000),
                        np.array([0.0, -0.0, np.inf, -np.inf, 1e-45, -1e-40, 3.3895314e38], dtype=np.float32)]).astype(np.float32)
    bits = ops.snapshot_bf16(a)
    ref = torch.tensor(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, ref)
    # ties go to the even mantissa: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    hand = np.array([1.0 + 2.0**-8, 1.0 + 2.0**-7 + 2.0**-8, 1.0 + 2.0**-8 + 2.0**-20], dtype=np.float32)
    np.testing.assert_array_equal(ops.snapshot_bf16(hand), [0x3F80, 0x3F82, 0x3F81])
    assert np.isnan(ops.bf16_to_f64(ops.snapshot_bf16(np.array([np.nan], dtype=np.float32))))[0]
    np.testing.assert_array_equal(ops.bf16_to_f64(np.array([0x3F80, 0xC000], dtype=np.uint16)), [1.0, -2.0])
