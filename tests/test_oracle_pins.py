"""Pins for the CPU oracle: everything here is fixed by mathematics or by the paper, not by the
oracle itself.  A dropped term, wrong sign, wrong index or transposed operand anywhere in
oracle/decoder_layer.py fails at least one of these."""
import numpy as np
import pytest

from oracle import decoder_layer as O


def tiny_weights(rng, H, I, sigma=0.3):
    return {
        "gamma_attn": 1.0 + 0.2 * rng.standard_normal(H),
        "w_qkv": sigma * rng.standard_normal((3 * H, H)),
        "w_o": sigma * rng.standard_normal((H, H)),
        "gamma_mlp": 1.0 + 0.2 * rng.standard_normal(H),
        "w_gate_up": sigma * rng.standard_normal((2 * I, H)),
        "w_down": sigma * rng.standard_normal((H, I)),
    }


B, S, H, NH, I = 2, 8, 16, 2, 24


def loss(W, x, dy):
    y, _ = O.layer_fwd(W, x, NH, 10000.0, 1e-6)
    return float(np.sum(y * dy))


# ------------------------------------------------------------------ finite differences (whole fwd+bwd)
@pytest.mark.parametrize("which", ["x", "gamma_attn", "w_qkv", "w_o", "gamma_mlp", "w_gate_up", "w_down"])
def test_finite_difference_directional(which):
    rng = np.random.default_rng(11)
    W = tiny_weights(rng, H, I)
    x = rng.standard_normal((B, S, H))
    dy = rng.standard_normal((B, S, H))
    y, cache = O.layer_fwd(W, x, NH, 10000.0, 1e-6)
    dx, G = O.layer_bwd(W, cache, dy)
    eps = 1e-5
    for trial in range(3):
        if which == "x":
            v = rng.standard_normal(x.shape)
            lp = loss(W, x + eps * v, dy)
            lm = loss(W, x - eps * v, dy)
            ana = float(np.sum(dx * v))
        else:
            v = rng.standard_normal(W[which].shape)
            Wp = dict(W); Wp[which] = W[which] + eps * v
            Wm = dict(W); Wm[which] = W[which] - eps * v
            lp, lm = loss(Wp, x, dy), loss(Wm, x, dy)
            ana = float(np.sum(G[which] * v))
        num = (lp - lm) / (2 * eps)
        assert abs(num - ana) <= 1e-7 * max(1.0, abs(ana)), (which, num, ana)


def test_finite_difference_elementwise_x():
    """Every single element of dx, not only random directions (catches index mix-ups)."""
    rng = np.random.default_rng(5)
    b, s, h, nh, i = 1, 4, 8, 2, 12
    W = tiny_weights(rng, h, i)
    x = rng.standard_normal((b, s, h))
    dy = rng.standard_normal((b, s, h))
    _, cache = O.layer_fwd(W, x, nh)
    dx, _ = O.layer_bwd(W, cache, dy)
    eps = 1e-6
    for idx in np.ndindex(x.shape):
        xp = x.copy(); xp[idx] += eps
        xm = x.copy(); xm[idx] -= eps
        num = (np.sum(O.layer_fwd(W, xp, nh)[0] * dy) - np.sum(O.layer_fwd(W, xm, nh)[0] * dy)) / (2 * eps)
        assert abs(num - dx[idx]) < 1e-6 * max(1.0, abs(dx[idx]))


# ------------------------------------------------------------------ causal mask
def test_causal_invariance_forward_and_backward():
    rng = np.random.default_rng(3)
    W = tiny_weights(rng, H, I)
    x = rng.standard_normal((B, S, H))
    dy = rng.standard_normal((B, S, H))
    y, cache = O.layer_fwd(W, x, NH)
    dx, _ = O.layer_bwd(W, cache, dy)
    t = 4
    x2 = x.copy(); x2[:, t + 1:, :] += rng.standard_normal((B, S - t - 1, H))
    y2, _ = O.layer_fwd(W, x2, NH)
    assert np.array_equal(y[:, :t + 1], y2[:, :t + 1])       # later tokens cannot be seen
    assert not np.allclose(y[:, t + 1:], y2[:, t + 1:])
    dy2 = dy.copy(); dy2[:, :t, :] += rng.standard_normal((B, t, H))
    dx2, _ = O.layer_bwd(W, cache, dy2)
    assert np.allclose(dx[:, t:], dx2[:, t:], rtol=0, atol=1e-13)   # gradient flows only backwards in time
    assert not np.allclose(dx[:, :t], dx2[:, :t])


def test_diagonal_is_unmasked():
    """Token 0 attends to itself only: o[0] = v[0] for every head."""
    rng = np.random.default_rng(4)
    q, k, v = (rng.standard_normal((1, 6, 2, 4)) for _ in range(3))
    o = O.attention_fwd(q, k, v)
    assert np.allclose(o[:, 0], v[:, 0], atol=1e-15)


# ------------------------------------------------------------------ softmax
def test_softmax_rows_sum_to_one_and_S1():
    rng = np.random.default_rng(6)
    q, k = (3.0 * rng.standard_normal((2, 9, 3, 4)) for _ in range(2))
    ones = np.ones((2, 9, 3, 4))
    assert np.max(np.abs(O.attention_fwd(q, k, ones) - 1.0)) < 1e-14
    q1, k1, v1 = (rng.standard_normal((2, 1, 3, 4)) for _ in range(3))
    assert np.array_equal(O.attention_fwd(q1, k1, v1), v1)


def test_attention_closed_form_zero_queries_is_running_mean():
    rng = np.random.default_rng(7)
    k, v = (rng.standard_normal((1, 10, 2, 4)) for _ in range(2))
    o = O.attention_fwd(np.zeros_like(k), k, v)
    run = np.cumsum(v, axis=1) / np.arange(1, 11)[None, :, None, None]
    assert np.allclose(o, run, atol=1e-14)


def test_softmax_scale_is_inv_sqrt_head_dim():
    """Two keys, hand-computed probabilities."""
    d = 4
    q = np.zeros((1, 2, 1, d)); k = np.zeros((1, 2, 1, d)); v = np.zeros((1, 2, 1, d))
    q[0, 1, 0, 0] = 2.0
    k[0, 0, 0, 0] = 1.0; k[0, 1, 0, 0] = 3.0
    v[0, 0, 0, 0] = 1.0; v[0, 1, 0, 1] = 1.0
    o = O.attention_fwd(q, k, v)
    s0, s1 = 2.0 * 1.0 / 2.0, 2.0 * 3.0 / 2.0          # / sqrt(4)
    p0 = np.exp(s0) / (np.exp(s0) + np.exp(s1))
    assert np.allclose(o[0, 1, 0, :2], [p0, 1 - p0], atol=1e-15)


# ------------------------------------------------------------------ brute force (different implementation)
def brute_attention(q, k, v):
    B_, S_, nh, d = q.shape
    o = np.zeros_like(q)
    P = np.zeros((B_, nh, S_, S_))
    for b in range(B_):
        for h in range(nh):
            for t in range(S_):
                sc = [sum(q[b, t, h, i] * k[b, u, h, i] for i in range(d)) / np.sqrt(d) for u in range(t + 1)]
                m = max(sc)
                e = [np.exp(s - m) for s in sc]
                z = sum(e)
                for u in range(t + 1):
                    P[b, h, t, u] = e[u] / z
                    for i in range(d):
                        o[b, t, h, i] += P[b, h, t, u] * v[b, u, h, i]
    return o, P


def test_attention_matches_bruteforce_fwd_and_bwd():
    rng = np.random.default_rng(8)
    q, k, v, do = (rng.standard_normal((2, 7, 2, 4)) for _ in range(4))
    o = O.attention_fwd(q, k, v)
    ob, P = brute_attention(q, k, v)
    assert np.max(np.abs(o - ob)) < 1e-12
    dq, dk, dv = O.attention_bwd(q, k, v, o, do)
    # scalar-loop gradient from the materialised P
    B_, S_, nh, d = q.shape
    dqb, dkb, dvb = np.zeros_like(q), np.zeros_like(q), np.zeros_like(q)
    for b in range(B_):
        for h in range(nh):
            for t in range(S_):
                D = float(np.dot(do[b, t, h], ob[b, t, h]))
                for u in range(t + 1):
                    dP = float(np.dot(do[b, t, h], v[b, u, h]))
                    dS = P[b, h, t, u] * (dP - D)
                    dvb[b, u, h] += P[b, h, t, u] * do[b, t, h]
                    dqb[b, t, h] += dS * k[b, u, h] / np.sqrt(d)
                    dkb[b, u, h] += dS * q[b, t, h] / np.sqrt(d)
    assert np.max(np.abs(dq - dqb)) < 1e-12
    assert np.max(np.abs(dk - dkb)) < 1e-12
    assert np.max(np.abs(dv - dvb)) < 1e-12


def test_attention_row_blocking_has_no_effect(monkeypatch):
    rng = np.random.default_rng(9)
    q, k, v, do = (rng.standard_normal((1, 37, 2, 4)) for _ in range(4))
    o_full = O.attention_fwd(q, k, v)
    g_full = O.attention_bwd(q, k, v, o_full, do)
    monkeypatch.setattr(O, "_ROW_BLOCK", 5)
    o_blk = O.attention_fwd(q, k, v)
    g_blk = O.attention_bwd(q, k, v, o_blk, do)
    assert np.max(np.abs(o_full - o_blk)) < 1e-14
    for a, b in zip(g_full, g_blk):
        assert np.max(np.abs(a - b)) < 1e-13


# ------------------------------------------------------------------ RoPE
def test_rope_properties():
    rng = np.random.default_rng(10)
    S_, d = 12, 8
    phi = O.rope_angles(S_, d, 10000.0)
    assert phi.shape == (S_, d // 2)
    assert np.allclose(phi[1], 10000.0 ** (-2.0 * np.arange(d // 2) / d))     # definition at p=1
    assert np.allclose(phi[5], 5 * phi[1])
    z = rng.standard_normal((2, S_, 3, d))
    r = O.rope_apply(z, phi)
    # norm preserved per pair and per vector; position 0 is the identity
    assert np.allclose(r[..., 0::2] ** 2 + r[..., 1::2] ** 2, z[..., 0::2] ** 2 + z[..., 1::2] ** 2, atol=1e-13)
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(z, axis=-1), atol=1e-13)
    assert np.array_equal(r[:, 0], z[:, 0])
    # inverse rotation undoes it (that is the backward map of an orthogonal transform)
    assert np.allclose(O.rope_apply(r, phi, inverse=True), z, atol=1e-13)
    # hand value: pair (1,0) at position p, frequency 0 -> (cos p, sin p): rotation is counter-clockwise
    e = np.zeros((1, S_, 1, d)); e[..., 0] = 1.0
    re = O.rope_apply(e, phi)
    assert np.allclose(re[0, :, 0, 0], np.cos(np.arange(S_)))
    assert np.allclose(re[0, :, 0, 1], np.sin(np.arange(S_)))
    # relative-position property: <rope(q,m), rope(k,n)> depends on m-n only
    qv = rng.standard_normal(d); kv = rng.standard_normal(d)
    Q = O.rope_apply(np.broadcast_to(qv, (1, S_, 1, d)).copy(), phi)[0, :, 0]
    K = O.rope_apply(np.broadcast_to(kv, (1, S_, 1, d)).copy(), phi)[0, :, 0]
    Gm = Q @ K.T
    for delta in range(-3, 4):
        diag = np.diagonal(Gm, offset=delta)
        assert np.allclose(diag, diag[0], atol=1e-12)


# ------------------------------------------------------------------ RMSNorm
def test_rmsnorm_properties():
    rng = np.random.default_rng(12)
    z = rng.standard_normal((5, 16)); gamma = 1 + 0.3 * rng.standard_normal(16)
    out, r = O.rmsnorm_fwd(z, gamma, 0.0)
    assert np.allclose(np.sqrt(np.mean((out / gamma) ** 2, axis=1)), 1.0, atol=1e-14)
    out3, _ = O.rmsnorm_fwd(3.7 * z, gamma, 0.0)
    assert np.allclose(out, out3, atol=1e-14)                      # scale invariance at eps=0
    dout = rng.standard_normal(z.shape)
    dz, dgamma = O.rmsnorm_bwd(dout, z, r, gamma)
    assert np.max(np.abs(np.sum(dz * z, axis=1))) < 1e-13          # gradient orthogonal to the input
    assert np.allclose(dgamma, np.sum(dout * out / gamma, axis=0), atol=1e-13)
    # eps sits inside the square root, added to the mean: one-row hand value
    o1, r1 = O.rmsnorm_fwd(np.array([[3.0, 4.0]]), np.ones(2), 0.5)
    assert np.allclose(r1, 1 / np.sqrt(12.5 + 0.5))
    assert np.allclose(o1, np.array([[3.0, 4.0]]) / np.sqrt(13.0))


# ------------------------------------------------------------------ SwiGLU
def test_swiglu_properties():
    rng = np.random.default_rng(13)
    u = rng.standard_normal(20); da = rng.standard_normal(20)
    assert np.array_equal(O.swiglu_fwd(np.zeros(20), u), np.zeros(20))
    dg, du = O.swiglu_bwd(da, np.zeros(20), u)
    assert np.allclose(dg, da * u / 2) and np.array_equal(du, np.zeros(20))
    g = rng.standard_normal(20)
    eps = 1e-6
    dg, du = O.swiglu_bwd(da, g, u)
    assert np.allclose(dg, da * (O.swiglu_fwd(g + eps, u) - O.swiglu_fwd(g - eps, u)) / (2 * eps), atol=1e-8)
    assert np.allclose(du, da * (O.swiglu_fwd(g, u + eps) - O.swiglu_fwd(g, u - eps)) / (2 * eps), atol=1e-8)
    assert np.allclose(O.swiglu_fwd(np.array([1.0]), np.array([2.0])), 2.0 / (1 + np.exp(-1.0)))


# ------------------------------------------------------------------ layer-level closed forms and symmetries
def test_layer_closed_form_zero_output_projections():
    rng = np.random.default_rng(14)
    W = tiny_weights(rng, H, I)
    W["w_o"] = np.zeros((H, H)); W["w_down"] = np.zeros((H, I))
    x = rng.standard_normal((B, S, H)); dy = rng.standard_normal((B, S, H))
    y, cache = O.layer_fwd(W, x, NH)
    dx, G = O.layer_bwd(W, cache, dy)
    assert np.array_equal(y, x) and np.array_equal(dx, dy)
    T = B * S
    assert np.allclose(G["w_o"], dy.reshape(T, H).T @ cache["o"].reshape(T, H), atol=1e-13)
    assert np.allclose(G["w_down"], dy.reshape(T, H).T @ cache["a"], atol=1e-13)
    assert np.all(G["w_qkv"] == 0) and np.all(G["w_gate_up"] == 0)


def test_backward_is_linear_in_dy():
    rng = np.random.default_rng(15)
    W = tiny_weights(rng, H, I)
    x = rng.standard_normal((B, S, H))
    d1, d2 = rng.standard_normal((2, B, S, H))
    _, cache = O.layer_fwd(W, x, NH)
    a, b = 0.7, -1.9
    dx1, G1 = O.layer_bwd(W, cache, d1)
    dx2, G2 = O.layer_bwd(W, cache, d2)
    dx3, G3 = O.layer_bwd(W, cache, a * d1 + b * d2)
    assert np.allclose(dx3, a * dx1 + b * dx2, atol=1e-12)
    for k in G3:
        assert np.allclose(G3[k], a * G1[k] + b * G2[k], atol=1e-12)


def test_batch_elements_independent_and_gradients_sum():
    rng = np.random.default_rng(16)
    W = tiny_weights(rng, H, I)
    x = rng.standard_normal((2, S, H)); dy = rng.standard_normal((2, S, H))
    y, cache = O.layer_fwd(W, x, NH)
    dx, G = O.layer_bwd(W, cache, dy)
    Gs = None
    for b in range(2):
        yb, cb = O.layer_fwd(W, x[b:b + 1], NH)
        dxb, Gb = O.layer_bwd(W, cb, dy[b:b + 1])
        assert np.allclose(yb, y[b:b + 1], atol=1e-13) and np.allclose(dxb, dx[b:b + 1], atol=1e-13)
        Gs = Gb if Gs is None else {k: O.grad_accum(Gs[k], Gb[k], 1.0) for k in Gb}
    for k in G:
        assert np.allclose(G[k], Gs[k], atol=1e-12)


def test_head_permutation_symmetry():
    rng = np.random.default_rng(17)
    W = tiny_weights(rng, H, I)
    x = rng.standard_normal((B, S, H))
    y, _ = O.layer_fwd(W, x, NH)
    d = H // NH
    perm = np.concatenate([np.arange(d) + d, np.arange(d)])     # swap the two heads
    W2 = dict(W)
    W2["w_qkv"] = np.concatenate([W["w_qkv"][0:H][perm], W["w_qkv"][H:2 * H][perm], W["w_qkv"][2 * H:][perm]])
    W2["w_o"] = W["w_o"][:, perm]
    y2, _ = O.layer_fwd(W2, x, NH)
    assert np.allclose(y, y2, atol=1e-13)


def test_grad_accum():
    G = np.array([1.0, 2.0, 3.0]); g = np.array([0.5, -1.0, 4.0])
    assert np.array_equal(O.grad_accum(G, g, 0.25), np.array([1.125, 1.75, 4.0]))
    assert np.array_equal(O.grad_accum(G, g), G + g)


def test_sampled_rows_agree_with_full_forward():
    rng = np.random.default_rng(18)
    h, nh, i, s = 32, 4, 40, 33
    W = tiny_weights(rng, h, i)
    x = rng.standard_normal((1, s, h))
    y, _ = O.layer_fwd(W, x, nh)
    rows = np.array([0, 5, 17, 32])
    yr = O.layer_fwd_rows(W, x[0], rows, nh)
    assert np.max(np.abs(yr - y[0, rows])) < 1e-12


@pytest.mark.parametrize("t0", [0, 1, 20, 32])
def test_backward_tail_agrees_with_full_backward(t0):
    """layer_bwd_tail (the closed sub-problem at the rows t >= t0, used for full-size parity of the
    layer's backward) against the complete layer_fwd + layer_bwd, and against central finite
    differences of the loss <dy, y> in x at those rows (which no oracle code path shares)."""
    rng = np.random.default_rng(23 + t0)
    h, nh, i, s = 32, 4, 40, 33
    W = tiny_weights(rng, h, i)
    x = rng.standard_normal((1, s, h))
    dy = rng.standard_normal((1, s, h))
    _, cache = O.layer_fwd(W, x, nh)
    dx, _ = O.layer_bwd(W, cache, dy)
    tail = O.layer_bwd_tail(W, x[0], dy[0], t0, nh)
    assert tail.shape == (s - t0, h)
    assert np.max(np.abs(tail - dx[0, t0:])) < 1e-11
    eps = 1e-5
    for _ in range(3):
        v = np.zeros_like(x)
        v[0, t0:] = rng.standard_normal((s - t0, h))
        lp = float(np.sum(O.layer_fwd(W, x + eps * v, nh)[0] * dy))
        lm = float(np.sum(O.layer_fwd(W, x - eps * v, nh)[0] * dy))
        ana = float(np.sum(tail * v[0, t0:]))
        assert abs((lp - lm) / (2 * eps) - ana) <= 1e-7 * max(1.0, abs(ana))


def test_backward_tail_catches_a_dropped_key_contribution(monkeypatch):
    """Planted mistake: if the tail form ignored the rotary backward, the comparison above must fail."""
    orig = O.rope_apply
    monkeypatch.setattr(O, "rope_apply", lambda z, phi, inverse=False: z if inverse else orig(z, phi))
    with pytest.raises(AssertionError):
        test_backward_tail_agrees_with_full_backward(20)


# ------------------------------------------------------------------ independent library implementation
def test_against_torch_fp64_autograd():
    """Same block written with torch CPU fp64 ops (complex-number RoPE, library SDPA, autograd
    for every gradient): an implementation that shares nothing with the oracle."""
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    rng = np.random.default_rng(19)
    b, s, h, nh, i = 2, 19, 32, 4, 40
    d = h // nh
    W = tiny_weights(rng, h, i)
    x = rng.standard_normal((b, s, h)); dy = rng.standard_normal((b, s, h))
    y, cache = O.layer_fwd(W, x, nh, 10000.0, 1e-6)
    dx, G = O.layer_bwd(W, cache, dy)

    tW = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in W.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)

    def rms(z, g):
        return z * torch.rsqrt(z.pow(2).mean(-1, keepdim=True) + 1e-6) * g

    def rope_c(z):  # z [b,s,nh,d] -> rotate as complex numbers (pair = re, im)
        zc = torch.view_as_complex(z.reshape(b, s, nh, d // 2, 2).contiguous())
        freqs = 1.0 / (10000.0 ** (torch.arange(0, d, 2, dtype=torch.float64) / d))
        ang = torch.outer(torch.arange(s, dtype=torch.float64), freqs)
        rot = torch.polar(torch.ones_like(ang), ang)[None, :, None, :]
        return torch.view_as_real(zc * rot).reshape(b, s, nh, d)

    xn = rms(tx, tW["gamma_attn"])
    qkv = F.linear(xn, tW["w_qkv"])
    q, k, v = qkv.split(h, dim=-1)
    q = rope_c(q.reshape(b, s, nh, d)).transpose(1, 2)
    k = rope_c(k.reshape(b, s, nh, d)).transpose(1, 2)
    v = v.reshape(b, s, nh, d).transpose(1, 2)
    o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(b, s, h)
    hh = tx + F.linear(o, tW["w_o"])
    hn = rms(hh, tW["gamma_mlp"])
    g, u = F.linear(hn, tW["w_gate_up"]).split(i, dim=-1)
    ty = hh + F.linear(F.silu(g) * u, tW["w_down"])
    ty.backward(torch.tensor(dy))
    assert np.max(np.abs(ty.detach().numpy() - y)) < 1e-11
    assert np.max(np.abs(tx.grad.numpy() - dx)) < 1e-10
    for kname in G:
        assert np.max(np.abs(tW[kname].grad.numpy() - G[kname])) < 1e-10, kname


# ------------------------------------------------------------------ facts printed in the paper
def test_parameter_count_matches_paper_12H2():
    """Theoretical Analysis: a LLaMA-style layer has about 12 H^2 parameters."""
    H_, I_ = 4096, 11008
    n = 4 * H_ * H_ + 3 * H_ * I_
    assert abs(n / (12 * H_ * H_) - 1.0) < 0.01
    assert n == 202_375_168


def test_flop_convention():
    assert abs(O.flops_fwd_bwd(1, 8192, 4096, 11008) / 1e12 - 11.60) < 0.01
    assert abs(O.flops_fwd_bwd(1, 32768, 4096, 11008) / 1e12 - 66.18) < 0.01


# ------------------------------------------------------------------ planted mistakes are caught
@pytest.mark.parametrize("mutation", ["mask_strict", "rope_sign", "drop_gamma", "scale"])
def test_pins_catch_planted_mistakes(monkeypatch, mutation):
    """Plant a plausible mistake in the oracle (on the CPU) and check a pin above notices."""
    if mutation == "mask_strict":
        # strict mask u < t would make row 0 empty; emulate "diagonal masked" on rows >= 1
        def bad_rows(q_blk, k, t0, scale):
            S_ = k.shape[0]
            s = (q_blk @ k.T) * scale
            t = np.arange(t0, t0 + q_blk.shape[0])[:, None]
            u = np.arange(S_)[None, :]
            keep = (u < t) | ((t == 0) & (u == 0))
            s = np.where(keep, s, -np.inf)
            e = np.exp(s - s.max(axis=1, keepdims=True))
            return e / e.sum(axis=1, keepdims=True)
        monkeypatch.setattr(O, "_softmax_rows", bad_rows)
        with pytest.raises(AssertionError):
            test_softmax_scale_is_inv_sqrt_head_dim()
    elif mutation == "rope_sign":
        orig = O.rope_apply
        monkeypatch.setattr(O, "rope_apply", lambda z, phi, inverse=False: orig(z, phi, not inverse))
        with pytest.raises(AssertionError):
            test_rope_properties()
    elif mutation == "drop_gamma":
        orig = O.rmsnorm_fwd
        monkeypatch.setattr(O, "rmsnorm_fwd", lambda z, g, e: orig(z, np.ones_like(g), e))
        with pytest.raises(AssertionError):
            test_against_torch_fp64_autograd()
    elif mutation == "scale":
        orig = O._softmax_rows
        monkeypatch.setattr(O, "_softmax_rows", lambda q, k, t0, sc: orig(q, k, t0, 1.0))
        with pytest.raises(AssertionError):
            test_softmax_scale_is_inv_sqrt_head_dim()


def test_sampled_attention_matches_the_full_definition():
    """attention_fwd_rows / attention_bwd_tail (used for full-size sampled parity) against the
    complete attention_fwd / attention_bwd on a size where both run, plus lse against a direct sum."""
    rng = np.random.default_rng(5)
    S, d = 97, 8
    q, k, v, do = (rng.standard_normal((1, S, 1, d)) for _ in range(4))
    o = O.attention_fwd(q, k, v)
    dq, dk, dv = O.attention_bwd(q, k, v, o, do)
    rows = np.array([0, 1, 13, 50, 96])
    o_r, lse = O.attention_fwd_rows(q[0, rows, 0], k[0, :, 0], v[0, :, 0], rows)
    np.testing.assert_allclose(o_r, o[0, rows, 0], rtol=1e-12, atol=1e-14)
    for n, t in enumerate(rows):
        direct = np.log(np.sum(np.exp(k[0, :t + 1, 0] @ q[0, t, 0] / np.sqrt(d))))
        assert abs(lse[n] - direct) < 1e-12
    t0 = 60
    dq_t, dk_t, dv_t = O.attention_bwd_tail(q[0, :, 0], k[0, :, 0], v[0, :, 0], do[0, :, 0], t0)
    np.testing.assert_allclose(dq_t, dq[0, t0:, 0], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dk_t, dk[0, t0:, 0], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dv_t, dv[0, t0:, 0], rtol=1e-11, atol=1e-13)


def test_adamw_step_against_closed_forms_and_a_library_optimizer():
    """adamw_step: the first step from zero state moves every weight by lr * g/(|g| + eps) (+ decay),
    zero gradient with zero state only decays, and five steps agree with torch.optim.AdamW in fp64."""
    import torch
    rng = np.random.default_rng(11)
    w0, g = rng.standard_normal(1000), rng.standard_normal(1000)
    z = np.zeros_like(w0)
    w1, m1, v1 = O.adamw_step(w0, z, z, g, 1, 1e-2, 0.9, 0.999, 1e-8, 0.0)
    np.testing.assert_allclose(w1, w0 - 1e-2 * g / (np.abs(g) + 1e-8), rtol=1e-12)
    np.testing.assert_allclose(m1, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v1, 0.001 * g * g, rtol=1e-12)
    w1, _, _ = O.adamw_step(w0, z, z, z, 1, 1e-2, 0.9, 0.999, 1e-8, 0.1)
    np.testing.assert_allclose(w1, w0 * (1 - 1e-3), rtol=1e-12)
    # grad_scale is the same as scaling the gradient
    a = O.adamw_step(w0, z, z, g, 3, 1e-3, 0.9, 0.95, 1e-6, 0.01, grad_scale=0.25)
    b = O.adamw_step(w0, z, z, 0.25 * g, 3, 1e-3, 0.9, 0.95, 1e-6, 0.01)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=1e-13)
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-6, weight_decay=0.05)
    w, m, v = w0.copy(), z.copy(), z.copy()
    for t in range(1, 6):
        gt = rng.standard_normal(1000)
        p.grad = torch.from_numpy(gt.copy())
        opt.step()
        w, m, v = O.adamw_step(w, m, v, gt, t, 3e-3, 0.9, 0.95, 1e-6, 0.05)
    np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-10, atol=1e-12)
