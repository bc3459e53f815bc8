"""CPU fp64 oracle for one LLaMA-2 style decoder layer: forward, backward, gradient accumulation.

TEST INFRASTRUCTURE ONLY.  This file is the independent reference that the HIP path is checked
against.  It shares no code with the HIP path and must never be imported by the product
package; only tests, the smoke check and the benchmark's cpu_baseline leg may call it.

What it follows.  The paper fixes the per-device computation only as "the layer applied to the
device's own micro-batch whenever the layer's weights arrive" (Methodology, Group-Based Weight
Pipeline Scheduler: forward caches activations A_j, backward yields the gradients G_j of W_j;
Table 1 symbols A, W, G), on models "derived from the LLaMA-2 architecture" (Experimental
Setup) whose layer has about 12 H^2 parameters (Theoretical Analysis) and whose attention is
exact (FlashAttention is an exact method).  Tiling, online softmax and fused epilogues do not
change that result, so the oracle is the plain definition of the block written out in fp64:

  forward:   xn = rmsnorm(x; gamma_attn)            q,k,v = xn Wq^T, xn Wk^T, xn Wv^T
             q,k <- rope(q), rope(k)                 o = softmax(q k^T / sqrt(d) + causal) v
             h = x + o Wo^T                          hn = rmsnorm(h; gamma_mlp)
             g,u = hn Wg^T, hn Wu^T                  a = silu(g) * u
             y = h + a Wd^T
  backward:  the chain rule through the same steps, for the implicit loss <dY, y>.

Readings adopted where the paper is silent (all are the LLaMA-2 conventions):
  pre-norm block with two residuals, no biases, no dropout, multi-head attention (no GQA);
  RMSNorm epsilon is added to the mean of squares inside the square root;
  RoPE rotates adjacent pairs (2i, 2i+1) of every head of q and k by pos * theta^(-2i/d),
  positions 0..S-1 in every batch element; softmax scale 1/sqrt(head_dim); the causal mask
  keeps u <= t; weights are [out, in] row-major and y = x W^T; w_qkv rows are [Q; K; V],
  w_gate_up rows are [gate; up].

numpy matmul (a library dgemm) serves as the matrix-product step; there is no tiling, no online
softmax and no fusion here: every attention row is normalised over its complete set of keys.
The only concession to memory is that attention rows are processed a block of rows at a time
(each row still sees all its keys at once).

Every function is pinned by tests/test_oracle_*.py (finite differences, closed forms,
invariants, brute force, and an independent library autograd); nothing here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

_ROW_BLOCK = 1024  # attention rows handled per step (memory only; no effect on the result)


# ----------------------------------------------------------------------------- RMSNorm
def rmsnorm_fwd(z, gamma, eps):
    """r_t = 1/sqrt(mean_i z[t,i]^2 + eps);  out[t,i] = z[t,i] r_t gamma_i.   z: [T, H]."""
    r = 1.0 / np.sqrt(np.mean(z * z, axis=-1, keepdims=True) + eps)
    return z * r * gamma, r[..., 0]


def rmsnorm_bwd(dout, z, r, gamma):
    """Gradient of rmsnorm_fwd.  c = dout*gamma;  dz = r c - z r^3 mean_j(c_j z_j);
    dgamma_i = sum_t dout[t,i] z[t,i] r_t."""
    c = dout * gamma
    rr = r[:, None]
    dz = rr * c - z * (rr ** 3) * np.mean(c * z, axis=-1, keepdims=True)
    dgamma = np.sum(dout * z * rr, axis=0)
    return dz, dgamma


# ----------------------------------------------------------------------------- RoPE
def rope_angles(S, head_dim, theta):
    """phi[p, i] = p * theta^(-2i/d), p in [0,S), i in [0,d/2)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = theta ** (-2.0 * i / head_dim)
    return np.arange(S, dtype=np.float64)[:, None] * inv_freq[None, :]


def rope_apply(z, phi, inverse=False):
    """Rotate adjacent pairs.  z: [B, S, n_heads, d];  phi: [S, d/2].
    (a, b) -> (a cos - b sin, a sin + b cos); inverse=True rotates by -phi (the backward map)."""
    c = np.cos(phi)[None, :, None, :]
    s = np.sin(phi)[None, :, None, :]
    if inverse:
        s = -s
    a = z[..., 0::2]
    b = z[..., 1::2]
    out = np.empty_like(z)
    out[..., 0::2] = a * c - b * s
    out[..., 1::2] = a * s + b * c
    return out


# ----------------------------------------------------------------------------- attention
def _softmax_rows(q_blk, k, t0, scale):
    """P[t, u] for rows t0..t0+len(q_blk)-1 over all keys u (zero for u > t)."""
    S = k.shape[0]
    s = (q_blk @ k.T) * scale
    t = np.arange(t0, t0 + q_blk.shape[0])[:, None]
    u = np.arange(S)[None, :]
    s = np.where(u <= t, s, -np.inf)
    m = np.max(s, axis=1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=1, keepdims=True)


def attention_fwd(q, k, v):
    """Causal softmax attention.  q,k,v: [B, S, n_heads, d] -> o of the same shape.
    o[t] = sum_{u<=t} P[t,u] v[u],  P = softmax over u<=t of q[t].k[u]/sqrt(d)."""
    B, S, nh, d = q.shape
    scale = 1.0 / np.sqrt(d)
    o = np.empty_like(q)
    for b in range(B):
        for h in range(nh):
            kk, vv = k[b, :, h, :], v[b, :, h, :]
            for t0 in range(0, S, _ROW_BLOCK):
                P = _softmax_rows(q[b, t0:t0 + _ROW_BLOCK, h, :], kk, t0, scale)
                o[b, t0:t0 + _ROW_BLOCK, h, :] = P @ vv
    return o


def attention_bwd(q, k, v, o, do):
    """Gradient of attention_fwd.  D_t = do[t].o[t];  dP = do v^T;  dS = P*(dP - D);
    dv = P^T do;  dq = dS k / sqrt(d);  dk = dS^T q / sqrt(d)."""
    B, S, nh, d = q.shape
    scale = 1.0 / np.sqrt(d)
    dq = np.zeros_like(q)
    dk = np.zeros_like(q)
    dv = np.zeros_like(q)
    for b in range(B):
        for h in range(nh):
            kk, vv = k[b, :, h, :], v[b, :, h, :]
            for t0 in range(0, S, _ROW_BLOCK):
                sl = slice(t0, t0 + _ROW_BLOCK)
                qq = q[b, sl, h, :]
                P = _softmax_rows(qq, kk, t0, scale)
                dO = do[b, sl, h, :]
                D = np.sum(dO * o[b, sl, h, :], axis=1, keepdims=True)
                dP = dO @ vv.T
                dS = P * (dP - D)
                dv[b, :, h, :] += P.T @ dO
                dq[b, sl, h, :] = (dS @ kk) * scale
                dk[b, :, h, :] += (dS.T @ qq) * scale
    return dq, dk, dv


# ----------------------------------------------------------------------------- SwiGLU
def swiglu_fwd(g, u):
    """a = g * sigmoid(g) * u."""
    return g / (1.0 + np.exp(-g)) * u


def swiglu_bwd(da, g, u):
    """dg = da u sig (1 + g (1 - sig));  du = da g sig."""
    sig = 1.0 / (1.0 + np.exp(-g))
    return da * u * sig * (1.0 + g * (1.0 - sig)), da * g * sig


# ----------------------------------------------------------------------------- the layer
def layer_fwd(W, x, n_heads, rope_theta=10000.0, rms_eps=1e-6):
    """Forward of the decoder layer.  W: dict of fp64 arrays (gamma_attn [H], w_qkv [3H,H],
    w_o [H,H], gamma_mlp [H], w_gate_up [2I,H], w_down [H,I]);  x: [B,S,H].
    Returns y [B,S,H] and the cache of intermediates the backward needs."""
    B, S, H = x.shape
    d = H // n_heads
    I = W["w_down"].shape[1]
    T = B * S
    x2 = x.reshape(T, H)
    xn, r1 = rmsnorm_fwd(x2, W["gamma_attn"], rms_eps)
    qkv = xn @ W["w_qkv"].T
    phi = rope_angles(S, d, rope_theta)
    q = rope_apply(qkv[:, 0:H].reshape(B, S, n_heads, d), phi)
    k = rope_apply(qkv[:, H:2 * H].reshape(B, S, n_heads, d), phi)
    v = qkv[:, 2 * H:3 * H].reshape(B, S, n_heads, d)
    o = attention_fwd(q, k, v)
    o2 = o.reshape(T, H)
    h = x2 + o2 @ W["w_o"].T
    hn, r2 = rmsnorm_fwd(h, W["gamma_mlp"], rms_eps)
    gu = hn @ W["w_gate_up"].T
    g, u = gu[:, :I], gu[:, I:]
    a = swiglu_fwd(g, u)
    y = h + a @ W["w_down"].T
    cache = dict(x=x2, xn=xn, r1=r1, q=q, k=k, v=v, o=o, h=h, hn=hn, r2=r2, g=g, u=u, a=a, phi=phi,
                 n_heads=n_heads)
    return y.reshape(B, S, H), cache


def layer_bwd(W, cache, dy):
    """Backward of the decoder layer for upstream gradient dy [B,S,H].
    Returns dx [B,S,H] and the weight gradients as a dict with the keys of W."""
    B, S, H = dy.shape
    T = B * S
    nh = cache["n_heads"]
    d = H // nh
    I = W["w_down"].shape[1]
    dy2 = dy.reshape(T, H)
    G = {}
    # y = h + a Wd^T
    da = dy2 @ W["w_down"]
    G["w_down"] = dy2.T @ cache["a"]
    dh = dy2.copy()
    # a = silu(g) u ; [g,u] = hn Wgu^T
    dg, du = swiglu_bwd(da, cache["g"], cache["u"])
    dgu = np.concatenate([dg, du], axis=1)
    dhn = dgu @ W["w_gate_up"]
    G["w_gate_up"] = dgu.T @ cache["hn"]
    # hn = rmsnorm(h)
    dz, G["gamma_mlp"] = rmsnorm_bwd(dhn, cache["h"], cache["r2"], W["gamma_mlp"])
    dh = dh + dz
    # h = x + o Wo^T
    do = dh @ W["w_o"]
    G["w_o"] = dh.T @ cache["o"].reshape(T, H)
    dq, dk, dv = attention_bwd(cache["q"], cache["k"], cache["v"], cache["o"], do.reshape(B, S, nh, d))
    dq = rope_apply(dq, cache["phi"], inverse=True)
    dk = rope_apply(dk, cache["phi"], inverse=True)
    dqkv = np.concatenate([dq.reshape(T, H), dk.reshape(T, H), dv.reshape(T, H)], axis=1)
    dxn = dqkv @ W["w_qkv"]
    G["w_qkv"] = dqkv.T @ cache["xn"]
    dz, G["gamma_attn"] = rmsnorm_bwd(dxn, cache["x"], cache["r1"], W["gamma_attn"])
    dx = dh + dz
    return dx.reshape(B, S, H), G


def grad_accum(G_dst, g_src, scale=1.0):
    """Owner-side aggregation of a gradient contribution into the fixed fp32 shard
    (Methodology, GWPS: gradients are transferred to the owner for final aggregation):
    G_dst[i] += scale * g_src[i].  Returns the new G_dst (fp64 arithmetic)."""
    return G_dst + scale * g_src


def adamw_step(w, m, v, g, step, lr, beta1, beta2, eps, weight_decay, grad_scale=1.0):
    """Owner-side update of a shard (Methodology, GWPS: the owner updates its shard in place from the
    optimizer state it keeps beside it; the optimizer itself is not named by the paper: AdamW with
    decoupled weight decay is the reading adopted).  All arrays fp64; step is 1-based.  Returns (w, m, v) after the step:
      g' = grad_scale g;  m = b1 m + (1-b1) g';  v = b2 v + (1-b2) g'^2
      w = w - lr ( m/(1-b1^t) / (sqrt(v/(1-b2^t)) + eps) + weight_decay w )"""
    g = grad_scale * g
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mh = m / (1.0 - beta1 ** step)
    vh = v / (1.0 - beta2 ** step)
    w = w - lr * (mh / (np.sqrt(vh) + eps) + weight_decay * w)
    return w, m, v


# ----------------------------------------------------------------------------- sampled evaluation
def layer_fwd_rows(W, x, rows, n_heads, rope_theta=10000.0, rms_eps=1e-6):
    """y at selected token rows of ONE batch element, by the same definition.
    x: [S, H]; rows: increasing int array.  Keys and values are projected for every token up to
    max(rows); queries, attention and the MLP only for the selected rows.  Returns y[rows]."""
    S, H = x.shape
    d = H // n_heads
    I = W["w_down"].shape[1]
    rows = np.asarray(rows)
    n = int(rows.max()) + 1
    xn, _ = rmsnorm_fwd(x[:n], W["gamma_attn"], rms_eps)
    phi = rope_angles(n, d, rope_theta)
    k = rope_apply((xn @ W["w_qkv"][H:2 * H].T).reshape(1, n, n_heads, d), phi)[0]
    v = (xn @ W["w_qkv"][2 * H:].T).reshape(n, n_heads, d)
    q_all = (xn[rows] @ W["w_qkv"][:H].T).reshape(1, len(rows), n_heads, d)
    # rotate each selected query by its own position
    c = np.cos(phi[rows])[None, :, None, :]
    s = np.sin(phi[rows])[None, :, None, :]
    q = np.empty_like(q_all)
    q[..., 0::2] = q_all[..., 0::2] * c - q_all[..., 1::2] * s
    q[..., 1::2] = q_all[..., 0::2] * s + q_all[..., 1::2] * c
    q = q[0]
    scale = 1.0 / np.sqrt(d)
    o = np.empty((len(rows), n_heads, d))
    for h in range(n_heads):
        sc = (q[:, h, :] @ k[:, h, :].T) * scale
        sc = np.where(np.arange(n)[None, :] <= rows[:, None], sc, -np.inf)
        e = np.exp(sc - sc.max(axis=1, keepdims=True))
        o[:, h, :] = (e / e.sum(axis=1, keepdims=True)) @ v[:, h, :]
    hrow = x[rows] + o.reshape(len(rows), H) @ W["w_o"].T
    hn, _ = rmsnorm_fwd(hrow, W["gamma_mlp"], rms_eps)
    gu = hn @ W["w_gate_up"].T
    return hrow + swiglu_fwd(gu[:, :I], gu[:, I:]) @ W["w_down"].T


def attention_fwd_rows(q_rows, k, v, rows):
    """Attention output and log-sum-exp at selected query rows of one (batch, head).
    q_rows: [n, d] (the queries at positions `rows`); k, v: [S, d].  Row t sees keys u <= t.
    Returns o [n, d] and lse [n] = log sum_{u<=t} exp(q[t].k[u]/sqrt(d))."""
    rows = np.asarray(rows)
    S, d = k.shape
    s = (q_rows @ k.T) / np.sqrt(d)
    s = np.where(np.arange(S)[None, :] <= rows[:, None], s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=1, keepdims=True)
    return (e / z) @ v, (m + np.log(z))[:, 0]


def attention_bwd_tail(q, k, v, do, t0):
    """Gradients of attention_fwd for one (batch, head), restricted to what the queries t >= t0
    determine completely: dq[t] for t >= t0 (a query's gradient needs only its own row of P) and
    dk[u], dv[u] for u >= t0 (a key is seen by the queries t >= u only).  q, k, v, do: [S, d].
    Returns dq [S-t0, d], dk [S-t0, d], dv [S-t0, d]."""
    S, d = q.shape
    scale = 1.0 / np.sqrt(d)
    rows = np.arange(t0, S)
    s = (q[t0:] @ k.T) * scale
    s = np.where(np.arange(S)[None, :] <= rows[:, None], s, -np.inf)
    e = np.exp(s - s.max(axis=1, keepdims=True))
    P = e / e.sum(axis=1, keepdims=True)
    o = P @ v
    D = np.sum(do[t0:] * o, axis=1, keepdims=True)
    dS = P * (do[t0:] @ v.T - D)
    dq = (dS @ k) * scale
    dk = (dS[:, t0:].T @ q[t0:]) * scale
    dv = P[:, t0:].T @ do[t0:]
    return dq, dk, dv


def layer_bwd_tail(W, x, dy, t0, n_heads, rope_theta=10000.0, rms_eps=1e-6):
    """dx at the token rows t >= t0 of ONE batch element, by the same definitions as layer_fwd / layer_bwd.
    x, dy: [S, H].  Causality makes this a closed sub-problem: the forward at a row t >= t0 needs the
    keys and values of every row (projected here for all of them) but queries, attention and the MLP
    only at the rows t >= t0; in the backward, dq[t] needs row t of the probabilities only, and
    dk[u], dv[u] for u >= t0 receive contributions from the queries t >= u >= t0 only.  Everything
    else (the residual path, both norms, the MLP) is row-wise.  Returns dx[t0:] as [S - t0, H]."""
    S, H = x.shape
    d = H // n_heads
    I = W["w_down"].shape[1]
    n = S - t0
    scale = 1.0 / np.sqrt(d)
    # ---- forward: k, v everywhere; the rest at rows t0..S-1
    xn, r1 = rmsnorm_fwd(x, W["gamma_attn"], rms_eps)
    phi = rope_angles(S, d, rope_theta)
    k = rope_apply((xn @ W["w_qkv"][H:2 * H].T).reshape(1, S, n_heads, d), phi)[0]
    v = (xn @ W["w_qkv"][2 * H:].T).reshape(S, n_heads, d)
    q = rope_apply((xn[t0:] @ W["w_qkv"][:H].T).reshape(1, n, n_heads, d), phi[t0:])[0]
    rows = np.arange(t0, S)
    P = np.empty((n_heads, n, S))
    o = np.empty((n, n_heads, d))
    for h in range(n_heads):
        sc = (q[:, h, :] @ k[:, h, :].T) * scale
        sc = np.where(np.arange(S)[None, :] <= rows[:, None], sc, -np.inf)
        e = np.exp(sc - sc.max(axis=1, keepdims=True))
        P[h] = e / e.sum(axis=1, keepdims=True)
        o[:, h, :] = P[h] @ v[:, h, :]
    o2 = o.reshape(n, H)
    hrow = x[t0:] + o2 @ W["w_o"].T
    hn, r2 = rmsnorm_fwd(hrow, W["gamma_mlp"], rms_eps)
    gu = hn @ W["w_gate_up"].T
    g, u = gu[:, :I], gu[:, I:]
    # ---- backward at the same rows
    dyt = dy[t0:]
    da = dyt @ W["w_down"]
    dg, du = swiglu_bwd(da, g, u)
    dhn = np.concatenate([dg, du], axis=1) @ W["w_gate_up"]
    dz, _ = rmsnorm_bwd(dhn, hrow, r2, W["gamma_mlp"])
    dh = dyt + dz
    do = (dh @ W["w_o"]).reshape(n, n_heads, d)
    dq = np.empty((n, n_heads, d))
    dk = np.empty((n, n_heads, d))
    dv = np.empty((n, n_heads, d))
    for h in range(n_heads):
        D = np.sum(do[:, h, :] * o[:, h, :], axis=1, keepdims=True)
        dS = P[h] * (do[:, h, :] @ v[:, h, :].T - D)
        dq[:, h, :] = (dS @ k[:, h, :]) * scale
        dk[:, h, :] = (dS[:, t0:].T @ q[:, h, :]) * scale
        dv[:, h, :] = P[h][:, t0:].T @ do[:, h, :]
    dq = rope_apply(dq[None], phi[t0:], inverse=True)[0]
    dk = rope_apply(dk[None], phi[t0:], inverse=True)[0]
    dqkv = np.concatenate([dq.reshape(n, H), dk.reshape(n, H), dv.reshape(n, H)], axis=1)
    dxn = dqkv @ W["w_qkv"]
    dz, _ = rmsnorm_bwd(dxn, x[t0:], r1[t0:], W["gamma_attn"])
    return dh + dz


def flops_fwd_bwd(B, S, H, I):
    """Model FLOPs of one forward+backward (counting convention, not arithmetic of the layer):
    GEMMs 6 T H (4H + 3I); attention 12 B (S(S+1)/2) H (causal pairs, backward = 2x forward)."""
    T = B * S
    return 6.0 * T * H * (4 * H + 3 * I) + 12.0 * B * (S * (S + 1) / 2.0) * H
