"""Oracle: GEMM, attention with dropout, and the transformer block, in float64.
TEST INFRASTRUCTURE ONLY.

Everything here is the plain definition.  Inputs are expected to hold values
already rounded to the dtype under test; all arithmetic is float64.
"""
import numpy as np

from . import philox as _philox


def gemm(A, Bm, transB=False):
    """C[m, n] = sum_k A[m, k] * B[k, n]  (paper Table 1, GEMM column).

    With transB the second operand is stored [N, K]."""
    A = np.asarray(A, dtype=np.float64)
    Bm = np.asarray(Bm, dtype=np.float64)
    return A @ (Bm.T if transB else Bm)


def gemm_entries(A, Bm, rows, cols, transB=False):
    """Selected entries C[rows[i], cols[i]] by explicit dot products."""
    A = np.asarray(A)
    Bm = np.asarray(Bm)
    out = np.empty(len(rows), dtype=np.float64)
    for i, (m, n) in enumerate(zip(rows, cols)):
        a = A[m, :].astype(np.float64)
        b = (Bm[n, :] if transB else Bm[:, n]).astype(np.float64)
        out[i] = float(np.dot(a, b))
    return out


def attention_dropout(Q, K, V, keep, p, causal=False, rows=None):
    """O = dropout(softmax(Q K^T / sqrt(d))) V  (paper Sec. 2.2: dropout is applied
    to the softmax output; kept probabilities are scaled by 1 / (1 - p)).

    Q: [B, S, H, d]; K, V: [B, S, Hkv, d] with H a multiple of Hkv (query head h
    uses key/value head h // (H // Hkv)).  keep: bool [B, H, S, S], or None for
    no dropout.  The softmax normaliser runs over every admissible column,
    dropped or not.  causal: column j is admissible for row i iff j <= i.
    rows: optional list of query indices; the result then has shape
    [B, len(rows), H, d].  A row whose kept set is empty gives zeros.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, S, H, d = Q.shape
    Hkv = K.shape[2]
    assert H % Hkv == 0 and K.shape == V.shape and K.shape[0] == B and K.shape[1] == S
    rep = H // Hkv
    ridx = np.arange(S) if rows is None else np.asarray(rows, dtype=np.int64)
    O = np.zeros((B, len(ridx), H, d), dtype=np.float64)
    scale = 1.0 / np.sqrt(float(d))
    keep_scale = 1.0 / (1.0 - float(np.float32(p))) if keep is not None else 1.0
    cols = np.arange(S)
    for b in range(B):
        for h in range(H):
            hk = h // rep
            s = (Q[b, ridx, h, :] @ K[b, :, hk, :].T) * scale          # [R, S]
            if causal:
                s = np.where(cols[None, :] <= ridx[:, None], s, -np.inf)
            m = np.max(s, axis=1, keepdims=True)
            e = np.exp(s - m)
            P = e / np.sum(e, axis=1, keepdims=True)
            if keep is not None:
                P = np.where(keep[b, h][ridx, :], P * keep_scale, 0.0)
            O[b, :, h, :] = P @ V[b, :, hk, :]
    return O


def attention_dropout_loops(Q, K, V, keep, p, causal=False):
    """The same definition as explicit scalar loops (tiny inputs only)."""
    import math
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, S, H, d = Q.shape
    Hkv = K.shape[2]
    rep = H // Hkv
    O = np.zeros((B, S, H, d), dtype=np.float64)
    inv_keep = 1.0 / (1.0 - float(np.float32(p))) if keep is not None else 1.0
    for b in range(B):
        for h in range(H):
            hk = h // rep
            for i in range(S):
                jmax = i + 1 if causal else S
                sc = [sum(Q[b, i, h, t] * K[b, j, hk, t] for t in range(d)) / math.sqrt(d)
                      for j in range(jmax)]
                mx = max(sc)
                ex = [math.exp(v - mx) for v in sc]
                den = sum(ex)
                for j in range(jmax):
                    if keep is not None and not keep[b, h, i, j]:
                        continue
                    wgt = ex[j] / den * inv_keep
                    for t in range(d):
                        O[b, i, h, t] += wgt * V[b, j, hk, t]
    return O


def rmsnorm(x, weight, eps):
    """y = x / sqrt(mean(x^2) + eps) * weight over the last axis."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(weight, dtype=np.float64)


def rope(x, theta):
    """Rotary embedding on [B, S, H, d]: adjacent pairs (2t, 2t+1) of token s are
    rotated by the angle s * theta^(-2t/d)."""
    x = np.asarray(x, dtype=np.float64)
    B, S, H, d = x.shape
    t = np.arange(d // 2, dtype=np.float64)
    ang = np.arange(S, dtype=np.float64)[:, None] * theta ** (-2.0 * t / d)[None, :]   # [S, d/2]
    c = np.cos(ang)[None, :, None, :]
    s = np.sin(ang)[None, :, None, :]
    xe, xo = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = xe * c - xo * s
    out[..., 1::2] = xe * s + xo * c
    return out


def silu(x):
    return x / (1.0 + np.exp(-x))


def block_forward(x, w, cfg, keep, rows=None):
    """Llama-style block (the paper's Fig. 2 block, Sec. 2.1, with RMSNorm, rotary
    embedding, grouped-query attention and a SwiGLU feed-forward, as the workload
    list asks):
        h1 = RMSNorm(x) ; [q|k|v] = h1 Wqkv^T ; q, k = RoPE(q), RoPE(k)
        a  = attention_dropout(q, k, v) ; x2 = x + a Wo^T
        h2 = RMSNorm(x2) ; y = x2 + (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T
    x: [B, S, hidden].  w: dict with 'norm1','norm2' [hidden], 'wqkv' [(H+2Hkv)d, hidden],
    'wo' [hidden, H d], 'wg','wu' [ffn, hidden], 'wd' [hidden, ffn].
    cfg: dict H, Hkv, d, eps, rope_theta, p, causal.
    rows: optional query-token subset; y is then returned only for those tokens
    (keys and values still come from every token)."""
    x = np.asarray(x, dtype=np.float64)
    B, S, hidden = x.shape
    H, Hkv, d = cfg["H"], cfg["Hkv"], cfg["d"]
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    h1 = rmsnorm(x, w["norm1"], cfg["eps"])
    qkv = h1 @ f64(w["wqkv"]).T
    q = qkv[..., : H * d].reshape(B, S, H, d)
    k = qkv[..., H * d: (H + Hkv) * d].reshape(B, S, Hkv, d)
    v = qkv[..., (H + Hkv) * d:].reshape(B, S, Hkv, d)
    q = rope(q, cfg["rope_theta"])
    k = rope(k, cfg["rope_theta"])
    a = attention_dropout(q, k, v, keep, cfg["p"], causal=cfg["causal"], rows=rows)
    xr = x if rows is None else x[:, np.asarray(rows), :]
    x2 = xr + a.reshape(B, a.shape[1], H * d) @ f64(w["wo"]).T
    h2 = rmsnorm(x2, w["norm2"], cfg["eps"])
    g = h2 @ f64(w["wg"]).T
    u = h2 @ f64(w["wu"]).T
    return x2 + (silu(g) * u) @ f64(w["wd"]).T


def fake_quant_e4m3(v, scale):
    """Per-tensor fp8 quantisation of an activation as the fp8 block applies it: the value is
    divided by its dequantisation scale, rounded to the nearest OCP e4m3 code (ties to even,
    saturating at +-448) and multiplied by the scale again."""
    from . import numerics as _num
    return _num.e4m3_decode(_num.e4m3_encode(np.asarray(v, dtype=np.float64) / scale)) * scale


def block_forward_fp8(x, w, w_scale, act_scale, cfg, keep, rows=None, stored_bf16=True):
    """The same block with fp8 (OCP e4m3) GEMMs, the precision the paper measures in (Sec. 1,
    Sec. 6); the paper does not say where values are quantised, so this is a reading: every GEMM
    takes both operands in e4m3 with one scale per tensor and accumulates exactly, everything
    between the GEMMs (normalisation, rotary embedding, attention, residuals) stays unquantised.
        h1 = Q0(RMSNorm(x))            ; [q|k|v] = h1 dq(Wqkv)^T ; RoPE(q, k)
        a  = Q1(attention_dropout(q, k, v)) ; x2 = x + a dq(Wo)^T
        h2 = Q2(RMSNorm(x2))           ; u = Q3(silu(h2 dq(Wg)^T) * (h2 dq(Wu)^T))
        y  = x2 + u dq(Wd)^T
    Qi(v) = fake_quant_e4m3(v, act_scale[i]); dq(W) = decode(codes) * w_scale[name].
    w: 'norm1', 'norm2' as floats, 'wqkv', 'wo', 'wg', 'wu', 'wd' as uint8 e4m3 codes [out, in];
    w_scale: dict name -> float; act_scale: 4 floats (for h1, a, h2, u).  rows as in block_forward.
    stored_bf16: the tensors the block keeps between its GEMMs in bf16 - the QKV projection, q and k
    after the rotary embedding, and the residual stream x2 - are rounded to bf16 here too.  They feed
    the quantisers Q1..Q3, i.e. they decide integer codes, and such a decision is taken on the stored
    value on both sides (a bf16 rounding error of 2^-9 would otherwise flip one code in thirty)."""
    from . import numerics as _num
    x = np.asarray(x, dtype=np.float64)
    B, S, hidden = x.shape
    H, Hkv, d = cfg["H"], cfg["Hkv"], cfg["d"]
    st = (lambda t: _num.bf16_round(t).astype(np.float64)) if stored_bf16 else (lambda t: t)
    dq = lambda name: _num.e4m3_decode(w[name]) * float(w_scale[name])
    h1 = fake_quant_e4m3(rmsnorm(x, w["norm1"], cfg["eps"]), act_scale[0])
    qkv = st(h1 @ dq("wqkv").T)
    q = qkv[..., : H * d].reshape(B, S, H, d)
    k = qkv[..., H * d: (H + Hkv) * d].reshape(B, S, Hkv, d)
    v = qkv[..., (H + Hkv) * d:].reshape(B, S, Hkv, d)
    q = st(rope(q, cfg["rope_theta"]))
    k = st(rope(k, cfg["rope_theta"]))
    a = attention_dropout(q, k, v, keep, cfg["p"], causal=cfg["causal"], rows=rows)
    a = fake_quant_e4m3(a, act_scale[1])
    xr = x if rows is None else x[:, np.asarray(rows), :]
    x2 = st(xr + a.reshape(B, a.shape[1], H * d) @ dq("wo").T)
    h2 = fake_quant_e4m3(rmsnorm(x2, w["norm2"], cfg["eps"]), act_scale[2])
    u = fake_quant_e4m3(silu(h2 @ dq("wg").T) * (h2 @ dq("wu").T), act_scale[3])
    return x2 + u @ dq("wd").T


def keep_from_words(words, S):
    return _philox.unpack_keep(words, S)
