"""fp64 oracle of one transformer layer's training step: forward, hand-derived
backward, and the loss seed.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

What it follows.  The paper defines a training workload as forward graph +
loss + backward graph + optimizer over learnable parameters (Section 2.1,
Fig. "Deep learning training workload"), and a backward graph as the chain of
adjoints, each giving the derivative w.r.t. an operator's inputs from the
derivative w.r.t. its outputs (Section 3.1.1).  The layer's own equations are
not in the paper (its models are stock BERT / GPT-2 layers, Section 5), so the
forward below is the textbook encoder/decoder layer and every adjoint is the
exact derivative of that forward; nothing is blocked, fused or reordered.

Notation: B batch, S sequence, H hidden, nh heads, dh = H/nh, F ffn width,
T = B*S, p dropout probability, alpha = 1/sqrt(dh).  Linear weights are
[out, in] row-major; w_qkv rows are the Q block, the K block, the V block.

Dropout has three sites per layer: 1 = attention probabilities [B,nh,S,S],
2 = attention output [T,H], 3 = ffn output [T,H]; masks come from
oracle.philox.dropout_keep and are scaled by 1/(1-p).
"""
import numpy as np
from scipy.special import erf

from .philox import dropout_keep

PARAM_NAMES = ("w_qkv", "b_qkv", "w_o", "b_o", "ln1_g", "ln1_b",
               "w_1", "b_1", "w_2", "b_2", "ln2_g", "ln2_b")


# ----------------------------------------------------------------- pieces --
def gelu(u, tanh_form=False):
    if tanh_form:
        k = np.sqrt(2.0 / np.pi)
        return 0.5 * u * (1.0 + np.tanh(k * (u + 0.044715 * u ** 3)))
    return 0.5 * u * (1.0 + erf(u / np.sqrt(2.0)))


def gelu_grad(u, tanh_form=False):
    if tanh_form:
        k = np.sqrt(2.0 / np.pi)
        t = np.tanh(k * (u + 0.044715 * u ** 3))
        return 0.5 * (1.0 + t) + 0.5 * u * (1.0 - t * t) * k * (1.0 + 3 * 0.044715 * u * u)
    Phi = 0.5 * (1.0 + erf(u / np.sqrt(2.0)))
    phi = np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)
    return Phi + u * phi


def layernorm(z, gamma, beta, eps):
    """Row-wise LayerNorm over the last axis with the biased variance.
    Returns (out, xhat, rstd)."""
    mu = z.mean(axis=-1, keepdims=True)
    var = ((z - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (z - mu) * rstd
    return xhat * gamma + beta, xhat, rstd


def layernorm_bwd(dout, xhat, rstd, gamma):
    """Adjoint of layernorm.  Returns (dz, dgamma, dbeta)."""
    dxhat = dout * gamma
    m1 = dxhat.mean(axis=-1, keepdims=True)
    m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    dz = rstd * (dxhat - m1 - xhat * m2)
    return dz, (dout * xhat).sum(axis=0), dout.sum(axis=0)


def attention_masked(B, S, seq_lens, causal):
    """Boolean [B,1,S,S]; True where key j may NOT be attended by query i:
    j >= len_b (key padding) or, if causal, j > i."""
    j = np.arange(S)[None, None, None, :]
    i = np.arange(S)[None, None, :, None]
    m = np.zeros((B, 1, S, S), dtype=bool)
    if seq_lens is not None:
        L = np.asarray(seq_lens).reshape(B, 1, 1, 1)
        m = m | (j >= L)
    if causal:
        m = m | (j > i)
    return m


def masked_softmax(s, masked):
    """softmax over the last axis with masked entries at probability exactly 0.
    A row with every key masked is defined as all zeros."""
    s = np.where(masked, -np.inf, s)
    mx = s.max(axis=-1, keepdims=True)
    mx = np.where(np.isfinite(mx), mx, 0.0)
    e = np.exp(s - mx)                      # exp(-inf) = 0 exactly
    den = e.sum(axis=-1, keepdims=True)
    return np.where(den > 0, e / np.where(den > 0, den, 1.0), 0.0)


def softmax_dropout_bwd(prob, keep, scale, dprob_d):
    """Adjoint of prob_d = softmax(s) * keep * scale with respect to s, given dprob_d:
    dprob = dprob_d * keep * scale;  ds = prob * (dprob - sum_j dprob * prob)."""
    dprob = dprob_d * keep * scale
    return prob * (dprob - (dprob * prob).sum(axis=-1, keepdims=True))


def _keep(cfg, site, step, shape):
    n = int(np.prod(shape))
    k = dropout_keep(cfg["seed"], cfg["layer_id"], site, step, n, cfg["dropout_p"])
    return k.reshape(shape).astype(np.float64)


def _split_heads(t, B, S, nh, dh):
    return t.reshape(B, S, nh, dh).transpose(0, 2, 1, 3)       # [B,nh,S,dh]


def _merge_heads(t, B, S, nh, dh):
    return t.transpose(0, 2, 1, 3).reshape(B * S, nh * dh)     # [T,H]


# ---------------------------------------------------- attention core --
def attention_core_forward(cfg, qkv, seq_lens=None, step=0):
    """qkv [T,3H] (column blocks Q | K | V, head h = columns 64h..) -> (c [T,H], cache):
    s = Q K^T / sqrt(dh), mask, softmax, dropout site 1, c = merge_heads(P~ V)."""
    B, S, H, nh = (cfg[k] for k in ("batch", "seq", "hidden", "heads"))
    dh = H // nh
    p = float(cfg["dropout_p"])
    alpha = 1.0 / np.sqrt(dh)
    scale = 1.0 / (1.0 - p)
    qkv = np.asarray(qkv, dtype=np.float64).reshape(B * S, 3 * H)
    q = _split_heads(qkv[:, 0 * H:1 * H], B, S, nh, dh)
    k = _split_heads(qkv[:, 1 * H:2 * H], B, S, nh, dh)
    v = _split_heads(qkv[:, 2 * H:3 * H], B, S, nh, dh)
    s = alpha * np.einsum("bhid,bhjd->bhij", q, k)
    masked = attention_masked(B, S, seq_lens, bool(cfg["causal"]))
    prob = masked_softmax(s, masked)
    keep1 = _keep(cfg, 1, step, (B, nh, S, S))
    prob_d = prob * keep1 * scale
    c = _merge_heads(np.einsum("bhij,bhjd->bhid", prob_d, v), B, S, nh, dh)
    return c, dict(q=q, k=k, v=v, prob=prob, keep1=keep1, prob_d=prob_d)


def attention_core_backward(cfg, A, dc):
    """Adjoint of attention_core_forward: dc [T,H] -> (dqkv [T,3H], ds [B,nh,S,S])."""
    B, S, H, nh = (cfg[k] for k in ("batch", "seq", "hidden", "heads"))
    dh = H // nh
    p = float(cfg["dropout_p"])
    alpha = 1.0 / np.sqrt(dh)
    scale = 1.0 / (1.0 - p)
    dc = _split_heads(np.asarray(dc, dtype=np.float64).reshape(B * S, H), B, S, nh, dh)   # [B,nh,S,dh]
    # c = prob_d V
    dprob_d = np.einsum("bhid,bhjd->bhij", dc, A["v"])
    dv = np.einsum("bhij,bhid->bhjd", A["prob_d"], dc)
    # prob_d = prob * keep1 * scale ; prob = softmax(s)
    ds = softmax_dropout_bwd(A["prob"], A["keep1"], scale, dprob_d)
    # s = alpha q k^T
    dq = alpha * np.einsum("bhij,bhjd->bhid", ds, A["k"])
    dk = alpha * np.einsum("bhij,bhid->bhjd", ds, A["q"])
    dqkv = np.concatenate([_merge_heads(t, B, S, nh, dh) for t in (dq, dk, dv)], axis=1)
    return dqkv, ds


# ---------------------------------------------------------------- forward --
def layer_forward(cfg, params, x, seq_lens=None, step=0):
    """x: [B,S,H] (or [T,H]).  Returns (y [T,H], cache dict)."""
    B, S, H, nh, F = (cfg[k] for k in ("batch", "seq", "hidden", "heads", "ffn"))
    dh = H // nh
    T = B * S
    p = float(cfg["dropout_p"])
    eps = float(cfg["ln_eps"])
    pre_ln = bool(cfg["pre_ln"])
    tanh_form = bool(cfg.get("gelu_tanh", 0))
    alpha = 1.0 / np.sqrt(dh)
    P64 = {k: np.asarray(params[k], dtype=np.float64) for k in PARAM_NAMES}
    x = np.asarray(x, dtype=np.float64).reshape(T, H)
    scale = 1.0 / (1.0 - p)
    C = {"x": x}

    if pre_ln:
        attn_in, C["xhat1"], C["rstd1"] = layernorm(x, P64["ln1_g"], P64["ln1_b"], eps)
    else:
        attn_in = x
    C["attn_in"] = attn_in

    qkv = attn_in @ P64["w_qkv"].T + P64["b_qkv"]
    c, A = attention_core_forward(cfg, qkv, seq_lens, step)
    a1 = c @ P64["w_o"].T + P64["b_o"]
    keep2 = _keep(cfg, 2, step, (T, H))
    z1 = x + a1 * keep2 * scale
    C.update(A)
    C.update(c=c, keep2=keep2, z1=z1)

    if pre_ln:
        ffn_in, C["xhat2"], C["rstd2"] = layernorm(z1, P64["ln2_g"], P64["ln2_b"], eps)
    else:
        ffn_in, C["xhat1"], C["rstd1"] = layernorm(z1, P64["ln1_g"], P64["ln1_b"], eps)
    C["ffn_in"] = ffn_in

    u = ffn_in @ P64["w_1"].T + P64["b_1"]
    g = gelu(u, tanh_form)
    a2 = g @ P64["w_2"].T + P64["b_2"]
    keep3 = _keep(cfg, 3, step, (T, H))
    z2 = (z1 if pre_ln else ffn_in) + a2 * keep3 * scale
    C.update(u=u, g=g, keep3=keep3, z2=z2)

    if pre_ln:
        y = z2
    else:
        y, C["xhat2"], C["rstd2"] = layernorm(z2, P64["ln2_g"], P64["ln2_b"], eps)
    C["params"] = P64
    return y, C


# ------------------------------------------------------------------- loss --
def loss_and_seed(y, G, loss_scale=1.0):
    """loss = sum(y * G); the gradient handed to backward is loss_scale * G."""
    y = np.asarray(y, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64).reshape(y.shape)
    return float((y * G).sum()), loss_scale * G


# --------------------------------------------------------------- backward --
def layer_backward(cfg, cache, dy):
    """Exact adjoint of layer_forward.  Returns (dx [T,H], grads dict)."""
    B, S, H, nh, F = (cfg[k] for k in ("batch", "seq", "hidden", "heads", "ffn"))
    dh = H // nh
    T = B * S
    p = float(cfg["dropout_p"])
    pre_ln = bool(cfg["pre_ln"])
    tanh_form = bool(cfg.get("gelu_tanh", 0))
    alpha = 1.0 / np.sqrt(dh)
    scale = 1.0 / (1.0 - p)
    C = cache
    W = C["params"]
    dy = np.asarray(dy, dtype=np.float64).reshape(T, H)
    gr = {}

    # ---- output side: y = LN2(z2) (post) or y = z2 (pre)
    if pre_ln:
        dz2 = dy
    else:
        dz2, gr["ln2_g"], gr["ln2_b"] = layernorm_bwd(dy, C["xhat2"], C["rstd2"], W["ln2_g"])

    # ---- z2 = res + a2 * keep3 * scale
    da2 = dz2 * C["keep3"] * scale
    dres = dz2
    # a2 = g W2^T + b2
    gr["w_2"] = da2.T @ C["g"]
    gr["b_2"] = da2.sum(axis=0)
    dg = da2 @ W["w_2"]
    du = dg * gelu_grad(C["u"], tanh_form)
    # u = ffn_in W1^T + b1
    gr["w_1"] = du.T @ C["ffn_in"]
    gr["b_1"] = du.sum(axis=0)
    dffn_in = du @ W["w_1"]

    if pre_ln:
        # ffn_in = LN2(z1); res = z1
        d_ln, gr["ln2_g"], gr["ln2_b"] = layernorm_bwd(dffn_in, C["xhat2"], C["rstd2"], W["ln2_g"])
        dz1 = dres + d_ln
    else:
        # ffn_in = h1 = LN1(z1); res = h1
        dz1, gr["ln1_g"], gr["ln1_b"] = layernorm_bwd(dres + dffn_in, C["xhat1"], C["rstd1"], W["ln1_g"])

    # ---- z1 = x + a1 * keep2 * scale
    da1 = dz1 * C["keep2"] * scale
    dx = dz1.copy()
    gr["w_o"] = da1.T @ C["c"]
    gr["b_o"] = da1.sum(axis=0)
    dqkv, ds = attention_core_backward(cfg, C, da1 @ W["w_o"])
    gr["w_qkv"] = dqkv.T @ C["attn_in"]
    gr["b_qkv"] = dqkv.sum(axis=0)
    dattn_in = dqkv @ W["w_qkv"]

    if pre_ln:
        d_ln, gr["ln1_g"], gr["ln1_b"] = layernorm_bwd(dattn_in, C["xhat1"], C["rstd1"], W["ln1_g"])
        dx = dx + d_ln
    else:
        dx = dx + dattn_in
    C["ds"] = ds          # kept for the masking tests
    C["dqkv"] = dqkv
    return dx, gr
