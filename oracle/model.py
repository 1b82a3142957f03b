"""fp64 oracle of the full encoder model of the largest workload: embedding,
a stack of layers, and the masked-language-model head with a tied decoder and
a summed softmax cross-entropy; forward, hand-derived backward, Adam.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Same basis as oracle/layer.py: the paper's training workload is forward graph
+ loss + backward graph + optimizer (Section 2.1) and the backward graph is the
chain of adjoints (Section 3.1.1); the model's equations are the textbook BERT
ones (the paper uses stock models, Section 5):

  e   = LN(Word[ids] + Pos[position]);  x0 = dropout_site4(e)
  x_l = layer_l(x_{l-1}),  l = 1..L
  r   = rows of x_L at the selected flat positions
  t   = LN(gelu(r Wt^T + bt));  logits = t Word^T + bv     (decoder tied to Word)
  loss = sum_i ( logsumexp(logits_i) - logits_i[label_i] )

No token-type embedding, no pooler.  Dropout site 4 uses the embedding's own
layer id.
"""
import numpy as np

from .layer import PARAM_NAMES, gelu, gelu_grad, layer_backward, layer_forward, layernorm, layernorm_bwd
from .philox import dropout_keep
from .adam import adam_step

EMBED_PARAMS = ("word", "pos", "emb_ln_g", "emb_ln_b")
HEAD_PARAMS = ("head_w", "head_b", "head_ln_g", "head_ln_b", "dec_b")


def layer_cfg(cfg, l):
    c = dict(cfg)
    c["layer_id"] = cfg["layer_id_base"] + l
    return c


def embed_forward(cfg, P, ids, step):
    B, S, H = cfg["batch"], cfg["seq"], cfg["hidden"]
    T = B * S
    ids = np.asarray(ids).reshape(T)
    pos_idx = np.tile(np.arange(S), B)
    z0 = P["word"][ids] + P["pos"][pos_idx]
    e, xhat, rstd = layernorm(z0, P["emb_ln_g"], P["emb_ln_b"], cfg["ln_eps"])
    p = float(cfg["dropout_p"])
    keep = dropout_keep(cfg["seed"], cfg["embed_layer_id"], 4, step, T * H, p).reshape(T, H).astype(np.float64)
    x0 = e * keep / (1.0 - p)
    return x0, dict(ids=ids, pos_idx=pos_idx, xhat=xhat, rstd=rstd, keep=keep)


def embed_backward(cfg, P, C, dx0):
    p = float(cfg["dropout_p"])
    de = dx0 * C["keep"] / (1.0 - p)
    dz0, dg, db = layernorm_bwd(de, C["xhat"], C["rstd"], P["emb_ln_g"])
    dword = np.zeros_like(P["word"])
    np.add.at(dword, C["ids"], dz0)
    dpos = np.zeros_like(P["pos"])
    np.add.at(dpos, C["pos_idx"], dz0)
    return dict(word=dword, pos=dpos, emb_ln_g=dg, emb_ln_b=db)


def head_forward(cfg, P, xL, sel, labels):
    """sel: flat positions (ascending), labels: vocabulary ids.  Returns loss, cache."""
    V = cfg["vocab"]
    r = xL[sel]
    t1 = r @ P["head_w"].T + P["head_b"]
    t2 = gelu(t1)
    t, xhat, rstd = layernorm(t2, P["head_ln_g"], P["head_ln_b"], cfg["ln_eps"])
    logits = t @ P["word"][:V].T + P["dec_b"]
    mx = logits.max(axis=-1, keepdims=True)
    lse = mx[:, 0] + np.log(np.exp(logits - mx).sum(axis=-1))
    loss = float((lse - logits[np.arange(len(sel)), labels]).sum())
    prob = np.exp(logits - lse[:, None])
    return loss, dict(r=r, t1=t1, t2=t2, t=t, xhat=xhat, rstd=rstd, prob=prob, sel=sel, labels=labels)


def head_backward(cfg, P, C, T, loss_scale):
    V = cfg["vocab"]
    n = len(C["sel"])
    dlogits = C["prob"].copy()
    dlogits[np.arange(n), C["labels"]] -= 1.0
    dlogits *= loss_scale
    gr = {}
    gr["dec_b"] = dlogits.sum(axis=0)
    dword = np.zeros_like(P["word"])
    dword[:V] = dlogits.T @ C["t"]
    dt = dlogits @ P["word"][:V]
    dt2, gr["head_ln_g"], gr["head_ln_b"] = layernorm_bwd(dt, C["xhat"], C["rstd"], P["head_ln_g"])
    dt1 = dt2 * gelu_grad(C["t1"])
    gr["head_w"] = dt1.T @ C["r"]
    gr["head_b"] = dt1.sum(axis=0)
    dr = dt1 @ P["head_w"]
    dxL = np.zeros((T, cfg["hidden"]))
    dxL[C["sel"]] = dr
    C["dlogits"] = dlogits
    return dxL, gr, dword


def model_forward_backward(cfg, P, layers, ids, seq_lens, sel, labels, step, loss_scale=1.0):
    """P: dict of embedding + head params (fp64); layers: list of per-layer param dicts.
    Returns dict(loss, grads (embedding/head dict, tied `word` summed), layer_grads list, xL)."""
    T = cfg["batch"] * cfg["seq"]
    x, EC = embed_forward(cfg, P, ids, step)
    caches = []
    for l, lp in enumerate(layers):
        x, C = layer_forward(layer_cfg(cfg, l), lp, x, seq_lens, step)
        caches.append(C)
    loss, HC = head_forward(cfg, P, x, sel, labels)
    dx, gr, dword_dec = head_backward(cfg, P, HC, T, loss_scale)
    layer_grads = [None] * len(layers)
    for l in reversed(range(len(layers))):
        dx, layer_grads[l] = layer_backward(layer_cfg(cfg, l), caches[l], dx)
        caches[l] = None
    eg = embed_backward(cfg, P, EC, dx)
    gr.update(eg)
    gr["word"] = eg["word"] + dword_dec
    return dict(loss=loss, grads=gr, layer_grads=layer_grads, xL=x, dlogits=HC["dlogits"])


def model_train_step(cfg, P, layers, mP, vP, mL, vL, ids, seq_lens, sel, labels, t, hyper):
    ls = float(hyper.get("loss_scale", 1.0))
    out = model_forward_backward(cfg, P, layers, ids, seq_lens, sel, labels, t, ls)
    a = (hyper["lr"], hyper["beta1"], hyper["beta2"], hyper["eps"], hyper.get("weight_decay", 0.0), 1.0 / ls)
    nP, nmP, nvP = {}, {}, {}
    for k in EMBED_PARAMS + HEAD_PARAMS:
        nP[k], nmP[k], nvP[k] = adam_step(P[k], out["grads"][k].reshape(P[k].shape), mP[k], vP[k], t, *a)
    nL, nmL, nvL = [], [], []
    for l, lp in enumerate(layers):
        p2, m2, v2 = {}, {}, {}
        for k in PARAM_NAMES:
            p2[k], m2[k], v2[k] = adam_step(lp[k], out["layer_grads"][l][k].reshape(np.shape(lp[k])), mL[l][k], vL[l][k],
                                            t, *a)
        nL.append(p2); nmL.append(m2); nvL.append(v2)
    out.update(P=nP, mP=nmP, vP=nvP, layers=nL, mL=nmL, vL=nvL)
    return out
