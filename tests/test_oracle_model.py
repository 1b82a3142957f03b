"""Pins for the full-model oracle (embedding, stack, MLM head, cross-entropy); CPU only."""
import numpy as np
import torch

from oracle import model as M
from oracle.layer import PARAM_NAMES
from workloads.synthetic import MODEL_CONFIGS, make_model_inputs


def small_cfg(**kw):
    cfg = dict(batch=2, seq=5, hidden=8, heads=1, ffn=12, pre_ln=0, causal=0, gelu_tanh=0, dropout_p=0.2,
               ln_eps=1e-5, seed=77, layer_id=0, layer_id_base=3, embed_layer_id=9, precision=0, layers=2,
               vocab=11, max_pos=7, loss_scale=1.0)
    cfg.update(kw)
    return cfg


def rand_model(cfg, seed):
    rng = np.random.default_rng(seed)
    H, V, F = cfg["hidden"], cfg["vocab"], cfg["ffn"]
    P = dict(word=0.5 * rng.standard_normal((V, H)), pos=0.5 * rng.standard_normal((cfg["max_pos"], H)),
             emb_ln_g=1 + 0.2 * rng.standard_normal(H), emb_ln_b=0.1 * rng.standard_normal(H),
             head_w=0.5 * rng.standard_normal((H, H)), head_b=0.1 * rng.standard_normal(H),
             head_ln_g=1 + 0.2 * rng.standard_normal(H), head_ln_b=0.1 * rng.standard_normal(H),
             dec_b=0.1 * rng.standard_normal(V))
    shapes = {"w_qkv": (3 * H, H), "b_qkv": (3 * H,), "w_o": (H, H), "b_o": (H,), "ln1_g": (H,), "ln1_b": (H,),
              "w_1": (F, H), "b_1": (F,), "w_2": (H, F), "b_2": (H,), "ln2_g": (H,), "ln2_b": (H,)}
    layers = []
    for _ in range(cfg["layers"]):
        layers.append({k: (1 + 0.2 * rng.standard_normal(s)) if k.endswith("_g") else 0.4 * rng.standard_normal(s)
                       for k, s in shapes.items()})
    T = cfg["batch"] * cfg["seq"]
    ids = rng.integers(0, V, size=T)
    ids[3] = ids[0]                      # duplicate ids must accumulate
    sel = np.array([1, 4, 7])
    labels = rng.integers(0, V, size=3)
    lens = np.array([5, 3])
    return P, layers, ids, lens, sel, labels


def test_model_gradients_by_finite_differences():
    cfg = small_cfg()
    P, layers, ids, lens, sel, labels = rand_model(cfg, 1)
    out = M.model_forward_backward(cfg, P, layers, ids, lens, sel, labels, step=3, loss_scale=1.0)
    rng = np.random.default_rng(5)

    def loss_with(name, delta, layer=None):
        P2 = dict(P)
        L2 = [dict(l) for l in layers]
        if layer is None:
            P2[name] = P[name] + delta
        else:
            L2[layer][name] = layers[layer][name] + delta
        return M.model_forward_backward(cfg, P2, L2, ids, lens, sel, labels, step=3)["loss"]

    eps = 1e-5
    for name in M.EMBED_PARAMS + M.HEAD_PARAMS:
        d = rng.standard_normal(P[name].shape)
        num = (loss_with(name, eps * d) - loss_with(name, -eps * d)) / (2 * eps)
        ana = float((out["grads"][name] * d).sum())
        assert abs(num - ana) <= 2e-6 * max(1.0, abs(ana)), (name, num, ana)
    for l in range(cfg["layers"]):
        for name in ("w_qkv", "b_1", "ln2_g", "w_2"):
            d = rng.standard_normal(layers[l][name].shape)
            num = (loss_with(name, eps * d, l) - loss_with(name, -eps * d, l)) / (2 * eps)
            ana = float((out["layer_grads"][l][name].reshape(d.shape) * d).sum())
            assert abs(num - ana) <= 2e-6 * max(1.0, abs(ana)), (l, name, num, ana)


def test_head_and_embedding_match_torch_autograd():
    cfg = small_cfg(layers=0, dropout_p=0.0)
    P, _, ids, lens, sel, labels = rand_model(cfg, 2)
    out = M.model_forward_backward(cfg, P, [], ids, lens, sel, labels, step=0, loss_scale=8.0)
    tp = {k: torch.tensor(v, requires_grad=True) for k, v in P.items()}
    F_ = torch.nn.functional
    H = cfg["hidden"]
    pos_idx = torch.arange(cfg["seq"]).repeat(cfg["batch"])
    e = F_.layer_norm(F_.embedding(torch.from_numpy(ids), tp["word"]) + tp["pos"][pos_idx], (H,), tp["emb_ln_g"],
                      tp["emb_ln_b"], cfg["ln_eps"])
    r = e[torch.from_numpy(sel)]
    t = F_.layer_norm(F_.gelu(F_.linear(r, tp["head_w"], tp["head_b"])), (H,), tp["head_ln_g"], tp["head_ln_b"],
                      cfg["ln_eps"])
    logits = F_.linear(t, tp["word"], tp["dec_b"])
    loss = F_.cross_entropy(logits, torch.from_numpy(labels), reduction="sum")
    (8.0 * loss).backward()
    assert np.isclose(out["loss"], loss.item(), rtol=1e-12)
    for k in P:
        assert np.allclose(out["grads"][k], tp[k].grad.numpy(), rtol=1e-9, atol=1e-11), k


def test_cross_entropy_invariants():
    cfg = small_cfg(layers=0, dropout_p=0.0)
    P, _, ids, lens, sel, labels = rand_model(cfg, 3)
    out = M.model_forward_backward(cfg, P, [], ids, lens, sel, labels, step=0)
    assert np.abs(out["dlogits"].sum(axis=1)).max() < 1e-12            # softmax - onehot sums to zero
    # uniform logits: tied table and decoder bias zero => loss = n_sel * ln(V)
    P0 = dict(P, word=np.zeros_like(P["word"]), dec_b=np.zeros_like(P["dec_b"]))
    out0 = M.model_forward_backward(cfg, P0, [], ids, lens, sel, labels, step=0)
    assert np.isclose(out0["loss"], len(sel) * np.log(cfg["vocab"]), rtol=1e-12)
    # unselected positions receive no gradient from the head: dWord from the embedding side only touches used ids
    used = np.zeros(cfg["vocab"], dtype=bool)
    used[ids] = True
    emb_only = out["grads"]["word"] - (out["dlogits"].T @ M.head_forward(cfg, P, M.embed_forward(cfg, P, ids, 0)[0],
                                                                          sel, labels)[1]["t"])
    assert np.abs(emb_only[~used]).max() < 1e-12
    # duplicate ids accumulate: position table gradient sums over the batch
    assert np.abs(out["grads"]["pos"][cfg["seq"]:]).max() == 0.0


def test_synthetic_model_inputs_shape_and_selection():
    cfg = MODEL_CONFIGS["tiny_model"]
    inp = make_model_inputs(cfg, seed=0)
    B, S = cfg["batch"], cfg["seq"]
    assert inp["ids"].shape == (B, S) and inp["sel"].ndim == 1 and len(inp["labels"]) == len(inp["sel"])
    assert (np.diff(inp["sel"]) > 0).all()
    b, s = np.divmod(inp["sel"], S)
    assert (s < inp["seq_lens"][b]).all()                    # only valid tokens are selected
    assert inp["P"]["word"].shape[0] % 32 == 0 and (inp["P"]["word"][cfg["vocab"]:] == 0).all()
    assert make_model_inputs(cfg, seed=0)["ids"].tobytes() == inp["ids"].tobytes()
