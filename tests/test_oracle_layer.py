"""Pins for the fp64 layer oracle (CPU only): finite differences, invariants,
closed forms and library second opinions.  None of them re-types the oracle's
own formulas: torch autograd differentiates an independently written forward,
torch.nn.TransformerEncoderLayer is a library layer, finite differences use
only the oracle's forward."""
import numpy as np
import pytest
import torch

from oracle import layer as L
from oracle.philox import dropout_keep
from workloads.synthetic import CONFIGS, PARAM_NAMES, make_layer_inputs, param_shapes


def micro_cfg(**kw):
    cfg = dict(batch=2, seq=6, hidden=16, heads=2, ffn=24, pre_ln=0, causal=0, gelu_tanh=0,
               dropout_p=0.0, ln_eps=1e-5, seed=1234, layer_id=3, precision=0,
               len_lo=None, len_hi=None, loss_scale=1.0)
    cfg.update(kw)
    return cfg


def rand_problem(cfg, seed=0, wscale=0.3):
    rng = np.random.default_rng(seed)
    B, S, H = cfg["batch"], cfg["seq"], cfg["hidden"]
    params = {}
    for k, shp in param_shapes(cfg).items():
        if k.endswith("_g"):
            params[k] = 1.0 + 0.2 * rng.standard_normal(shp)
        else:
            params[k] = wscale * rng.standard_normal(shp)
    x = rng.standard_normal((B * S, H))
    G = rng.standard_normal((B * S, H))
    return params, x, G


def loss_of(cfg, params, x, G, lens, step):
    y, _ = L.layer_forward(cfg, params, x, lens, step)
    return float((y * G).sum())


VARIANTS = [
    dict(),
    dict(pre_ln=1),
    dict(causal=1),
    dict(pre_ln=1, causal=1, gelu_tanh=1),
    dict(dropout_p=0.25),
    dict(dropout_p=0.25, pre_ln=1, causal=1),
    dict(gelu_tanh=1),
]


@pytest.mark.parametrize("var", VARIANTS)
@pytest.mark.parametrize("with_lens", [False, True])
def test_finite_differences_every_input(var, with_lens):
    cfg = micro_cfg(**var)
    params, x, G = rand_problem(cfg, seed=3)
    lens = np.array([4, 6], dtype=np.int32) if with_lens else None
    step = 5
    y, cache = L.layer_forward(cfg, params, x, lens, step)
    dx, grads = L.layer_backward(cfg, cache, G)
    rng = np.random.default_rng(8)
    eps = 1e-5

    def fd_dir(name, direction):
        def at(h):
            p2 = dict(params)
            x2 = x
            if name == "x":
                x2 = x + h * direction
            else:
                p2[name] = params[name] + h * direction
            return loss_of(cfg, p2, x2, G, lens, step)
        return (at(eps) - at(-eps)) / (2 * eps)

    for name in ("x",) + PARAM_NAMES:
        an = dx if name == "x" else grads[name].reshape(np.shape(params[name]))
        base = x if name == "x" else params[name]
        # random direction
        d = rng.standard_normal(base.shape)
        num = fd_dir(name, d)
        ana = float((an * d).sum())
        assert abs(num - ana) <= 1e-6 * max(1.0, abs(ana)), (name, num, ana)
        # a few single coordinates
        flat = np.arange(base.size)
        for idx in rng.choice(flat, size=min(3, base.size), replace=False):
            e = np.zeros(base.size)
            e[idx] = 1.0
            num = fd_dir(name, e.reshape(base.shape))
            ana = float(an.reshape(-1)[idx])
            assert abs(num - ana) <= 1e-6 * max(1.0, abs(ana)), (name, idx, num, ana)


def torch_forward(cfg, tp, x, lens, keeps):
    """Independently typed forward in torch fp64 (library ops + autograd)."""
    B, S, H, nh = cfg["batch"], cfg["seq"], cfg["hidden"], cfg["heads"]
    dh = H // nh
    p = cfg["dropout_p"]
    F_ = torch.nn.functional
    act = (lambda t: F_.gelu(t, approximate="tanh")) if cfg["gelu_tanh"] else F_.gelu
    xx = x.view(B, S, H)
    a_in = F_.layer_norm(xx, (H,), tp["ln1_g"], tp["ln1_b"], cfg["ln_eps"]) if cfg["pre_ln"] else xx
    qkv = F_.linear(a_in, tp["w_qkv"], tp["b_qkv"])
    q, k, v = [t.view(B, S, nh, dh).permute(0, 2, 1, 3) for t in qkv.split(H, dim=-1)]
    s = torch.matmul(q, k.transpose(-1, -2)) / dh ** 0.5
    bias = torch.zeros(B, 1, S, S, dtype=torch.float64)
    if lens is not None:
        for b in range(B):
            bias[b, :, :, int(lens[b]):] = float("-inf")
    if cfg["causal"]:
        bias = bias + torch.full((S, S), float("-inf"), dtype=torch.float64).triu(1)
    pr = torch.softmax(s + bias, dim=-1)
    pr = pr * keeps[0].view(B, nh, S, S) / (1 - p)
    c = torch.matmul(pr, v).permute(0, 2, 1, 3).reshape(B, S, H)
    a1 = F_.linear(c, tp["w_o"], tp["b_o"]) * keeps[1].view(B, S, H) / (1 - p)
    z1 = xx + a1
    if cfg["pre_ln"]:
        f_in = F_.layer_norm(z1, (H,), tp["ln2_g"], tp["ln2_b"], cfg["ln_eps"])
        res = z1
    else:
        f_in = F_.layer_norm(z1, (H,), tp["ln1_g"], tp["ln1_b"], cfg["ln_eps"])
        res = f_in
    a2 = F_.linear(act(F_.linear(f_in, tp["w_1"], tp["b_1"])), tp["w_2"], tp["b_2"])
    z2 = res + a2 * keeps[2].view(B, S, H) / (1 - p)
    if cfg["pre_ln"]:
        return z2.reshape(B * S, H)
    return F_.layer_norm(z2, (H,), tp["ln2_g"], tp["ln2_b"], cfg["ln_eps"]).reshape(B * S, H)


@pytest.mark.parametrize("var", VARIANTS)
def test_matches_torch_autograd_second_opinion(var):
    cfg = micro_cfg(batch=3, seq=10, hidden=32, heads=4, ffn=48, **var)
    params, x, G = rand_problem(cfg, seed=5)
    lens = np.array([10, 3, 7], dtype=np.int32)
    step = 2
    B, S, H, nh = cfg["batch"], cfg["seq"], cfg["hidden"], cfg["heads"]
    y, cache = L.layer_forward(cfg, params, x, lens, step)
    dx, grads = L.layer_backward(cfg, cache, G)
    keeps = [torch.from_numpy(dropout_keep(cfg["seed"], cfg["layer_id"], site, step, n, cfg["dropout_p"])
                              .astype(np.float64))
             for site, n in ((1, B * nh * S * S), (2, B * S * H), (3, B * S * H))]
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in params.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ty = torch_forward(cfg, tp, tx, lens, keeps)
    (ty * torch.from_numpy(G)).sum().backward()
    assert np.allclose(y, ty.detach().numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-9, atol=1e-11)
    for k in PARAM_NAMES:
        assert np.allclose(grads[k].reshape(params[k].shape), tp[k].grad.numpy(), rtol=1e-9, atol=1e-11), k


@pytest.mark.parametrize("norm_first", [False, True])
def test_matches_torch_library_encoder_layer(norm_first):
    cfg = micro_cfg(batch=2, seq=9, hidden=32, heads=4, ffn=40, pre_ln=int(norm_first))
    params, x, G = rand_problem(cfg, seed=9)
    lens = np.array([9, 5], dtype=np.int32)
    B, S, H = cfg["batch"], cfg["seq"], cfg["hidden"]
    lay = torch.nn.TransformerEncoderLayer(H, cfg["heads"], cfg["ffn"], dropout=0.0, activation="gelu",
                                           layer_norm_eps=cfg["ln_eps"], batch_first=True,
                                           norm_first=norm_first, dtype=torch.float64)
    sd = {"self_attn.in_proj_weight": "w_qkv", "self_attn.in_proj_bias": "b_qkv",
          "self_attn.out_proj.weight": "w_o", "self_attn.out_proj.bias": "b_o",
          "linear1.weight": "w_1", "linear1.bias": "b_1", "linear2.weight": "w_2", "linear2.bias": "b_2",
          "norm1.weight": "ln1_g", "norm1.bias": "ln1_b", "norm2.weight": "ln2_g", "norm2.bias": "ln2_b"}
    with torch.no_grad():
        for tname, oname in sd.items():
            dict(lay.named_parameters())[tname].copy_(torch.from_numpy(params[oname]))
    lay.train()
    pad = torch.zeros(B, S, dtype=torch.bool)
    for b in range(B):
        pad[b, int(lens[b]):] = True
    tx = torch.tensor(x.reshape(B, S, H), requires_grad=True)
    ty = lay(tx, src_key_padding_mask=pad)
    (ty.reshape(B * S, H) * torch.from_numpy(G)).sum().backward()
    y, cache = L.layer_forward(cfg, params, x, lens, 0)
    dx, grads = L.layer_backward(cfg, cache, G)
    assert np.allclose(y, ty.detach().numpy().reshape(B * S, H), rtol=1e-9, atol=1e-11)
    assert np.allclose(dx, tx.grad.numpy().reshape(B * S, H), rtol=1e-8, atol=1e-10)
    named = dict(lay.named_parameters())
    for tname, oname in sd.items():
        assert np.allclose(grads[oname].reshape(params[oname].shape), named[tname].grad.numpy(),
                           rtol=1e-8, atol=1e-10), oname


def test_pieces_against_library_routines():
    rng = np.random.default_rng(1)
    u = rng.standard_normal((7, 33)) * 3
    F_ = torch.nn.functional
    tu = torch.from_numpy(u).requires_grad_()
    assert np.allclose(L.gelu(u), F_.gelu(tu).detach().numpy(), rtol=1e-12, atol=1e-14)
    F_.gelu(tu).sum().backward()
    assert np.allclose(L.gelu_grad(u), tu.grad.numpy(), rtol=1e-11, atol=1e-13)
    tu2 = torch.from_numpy(u).requires_grad_()
    F_.gelu(tu2, approximate="tanh").sum().backward()
    assert np.allclose(L.gelu(u, True), F_.gelu(tu2, approximate="tanh").detach().numpy(), rtol=1e-12)
    assert np.allclose(L.gelu_grad(u, True), tu2.grad.numpy(), rtol=1e-11, atol=1e-13)
    g, b = rng.standard_normal(33), rng.standard_normal(33)
    out, xhat, rstd = L.layernorm(u, g, b, 1e-5)
    ref = F_.layer_norm(torch.from_numpy(u), (33,), torch.from_numpy(g), torch.from_numpy(b), 1e-5)
    assert np.allclose(out, ref.numpy(), rtol=1e-12, atol=1e-13)
    s = rng.standard_normal((2, 3, 5, 5))
    msk = np.zeros((2, 1, 5, 5), dtype=bool)
    pr = L.masked_softmax(s, msk)
    assert np.allclose(pr, torch.softmax(torch.from_numpy(s), -1).numpy(), rtol=1e-12)


@pytest.mark.parametrize("causal,with_lens", [(0, False), (1, False), (0, True), (1, True)])
def test_attention_core_against_library_attention(causal, with_lens):
    """attention_core_forward / _backward against torch's scaled_dot_product_attention (library routine, its own
    autograd) without dropout, and with dropout against autograd through an independently typed forward that takes
    the same keep mask."""
    B, S, nh, dh = 2, 12, 2, 64
    H = nh * dh
    cfg = micro_cfg(batch=B, seq=S, hidden=H, heads=nh, ffn=4 * H, causal=causal, dropout_p=0.0)
    rng = np.random.default_rng(5 + causal)
    qkv = rng.standard_normal((B * S, 3 * H))
    dc = rng.standard_normal((B * S, H))
    lens = np.array([S, 7], dtype=np.int32) if with_lens else None
    c, A = L.attention_core_forward(cfg, qkv, lens, step=3)
    dqkv, _ = L.attention_core_backward(cfg, A, dc)
    t = torch.tensor(qkv, requires_grad=True)
    q, k, v = [t[:, i * H:(i + 1) * H].reshape(B, S, nh, dh).permute(0, 2, 1, 3) for i in range(3)]
    allowed = torch.ones(B, 1, S, S, dtype=torch.bool)
    if with_lens:
        allowed = allowed & (torch.arange(S)[None, None, None, :] < torch.from_numpy(lens.astype(np.int64))[:, None, None, None])
    if causal:
        allowed = allowed & torch.ones(S, S, dtype=torch.bool).tril()
    o = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=allowed)
    tc = o.permute(0, 2, 1, 3).reshape(B * S, H)
    (tc * torch.from_numpy(dc)).sum().backward()
    assert np.allclose(c, tc.detach().numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dqkv, t.grad.numpy(), rtol=1e-9, atol=1e-11)
    # dropout at site 1: same keep mask fed to an independent forward
    cfg_d = dict(cfg, dropout_p=0.25)
    c2, A2 = L.attention_core_forward(cfg_d, qkv, lens, step=3)
    dqkv2, _ = L.attention_core_backward(cfg_d, A2, dc)
    keep = torch.from_numpy(dropout_keep(cfg_d["seed"], cfg_d["layer_id"], 1, 3, B * nh * S * S, 0.25)
                            .reshape(B, nh, S, S).astype(np.float64))
    t2 = torch.tensor(qkv, requires_grad=True)
    q, k, v = [t2[:, i * H:(i + 1) * H].reshape(B, S, nh, dh).permute(0, 2, 1, 3) for i in range(3)]
    sc = torch.matmul(q, k.transpose(-1, -2)) / dh ** 0.5
    pr = torch.softmax(sc.masked_fill(~allowed, float("-inf")), dim=-1)
    tc2 = torch.matmul(pr * keep / 0.75, v).permute(0, 2, 1, 3).reshape(B * S, H)
    (tc2 * torch.from_numpy(dc)).sum().backward()
    assert np.allclose(c2, tc2.detach().numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dqkv2, t2.grad.numpy(), rtol=1e-9, atol=1e-11)


def test_softmax_invariants_and_masking():
    cfg = micro_cfg(batch=3, seq=12, hidden=16, heads=2, causal=0)
    params, x, G = rand_problem(cfg, seed=2)
    lens = np.array([12, 1, 7], dtype=np.int32)
    y, C = L.layer_forward(cfg, params, x, lens, 0)
    pr = C["prob"]
    assert np.abs(pr.sum(-1) - 1.0).max() < 1e-12
    for b in range(3):
        assert (pr[b, :, :, lens[b]:] == 0.0).all()
        assert (pr[b, :, :, :lens[b]] > 0.0).all()
    # shift invariance
    s = np.random.default_rng(0).standard_normal((2, 2, 5, 5))
    m = L.attention_masked(2, 5, np.array([5, 3]), True)
    assert np.allclose(L.masked_softmax(s, m), L.masked_softmax(s + 123.0, m), rtol=1e-12, atol=1e-15)
    # causal structure
    pc = L.masked_softmax(s, m)
    assert (np.triu(pc[0, 0], 1) == 0).all() and (pc[1, :, :, 3:] == 0).all()
    # a row with no admissible key is all zeros by definition (length 0)
    m0 = L.attention_masked(1, 4, np.array([0]), False)
    assert (L.masked_softmax(np.zeros((1, 1, 4, 4)), m0) == 0).all()
    # backward: ds is exactly zero at masked positions; padded keys get no attention gradient
    dx, gr = L.layer_backward(cfg, C, G)
    H = cfg["hidden"]
    for b in range(3):
        assert (C["ds"][b, :, :, lens[b]:] == 0.0).all()
        rows = slice(b * 12 + int(lens[b]), (b + 1) * 12)
        assert (C["dqkv"][rows, H:3 * H] == 0.0).all()      # dK and dV rows of padded keys


def test_causal_future_independence():
    cfg = micro_cfg(batch=1, seq=8, causal=1, pre_ln=1)
    params, x, G = rand_problem(cfg, seed=4)
    y0, _ = L.layer_forward(cfg, params, x, None, 0)
    x2 = x.copy()
    x2[5:] += np.random.default_rng(1).standard_normal((3, cfg["hidden"]))
    y1, _ = L.layer_forward(cfg, params, x2, None, 0)
    assert np.array_equal(y0[:5], y1[:5])
    assert not np.allclose(y0[5:], y1[5:])


def test_layernorm_invariants_on_tiny_config():
    cfg = CONFIGS["tiny"]
    inp = make_layer_inputs(cfg, seed=0)
    y, C = L.layer_forward(cfg, inp["params"], inp["x"], inp["seq_lens"], 0)
    # gamma=1, beta=0: every output row has mean 0 and variance var/(var+eps)
    assert np.abs(y.mean(-1)).max() < 1e-12
    var_z = C["z2"].var(-1)
    assert np.allclose(y.var(-1), var_z / (var_z + cfg["ln_eps"]), rtol=1e-12)
    dx, gr = L.layer_backward(cfg, C, inp["G"].reshape(y.shape))
    # LN-backward invariants on a direct call
    rng = np.random.default_rng(0)
    z = rng.standard_normal((9, 40)) * 2 + 1
    gmm = rng.standard_normal(40)
    out, xhat, rstd = L.layernorm(z, gmm, rng.standard_normal(40), 1e-14)   # exact only as eps -> 0
    dz, dg, db = L.layernorm_bwd(rng.standard_normal((9, 40)), xhat, rstd, gmm)
    assert np.abs(dz.sum(-1)).max() < 1e-12
    assert np.abs((dz * xhat).sum(-1)).max() < 1e-11


def test_zero_projection_closed_form():
    # W_o = 0 and W_2 = 0 (biases 0): the post-LN layer is LN2(LN1(x)); the pre-LN layer is the identity.
    for pre in (0, 1):
        cfg = micro_cfg(pre_ln=pre, dropout_p=0.3)
        params, x, G = rand_problem(cfg, seed=6)
        for k in ("w_o", "b_o", "w_2", "b_2"):
            params[k] = np.zeros_like(params[k])
        y, _ = L.layer_forward(cfg, params, x, None, 1)
        if pre:
            assert np.array_equal(y, x)
        else:
            def ln(z, g, b):
                mu = z.mean(-1, keepdims=True)
                return (z - mu) / np.sqrt(z.var(-1, keepdims=True) + cfg["ln_eps"]) * g + b
            ref = ln(ln(x, params["ln1_g"], params["ln1_b"]), params["ln2_g"], params["ln2_b"])
            assert np.allclose(y, ref, rtol=1e-12, atol=1e-13)


def test_dropout_sites_are_wired():
    # p>0 changes the output, and the mask of each site is the one the generator defines
    cfg = micro_cfg(dropout_p=0.5)
    params, x, G = rand_problem(cfg, seed=7)
    y, C = L.layer_forward(cfg, params, x, None, 3)
    B, S, H, nh = cfg["batch"], cfg["seq"], cfg["hidden"], cfg["heads"]
    for site, key, n in ((1, "keep1", B * nh * S * S), (2, "keep2", B * S * H), (3, "keep3", B * S * H)):
        assert np.array_equal(C[key].reshape(-1) != 0,
                              dropout_keep(cfg["seed"], cfg["layer_id"], site, 3, n, 0.5))
    assert np.array_equal(C["prob_d"] == 0, (C["keep1"] == 0) | (C["prob"] == 0))
    y2, _ = L.layer_forward(cfg, params, x, None, 4)
    assert not np.allclose(y, y2)
