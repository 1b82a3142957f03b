"""Seeded synthetic transformer-layer workloads.

These stand in for the paper's evaluation inputs (tokenised WikiText-2 fed to
pretrained BERT / GPT-2 checkpoints, Section 5.1), which are not available
offline: the shapes are those of the same model families, values are drawn
from a seeded generator.  Nothing here computes any part of the training
step; it only draws numbers and rounds inputs to the storage type.

Draw order (fixed, so a seed names one workload): x, G, the twelve parameter
tensors in PARAM_NAMES order, then seq_lens.
"""
import numpy as np

PARAM_NAMES = ("w_qkv", "b_qkv", "w_o", "b_o", "ln1_g", "ln1_b",
               "w_1", "b_1", "w_2", "b_2", "ln2_g", "ln2_b")

F32, BF16_AMP = 0, 1

_BASE = dict(pre_ln=0, causal=0, gelu_tanh=0, seed=0x5EED2303, layer_id=0)

CONFIGS = {
    # tiny post-LN layer, fp32, no dropout, full-length sequences
    "tiny": dict(_BASE, batch=2, seq=32, hidden=128, heads=2, ffn=512, precision=F32,
                 dropout_p=0.0, ln_eps=1e-12, len_lo=None, len_hi=None, loss_scale=1.0),
    # BERT-base-shaped encoder layer, bf16 AMP, padding lengths U[64,128]
    "bert_base": dict(_BASE, batch=32, seq=128, hidden=768, heads=12, ffn=3072, precision=BF16_AMP,
                      dropout_p=0.1, ln_eps=1e-12, len_lo=64, len_hi=128, loss_scale=1024.0),
    # BERT-large-shaped encoder layer, bf16 AMP, padding lengths U[256,512]
    "bert_large": dict(_BASE, batch=8, seq=512, hidden=1024, heads=16, ffn=4096, precision=BF16_AMP,
                       dropout_p=0.1, ln_eps=1e-12, len_lo=256, len_hi=512, loss_scale=1024.0),
    # GPT-2-medium-shaped pre-LN decoder layer, causal, no padding
    "gpt2_medium": dict(_BASE, batch=4, seq=1024, hidden=1024, heads=16, ffn=4096, precision=BF16_AMP,
                        pre_ln=1, causal=1, dropout_p=0.1, ln_eps=1e-5, len_lo=None, len_hi=None,
                        loss_scale=1024.0),
}

ADAM = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)


def param_shapes(cfg):
    H, F = cfg["hidden"], cfg["ffn"]
    return {"w_qkv": (3 * H, H), "b_qkv": (3 * H,), "w_o": (H, H), "b_o": (H,),
            "ln1_g": (H,), "ln1_b": (H,), "w_1": (F, H), "b_1": (F,),
            "w_2": (H, F), "b_2": (H,), "ln2_g": (H,), "ln2_b": (H,)}


def round_to_bf16(a):
    """fp32 array -> nearest-even bfloat16 value, returned as fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a):
    """fp32 array holding bf16-representable values -> uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def make_layer_inputs(cfg, seed=0, random_affine=False):
    """Returns dict(x [B,S,H] f32, G [B,S,H] f32, params {name: f32}, seq_lens int32 or None).

    x, G ~ N(0,1); weights ~ N(0,0.02); biases 0; LayerNorm gamma 1, beta 0.
    With random_affine=True biases and LayerNorm parameters are drawn too
    (N(0,0.02) and 1+N(0,0.1)), for tests that must see those gradients move.
    In AMP configs x and G are rounded once to bf16 so both sides read the
    same numbers.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    B, S, H = cfg["batch"], cfg["seq"], cfg["hidden"]
    x = rng.standard_normal((B, S, H), dtype=np.float32)
    G = rng.standard_normal((B, S, H), dtype=np.float32)
    params = {}
    for name, shape in param_shapes(cfg).items():
        if name.startswith("w_"):
            params[name] = (0.02 * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)
        elif name.endswith("_g"):
            params[name] = np.ones(shape, dtype=np.float32)
            if random_affine:
                params[name] += (0.1 * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)
        else:
            params[name] = np.zeros(shape, dtype=np.float32)
            if random_affine:
                params[name] += (0.02 * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)
    seq_lens = None
    if cfg.get("len_lo") is not None:
        seq_lens = rng.integers(cfg["len_lo"], cfg["len_hi"], size=B, endpoint=True).astype(np.int32)
    if cfg["precision"] == BF16_AMP:
        x = round_to_bf16(x)
        G = round_to_bf16(G)
    return dict(x=x, G=G, params=params, seq_lens=seq_lens)


# ---------------------------------------------------------------- full model --
MODEL_CONFIGS = {
    # 12-layer BERT-base-shaped encoder + MLM head, tied 30522 x 768 embedding, bf16 AMP
    "bert_base_12l_mlm": dict(CONFIGS["bert_base"], batch=64, layers=12, vocab=30522, max_pos=512,
                              layer_id_base=0, embed_layer_id=0xE0, mlm_prob=0.15),
    # small fp32 model for parity tests that the oracle finishes in seconds
    "tiny_model": dict(CONFIGS["tiny"], layers=2, vocab=1000, max_pos=64, layer_id_base=0, embed_layer_id=0xE0,
                       mlm_prob=0.15, dropout_p=0.1, loss_scale=4.0, len_lo=8, len_hi=32),
}

EMBED_PARAMS = ("word", "pos", "emb_ln_g", "emb_ln_b")
HEAD_PARAMS = ("head_w", "head_b", "head_ln_g", "head_ln_b", "dec_b")


def vocab_padded(cfg):
    """Rows of the word table as stored: the vocabulary rounded up to a multiple of 32 (extra rows zero)."""
    return (cfg["vocab"] + 31) // 32 * 32


def make_model_inputs(cfg, seed=0):
    """Returns dict(ids [B,S] int32, seq_lens, sel int32 (ascending flat positions), labels int32,
    P {embedding/head name: f32}, layers [ {layer param: f32} ]).

    Draw order: seq_lens, ids, selection mask, labels, embedding/head parameters, then each layer's
    twelve tensors.  Selected positions: Bernoulli(mlm_prob) on valid tokens (at least one); labels
    and ids uniform over the vocabulary; tables ~ N(0,0.02); LayerNorm gamma 1, beta 0; biases 0.
    These stand in for tokenised text and a pretrained checkpoint.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    B, S, H, V = cfg["batch"], cfg["seq"], cfg["hidden"], cfg["vocab"]
    seq_lens = rng.integers(cfg["len_lo"], cfg["len_hi"], size=B, endpoint=True).astype(np.int32)
    ids = rng.integers(0, V, size=(B, S)).astype(np.int32)
    valid = np.arange(S)[None, :] < seq_lens[:, None]
    pick = (rng.random((B, S)) < cfg["mlm_prob"]) & valid
    if not pick.any():
        pick[0, 0] = True
    sel = np.flatnonzero(pick.reshape(-1)).astype(np.int32)
    labels = rng.integers(0, V, size=sel.size).astype(np.int32)
    Vp = vocab_padded(cfg)
    P = {}
    word = np.zeros((Vp, H), dtype=np.float32)
    word[:V] = 0.02 * rng.standard_normal((V, H), dtype=np.float32)
    P["word"] = word
    P["pos"] = (0.02 * rng.standard_normal((cfg["max_pos"], H), dtype=np.float32)).astype(np.float32)
    P["emb_ln_g"] = np.ones(H, dtype=np.float32)
    P["emb_ln_b"] = np.zeros(H, dtype=np.float32)
    P["head_w"] = (0.02 * rng.standard_normal((H, H), dtype=np.float32)).astype(np.float32)
    P["head_b"] = np.zeros(H, dtype=np.float32)
    P["head_ln_g"] = np.ones(H, dtype=np.float32)
    P["head_ln_b"] = np.zeros(H, dtype=np.float32)
    P["dec_b"] = np.zeros(V, dtype=np.float32)
    layers = []
    for _ in range(cfg["layers"]):
        lp = {}
        for name, shape in param_shapes(cfg).items():
            if name.startswith("w_"):
                lp[name] = (0.02 * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)
            elif name.endswith("_g"):
                lp[name] = np.ones(shape, dtype=np.float32)
            else:
                lp[name] = np.zeros(shape, dtype=np.float32)
        layers.append(lp)
    return dict(ids=ids, seq_lens=seq_lens, sel=sel, labels=labels, P=P, layers=layers)
