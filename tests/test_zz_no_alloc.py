"""The entry point that allocates nothing (raf_op_dropout_residual_ln_bwd_noalloc) against the entry point it is a
variant of: same kernels, so every output must be bit-identical.  Two calls in a row on the one device-resident
partial-sum array, the second with a smaller input, then the size limit."""
import numpy as np
import pytest
import torch

import paper_2303_04759_amd as raf

from gpu_util import announce, cdtype, to_dev

pytestmark = pytest.mark.gpu


def one_case(precision, rows, H, p, seed):
    cfg = dict(batch=1, seq=32, hidden=H, heads=H // 64, ffn=4 * H, pre_ln=0, causal=0, gelu_tanh=0,
               precision=precision, ln_eps=1e-5, dropout_p=p, seed=1234, layer_id=3)
    desc = raf.make_desc(cfg)
    rng = np.random.default_rng(seed)
    dt = cdtype(precision)
    z, dout, dout2, dres = (to_dev(rng.standard_normal((rows, H)), dt) for _ in range(4))
    gamma = torch.from_numpy((1 + 0.2 * rng.standard_normal(H)).astype(np.float32)).cuda()
    mu = z.float().mean(-1).contiguous()
    rstd = (1.0 / torch.sqrt(z.float().var(-1, unbiased=False) + 1e-5)).contiguous()
    step = 9
    outs = []
    for variant in ("workspace", "noalloc"):
        dz, da = torch.full_like(z, 3.0), torch.full_like(z, 3.0)
        dg, db, dbias = (torch.full((H,), 3.0, device="cuda") for _ in range(3))
        if variant == "workspace":
            partial = torch.zeros(raf.raf_op_ln_bwd_partial_floats(H, rows), device="cuda")
            raf.raf_op_dropout_residual_ln_bwd(desc, 2, rows, dout, dout2, z, mu, rstd, gamma, dres, dz, da, dg, db,
                                               dbias, partial, step)
        else:
            raf.raf_op_dropout_residual_ln_bwd_noalloc(desc, 2, rows, dout, dout2, z, mu, rstd, gamma, dres, dz, da,
                                                       dg, db, dbias, step)
        torch.cuda.synchronize()
        outs.append((dz, da, dg, db, dbias))
    for a, b, name in zip(outs[0], outs[1], ("dz", "da", "dgamma", "dbeta", "dbias")):
        assert torch.isfinite(b.float()).all(), name
        assert torch.equal(a, b), (name, precision, rows, H)


def test_noalloc_entry_point_matches_the_workspace_one():
    announce("no-alloc LayerNorm adjoint: bf16 4096x768, then 100x256, then fp32 37x1024")
    one_case(1, 4096, 768, 0.1, seed=0)      # fills the partial array of 256 workgroups
    one_case(1, 100, 256, 0.1, seed=1)       # smaller input right after: stale partials must not leak in
    one_case(0, 37, 1024, 0.0, seed=2)


def test_noalloc_entry_point_rejects_what_its_array_cannot_hold():
    announce("no-alloc LayerNorm adjoint: size limit")
    H, rows = 2048, 4096
    assert raf.raf_op_ln_bwd_partial_floats(H, rows) > raf.RAF_NOALLOC_LN_BWD_PARTIAL_FLOATS
    cfg = dict(batch=1, seq=32, hidden=H, heads=H // 64, ffn=4 * H, pre_ln=0, causal=0, gelu_tanh=0, precision=1,
               ln_eps=1e-5, dropout_p=0.0, seed=1, layer_id=0)
    t = torch.zeros(rows, H, device="cuda", dtype=torch.bfloat16)
    v = torch.zeros(H, device="cuda")
    r = torch.zeros(rows, device="cuda")
    with pytest.raises(raf.RafError) as e:
        raf.raf_op_dropout_residual_ln_bwd_noalloc(raf.make_desc(cfg), 2, rows, t, None, t, r, r, v, None, t, t, v, v,
                                                   v, 0)
    assert e.value.status == raf.RAF_EWORKSPACE
