"""CPU-only checks of the boundary: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before any launch."""
import ctypes as C
import os
import re

import pytest

import paper_2303_04759_amd as raf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(raf.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return raf.load_library()


def header_symbols():
    text = open(os.path.join(ROOT, "include", "raf_mi355.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(raf_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    syms = header_symbols()
    assert len(syms) >= 14
    for s in syms:
        assert hasattr(lib, s), s
    assert sorted(raf.EXPORTS) == syms


def test_struct_layout_matches_header():
    assert C.sizeof(raf.LayerDesc) == 64
    assert raf.LayerDesc.dropout_p.offset == 40 and raf.LayerDesc.seed.offset == 48
    assert C.sizeof(raf.LayerTensors) == 136 and raf.LayerTensors.wt_qkv.offset == 96 and raf.LayerTensors.nonfinite.offset == 128
    assert C.sizeof(raf.AdamTensor) == 64 and raf.AdamTensor.lowp_t.offset == 48 and raf.AdamTensor.cols.offset == 60
    assert C.sizeof(raf.ScalerState) == 32 and raf.ScalerState.t.offset == 16 and raf.ScalerState.inv_bc2.offset == 28


def good_cfg(**kw):
    cfg = dict(batch=2, seq=32, hidden=128, heads=2, ffn=512, pre_ln=0, causal=0, gelu_tanh=0, precision=0,
               ln_eps=1e-5, dropout_p=0.1, seed=1, layer_id=0)
    cfg.update(kw)
    return cfg


def test_workspace_and_descriptor_validation(lib):
    sv, sc = raf.raf_layer_workspace(raf.make_desc(good_cfg()))
    assert sv > 0 and sc > 0 and sv % 256 == 0 and sc % 256 == 0
    sv2, _ = raf.raf_layer_workspace(raf.make_desc(good_cfg(precision=1)))
    assert sv2 < sv
    for bad, code in ((dict(heads=4), raf.RAF_ENOTSUP), (dict(seq=33), raf.RAF_ENOTSUP),
                      (dict(dropout_p=1.0), raf.RAF_EINVAL), (dict(batch=0), raf.RAF_EINVAL),
                      (dict(precision=7), raf.RAF_EINVAL), (dict(hidden=8192, heads=128), raf.RAF_ENOTSUP),
                      (dict(pre_ln=2), raf.RAF_EINVAL)):
        with pytest.raises(raf.RafError) as e:
            raf.raf_layer_workspace(raf.make_desc(good_cfg(**bad)))
        assert e.value.status == code, bad


def test_keep_bits_of_the_blockwise_attention_are_accounted_for(lib):
    """Host arithmetic only: one keep bit per score for seq > 128 with dropout (16 bytes per query row and 128-key
    block), none otherwise, and raf_layer_workspace reserves exactly that much more of `saved`."""
    big = good_cfg(batch=2, seq=416, hidden=128, heads=2, ffn=512, precision=1)
    nbytes = raf.raf_op_attention_keep_bytes(raf.make_desc(big))
    assert nbytes == 2 * 2 * 416 * 4 * 16
    assert raf.raf_op_attention_keep_bytes(raf.make_desc(dict(big, dropout_p=0.0))) == 0
    assert raf.raf_op_attention_keep_bytes(raf.make_desc(dict(big, seq=128))) == 0
    assert raf.raf_op_attention_keep_bytes(raf.make_desc(dict(big, precision=0))) == 0
    with_bits, _ = raf.raf_layer_workspace(raf.make_desc(big))
    without, _ = raf.raf_layer_workspace(raf.make_desc(dict(big, dropout_p=0.0)))
    assert with_bits - without == (nbytes + 255) // 256 * 256


def test_null_and_misaligned_pointers_are_rejected_on_host(lib):
    d = raf.make_desc(good_cfg())
    w = raf.LayerTensors()          # all NULL
    rc = lib.raf_layer_fwd(C.byref(d), C.byref(w), 256, None, 256, 256, 256, 0, None)
    assert rc == raf.RAF_EINVAL
    for n in raf.PARAM_NAMES:
        setattr(w, n, 4096)
    rc = lib.raf_layer_fwd(C.byref(d), C.byref(w), 4096 + 8, None, 4096, 4096, 4096, 0, None)   # x misaligned
    assert rc == raf.RAF_EINVAL
    rc = lib.raf_layer_bwd(C.byref(d), C.byref(w), 4096, None, None, 4096, 4096, C.byref(w), 4096, 0, None)
    assert rc == raf.RAF_EINVAL
    assert lib.raf_adam_step(None, 0, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, 1.0, None) == raf.RAF_OK     # empty list
    assert lib.raf_adam_step(None, 1, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, 1.0, None) == raf.RAF_EINVAL
    t = (raf.AdamTensor * 1)(raf.AdamTensor(4096, 4096, 4096, 4096 + 4, None, 10))
    assert lib.raf_adam_step(t, 1, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, 1.0, None) == raf.RAF_EINVAL
    assert lib.raf_adam_step(t, 1, 1e-3, 0.9, 0.999, 1e-8, 0.0, 0, 1.0, None) == raf.RAF_EINVAL    # t is 1-based
    assert lib.raf_op_gemm(1, 64, 64, 48, 4096, 64, 1, 4096, 64, 1, 4096, 64, 0, 1.0, 0, None, None, 0,
                           None) == raf.RAF_ENOTSUP
    # dynamic loss scaler and attention operations: argument checks happen before any launch
    assert lib.raf_scaler_init(None, 128.0, None) == raf.RAF_EINVAL
    assert lib.raf_scaler_init(4096, 0.0, None) == raf.RAF_EINVAL
    assert lib.raf_scaler_init(4096 + 4, 128.0, None) == raf.RAF_EINVAL
    assert lib.raf_scaler_update(4096, 0.5, 0.5, 10, None) == raf.RAF_EINVAL        # growth factor below 1
    assert lib.raf_scaler_update(4096, 2.0, 0.5, 0, None) == raf.RAF_EINVAL          # interval below 1
    assert lib.raf_grads_check(None, 1, 4096, None) == raf.RAF_EINVAL
    assert lib.raf_adam_step_scaled(None, 0, 1e-3, 0.9, 0.999, 1e-8, 0.0, None, None) == raf.RAF_EINVAL
    assert lib.raf_loss_seed_scaled(1, 4096, 4096, 64, None, 4096, 4096, 4096, None) == raf.RAF_EINVAL
    d32 = raf.make_desc(good_cfg())                                                  # fp32: no on-chip attention path
    assert lib.raf_op_attention_fwd(C.byref(d32), 4096, None, 4096, None, None, 0, None) == raf.RAF_ENOTSUP
    dbf = raf.make_desc(good_cfg(precision=1))
    assert lib.raf_op_attention_fwd(C.byref(dbf), None, None, 4096, None, None, 0, None) == raf.RAF_EINVAL
    assert lib.raf_op_attention_bwd(C.byref(dbf), 4096, 4096 + 2, None, None, None, None, 4096, None, 0, None) == raf.RAF_EINVAL
    assert raf.status_string(raf.RAF_ENOTSUP) == "unsupported shape or mode"
    assert raf.version().startswith("raf_mi355")


def test_mlm_head_rejects_zero_layernorm_eps(lib):
    """The head pads the selected rows with rows of zero variance; eps = 0 would turn them into NaN."""
    cfg = dict(batch=2, seq=32, hidden=128, vocab=1000, precision=1, ln_eps=1e-12)
    assert raf.raf_mlm_workspace(raf.make_mlm_desc(cfg, 9)) > 0
    with pytest.raises(raf.RafError) as e:
        raf.raf_mlm_workspace(raf.make_mlm_desc(dict(cfg, ln_eps=0.0), 9))
    assert e.value.status == raf.RAF_EINVAL


def test_product_path_has_no_oracle_or_cpu_fallback():
    """No file of the package (Python or HIP source) may name the oracle: it is test infrastructure only."""
    pkg = os.path.join(ROOT, "paper_2303_04759_amd")
    seen = 0
    for base, _, files in os.walk(pkg):
        if "__pycache__" in base:
            continue
        for fn in files:
            if not fn.endswith((".py", ".hip", ".hpp", ".h", ".cpp", ".c")):
                continue
            seen += 1
            src = open(os.path.join(base, fn)).read()
            assert not re.search(r"\boracle\b", src), os.path.join(base, fn)
            assert "_work/" not in src, os.path.join(base, fn)
    assert seen >= 10