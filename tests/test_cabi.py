"""CPU-only checks of the C boundary: the library loads, exports every symbol the header declares, and its host-side
logic (configuration checks, workspace sizing, dropout keys) behaves.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def T():
    import paper_1904_01038_amd as T
    if not os.path.exists(T.lib_path()):
        from paper_1904_01038_amd import build
        build.build(verbose=False)
    return T


def declared_functions():
    text = open(os.path.join(ROOT, "include", "tfm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tfm_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(T):
    names = declared_functions()
    assert len(names) >= 25 and "tfm_train_step" in names and "tfm_apply_update" in names and "tfm_create" in names
    lib = C.CDLL(T.lib_path())
    missing = [n for n in names if not hasattr(lib, n)]
    assert not missing, missing


def test_workspace_sizing_and_config_validation(T):
    from synth import PRESETS, count_params
    L = T.lib()
    n = C.c_size_t()
    sizes = {}
    for name, prec in [("tiny", T.FP32), ("base", T.BF16), ("big", T.FP16), ("lm16", T.FP16)]:
        cfg = T.make_config(PRESETS[name], precision=prec, max_sentences=256, max_len=128, max_tokens=4096)
        assert L.tfm_workspace_bytes(C.byref(cfg), C.byref(n)) == 0
        sizes[name] = n.value
        # at least master + two moments + accumulator in fp32
        assert n.value >= 16 * count_params(PRESETS[name])
    assert sizes["tiny"] < sizes["base"] < sizes["big"]
    assert sizes["big"] < 12 * 2 ** 30              # a small fraction of 288 GB
    bad = [dict(d_model=100), dict(n_heads=3), dict(dec_layers=0), dict(vocab=2), dict(dropout=1.0), dict(precision=7),
           dict(max_tokens=0), dict(label_smoothing=-0.1), dict(init_loss_scale=0.0), dict(scale_window=0), dict(pad_id=-1)]
    for change in bad:
        cfg = T.make_config(PRESETS["tiny"], precision=T.FP32, max_sentences=8, max_len=16, max_tokens=128)
        for k, v in change.items():
            setattr(cfg, k, v)
        assert L.tfm_workspace_bytes(C.byref(cfg), C.byref(n)) == -1, change
        assert L.tfm_last_error(None)
    # a null workspace is rejected before anything touches the GPU
    cfg = T.make_config(PRESETS["tiny"], precision=T.FP32, max_sentences=8, max_len=16, max_tokens=128)
    h = C.c_void_p()
    assert L.tfm_create(C.byref(cfg), None, 0, None, C.byref(h)) == -1


def test_dropout_site_keys_match_the_oracle(T):
    from oracle.transformer import dropout_key, site_id
    L = T.lib()
    rng = np.random.default_rng(0)
    for _ in range(50):
        seed, step = int(rng.integers(0, 2 ** 62)), int(rng.integers(0, 2 ** 40))
        stream, layer, sub = int(rng.integers(0, 2)), int(rng.integers(-1, 16)), int(rng.integers(0, 3))
        assert L.tfm_dropout_key(seed, step, stream, layer, sub) == int(dropout_key(seed, step, site_id(stream, layer, sub)))


def test_parameter_list_matches_the_shared_shape_module(T):
    # the C side enumerates its parameters only for a live context; compare the count it needs with the shape module
    from synth import PRESETS, param_specs
    for name in ("tiny", "big", "lm16"):
        specs = param_specs(PRESETS[name])
        assert len({n for n, _ in specs}) == len(specs)
        assert specs[0][0] == "embed"
