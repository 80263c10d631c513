"""Host-only checks: the shared library loads, exports every symbol the headers declare, and its
layout / workspace queries are pure functions of the configuration that agree with the input
recipe's inventory.  No kernel is launched."""
import os
import re

import pytest

import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def tm():
    import paper_2412_12636_amd as tm
    if not os.path.exists(tm.LIB_PATH):
        from paper_2412_12636_amd import build
        build.build()
    return tm


def declared_symbols():
    names = set()
    for hdr in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not hdr.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", hdr)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(tm_[a-z0-9_]+)\s*\(", text))
    return names


def test_every_declared_symbol_is_exported_and_bound(tm):
    lib = tm.lib()
    decl = declared_symbols()
    assert decl, "no declarations found"
    for name in decl:
        assert hasattr(lib, name), name
    assert decl == set(tm.EXPORTS), decl ^ set(tm.EXPORTS)
    for name in decl:
        assert callable(getattr(tm, name)), f"binding lacks {name}"


@pytest.mark.parametrize("preset", list(si.PRESETS))
def test_layout_matches_inventory(tm, preset):
    cfg = si.PRESETS[preset]
    assert tm.tm_stage_param_count(cfg) == si.stage_param_count(cfg)
    layout = tm.tm_stage_param_layout(cfg)
    inv = si.layer_inventory(cfg)
    assert len(layout) == cfg.n_layers * len(inv)
    off = 0
    for l in range(cfg.n_layers):
        for (name, shape) in inv:
            lname, loff, lshape = layout[l * len(inv) + inv.index((name, shape))]
            assert lname == f"layer{l}.{name}"
            assert loff == off and off % 8 == 0
            assert lshape == (shape[0], shape[1] if len(shape) == 2 else 1)
            off += shape[0] * (shape[1] if len(shape) == 2 else 1)
    # queries are pure: asking twice gives the same answers
    assert tm.tm_stage_param_layout(cfg) == layout
    assert tm.tm_stage_workspace_bytes(cfg) == tm.tm_stage_workspace_bytes(cfg) > 0


def test_config_errors(tm):
    cfg = si.PRESETS["tiny"]
    for bad, code in ((cfg.replace(hidden=100), tm.TM_ESIZE), (cfg.replace(n_layers=0), tm.TM_EINVAL),
                      (cfg.replace(n_q_heads=3, n_kv_heads=2), tm.TM_ESIZE), (cfg.replace(dtype=7), tm.TM_EINVAL),
                      (cfg.replace(hidden=32768, dtype=si.DTYPE_BF16), tm.TM_ESIZE),
                      (cfg.replace(seq=10000), tm.TM_ESIZE)):
        with pytest.raises(tm.TmError) as e:
            tm.tm_stage_param_count(bad)
        assert e.value.code == code
        assert tm.tm_last_error()


def test_long_sequences_need_the_matrix_core_attention(tm):
    """Sequences above the plain-ALU attention's limit are accepted only where the flash kernels run (bf16, head size
    128): tm_stage_init must refuse the others itself, before anything is enqueued, with the dispatch's own condition."""
    long_cfg = si.PRESETS["longctx"].replace(n_layers=1)
    assert tm.tm_stage_param_count(long_cfg) > 0
    for bad in (long_cfg.replace(head_dim=64, n_q_heads=16, n_kv_heads=2), long_cfg.replace(dtype=si.DTYPE_FP32),
                long_cfg.replace(head_dim=256, n_q_heads=4)):
        for call in (lambda: tm.tm_stage_param_count(bad), lambda: tm.tm_stage_workspace_bytes(bad),
                     lambda: tm.tm_stage_init(bad, 256, 256, 256, 256, 256, 256, 1 << 40)):
            with pytest.raises(tm.TmError) as e:
                call()
            assert e.value.code == tm.TM_ESIZE
    # at the limit itself every head size is fine
    assert tm.tm_stage_param_count(long_cfg.replace(head_dim=64, n_q_heads=16, n_kv_heads=2, seq=8192)) > 0


def test_reduce_scratch_query(tm):
    assert tm.tm_op_reduce_scratch_bytes(2048, 12288) == 256 * 12288 * 4
    assert tm.tm_op_reduce_scratch_bytes(5, 8) == 5 * 8 * 4
