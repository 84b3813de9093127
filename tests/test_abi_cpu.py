"""The C-ABI library loads and exports every symbol its header declares; host-only entry points behave.
CPU only (no kernel is launched)."""
import ctypes as C
import os
import re

import pytest

import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2505_15380_amd as pkg
    if not os.path.exists(pkg.library_path()):
        import __graft_entry__ as g
        g.build()
    return pkg.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ssd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ssd_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    import paper_2505_15380_amd as pkg
    names = declared_symbols()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/ssd.h but not exported"
    assert sorted(pkg.EXPORTED_SYMBOLS) == names


def test_host_only_calls(lib):
    from paper_2505_15380_amd.binding import ModelConfig
    sh = si.model_shape("half_b")
    cfg = ModelConfig(sh["n_layers"], sh["d_model"], sh["n_q_heads"], sh["n_kv_heads"], sh["head_dim"], sh["d_ffn"],
                      sh["vocab"], sh["n_embed"], 1, 1, 1e6, 1e-6)
    need = lib.ssd_model_workspace_bytes(C.byref(cfg), 2048)
    params = sh["n_layers"] * (sh["d_model"] * (1152 + 896) + 3 * sh["d_model"] * sh["d_ffn"]) + \
        sh["d_model"] * (sh["vocab"] + sh["n_embed"])
    assert 2 * params <= need <= 2 * params * 1.01 + (1 << 20)       # bf16 weights + small tables
    cfg.head_dim = 48
    assert lib.ssd_model_workspace_bytes(C.byref(cfg), 2048) == 0
    assert b"head_dim" in lib.ssd_last_error()
    assert lib.ssd_strerror(0) == b"ok" and lib.ssd_strerror(-2) != lib.ssd_strerror(-1)
    # null handles are rejected without touching a device
    assert lib.ssd_kv_rollback(None, 0, 0, 0, None) == -1
    assert lib.ssd_verify(None, None, 1, None, None, None, 0, None, 0, None, None, None, None, None) == -1
    assert lib.ssd_kv_pool_bytes(None, 4, 16) == 0


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2505_15380_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f"{f} mentions the oracle"
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            assert "paper_2505_15380_amd" not in open(os.path.join(ROOT, "oracle", f)).read()
