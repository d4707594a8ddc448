"""The C-ABI library loads and exports every symbol the public header declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    src = open(os.path.join(ROOT, "include", "dlayer.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b([a-z_][a-z0-9_]*)\s*\(", src)
    return sorted({n for n in names if n not in ("defined",)})


def test_header_symbols_are_exported_and_bound():
    import paper_2602_08387_amd as K
    declared = _declared_functions()
    assert "dlayer_forward" in declared and "ce_loss_fwd_bwd" in declared and len(declared) >= 20
    lib = ctypes.CDLL(K.lib_path)
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in dlayer.h but not exported"
        assert name in K.EXPORTED_SYMBOLS, f"{name} has no Python binding"
        assert name == "dlayer_last_error" or hasattr(K, name)
    assert sorted(K.EXPORTED_SYMBOLS) == declared
    assert K.dlayer_version() == 1


def test_size_queries_and_cfg_validation_on_host():
    import paper_2602_08387_amd as K
    from synth import inputs as si
    cfg = si.CONFIGS["8b"]
    T, D, F = cfg.tokens, cfg.d_model, cfg.d_ff
    qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    # everything the backward needs is kept: bf16 h1,q,k,v,o,y1,h2,g,u,a + fp32 rstd x2 + lse + the
    # rotary cos / sin tables (a is stored with rows of d_ff + 64 elements)
    expect = (2 * T * (3 * D + 2 * qd + 2 * kd + 3 * F + 64) + 4 * T * (2 + cfg.n_q_heads)
              + 2 * 4 * cfg.seq * cfg.head_dim // 2)
    got = K.dlayer_saved_bytes(cfg)
    assert expect <= got <= expect + 15 * 256
    assert K.dlayer_workspace_bytes(cfg) > 0
    for bad in (cfg.with_(head_dim=96), cfg.with_(n_kv_heads=5), cfg.with_(seq=100), cfg.with_(d_ff=1000),
                cfg.with_(rope_layout=2), cfg.with_(batch=0), cfg.with_(d_model=16448),
                # few tokens, but w_gate alone is 16384 x 131072 x 2 B = 4 GiB
                cfg.with_(batch=1, seq=128, d_model=16384, d_ff=131072, n_q_heads=8, n_kv_heads=8),
                # batch * seq * width * 2 wraps around 64 bits to a small number: still too large
                cfg.with_(batch=2 ** 31 - 1, seq=2 ** 31 - 128, d_model=4096),
                cfg.with_(batch=2 ** 20, seq=2 ** 22)):
        assert K.dlayer_saved_bytes(bad) == 0 and K.dlayer_workspace_bytes(bad) == 0
    assert K.ce_loss_workspace_bytes(8192, 128256) == 8192 * 4
    assert K.rmsnorm_backward_workspace_bytes(16384, 4096) == 512 * 4096 * 4
    # chunked LM head: one chunk of logits (1 GiB's worth of rows by default, a multiple of 256), W_lm^T, T floats
    T, D, V = 8192, 4096, 128256
    assert K.lm_head_ce_workspace_bytes(T, D, V, 0) == 4096 * V * 2 + V * D * 2 + T * 4
    assert K.lm_head_ce_workspace_bytes(T, D, V, 1024) == 1024 * V * 2 + V * D * 2 + T * 4
    assert K.lm_head_ce_workspace_bytes(512, D, V, 0) == 512 * V * 2 + V * D * 2 + 512 * 4   # fewer rows than a chunk
    assert K.lm_head_ce_workspace_bytes(T, D, V, 100) == 0                                    # chunk not a multiple of 64
    assert K.linear_swiglu_backward_workspace_bytes(T, D, 14336) == D * 14336 * 2
    # rows wider than one 4096-column chunk also need one float per row
    assert K.rmsnorm_backward_workspace_bytes(16384, 8192) == 512 * 8192 * 4 + 16384 * 4


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2602_08387_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f"{f} mentions the oracle"
