"""CPU-only checks of the C-ABI library: it loads, exports every symbol include/stairs.h
declares, and rejects bad arguments before touching the GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2407_19947_amd as pkg
from paper_2407_19947_amd import binding
import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "stairs.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:stairs_|draft_)[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = pkg.lib()
    declared = _declared_symbols()
    assert len(declared) >= 12
    for name in declared:
        assert hasattr(L, name), f"{name} is declared in stairs.h but not exported"
    assert sorted(pkg.EXPORTED_SYMBOLS) == declared


def test_strerror():
    assert pkg.stairs_strerror(0) == "ok"
    assert "argument" in pkg.stairs_strerror(-1)
    assert pkg.stairs_last_error(None) == "context is NULL"


def test_init_rejects_bad_shapes_without_gpu():
    m = si.make_model(1, 1, 64, 1, 64, 64, "fp32")
    keep = []
    cfg, w = binding._marshal(m, 64, keep)
    ctx = C.c_void_p()
    L = pkg.lib()

    def init(cfg_, k_max=0, dcfg=None, dw=None):
        return L.stairs_init(C.byref(ctx), C.byref(cfg_), C.byref(w), dcfg, dw, k_max, None)

    bad = binding._ModelCfg.from_buffer_copy(cfg); bad.n_heads = 3          # d % heads
    assert init(bad) == -1 and not ctx.value
    bad = binding._ModelCfg.from_buffer_copy(cfg); bad.n_heads = 2          # head_dim 32 unsupported
    assert init(bad) == -1
    bad = binding._ModelCfg.from_buffer_copy(cfg); bad.dtype = 7
    assert init(bad) == -1
    bad = binding._ModelCfg.from_buffer_copy(cfg); bad.dtype = 1            # bf16 needs d % 256
    assert init(bad) == -1
    bad = binding._ModelCfg.from_buffer_copy(cfg); bad.vocab = 0
    assert init(bad) == -1
    assert init(cfg, k_max=32) == -1                                         # k_max >= STAIRS_MAX_ROWS
    assert init(cfg, k_max=2) == -1                                          # k_max > 0 without a draft
    assert L.stairs_init(None, C.byref(cfg), C.byref(w), None, None, 0, None) == -1
    assert L.stairs_init(C.byref(ctx), None, C.byref(w), None, None, 0, None) == -1
    wbad = binding._Weights.from_buffer_copy(w); wbad.lm_head = None
    assert L.stairs_init(C.byref(ctx), C.byref(cfg), C.byref(wbad), None, None, 0, None) == -1


def test_null_context_calls_return_einval():
    L = pkg.lib()
    buf = (C.c_int32 * 4)()
    assert L.stairs_prefill(None, buf, 4) == -1
    assert L.draft_propose(None, 1, buf) == -1
    assert L.stairs_verify(None, 0, buf, buf, None) == -1
    assert L.stairs_verify_tokens(None, buf, 1, buf, buf, None) == -1
    assert L.stairs_generate(None, buf, 4, 1, 0, buf, None) == -1
    assert L.stairs_get_tokens(None, buf, 4, buf) == -1
    L.stairs_free(None)


def test_gemm_host_rejects_bad_shapes():
    W = np.zeros((16, 100), np.uint16)
    X = np.zeros((1, 100), np.float32)
    with pytest.raises(pkg.StairsError):
        pkg.stairs_gemm_host(W, X)                      # K % 256 != 0 for bf16
    with pytest.raises(pkg.StairsError):
        pkg.stairs_gemm_host(np.zeros((16, 256), np.uint16), np.zeros((33, 256), np.float32))   # M > 32


@pytest.mark.parametrize("buckets,maxd", [(32, 128), (16, 64), (64, 256)])
def test_host_bucket_rule_equals_the_oracles(buckets, maxd):
    """The bias tables the library builds on the host use the same buckets as the oracle's own implementation of
    the rule (itself pinned in test_oracle_encdec.py), for every distance a table can hold."""
    from oracle import encdec_oracle as eo
    rel = np.arange(-5000, 5001)
    for two_sided in (True, False):
        want = eo.relative_position_bucket(rel, two_sided, buckets, maxd)
        got = np.array([pkg.stairs_rel_bucket(int(r), two_sided, buckets, maxd) for r in rel])
        assert np.array_equal(got, want), two_sided
    assert pkg.stairs_rel_bucket(1, True, 30, 128) == -1 and pkg.stairs_rel_bucket(1, True, 32, 16) == -1


def test_encdec_init_rejects_bad_shapes_without_gpu():
    m = si.make_encdec_model(1, 1, 1, 256, 4, 64, 256, 512)
    keep = []
    cfg, w = binding._marshal_encdec(m, 16, 16, keep)
    ctx = C.c_void_p()
    L = pkg.lib()

    def init(cfg_, k_max=0, start=0):
        return L.stairs_encdec_init(C.byref(ctx), C.byref(cfg_), C.byref(w), None, None, k_max, start, None)

    for field, value in (("head_dim", 32), ("d_model", 128), ("d_ffn", 100), ("vocab", 500), ("rel_buckets", 30),
                         ("rel_max_distance", 8), ("max_src", 5000), ("max_seq", 1), ("n_enc_layers", 0)):
        bad = binding._EncDecCfg.from_buffer_copy(cfg)
        setattr(bad, field, value)
        assert init(bad) == -1 and not ctx.value, field
    assert init(cfg, k_max=1) == -1                                          # k_max > 0 without a draft
    assert init(cfg, start=512) == -1                                        # start token outside the vocabulary
