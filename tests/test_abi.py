"""The C ABI on a machine without a GPU: the library loads, exports every
function include/arb.h declares, and its host-side validation returns the
documented status codes before anything is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2512_05033_amd import binding, build
    if not os.path.exists(build.LIB):
        build.build_library(verbose=False)
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "arb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(arb_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2512_05033_amd import binding
    names = declared_functions()
    assert "arb_prefill" in names and "arb_score_steps" in names and "arb_route" in names
    for n in names:
        assert getattr(lib, n) is not None
    assert sorted(binding.EXPORTS) == names


def _cfg(**over):
    from paper_2512_05033_amd.binding import _Cfg
    v = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=1024, vocab=32000,
             rms_eps=1e-6, rope_base=10000.0, kv_block=16, pool=0, has_router_head=1)
    v.update(over)
    return _Cfg(*[v[k] for k, _ in _Cfg._fields_])


def _weights(n_layers=2, head=True):
    from paper_2512_05033_amd.binding import _Weights
    arr = (C.c_void_p * n_layers)(*([0x1000] * n_layers))      # never dereferenced by arb_model_create
    return _Weights(0x1000, arr, arr, arr, arr, arr, arr, 0x1000, 0x1000 if head else None, 0.0), arr


def _create(lib, cfg, w):
    h = C.c_void_p()
    st = lib.arb_model_create(C.byref(cfg), C.byref(w), C.byref(h))
    return st, h


def test_model_create_validation(lib):
    from paper_2512_05033_amd import binding as B
    w, _keep = _weights()
    st, h = _create(lib, _cfg(), w)
    assert st == B.ARB_OK and h.value
    assert lib.arb_workspace_bytes(h, 4, 128, 544) > 128 * 256 * 4
    assert lib.arb_workspace_bytes(h, 4, -1, 544) == 0
    lib.arb_model_destroy(h)
    assert _create(lib, _cfg(n_q_heads=5), w)[0] == B.ARB_ESHAPE
    assert _create(lib, _cfg(head_dim=63), w)[0] == B.ARB_ESHAPE
    assert _create(lib, _cfg(n_layers=0), w)[0] == B.ARB_ESHAPE
    assert _create(lib, _cfg(head_dim=32, n_q_heads=8, n_kv_heads=4), w)[0] == B.ARB_EUNSUPPORTED
    assert _create(lib, _cfg(kv_block=32), w)[0] == B.ARB_EUNSUPPORTED
    assert _create(lib, _cfg(d_model=200), w)[0] == B.ARB_EUNSUPPORTED
    assert b"d_model" in lib.arb_last_error()
    assert _create(lib, _cfg(pool=7), w)[0] == B.ARB_EINVAL
    assert _create(lib, _cfg(has_router_head=3), w)[0] == B.ARB_EINVAL
    assert _create(lib, _cfg(has_router_head=B.ARB_HEAD_TWO_CLASS), w)[0] == B.ARB_OK
    wn, _k2 = _weights(head=False)
    assert _create(lib, _cfg(), wn)[0] == B.ARB_EINVAL
    assert _create(lib, _cfg(has_router_head=0), wn)[0] == B.ARB_OK
    assert lib.arb_model_create(None, None, None) == B.ARB_EINVAL
    # optional K-blocked gate/up copies: one pointer per layer or none at all
    wb, keep_b = _weights()
    wb.wgu_blocked = keep_b
    assert _create(lib, _cfg(), wb)[0] == B.ARB_OK
    holes = (C.c_void_p * 2)(0x1000, None)
    wb.wgu_blocked = holes
    assert _create(lib, _cfg(), wb)[0] == B.ARB_EINVAL and b"wgu_blocked" in lib.arb_last_error()
    assert lib.arb_pack_k_blocked(0x1000, 4, 48, 0x1000, None) == B.ARB_EUNSUPPORTED       # K % 32
    assert lib.arb_pack_k_blocked(None, 4, 64, 0x1000, None) == B.ARB_EINVAL
    assert lib.arb_pack_k_blocked(None, 0, 64, None, None) == B.ARB_OK


def test_batch_validation_happens_on_the_host(lib):
    """Bad descriptors are refused from the host copies of the lengths, before
    any device pointer is touched (all device pointers here are fake)."""
    from paper_2512_05033_amd import binding as B
    w, _keep = _weights()
    st, h = _create(lib, _cfg(), w)
    pools = (C.c_void_p * 2)(0x1000, 0x1000)
    kv = B._KV(pools, pools, 8)

    def call(prefix, cu, max_blocks, total=None, ws_bytes=1 << 30, scores=0x1000):
        p, c = np.asarray(prefix, np.int32), np.asarray(cu, np.int32)
        bt = B._Batch(len(p), int(c[-1]) if total is None else total, max_blocks, 0x1000, 0x1000, 0x1000, 0x1000,
                      p.ctypes.data, c.ctypes.data)
        return lib.arb_score_steps(h, C.byref(kv), C.byref(bt), 0.0, scores, None, None, 0x1000, ws_bytes, None)

    assert call([10, 10], [0, 4, 4], 4) == B.ARB_EINVAL            # empty step
    assert b"step" in lib.arb_last_error()
    assert call([10, 10], [1, 4, 8], 4) == B.ARB_EINVAL            # cu[0] != 0
    assert call([10, -1], [0, 4, 8], 4) == B.ARB_EINVAL            # negative prefix
    assert call([10, 10], [0, 4, 8], 4, total=9) == B.ARB_EINVAL   # total mismatch
    assert call([60, 10], [0, 5, 8], 4) == B.ARB_ECAPACITY         # 65 tokens need 5 blocks
    assert call([59, 10], [0, 5, 8], 4, ws_bytes=16) == B.ARB_ECAPACITY   # workspace too small
    assert call([10, 10], [0, 4, 8], 4, scores=None) == B.ARB_EINVAL      # head but no scores buffer
    assert lib.arb_route(None, -1, 0.0, 0, None, None) == B.ARB_EINVAL
    assert lib.arb_route(None, 0, 0.0, 0, None, None) == B.ARB_OK
    assert lib.arb_route(0x1000, 4, 0.0, 9, 0x1000, None) == B.ARB_EINVAL
    assert lib.arb_advantage_route(None, None, 0, 0.0, None, None, None, None, None) == B.ARB_OK
    assert lib.arb_advantage_route(None, 0x1000, 4, 0.0, None, 0x1000, None, None, None) == B.ARB_EINVAL
    assert lib.arb_advantage_route(0x1000, 0x1000, 4, 0.0, None, None, None, None, None) == B.ARB_EINVAL   # no output
    assert lib.arb_budget_threshold(0x1000, -1, 0, 0x1000, None) == B.ARB_EINVAL
    assert lib.arb_budget_threshold(0x1000, 4, 1, None, None) == B.ARB_EINVAL
    assert lib.arb_stage_layers(None, None, None, 0, 1, None, None, None, 0, None) == B.ARB_EINVAL
    assert lib.arb_stage_gemm(0x1000, 0x1000, None, 0x1000, 8, 128, 96, 0, None) == B.ARB_EUNSUPPORTED
    assert lib.arb_stage_gemm(0x1000, 0x1000, None, 0x1000, 8, 100, 128, 0, None) == B.ARB_EUNSUPPORTED
    lib.arb_model_destroy(h)


def test_binding_refuses_to_run_without_the_library(tmp_path):
    from paper_2512_05033_amd import binding
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load_library(str(tmp_path / "libarb.so"))


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2512_05033_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
