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
    # step bookkeeping of the decode loop
    assert lib.arb_step_advance(None, None, 0, 4, 8, 1, 2, None, None, None, None, None, None, None) == B.ARB_EINVAL   # no n_next
    assert lib.arb_step_advance(0x1000, 0x1000, 5, 4, 8, 1, 2, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, None) == B.ARB_EINVAL
    assert lib.arb_step_advance(0x1000, 0x1000, 2, 4, 0, 1, 2, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, None) == B.ARB_EINVAL
    assert lib.arb_step_advance(0x1000, None, 2, 4, 8, 1, 2, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, None) == B.ARB_EINVAL
    assert lib.arb_pack_steps(None, 8, None, None, 0, None, None) == B.ARB_OK
    assert lib.arb_pack_steps(0x1000, 0, 0x1000, 0x1000, 2, 0x1000, None) == B.ARB_EINVAL
    assert lib.arb_pack_steps(0x1000, 8, None, 0x1000, 2, 0x1000, None) == B.ARB_EINVAL
    assert lib.arb_stage_gemm(0x1000, 0x1000, None, 0x1000, 8, 128, 96, 0, None) == B.ARB_EUNSUPPORTED
    assert lib.arb_stage_gemm(0x1000, 0x1000, None, 0x1000, 8, 100, 128, 0, None) == B.ARB_EUNSUPPORTED
    lib.arb_model_destroy(h)


def test_launch_plan_of_the_projection_gemm_is_host_arithmetic(lib):
    """arb_gemm_large_tile_columns: whole rounds of 256 large tiles go to the large-tile kernel, the rest
    (or everything, when there is less than a round) to small tiles."""
    from paper_2512_05033_amd import binding as B
    cols = lambda M, N, K, e: lib.arb_gemm_large_tile_columns(M, N, K, e)
    # C2 gate/up: 4 x 70 large tiles -> one round of 4 x 64, 6 columns (768 features) left to small tiles
    assert cols(1024, 8960, 1536, B.ARB_EPI_SWIGLU_BF16) == 64
    # less than 205 large tiles: small tiles only
    assert cols(130, 64, 128, B.ARB_EPI_SWIGLU_BF16) == 0
    assert cols(1024, 2048, 1536, B.ARB_EPI_STORE_BF16) == 0
    # 13 x 16 = 208 large tiles: one round, at least 80 % full -> all 16 columns
    assert cols(3300, 4096, 256, B.ARB_EPI_STORE_BF16) == 16
    # 16 x 35 = 560: two rounds = 32 columns, the other 3 columns in small tiles
    assert cols(4000, 8960, 128, B.ARB_EPI_STORE_BF16) == 32
    # a width that is not a multiple of the large tile never uses it; bad sizes give 0
    assert cols(4000, 8960 + 128, 128, B.ARB_EPI_STORE_BF16) == 0
    assert cols(0, 4096, 256, B.ARB_EPI_STORE_BF16) == 0 and cols(-5, 4096, 256, B.ARB_EPI_STORE_BF16) == 0


def test_workspace_size_grows_with_every_argument(lib):
    w, _keep = _weights()
    st, h = _create(lib, _cfg(), w)
    base = lib.arb_workspace_bytes(h, 4, 128, 544)
    assert base > 0 and base % 256 == 0
    assert lib.arb_workspace_bytes(h, 4, 256, 544) > base
    assert lib.arb_workspace_bytes(h, 4, 128, 40000) > base            # more key splits to merge
    assert lib.arb_workspace_bytes(h, 4, 0, 0) >= 0
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
