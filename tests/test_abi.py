"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2603_25702_amd import binding as Bd
from s2d2_inputs import CONFIGS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(Bd.lib_path()):
        from paper_2603_25702_amd.build import build_lib
        build_lib()
    return Bd.load_library()


def header_functions():
    names = set()
    for h in ("s2d2.h", "s2d2_aux.h"):   # the step's boundary, and the inspection / measurement aids
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(s2d2_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = header_functions()
    assert set(names) == set(Bd.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_sizes_match_the_header_layout():
    assert C.sizeof(Bd.ModelDesc) == 14 * 4 + 8
    assert C.sizeof(Bd.LayerWeights) == 9 * 8
    assert C.sizeof(Bd.KvView) == 5 * 8 + 3 * 4 + 4
    assert C.sizeof(Bd.ParamsC) == 56
    assert C.sizeof(Bd.RouteParamsC) == 10 * 4 and C.sizeof(Bd.RouteOutC) == 4 * 8
    assert C.sizeof(Bd.DraftOutC) == 11 * 8 and C.sizeof(Bd.VerifyOutC) == 8 * 8 and C.sizeof(Bd.AcceptOutC) == 4 * 8


def test_workspace_bytes_and_limits(lib):
    for k in (1, 2, 3, 4):
        wl = CONFIGS[k]
        d = Bd.model_desc(wl.cfg)
        n = lib.s2d2_workspace_bytes(C.byref(d), wl.batch, wl.block)
        assert n > 0 and n % 256 == 0
        assert lib.s2d2_workspace_bytes(C.byref(d), 2 * wl.batch, wl.block) > n
    d = Bd.model_desc(CONFIGS[2].cfg)
    assert lib.s2d2_workspace_bytes(C.byref(d), 0, 4) == Bd.S2D2_EINVAL
    assert lib.s2d2_workspace_bytes(C.byref(d), 1, 65) == Bd.S2D2_EINVAL
    assert b"max_block" in lib.s2d2_last_error()
    assert lib.s2d2_stage_rows(2, 8) == 48
    assert lib.s2d2_workspace_bytes(None, 1, 4) == Bd.S2D2_EINVAL
    d2 = Bd.model_desc(CONFIGS[2].cfg)
    assert lib.s2d2_packed_bytes(C.byref(d2)) == 2 * (CONFIGS[2].cfg.n_params())  # every tile is full
    assert lib.s2d2_packed_bytes(C.byref(Bd.model_desc(CONFIGS[1].cfg))) == 0    # fp32: canonical layouts


@pytest.mark.parametrize("field,value", [("dtype", 7), ("head_dim", 48), ("n_kv_heads", 3), ("mask_id", -1),
                                         ("d_model", 2050), ("d_ffn", 0), ("vocab", 1), ("n_layers", 0)])
def test_bad_descriptions_are_rejected(lib, field, value):
    d = Bd.model_desc(CONFIGS[2].cfg)
    setattr(d, field, value)
    assert lib.s2d2_workspace_bytes(C.byref(d), 1, 4) == Bd.S2D2_EINVAL
    assert len(lib.s2d2_last_error()) > 0


def test_create_rejects_null_and_misaligned_arguments_without_a_device(lib):
    d = Bd.model_desc(CONFIGS[1].cfg)
    ctx = C.c_void_p()
    assert lib.s2d2_create(C.byref(d), None, 1, 4, None, None, 0, None, 0, C.byref(ctx)) == Bd.S2D2_EINVAL
    layers = (Bd.LayerWeights * d.n_layers)()
    for l in range(d.n_layers):
        layers[l] = Bd.LayerWeights(*([0x1000] * 6), None, None, None)
    w = Bd.Weights(0x1000, 0x1000, 0x1000, layers)
    assert lib.s2d2_create(C.byref(d), C.byref(w), 1, 4, None, None, 0, None, 0, C.byref(ctx)) == Bd.S2D2_EINVAL  # no workspace
    assert lib.s2d2_create(C.byref(d), C.byref(w), 1, 4, None, 0x1010, 1 << 30, None, 0, C.byref(ctx)) == Bd.S2D2_EINVAL  # misaligned
    assert lib.s2d2_create(C.byref(d), C.byref(w), 1, 4, None, 0x1000, 16, None, 0, C.byref(ctx)) == Bd.S2D2_ENOSPC
    layers[1].wo = 0x1004
    assert lib.s2d2_create(C.byref(d), C.byref(w), 1, 4, None, 0x1000, 1 << 30, None, 0, C.byref(ctx)) == Bd.S2D2_EINVAL
    assert b"layer 1" in lib.s2d2_last_error()
    assert ctx.value is None


def test_calls_reject_null_context(lib):
    assert lib.s2d2_destroy(None) == Bd.S2D2_EINVAL
    assert lib.s2d2_draft(None, None, None, 1, 4, None, None) == Bd.S2D2_EINVAL
    assert lib.s2d2_verify(None, None, None, 1, 4, None, None, None) == Bd.S2D2_EINVAL
    assert lib.s2d2_accept(None, None, 1, 4, None, None, None, None) == Bd.S2D2_EINVAL
    assert lib.s2d2_kv_append(None, None, 1, 4, None, None, None) == Bd.S2D2_EINVAL
    assert lib.s2d2_block_advance(None, None, None, 1, 4, None) == Bd.S2D2_EINVAL


def test_product_does_not_import_the_oracle():
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2603_25702_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower().replace("no oracle", ""), f
    src = open(os.path.join(ROOT, "oracle", "s2d2_oracle.py")).read()
    assert "paper_2603_25702_amd" not in src and "ctypes" not in src
