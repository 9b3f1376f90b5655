"""The C-ABI library loads on a machine without a GPU, exports every symbol the header
declares, and rejects bad arguments from the host before any device work (CPU only)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def m():
    import paper_2401_14361_amd as mod
    if not os.path.exists(mod.lib_path()):          # build only if nothing is built
        from paper_2401_14361_amd.build import build
        build()
    mod.lib()
    return mod


def _declared():
    src = open(os.path.join(ROOT, "include", "moei.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(?:int|const char\*)\s+(\w+)\s*\(", src)))


def test_every_declared_symbol_is_exported_and_bound(m):
    names = _declared()
    assert {"moe_route_topk", "eam_update", "eamc_match", "expert_priority", "expert_ffn_gemv",
            "moe_decode_layer"} <= set(names)
    L = m.lib()
    for n in names:
        assert getattr(L, n) is not None, n
    assert sorted(m.EXPORTS) == names
    assert b"gfx950" in L.moei_version()


def test_model_desc_layout_matches_header(m):
    assert C.sizeof(m.ModelDesc) == 9 * 4
    assert [f[0] for f in m.ModelDesc._fields_] == ["L", "E", "k", "n_shared", "H", "I", "wdtype", "renorm_topk", "eps"]


def test_bad_arguments_are_refused_on_the_host(m):
    L = m.lib()
    null = C.c_void_p(0)
    one = C.c_void_p(16)        # never dereferenced: validation fails first

    def err(rc):
        assert rc < 0
        return L.moei_last_error().decode()

    assert "k = 9" in err(L.moe_route_topk(one, 1, 8, 9, 0, one, one, null))          # k > E
    assert "null" in err(L.moe_route_topk(null, 1, 8, 2, 0, one, one, null))
    assert "E = 5000" in err(L.moe_route_topk(one, 1, 5000, 2, 0, one, one, null))
    assert "layer 4" in err(L.eam_update(one, 1, 4, 8, 4, one, 2, null))               # layer >= L
    assert "null" in err(L.eam_update(null, 1, 4, 8, 0, one, 2, null))
    assert "null" in err(L.eamc_match(null, one, 1, 0, one, one, null, null))
    assert "null" in err(L.expert_priority(null, one, 1, 0, one, C.c_float(0), null, 0, one, one, one, one, one, one, null))
    assert "null" in err(L.expert_ffn_gemv(null, one, one, 1, one, one, null))
    assert "null" in err(L.moe_decode_layer(null, null, one, 0, one, null, one, one, null, null, null, null))
    h = C.c_void_p(0)
    bad = m.ModelDesc(4, 8, 9, 0, 64, 64, 1, 0, 1e-6)                                   # k > E
    assert L.moei_eamc_create(C.byref(bad), 10, 4, C.byref(h)) == -1 and not h.value
    ok = m.ModelDesc(4, 8, 2, 0, 64, 64, 1, 0, 1e-6)
    assert "cell_bytes" in err(L.moei_eamc_create(C.byref(ok), 10, 3, C.byref(h)))
    assert "n_cap" in err(L.moei_eamc_create(C.byref(ok), 0, 4, C.byref(h)))
    assert L.moei_cache_create(C.byref(ok), 1, null, 0, null, C.byref(h)) == -5          # fewer slots than k
    assert "wdtype" in err(L.moei_cache_create(C.byref(m.ModelDesc(4, 8, 2, 0, 64, 64, 7, 0, 0.0)), 4, null, 0, null, C.byref(h)))
    assert L.moei_eamc_destroy(null) == 0 and L.moei_cache_destroy(null) == 0


def test_product_path_does_not_reach_the_oracle():
    # the package and the HIP sources never import, include or name anything under oracle/
    pkg = os.path.join(ROOT, "paper_2401_14361_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in txt.lower(), os.path.join(dirpath, f)
    assert "paper_2401_14361_amd" not in open(os.path.join(ROOT, "oracle", "moei_oracle.py")).read()
