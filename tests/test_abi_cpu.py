"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and its pure-host entry points validate their arguments."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def P():
    from paper_1705_04862_amd import paac
    if not os.path.exists(paac.LIB_PATH):
        from paper_1705_04862_amd import build
        build.build_lib()
    return paac


def test_library_exports_every_declared_symbol(P):
    L = P.lib()
    header = open(os.path.join(ROOT, "include", "paac.h")).read()
    declared = sorted(set(re.findall(r"\b(paac_[a-z_]+)\s*\(", header)))
    assert declared == sorted(P.SYMBOLS)
    for name in declared:
        assert hasattr(L, name), name


def test_struct_layouts_match_header(P):
    assert C.sizeof(P.paac_config) == 32
    assert C.sizeof(P.paac_hparams) == 28
    assert C.sizeof(P.paac_train_stats) == 28


@pytest.mark.parametrize("arch,n_e,t_max,A,expect_p", [(0, 4, 5, 6, 677943), (1, 32, 5, 18, 1693875)])
def test_workspace_bytes(P, arch, n_e, t_max, A, expect_p):
    L = P.lib()
    cfg = P.paac_config(arch, n_e, t_max, A, 4, 84, 84, 0)
    n = C.c_size_t()
    assert L.paac_workspace_bytes(C.byref(cfg), C.byref(n)) == 0
    # at least parameters + RMSProp state + gradients, and a multiple of the 256-byte alignment
    assert n.value >= 3 * 4 * expect_p and n.value % 256 == 0
    cfg2 = P.paac_config(arch, 2 * n_e, t_max, A, 4, 84, 84, 0)
    n2 = C.c_size_t()
    assert L.paac_workspace_bytes(C.byref(cfg2), C.byref(n2)) == 0 and n2.value > n.value


@pytest.mark.parametrize("field,value", [("arch", 2), ("n_e", 0), ("t_max", 0), ("n_actions", 1),
                                         ("n_actions", 33), ("in_c", 3), ("in_h", 80), ("precision", 7)])
def test_bad_config_is_rejected(P, field, value):
    L = P.lib()
    cfg = P.paac_config(0, 4, 5, 6, 4, 84, 84, 0)
    setattr(cfg, field, value)
    n = C.c_size_t()
    assert L.paac_workspace_bytes(C.byref(cfg), C.byref(n)) == -2
    h = C.c_void_p()
    assert L.paac_create(C.byref(cfg), None, 0, None, C.byref(h)) == -2


def test_null_arguments(P):
    L = P.lib()
    n = C.c_size_t()
    assert L.paac_workspace_bytes(None, C.byref(n)) == -1
    assert L.paac_create(None, None, 0, None, None) == -1
    assert L.paac_param_count(None) == 0
    assert L.paac_last_error(None) == b"null context"
    L.paac_destroy(None)
