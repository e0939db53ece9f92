"""The C-ABI library builds, loads and exports every symbol the header declares (no GPU needed)."""
import os
import re

import pytest

import paper_1911_13252_amd as elm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "elm_rnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(elm_rnn_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(elm.lib_path()):
        from paper_1911_13252_amd.build import build_library
        build_library()
    return elm.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 14
    assert sorted(elm.DECLARED_SYMBOLS) == names
    for n in names:
        assert hasattr(lib, n), n


def test_host_only_entry_points(lib):
    assert lib.elm_rnn_strerror(0) == b"ok"
    assert b"rank" in lib.elm_rnn_strerror(-3)
    assert lib.elm_rnn_strerror(-99) == b"unknown error code"
    # workspace sizes: O(1) in N once the level-0 grid is full, zero for unsupported sizes
    a = elm.solve_workspace_bytes(4_000_000, 512, 2)
    b = elm.solve_workspace_bytes(8_000_000, 512, 2)
    assert a == b and 0 < a < (1 << 30)
    assert elm.solve_workspace_bytes(1000, 513, 1) == 0
    assert elm.solve_workspace_bytes(0, 10, 1) == 0
    assert elm.fit_workspace_bytes(1000, 16, 1, True) >= elm.fit_workspace_bytes(1000, 16, 1, False) + 1000 * 16 * 4
    # the streamed fit holds one chunk of H: whole 128-row blocks, at most N rows, 128 MiB by default
    assert elm.fit_streamed_workspace_bytes(4_000_000, 512, 2, 1000) - a == 1024 * 512 * 4
    assert elm.fit_streamed_workspace_bytes(4_000_000, 512, 2) - a == 65536 * 512 * 4
    # (a narrow layer's in-kernel hand-off may bring up to two R factors per compute unit)
    assert elm.fit_streamed_workspace_bytes(1000, 16, 1) >= elm.fit_workspace_bytes(1000, 16, 1, True)
    assert elm.fit_streamed_workspace_bytes(1000, 16, 1) - elm.fit_workspace_bytes(1000, 16, 1, True) <= 1024 * 32 * 32 * 4 * 2
    assert elm.fit_streamed_workspace_bytes(1000, 513, 1, 0) == 0


def test_no_cpu_fallback_and_no_oracle_in_the_product():
    pkg = os.path.join(ROOT, "paper_1911_13252_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src, f
