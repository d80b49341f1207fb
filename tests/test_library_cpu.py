"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the
header declares, sizes its workspace, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2605_06374_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "varlen_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(varlen_attn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"varlen_attn_fwd", "varlen_attn_bwd", "varlen_attn_plan", "varlen_attn_check",
            "varlen_attn_workspace_bytes", "varlen_attn_status_string"} <= set(names)
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"


def test_struct_sizes_match_header():
    assert ctypes.sizeof(B.Params) == 28
    assert ctypes.sizeof(B.PlanHeader) == 64
    assert ctypes.sizeof(B.Unit) == 32
    assert ctypes.sizeof(B.CombineItem) == 16


def test_workspace_bytes():
    p = B.make_params(8192, 9, 4, 4, 128, 0.0884)
    n = B.varlen_attn_workspace_bytes(p)
    L = B.varlen_attn_workspace_regions(p)
    tiles = 8192 // 128 + 9
    assert L.total_bytes == n and n % 256 == 0
    assert L.max_combine == tiles and L.max_units >= tiles + L.max_row_slots
    assert L.row_units_offset >= 64
    offs = [L.row_units_offset, L.col_units_offset, L.row_combine_offset, L.col_combine_offset,
            L.dsum_offset, L.row_partials_offset, L.col_partials_offset, L.total_bytes]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert L.col_units_offset - L.row_units_offset >= 32 * L.max_units
    assert L.row_partials_offset - L.dsum_offset >= 2 * 4 * 4 * 8192
    assert L.col_partials_offset - L.row_partials_offset >= (128 * 128 + 512) * 4 * 4 * L.max_row_slots
    assert L.total_bytes - L.col_partials_offset >= 2 * 128 * 128 * 4 * 4 * L.max_col_slots
    # grouped-query attention: every column tile needs a partial slot
    pg = B.make_params(16384, 7, 8, 1, 128, 0.0884)
    Lg = B.varlen_attn_workspace_regions(pg)
    assert Lg.max_col_slots >= Lg.max_row_slots + 16384 // 128 + 7
    for bad in (B.make_params(0, 1, 1, 1, 64, 1.0), B.make_params(8, 0, 1, 1, 64, 1.0),
                B.make_params(8, 1, 3, 2, 64, 1.0), B.make_params(8, 1, 1, 1, 96, 1.0),
                B.make_params(8, 1, 1, 1, 64, 0.0), B.make_params(8, 1, 1, 1, 64, float("nan")),
                B.make_params(8, 1, 1, 1, 64, float("inf")), B.make_params(8, 1, 0, 1, 64, 1.0)):
        assert B.varlen_attn_workspace_bytes(bad) == 0


def test_argument_errors_are_reported_on_the_host():
    good = B.make_params(256, 2, 2, 1, 128, 0.1)
    fake = 0x10000  # 16-byte aligned, never dereferenced: validation fails first
    L = B.lib()
    ws = B.varlen_attn_workspace_bytes(good)

    def fwd(p, q=fake, k=fake, v=fake, cu=fake, o=fake, lse=fake, w=fake, wb=ws):
        return L.varlen_attn_fwd(ctypes.byref(p), q, k, v, cu, o, lse, w, wb, None)

    def bwd(p, **kw):
        a = dict(q=fake, k=fake, v=fake, o=fake, lse=fake, do=fake, cu=fake, dq=fake, dk=fake,
                 dv=fake, w=fake, wb=ws)
        a.update(kw)
        return L.varlen_attn_bwd(ctypes.byref(p), a["q"], a["k"], a["v"], a["o"], a["lse"], a["do"],
                                 a["cu"], a["dq"], a["dk"], a["dv"], a["w"], a["wb"], None)

    assert fwd(good, q=None) == B.INVALID_ARG
    assert fwd(good, lse=None) == B.INVALID_ARG
    assert fwd(good, w=None) == B.INVALID_ARG
    assert fwd(B.make_params(256, 2, 3, 2, 128, 0.1)) == B.INVALID_ARG
    assert fwd(B.make_params(256, 2, 2, 1, 128, -1.0)) == B.INVALID_ARG
    assert fwd(B.make_params(256, 2, 2, 1, 80, 0.1)) == B.UNSUPPORTED
    assert fwd(good, k=fake + 8) == B.UNSUPPORTED
    assert fwd(good, wb=ws - 1) == B.WORKSPACE_TOO_SMALL
    assert bwd(good, dv=None) == B.INVALID_ARG
    assert bwd(good, do=fake + 2) == B.UNSUPPORTED
    assert bwd(good, wb=16) == B.WORKSPACE_TOO_SMALL
    assert L.varlen_attn_plan(ctypes.byref(good), None, fake, ws, None) == B.INVALID_ARG
    assert L.varlen_attn_check(None, None) == B.INVALID_ARG


def test_status_strings():
    seen = set()
    for code in (0, -1, -2, -3, -4, -5):
        s = B.varlen_attn_status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 6
    assert B.varlen_attn_status_string(-99) == "unknown status"
