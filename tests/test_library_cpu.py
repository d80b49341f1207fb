"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the
header declares, sizes its workspace, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2605_06374_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="varlen_attn.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(varlen_attn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"varlen_attn_fwd", "varlen_attn_bwd", "varlen_attn_plan", "varlen_attn_check",
            "varlen_attn_workspace_bytes", "varlen_attn_status_string"} <= set(names)
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"
    # the product header declares no measurement aid
    assert not [n for n in names if "rate" in n or "profile" in n or "bench" in n]


def test_bench_header_symbols_are_exported_by_the_two_libraries():
    """include/varlen_attn_bench.h: the event profiler lives in the attention library (its
    launch sites are there), the rate probes in a library of their own."""
    names = declared_functions("varlen_attn_bench.h")
    assert {"varlen_attn_profile", "varlen_attn_profile_read", "varlen_attn_bench_mfma_rate",
            "varlen_attn_bench_lds_rate"} <= set(names)
    lib, bench = ctypes.CDLL(B.LIB_PATH), ctypes.CDLL(B.BENCH_LIB_PATH)
    for n in names:
        owner = bench if n.startswith("varlen_attn_bench_") else lib
        assert hasattr(owner, n), n
    assert not hasattr(lib, "varlen_attn_bench_mfma_rate")


def test_status_strings():
    seen = set()
    for code in (B.OK, B.INVALID_ARG, B.UNSUPPORTED, B.WORKSPACE_TOO_SMALL, B.LAUNCH_FAILED,
                 B.BAD_CU_SEQLENS, B.PLAN_OVERFLOW, B.STATIC_TOO_LARGE):
        text = B.varlen_attn_status_string(code)
        assert text and text != "unknown status" and text not in seen
        seen.add(text)
    assert B.varlen_attn_status_string(-99) == "unknown status"


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


# ------------------------------------------------------------------ capacities of the workspace
def _adversarial_cu_lists():
    import numpy as np
    rng = np.random.default_rng(7)
    yield [1] * 5000                                   # many one-token documents
    yield [129] * 200                                  # every document spills one row into a second tile
    yield [100000]                                     # one huge document
    yield [0, 0, 40000, 0, 1, 127, 128, 129, 0]        # empties next to a long one
    yield [65] * 300 + [9000]
    for _ in range(6):
        yield [int(x) for x in rng.integers(0, 700, size=int(rng.integers(1, 400)))] + [1]


@pytest.mark.parametrize("hq,hkv", [(1, 1), (4, 4), (8, 1), (32, 8)])
def test_workspace_capacities_bound_every_plan(hq, hkv):
    """The capacities depend on (N, B, Hq, Hkv, d) only.  Against the oracle's tile set and
    chain lengths: every tile fits the reduction list; for every chunk length whose cut chains
    fit the slot budget, the units fit the unit arrays (uncut tiles + slots); the chunk length
    the plan starts from (2 * steps / ch <= budget) always fits; and some chunk length fits."""
    from itertools import accumulate
    from oracle import plan as oplan
    for lengths in _adversarial_cu_lists():
        cu = [0] + list(accumulate(lengths))
        n = cu[-1]
        p = B.make_params(n, len(lengths), hq, hkv, 128, 0.1)
        L = B.varlen_attn_workspace_regions(p)
        cap = L.max_row_slots
        tiles = oplan.row_tiles(cu, B.TILE_ROWS)
        assert len(tiles) <= L.max_combine <= n // B.TILE_ROWS + len(lengths)
        for chains in (oplan.row_chain_steps(cu, B.TILE_ROWS, B.STEP_ROWS),
                       oplan.col_chain_steps(cu, B.TILE_ROWS, B.STEP_ROWS)):
            lens = list(chains.values())
            steps = sum(lens)
            assert len(lens) == len(tiles)
            fitting = 0
            for ch in sorted(set([1, 2, 3, 4, 5, 8, 13, 64, 1000] + lens)):
                slots = sum(-(-x // ch) for x in lens if x > ch)
                units = sum(-(-x // ch) for x in lens)
                assert slots <= 2 * steps // ch + 1          # what the plan's first guess relies on
                if slots <= cap:
                    fitting += 1
                    assert units <= L.max_units
                    if hq > hkv:                            # grouped: every tile takes slots
                        assert units <= L.max_col_slots
                if 2 * steps <= ch * cap:
                    assert slots <= cap
            assert fitting >= 1 and sum(-(-x // max(lens)) for x in lens if x > max(lens)) == 0


# ------------------------------------------------------------------ separation of product and checker
def _sources(*roots, suffixes=(".py", ".h", ".hpp", ".hip", ".c", ".cpp")):
    for root in roots:
        for dirpath, _, names in os.walk(os.path.join(ROOT, root)):
            for n in names:
                if n.endswith(suffixes):
                    yield os.path.join(dirpath, n)


def test_product_and_oracle_do_not_reach_into_each_other():
    """The package never imports, includes or loads anything of oracle/, and oracle/ nothing of the
    package; only the tests, the smoke entry and the benchmark's baseline leg use the oracle."""
    import re
    for path in _sources("paper_2605_06374_amd", "include"):
        text = open(path).read()
        assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), path
        assert "oracle/" not in text and "libvarlen_attn_oracle" not in text, path
    for path in _sources("oracle"):
        text = open(path).read()
        assert not re.search(r"^\s*(from|import)\s+paper_2605_06374_amd\b", text, re.M), path
        assert "csrc/" not in text and "libvarlen_attn.so" not in text, path
    bench = open(os.path.join(ROOT, "bench.py")).read()
    first = bench.index("from oracle import")
    assert bench.index("if not args.no_cpu_baseline") < first          # only inside the baseline leg
    assert bench.count("from oracle import") + bench.count("import oracle") == 1
