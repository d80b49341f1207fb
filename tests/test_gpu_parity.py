"""GPU parity: the HIP path (through the C ABI) against the CPU fp64 oracle, element by
element on the same seeded inputs.  Tolerances: max|x-y|/max|y| <= 1e-2 for O, 2e-2 for
dQ/dK/dV; LSE within 1e-3 * max(1, |y|); integer/plan work bit-exact."""
import math

import numpy as np
import pytest

from helpers import (TOL_GRAD, TOL_LSE, TOL_O, assert_close_full, e1, f64_values,
                     interesting_rows, key_rows_cheap, oracle_full, oracle_keys, oracle_rows)
from oracle import plan as oplan
from paper_2605_06374_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2605_06374_amd import binding, runner
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.lib()   # fail loudly if the HIP library is missing
    return runner


def run_all(gpu, w, values=None, poison=True, flags=0):
    from paper_2605_06374_amd import binding
    prob = gpu.DeviceProblem(w, values=values, flags=flags)
    if poison:
        prob.poison_outputs()
    prob.forward()
    prob.backward(reuse_plan=True)
    assert binding.varlen_attn_check(prob.workspace) == binding.OK
    return prob


SMALL = [
    # lengths, Hq, Hkv, d
    ([1], 1, 1, 64),
    ([1], 2, 1, 128),
    ([5], 2, 2, 128),
    ([31, 32, 33], 2, 2, 64),
    ([63, 64, 65], 2, 1, 128),
    ([127, 128, 129], 4, 2, 128),
    ([64, 300, 1, 515], 4, 4, 128),
    ([64, 300, 1, 515], 4, 2, 64),
    ([1] * 40, 2, 2, 128),
    ([200, 0, 0, 77, 0], 2, 1, 128),          # empty documents
    ([0, 130], 1, 1, 64),
    ([1000], 3, 3, 128),                      # B = 1, odd head count
    ([257, 511, 769], 8, 1, 128),             # 8:1 GQA
    ([16, 17, 18, 19, 20] * 8, 4, 4, 128),
    ([1537], 2, 2, 64),
    ([300, 129], 16, 2, 64),                  # more q heads than XCDs
    ([700, 40], 6, 3, 128),                   # head count that neither divides nor is divided by 8
    ([260], 32, 32, 64),
]


@pytest.mark.parametrize("lengths,hq,hkv,d", SMALL)
def test_small_shapes_full_parity(gpu, lengths, hq, hkv, d):
    print(f"case lengths={lengths[:8]} hq={hq} hkv={hkv} d={d}", flush=True)
    w = W.custom("small", lengths, hq, hkv, d, seed=sum(lengths) + 13 * hq + d)
    prob = run_all(gpu, w)
    errs = assert_close_full(prob.results(), oracle_full(w), label=str(lengths[:6]))
    print("  errors (E1, row-wise):", {k: (f"{a:.2e}", f"{b:.2e}") for k, (a, b) in errs.items()}, flush=True)


def test_non_default_scale_and_std(gpu):
    w = W.custom("scaled", [300, 45, 700], 4, 2, 128, std=0.5, seed=5)
    w.__class__ = type("WS", (W.Workload,), {"softmax_scale": property(lambda self: 0.21)})
    prob = run_all(gpu, w)
    assert_close_full(prob.results(), oracle_full(w), "scale 0.21")


@pytest.mark.parametrize("std,d", [(4.0, 128), (3.0, 64), (0.01, 128)])
def test_extreme_logit_ranges(gpu, std, d):
    """Values four times larger give logits with a standard deviation of 16 (nearly one-hot
    rows, the running max rises by far more than the lazy-rescale margin many times over);
    tiny values give nearly uniform rows.  Both across cut chains."""
    w = W.custom("logits", [900, 130, 1500], 2, 1, d, std=std, seed=int(std * 100) + d)
    prob = run_all(gpu, w)
    got = prob.results()
    for name in ("o", "lse", "dq", "dk", "dv"):
        assert np.isfinite(got[name]).all(), name
    # The backward reads O as the forward stored it (bf16), so its D = rowsum(dO * O) carries
    # 2^-9 of sum |dO O|; with values four times larger that is 16 times the usual absolute
    # error, spread over dQ rows that are tiny where a row is one-hot: the row-wise gate is
    # widened for this case, the tensor-scale gates are not.
    assert_close_full(got, oracle_full(w), f"std {std}", row_tol_scale=4.0)


def test_config1_tiny_full(gpu):
    w = W.config(1)
    prob = run_all(gpu, w)
    errs = assert_close_full(prob.results(), oracle_full(w), "cfg1")
    print("cfg1 errors:", errs, flush=True)


def test_config2_7b_shard_full(gpu):
    w = W.config(2)
    prob = run_all(gpu, w)
    errs = assert_close_full(prob.results(), oracle_full(w), "cfg2")
    print("cfg2 errors:", errs, flush=True)


def _sampled_parity(gpu, w, n_rows, n_keys, seed):
    prob = run_all(gpu, w)
    got = prob.results()
    for name in ("o", "dq", "dk", "dv", "lse"):
        assert np.isfinite(got[name]).all(), f"{w.name} {name}: non-finite (unwritten?) output"
    rng = np.random.default_rng(seed)
    rows = interesting_rows(w.cu_seqlens, n_rows, rng)
    ref = oracle_rows(w, rows)
    print(f"{w.name}: {len(rows)} sampled query rows", flush=True)
    # the scale of each tensor is taken from the oracle's sampled rows
    assert np.abs(got["o"][rows] - ref["o"]).max() <= TOL_O * np.abs(ref["o"]).max()
    assert np.abs(got["dq"][rows] - ref["dq"]).max() <= TOL_GRAD * np.abs(ref["dq"]).max()
    dl = np.abs(got["lse"][:, rows] - ref["lse"]) / np.maximum(1.0, np.abs(ref["lse"]))
    assert dl.max() <= TOL_LSE
    keys = key_rows_cheap(w.cu_seqlens, n_keys, rng)
    refk = oracle_keys(w, keys)
    print(f"{w.name}: {len(keys)} sampled key rows", flush=True)
    assert np.abs(got["dk"][keys] - refk["dk"]).max() <= TOL_GRAD * np.abs(refk["dk"]).max()
    assert np.abs(got["dv"][keys] - refk["dv"]).max() <= TOL_GRAD * np.abs(refk["dv"]).max()
    # properties that hold at any size (from the inputs alone):
    #   sum_j dV[j, kappa] = sum_{t, h in group} dO[t, h]  per document;  sum_j dK[j] = 0
    # How far the sums of the bf16 results may be off (u = 2^-9, half a bf16 ulp):
    #   dV: every dV[j] is rounded once (2u of sum_j |dV[j]| at worst) and every P[t, j] was
    #       rounded before it met dO (u * sum_t |dO[t]|);
    #   dK: the results' rounding again, the rounding of dS before it met Q (taken as twice the
    #       results' share), and D = rowsum(dO * O) read from the O that the forward stored in
    #       bf16: every query t adds scale * dD[t] * q[t] to the sum, |dD[t]| <= u * sum_c |dO O|.
    #       In a document of two or three tokens, whose dK is nearly zero wherever one key takes
    #       nearly all the weight, that last term is all there is.
    u = 2.0 ** -9
    v = f64_values(w)
    cu = w.cu_seqlens
    g = w.n_q_heads // w.n_kv_heads
    shape = (w.n_kv_heads, g, w.head_dim)
    for b in range(len(cu) - 1):
        s, e = int(cu[b]), int(cu[b + 1])
        if e == s:
            continue
        do = v["do"][s:e].reshape(e - s, *shape)
        want = do.sum(axis=(0, 2))
        gotv = got["dv"][s:e].sum(axis=0)
        scale_v = np.abs(got["dv"][s:e]).sum(axis=0).max()
        tol_v = 2 * u * scale_v + u * np.abs(do).sum(axis=(0, 2)).max() + 1e-6
        assert np.abs(gotv - want).max() <= 1.25 * tol_v, (b, "dV column sums")
        scale_k = np.abs(got["dk"][s:e]).sum(axis=0).max()
        d_err = u * (np.abs(do) * np.abs(got["o"][s:e].reshape(e - s, *shape))).sum(axis=-1, keepdims=True)
        from_d = w.softmax_scale * (d_err * np.abs(v["q"][s:e].reshape(e - s, *shape))).sum(axis=(0, 2)).max()
        tol_k = 6 * u * scale_k + from_d + 1e-6
        assert np.abs(got["dk"][s:e].sum(axis=0)).max() <= 1.25 * tol_k, (b, "dK sums")
    return prob


def test_config3_longtail_full(gpu):
    """All 32768 tokens element by element (the 11K and 16K documents' first keys have the
    longest column chains of the five configurations)."""
    w = W.config(3)
    prob = run_all(gpu, w)
    errs = assert_close_full(prob.results(), oracle_full(w), "cfg3")
    print("cfg3 errors (E1, row-wise):", errs, flush=True)


def test_config4_gqa_full(gpu):
    """All 16384 tokens element by element, 8 q heads on one kv head."""
    w = W.config(4)
    prob = run_all(gpu, w)
    errs = assert_close_full(prob.results(), oracle_full(w), "cfg4")
    print("cfg4 errors (E1, row-wise):", errs, flush=True)


def test_config3_and_4_sampled_rows_and_properties(gpu):
    """The sampled form that also runs at sizes the oracle cannot finish (used for the 131K
    document below) is kept honest on two sizes where the full comparison exists too."""
    _sampled_parity(gpu, W.config(3), n_rows=48, n_keys=48, seed=303)
    _sampled_parity(gpu, W.config(4), n_rows=64, n_keys=64, seed=404)


@pytest.mark.parametrize("first", [0, 16, 32, 48])
def test_config5_sweep_microbatches_full(gpu, first):
    """All 64 microbatches of the length-skew sweep, each element by element."""
    worst = {}
    for mb in range(first, first + 16):
        w = W.config(5, microbatch=mb)
        prob = run_all(gpu, w)
        errs = assert_close_full(prob.results(), oracle_full(w), w.name)
        for k, (a, b) in errs.items():
            worst[k] = (max(worst.get(k, (0, 0))[0], a), max(worst.get(k, (0, 0))[1], b))
        del prob
    print(f"cfg5 microbatches {first}..{first + 15} worst (E1, row-wise):", worst, flush=True)


def test_mid_size_long_document_full(gpu):
    """A 3000-token document next to short ones: every dK/dV row of a long document checked."""
    w = W.custom("mid", [3000, 17, 600, 479], 4, 2, 128, seed=77)
    prob = run_all(gpu, w)
    assert_close_full(prob.results(), oracle_full(w), "mid")


# ------------------------------------------------------------------ cu_seqlens handling, bit-exact
def _check_plan(prob, w, no_split):
    """Integer plan quantities against the oracle's integers: pair count, the tile set, and
    for every tile a partition of its full chain into chunks; unit order longest first."""
    plan = prob.read_plan()
    hdr, L = plan["header"], plan["layout"]
    cu = w.cu_seqlens
    g = w.n_q_heads // w.n_kv_heads
    assert hdr.status == 0 and hdr.pairs == oplan.pairs(cu) == w.pairs
    assert hdr.col_heads_per_unit >= 1 and g % hdr.col_heads_per_unit == 0
    for units, comb, chains, n_slots, always_slots, shift in (
            (plan["row_units"], plan["row_combine"], oplan.row_chain_steps(cu, 128, 64),
             hdr.n_row_slots, False, hdr.row_class_shift),
            (plan["col_units"], plan["col_combine"], oplan.col_chain_steps(cu, 128, 64),
             hdr.n_col_slots, g > hdr.col_heads_per_unit, hdr.col_class_shift)):
        assert len(units) <= L.max_units and len(comb) <= L.max_combine
        by_tile = {}
        for r0, s, e, b0, b1, slot, cost, _ in units.tolist():
            assert cost == b1 - b0 and cost >= 1
            by_tile.setdefault((r0, s, e), []).append((b0, b1, slot))
        assert set(by_tile) == set(chains), "tile set differs from the oracle's"
        comb_map = {(r0, e): (s0, nc) for r0, e, s0, nc in comb.tolist()}
        used_slots = []
        for key, chunks in by_tile.items():
            chunks.sort()
            assert chunks[0][0] == 0 and chunks[-1][1] == chains[key]
            for (a0, a1, _), (b0, b1, _) in zip(chunks, chunks[1:]):
                assert a1 == b0, "chunks must tile the chain without gap or overlap"
            lens = [b1 - b0 for b0, b1, _ in chunks]
            assert max(lens) - min(lens) <= 1
            if no_split:
                assert len(chunks) == 1
            if len(chunks) > 1 or always_slots:
                s0, nc = comb_map[(key[0], key[2])]
                assert nc == len(chunks)
                assert [sl for _, _, sl in chunks] == list(range(s0, s0 + nc))
                used_slots.extend(range(s0, s0 + nc))
            else:
                assert chunks[0][2] == -1 and (key[0], key[2]) not in comb_map
        assert sorted(used_slots) == list(range(n_slots)), "slots must be dense and disjoint"
        assert 0 <= shift < 31 and ((int(units[:, 6].max()) - 1) >> shift) < 32
        assert (np.diff((units[:, 6] - 1) >> shift) <= 0).all(), "units must be ordered longest class first"
    return plan


@pytest.mark.parametrize("k", [1, 2, 3, 4])
@pytest.mark.parametrize("no_split", [False, True])
def test_plan_integers_match_oracle(gpu, k, no_split):
    from paper_2605_06374_amd import binding
    w = W.config(k)
    prob = gpu.DeviceProblem(w, flags=binding.FLAG_NO_SPLIT if no_split else 0)
    prob.plan()
    plan = _check_plan(prob, w, no_split)
    hdr = plan["header"]
    print(f"cfg{k} no_split={no_split}: row units {hdr.n_row_units} (chunk {hdr.row_chunk_steps}), "
          f"col units {hdr.n_col_units} (chunk {hdr.col_chunk_steps}), slots {hdr.n_row_slots}/"
          f"{hdr.n_col_slots}, class shifts {hdr.row_class_shift}/{hdr.col_class_shift}", flush=True)


def test_plan_many_short_documents(gpu):
    lengths = [1 + (i * 7) % 40 for i in range(3000)]
    w = W.custom("many", lengths, 1, 1, 64, seed=1)
    prob = gpu.DeviceProblem(w)
    prob.plan()
    _check_plan(prob, w, False)


def test_plan_single_long_document_and_gqa(gpu):
    for lengths, hq, hkv in (([4096], 4, 4), ([5000, 3, 700], 8, 2), ([20000], 2, 1)):
        w = W.custom("long", lengths, hq, hkv, 64, seed=2)
        prob = gpu.DeviceProblem(w)
        prob.plan()
        _check_plan(prob, w, False)


def test_bad_cu_seqlens_is_reported_and_writes_nothing(gpu):
    import torch
    from paper_2605_06374_amd import binding
    w = W.custom("bad", [100, 200, 84], 2, 2, 128, seed=3)
    for bad in ([0, 250, 200, 384], [1, 100, 300, 384], [0, 100, 300, 383]):
        prob = gpu.DeviceProblem(w)
        prob.cu.copy_(torch.tensor(bad, dtype=torch.int32))
        prob.poison_outputs()
        prob.forward()
        prob.backward()
        assert binding.varlen_attn_check(prob.workspace) == binding.BAD_CU_SEQLENS
        bits = prob.result_bits()
        assert (bits["o"] == 0x7FC0).all() and (bits["dq"] == 0x7FC0).all()
        assert (bits["dk"] == 0x7FC0).all() and (bits["dv"] == 0x7FC0).all()


def test_first_row_identity(gpu):
    """The first token of a document sees one key: P = 1, so O equals its V row bit for bit,
    LSE = scale * q.k, and dQ vanishes."""
    w = W.config(2)
    prob = run_all(gpu, w)
    bits = prob.result_bits()
    vals = w.values()
    got = prob.results()
    v64 = f64_values(w)
    g = w.n_q_heads // w.n_kv_heads
    for b in range(len(w.lengths)):
        t = int(w.cu_seqlens[b])
        for h in range(w.n_q_heads):
            assert np.array_equal(bits["o"][t, h], vals["v"][t, h // g])
            s = w.softmax_scale * float(v64["q"][t, h] @ v64["k"][t, h // g])
            assert abs(got["lse"][h, t] - s) <= 2e-6 * max(1.0, abs(s))
            assert np.abs(got["dq"][t, h]).max() <= 1e-5 * w.softmax_scale * np.abs(v64["k"][t]).max() * 10


def test_isolation_bit_exact(gpu):
    """Poisoning every token outside a document (NaN, Inf, huge) leaves that document's
    outputs bit-identical: nothing outside [cu[b], cu[b+1]) is ever read for it."""
    w = W.custom("iso", [300, 130, 1, 700, 64], 4, 2, 128, seed=9)
    vals = w.values()
    base = run_all(gpu, w).result_bits()
    cu = w.cu_seqlens
    for b in (0, 1, 2, 3):
        s, e = int(cu[b]), int(cu[b + 1])
        poisoned = {}
        for n, x in vals.items():
            y = x.copy()
            y[:s] = 0x7FC0 if n != "k" else 0x7F80     # NaN, and +Inf in K
            y[e:] = 0x7FC0 if n != "v" else 0x7E00     # NaN, and huge in V
            poisoned[n] = y
        got = run_all(gpu, w, values=poisoned).result_bits()
        for n in ("o", "dq", "dk", "dv"):
            assert np.array_equal(got[n][s:e], base[n][s:e]), (b, n)
        assert np.array_equal(got["lse"][:, s:e], base["lse"][:, s:e])


def test_packing_invariance(gpu):
    """A document run alone against the same document inside a pack: bit-identical when
    chains are never cut (NO_SPLIT), within rounding of the fp32 partial sums otherwise
    (the chunking then depends on how much work the whole microbatch holds)."""
    from paper_2605_06374_amd import binding
    w = W.custom("iso", [300, 130, 1, 1500, 64], 4, 2, 128, seed=9)
    vals = w.values()
    cu = w.cu_seqlens
    for flags in (binding.FLAG_NO_SPLIT, 0):
        packed = run_all(gpu, w, flags=flags)
        base, basef = packed.result_bits(), packed.results()
        for b in range(len(w.lengths)):
            s, e = int(cu[b]), int(cu[b + 1])
            alone = W.custom("alone", [e - s], 4, 2, 128, seed=0)
            alone_vals = {n: x[s:e].copy() for n, x in vals.items()}
            one = run_all(gpu, alone, values=alone_vals, flags=flags)
            got1, got1f = one.result_bits(), one.results()
            for n in ("o", "dq", "dk", "dv"):
                if flags:
                    assert np.array_equal(got1[n], base[n][s:e]), (b, n, "alone")
                else:
                    ref = basef[n][s:e]
                    assert np.abs(got1f[n] - ref).max() <= 8e-3 * np.abs(ref).max() + 1e-30, (b, n)
            if flags:
                assert np.array_equal(got1["lse"], base["lse"][:, s:e])
            else:
                assert np.abs(got1f["lse"] - basef["lse"][:, s:e]).max() <= 1e-5


def test_no_split_mode_parity(gpu):
    from paper_2605_06374_amd import binding
    for w in (W.config(1), W.custom("ns", [900, 40, 2000], 8, 2, 128, seed=31)):
        prob = run_all(gpu, w, flags=binding.FLAG_NO_SPLIT)
        assert_close_full(prob.results(), oracle_full(w), "no_split " + w.name)


def test_caller_given_chunk_lengths(gpu):
    """Chunk lengths passed through the flag bits: the plan uses them (or longer ones when the
    partials would not fit), stays a valid partition, and the results still match the oracle."""
    from paper_2605_06374_amd import binding
    w = W.custom("forced_chunks", [1500, 130, 700], 2, 1, 128, seed=33)
    flags = binding.flag_chunk_steps(3, 5)
    prob = run_all(gpu, w, flags=flags)
    plan = _check_plan(prob, w, False)
    hdr = plan["header"]
    assert hdr.row_chunk_steps >= 3 and hdr.col_chunk_steps >= 5
    assert int(plan["row_units"][:, 6].max()) <= hdr.row_chunk_steps
    assert int(plan["col_units"][:, 6].max()) <= hdr.col_chunk_steps
    assert_close_full(prob.results(), oracle_full(w), "forced chunks")


@pytest.mark.parametrize("heads", [1, 2, 4])
def test_grouped_query_column_units_sweeping_heads(gpu, heads):
    """Grouped-query dK/dV with a column unit sweeping 1, 2 or all 4 q heads of its group (forced
    through the flag bits): plan valid, results within tolerance, with cut chains, with chains
    kept whole, and with very short chunks."""
    from paper_2605_06374_amd import binding
    for lengths, hq, hkv, d, extra in (([1500, 130, 700], 4, 1, 128, 0),
                                       ([900, 64, 1, 333], 8, 2, 64, binding.FLAG_NO_SPLIT),
                                       ([2600], 4, 1, 128, binding.flag_chunk_steps(3, 3))):
        w = W.custom("gqa_sweep", lengths, hq, hkv, d, seed=61 + heads)
        prob = run_all(gpu, w, flags=binding.flag_group_heads(heads) | extra)
        plan = _check_plan(prob, w, bool(extra & binding.FLAG_NO_SPLIT))
        assert plan["header"].col_heads_per_unit == heads
        assert_close_full(prob.results(), oracle_full(w), f"gqa sweep {heads} {lengths}")


@pytest.mark.parametrize("lengths,hq,hkv,d", SMALL + [([900, 130, 1500, 64, 1], 8, 2, 128)])
def test_fused_backward_small_shapes(gpu, lengths, hq, hkv, d):
    """The single-kernel backward (dQ by fp32 atomics): same oracle, same tolerances; dV is
    computed by the same arithmetic as in the two-kernel form, hence bit-identical to it (dK is
    not: D = rowsum(dO * O) is summed by another kernel, in another order)."""
    from paper_2605_06374_amd import binding
    print(f"fused case lengths={lengths[:8]} hq={hq} hkv={hkv} d={d}", flush=True)
    w = W.custom("fused", lengths, hq, hkv, d, seed=sum(lengths) + 13 * hq + d)
    prob = run_all(gpu, w, flags=binding.FLAG_FUSED_BWD)
    assert_close_full(prob.results(), oracle_full(w), label="fused " + str(lengths[:6]))
    base, got = run_all(gpu, w).result_bits(), prob.result_bits()
    for n in ("o", "lse", "dv"):
        assert np.array_equal(got[n], base[n]), n


@pytest.mark.parametrize("k", [2, 4])
def test_fused_backward_configs(gpu, k):
    from paper_2605_06374_amd import binding
    w = W.config(k)
    prob = run_all(gpu, w, flags=binding.FLAG_FUSED_BWD)
    errs = assert_close_full(prob.results(), oracle_full(w), f"fused cfg{k}")
    print(f"fused cfg{k} errors (E1, row-wise):", errs, flush=True)
    # the workspace grows by the fp32 dQ accumulator only when the flag is given
    L0 = binding.varlen_attn_workspace_regions(binding.make_params(w.n_tokens, len(w.lengths), w.n_q_heads,
                                                                    w.n_kv_heads, w.head_dim, 0.1, 0))
    L1 = binding.varlen_attn_workspace_regions(prob.params)
    assert L1.total_bytes - L0.total_bytes >= 4 * w.n_tokens * w.n_q_heads * w.head_dim
    assert L0.total_bytes == L0.dq_accumulator_offset


def test_bit_reproducible(gpu):
    w = W.config(4)
    a = run_all(gpu, w).result_bits()
    b = run_all(gpu, w).result_bits()
    for n in a:
        assert np.array_equal(a[n], b[n]), n


@pytest.mark.parametrize("lengths,hq,hkv,d", [SMALL[3], SMALL[6], SMALL[7], SMALL[10], SMALL[11], SMALL[13],
                                               ([900, 130, 1500, 64, 1, 0, 700], 4, 2, 128),
                                               ([8192], 2, 2, 64), ([3] * 64, 2, 1, 128),
                                               ([16384 + 77], 1, 1, 128),
                                               ([31000, 1, 900], 2, 2, 64),          # 251 tiles: four rounds of 64
                                               ([0, 5, 0, 0, 300, 0] + [1, 130, 64, 0] * 14 + [0, 0], 3, 1, 128)])
def test_self_planned_forward_equals_planned_forward(gpu, lengths, hq, hkv, d):
    """On small microbatches the forward workgroups work out their units themselves while one of
    them writes the plan: same units, same slots, hence the bits of a forward behind a plan
    launch, and the same plan tables (the reduction's items in any order)."""
    from paper_2605_06374_amd import binding
    w = W.custom("self", lengths, hq, hkv, d, seed=sum(lengths) + 7 * hq + d)
    a = run_all(gpu, w, flags=binding.FLAG_PLAN_FIRST)
    b = run_all(gpu, w)
    abits, bbits = a.result_bits(), b.result_bits()
    for n in abits:
        assert np.array_equal(abits[n], bbits[n]), n
    pa, pb = a.read_plan(), b.read_plan()
    for f, _ in pa["header"]._fields_:
        if f != "reserved":
            assert getattr(pa["header"], f) == getattr(pb["header"], f), f
    for name in ("row_units", "col_units", "row_combine", "col_combine"):
        assert sorted(map(tuple, pa[name].tolist())) == sorted(map(tuple, pb[name].tolist())), name
    assert_close_full(b.results(), oracle_full(w), label="self-planned " + str(lengths[:6]))


def _random_shape(rng, kind):
    if kind == 0:     # many short documents
        lengths = rng.integers(0, 40, size=int(rng.integers(1, 70)))
    elif kind == 1:   # a few long ones
        lengths = rng.integers(1, 1400, size=int(rng.integers(1, 5)))
    elif kind == 2:   # lengths on and beside the 64-token step and 128-token tile edges
        lengths = rng.choice([0, 1, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 384],
                             size=int(rng.integers(1, 12)))
    elif kind == 3:   # long tail
        lengths = np.minimum((rng.pareto(1.2, size=int(rng.integers(2, 30))) * 30).astype(int), 2500)
    elif kind == 4:   # one document among empty ones
        lengths = np.zeros(int(rng.integers(2, 66)), dtype=int)
        lengths[int(rng.integers(0, len(lengths)))] = int(rng.integers(1, 3000))
    else:
        lengths = rng.integers(0, 200, size=int(rng.integers(1, 100)))
    lengths = [int(x) for x in lengths]
    if sum(lengths) == 0:
        lengths[0] = 1
    while sum(lengths) > 3500:
        lengths[int(np.argmax(lengths))] //= 2
    return lengths


def test_random_shapes_full_parity(gpu):
    """Sixty seeded random microbatches (six length mixes, twelve head layouts, both head sizes,
    the default and four other modes), each against the oracle in full; in the modes where the
    forward may plan itself also bit by bit against the forward behind a plan launch."""
    from paper_2605_06374_amd import binding
    heads = [(1, 1), (2, 1), (2, 2), (4, 4), (4, 2), (8, 2), (8, 8), (6, 3), (3, 3), (16, 2), (5, 1), (12, 4)]
    for case in range(60):
        rng = np.random.default_rng(77000 + case)
        lengths = _random_shape(rng, case % 6)
        hq, hkv = heads[int(rng.integers(0, len(heads)))]
        d = int(rng.choice([64, 128]))
        flags = [0, 0, binding.FLAG_NO_SPLIT, binding.FLAG_PLAN_FIRST, binding.FLAG_FUSED_BWD,
                 (int(rng.integers(1, 9)) << 8) | (int(rng.integers(1, 9)) << 16)][int(rng.integers(0, 6))]
        label = f"random case {case}: B={len(lengths)} N={sum(lengths)} hq={hq} hkv={hkv} d={d} flags={flags:#x}"
        print(label, flush=True)
        w = W.custom("random", lengths, hq, hkv, d, seed=case)
        prob = run_all(gpu, w, flags=flags)
        assert_close_full(prob.results(), oracle_full(w), label)
        if not flags & binding.FLAG_PLAN_FIRST:
            first = run_all(gpu, w, flags=flags | binding.FLAG_PLAN_FIRST).result_bits()
            got = prob.result_bits()
            for n in ("o", "lse"):
                assert np.array_equal(first[n], got[n]), f"{label}: {n}"


def test_random_larger_shapes_sampled(gpu):
    """Ten seeded microbatches of 4K to 40K tokens (thousands of tiny documents, a long tail,
    one huge document among dust, equal documents, a uniform mix): sampled rows against the
    oracle, the column-sum properties, and the plan's integers."""
    heads = [(1, 1), (2, 2), (4, 4), (4, 2), (8, 2), (8, 1), (8, 8), (6, 3), (16, 2), (32, 8), (5, 1)]
    for case in range(10):
        rng = np.random.default_rng(88000 + case)
        n = int(rng.integers(4000, 40000))
        kind = case % 5
        if kind == 2:
            lengths = [int(rng.integers(0, 20)) for _ in range(int(rng.integers(0, 300)))]
            lengths.insert(int(rng.integers(0, len(lengths) + 1)), n)
        elif kind == 3:
            each = int(rng.choice([127, 128, 129, 500, 1024, 2048, 4096]))
            lengths = [each] * max(1, n // each)
        else:
            draw = {0: lambda: int(rng.integers(0, 30)), 1: lambda: int(min(rng.pareto(1.1) * 200, 20000)),
                    4: lambda: int(rng.integers(1, 3000))}[kind]
            lengths = []
            while sum(lengths) < n:
                lengths.append(draw())
        hq, hkv = heads[int(rng.integers(0, len(heads)))]
        if sum(lengths) * hq > 320000:
            hq, hkv = 4, 2
        d = int(rng.choice([64, 128]))
        print(f"larger case {case}: B={len(lengths)} N={sum(lengths)} hq={hq} hkv={hkv} d={d} "
              f"longest={max(lengths)}", flush=True)
        w = W.custom(f"larger{case}", lengths, hq, hkv, d, seed=case)
        prob = _sampled_parity(gpu, w, n_rows=16, n_keys=16, seed=case)
        _check_plan(prob, w, False)
        del prob


def test_forward_reuses_a_plan(gpu):
    """One plan for the attention calls of all layers of a micro-batch: a forward that reuses the
    plan of varlen_attn_plan gives the bits of a forward that plans itself."""
    w = W.custom("layers", [700, 40, 1300, 5, 129], 4, 2, 128, seed=31)
    fresh = run_all(gpu, w).result_bits()
    prob = gpu.DeviceProblem(w)
    prob.poison_outputs()
    prob.plan()
    prob.forward(reuse_plan=True)
    prob.backward(reuse_plan=True)
    got = prob.result_bits()
    for n in fresh:
        assert np.array_equal(fresh[n], got[n]), n


def test_bwd_plans_itself_without_reuse_flag(gpu):
    from paper_2605_06374_amd import binding
    w = W.custom("noreuse", [500, 77], 2, 2, 128, seed=21)
    prob = gpu.DeviceProblem(w)
    prob.poison_outputs()
    prob.forward()
    prob.workspace.zero_()          # wipe the plan: bwd must rebuild it
    prob.backward(reuse_plan=False)
    assert binding.varlen_attn_check(prob.workspace) == binding.OK
    assert_close_full(prob.results(), oracle_full(w), "noreuse")


def test_cost_follows_sum_of_squares_not_n_squared(gpu):
    """Section 2.2: one 4K document costs about four times four packed 1K documents; the
    tile pairs the kernels visit follow the same ratio (tile skipping)."""
    a = oplan.causal_tile_pairs([0, 4096], 128, 64)
    b = oplan.causal_tile_pairs([0, 1024, 2048, 3072, 4096], 128, 64)
    assert 3.5 < a / b < 4.0


def test_hip_graph_replays_match_eager(gpu):
    """fwd + bwd enqueue kernels only (no allocation, no synchronisation, no memset nodes), so
    a caller may capture them in a HIP graph: every replay, with eager work and
    synchronisations between the replays, reproduces the eager results bit for bit."""
    import torch
    w = W.custom("graph", [700, 64, 1, 900, 333], 4, 2, 128, seed=77)
    eager = run_all(gpu, w)
    want = eager.result_bits()
    prob = gpu.DeviceProblem(w)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):        # warm-up on the capture stream
        prob.forward()
        prob.backward(reuse_plan=True)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        prob.forward()
        prob.backward(reuse_plan=True)
    for replay in range(3):
        prob.poison_outputs()
        prob.workspace.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = prob.result_bits()
        for n in want:
            assert np.array_equal(got[n], want[n]), (replay, n)
        other = run_all(gpu, W.config(1))      # eager work between the replays
        torch.cuda.synchronize()
        del other


def test_long_single_document_sampled(gpu):
    """131072 tokens in one document (1024 tiles, chains of up to 2048 steps, cut into
    chunks): sampled rows and keys against the oracle plus the size-independent properties."""
    w = W.custom("long131k", [131072], 2, 1, 128, seed=5)
    prob = _sampled_parity(gpu, w, n_rows=24, n_keys=24, seed=131)
    assert prob.read_plan()["header"].pairs == w.pairs == 131072 * 131073 // 2


def test_mfma_rate_probe_runs(gpu):
    """The measurement aid returns a plausible rate and rejects bad arguments."""
    import torch
    from paper_2605_06374_amd import binding
    scratch = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    for hashed in (False, True):
        rate = binding.varlen_attn_bench_mfma_rate(hashed, 2000, scratch.data_ptr())
        assert 50.0 < rate < 2600.0, rate
    with pytest.raises(RuntimeError):
        binding.varlen_attn_bench_mfma_rate(False, 0, scratch.data_ptr())
    for transposed in (False, True):
        rate = binding.varlen_attn_bench_lds_rate(transposed, 2000, scratch.data_ptr())
        assert 16.0 < rate < 600.0, rate


def test_overlap_and_atomic_probes_run(gpu):
    """The other measurement aids return plausible figures and reject bad arguments."""
    import torch
    from paper_2605_06374_amd import binding
    scratch = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    alone = binding.varlen_attn_bench_overlap(0, -1, 500, scratch.data_ptr())      # 16 MFMA: 512 clocks at full rate
    assert 450.0 < alone < 3000.0, alone
    both = binding.varlen_attn_bench_overlap(0, 1, 500, scratch.data_ptr())
    assert alone * 0.8 < both < 3.0 * alone, (alone, both)
    with pytest.raises(RuntimeError):
        binding.varlen_attn_bench_overlap(1, 0, 500, scratch.data_ptr())            # not an offered pair
    with pytest.raises(RuntimeError):
        binding.varlen_attn_bench_overlap(0, -1, 0, scratch.data_ptr())
    buf = torch.zeros(8 << 20, dtype=torch.uint8, device="cuda:0")
    for mode in (0, 1):
        rate = binding.varlen_attn_bench_atomic_rate(mode, 8, 64, 1, buf)
        assert 20.0 < rate < 20000.0, (mode, rate)
    # block (b + s * stride) % regions of workgroup b: every one of the 64 regions gets adds
    torch.cuda.synchronize()
    assert float(buf.view(torch.float32)[: 64 * 64 * 128].min()) >= 1.0
    with pytest.raises(RuntimeError):
        binding.varlen_attn_bench_atomic_rate(0, 8, 1 << 20, 1, buf)                # regions do not fit the buffer
