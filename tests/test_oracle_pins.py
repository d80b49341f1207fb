"""Pins of the CPU fp64 oracle against things other than itself: dense brute force with an
explicit mask, torch autograd, finite differences, closed forms and invariants.  Each pin
is chosen so that a plausible mistake (dropped term, wrong sign or index, transposed
operand, wrong head mapping, off-by-one at a document edge) fails at least one of them."""
import math
import os

import numpy as np
import pytest

from oracle import plan as oplan

HERE = os.path.dirname(os.path.abspath(__file__))


def rand_problem(rng, lengths, hq, hkv, d, scale_in=1.0):
    n = int(sum(lengths))
    q = rng.standard_normal((n, hq, d)) * scale_in
    k = rng.standard_normal((n, hkv, d)) * scale_in
    v = rng.standard_normal((n, hkv, d))
    do = rng.standard_normal((n, hq, d))
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lengths)
    return q, k, v, do, cu


def dense_reference(q, k, v, do, cu, scale):
    """Dense N x N masked softmax attention and its gradient, written with whole-matrix
    numpy operations and an explicit mask built from per-token document ids."""
    n, hq, d = q.shape
    hkv = k.shape[1]
    g = hq // hkv
    doc = np.asarray(oplan.doc_of_token(cu))
    idx = np.arange(n)
    allowed = (doc[:, None] == doc[None, :]) & (idx[None, :] <= idx[:, None])
    o = np.zeros_like(q); lse = np.zeros((hq, n))
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    for h in range(hq):
        kap = h // g
        s = scale * q[:, h, :] @ k[:, kap, :].T
        s = np.where(allowed, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        z = e.sum(axis=1, keepdims=True)
        p = e / z
        lse[h] = (m + np.log(z))[:, 0]
        o[:, h, :] = p @ v[:, kap, :]
        dp = do[:, h, :] @ v[:, kap, :].T
        ds = p * (dp - (p * dp).sum(axis=1, keepdims=True))
        dq[:, h, :] = scale * ds @ k[:, kap, :]
        dk[:, kap, :] += scale * ds.T @ q[:, h, :]
        dv[:, kap, :] += p.T @ do[:, h, :]
    return o, lse, dq, dk, dv


CASES = [
    ([1], 1, 1, 4),
    ([5], 2, 2, 8),
    ([1, 1, 1], 2, 1, 4),
    ([3, 1, 7, 2], 4, 2, 8),
    ([17, 1, 30, 16], 4, 1, 16),
    ([9, 0, 4, 0, 11], 2, 2, 8),      # empty documents
    ([64], 3, 3, 16),
]


@pytest.mark.parametrize("lengths,hq,hkv,d", CASES)
def test_brute_force_dense(oracle, lengths, hq, hkv, d):
    rng = np.random.default_rng(7 + sum(lengths) + hq)
    q, k, v, do, cu = rand_problem(rng, lengths, hq, hkv, d)
    scale = 1.0 / math.sqrt(d)
    o, lse = oracle.fwd(q, k, v, cu, scale)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, scale)
    ro, rlse, rdq, rdk, rdv = dense_reference(q, k, v, do, cu, scale)
    for a, b in ((o, ro), (lse, rlse), (dq, rdq), (dk, rdk), (dv, rdv)):
        np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-12)


def test_torch_autograd_block_diagonal(oracle):
    """Independent second opinion: torch's own softmax + autograd in fp64 on CPU."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(11)
    lengths, hq, hkv, d = [13, 1, 40, 10], 4, 2, 16
    q, k, v, do, cu = rand_problem(rng, lengths, hq, hkv, d)
    scale = 0.37   # deliberately not 1/sqrt(d): the scale must be taken from the argument
    n = q.shape[0]
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    doc = torch.tensor(oplan.doc_of_token(cu))
    idx = torch.arange(n)
    allowed = (doc[:, None] == doc[None, :]) & (idx[None, :] <= idx[:, None])
    kk = tk.repeat_interleave(hq // hkv, dim=1)
    vv = tv.repeat_interleave(hq // hkv, dim=1)
    s = torch.einsum("thc,jhc->htj", tq, kk) * scale
    s = s.masked_fill(~allowed[None], float("-inf"))
    to = torch.einsum("htj,jhc->thc", torch.softmax(s, dim=-1), vv)
    tlse = torch.logsumexp(s, dim=-1)
    (to * torch.tensor(do)).sum().backward()
    o, lse = oracle.fwd(q, k, v, cu, scale)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, scale)
    np.testing.assert_allclose(o, to.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(lse, tlse.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_single_document_is_plain_causal_sdpa(oracle):
    """B = 1 reduces to textbook causal scaled-dot-product attention (library routine)."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(12)
    q, k, v, do, cu = rand_problem(rng, [48], 2, 2, 32)
    scale = 1.0 / math.sqrt(32)
    tq, tk, tv = (torch.tensor(x.transpose(1, 0, 2)[None], dtype=torch.float64) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    o, _ = oracle.fwd(q, k, v, cu, scale)
    np.testing.assert_allclose(o, ref[0].numpy().transpose(1, 0, 2), rtol=1e-11, atol=1e-12)


def test_softmax_rows_sum_to_one(oracle):
    rng = np.random.default_rng(13)
    lengths, hq, hkv, d = [33, 7, 1, 90], 4, 2, 16
    q, k, v, do, cu = rand_problem(rng, lengths, hq, hkv, d, scale_in=2.0)
    scale = 1.0 / math.sqrt(d)
    _, lse = oracle.fwd(q, k, v, cu, scale)
    doc = oplan.doc_of_token(cu)
    for h in range(hq):
        kap = h // (hq // hkv)
        for t in range(q.shape[0]):
            s = scale * k[cu[doc[t]]:t + 1, kap, :] @ q[t, h, :]
            assert abs(np.exp(s - lse[h, t]).sum() - 1.0) < 1e-13


def test_packing_invariance(oracle):
    rng = np.random.default_rng(14)
    lengths, hq, hkv, d = [20, 3, 41, 1, 16], 4, 2, 8
    q, k, v, do, cu = rand_problem(rng, lengths, hq, hkv, d)
    scale = 1.0 / math.sqrt(d)
    o, lse = oracle.fwd(q, k, v, cu, scale)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, scale)
    for b, l in enumerate(lengths):
        sl = slice(cu[b], cu[b + 1])
        cu1 = np.array([0, l], dtype=np.int32)
        o1, lse1 = oracle.fwd(q[sl], k[sl], v[sl], cu1, scale)
        dq1, dk1, dv1 = oracle.bwd(q[sl], k[sl], v[sl], do[sl], cu1, scale)
        assert np.array_equal(o[sl], o1) and np.array_equal(lse[:, sl], lse1)
        assert np.array_equal(dq[sl], dq1) and np.array_equal(dk[sl], dk1)
        assert np.array_equal(dv[sl], dv1)


def test_gqa_equals_explicit_replication(oracle):
    rng = np.random.default_rng(15)
    lengths, hq, hkv, d = [25, 6, 33], 8, 2, 8
    g = hq // hkv
    q, k, v, do, cu = rand_problem(rng, lengths, hq, hkv, d)
    scale = 1.0 / math.sqrt(d)
    o, lse = oracle.fwd(q, k, v, cu, scale)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, scale)
    kr, vr = np.repeat(k, g, axis=1), np.repeat(v, g, axis=1)   # head h <- kv head h // g
    o2, lse2 = oracle.fwd(q, kr, vr, cu, scale)
    dq2, dk2, dv2 = oracle.bwd(q, kr, vr, do, cu, scale)
    np.testing.assert_allclose(o, o2, rtol=0, atol=0)
    np.testing.assert_allclose(lse, lse2, rtol=0, atol=0)
    np.testing.assert_allclose(dq, dq2, rtol=1e-13, atol=1e-14)
    n = q.shape[0]
    np.testing.assert_allclose(dk, dk2.reshape(n, hkv, g, d).sum(axis=2), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dv, dv2.reshape(n, hkv, g, d).sum(axis=2), rtol=1e-12, atol=1e-13)


def _loss(oracle, q, k, v, do, cu, scale):
    o, _ = oracle.fwd(q, k, v, cu, scale)
    return float((o * do).sum())


def test_finite_differences_all_coordinates(oracle):
    rng = np.random.default_rng(16)
    lengths, hq, hkv, d = [7, 1, 11, 4], 2, 1, 4
    q, k, v, do, cu = rand_problem(rng, lengths, hq, hkv, d)
    scale = 0.5
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, scale)
    for name, x, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            x0 = x[i]
            h = 1e-5 * max(1.0, abs(x0))
            x[i] = x0 + h; lp = _loss(oracle, q, k, v, do, cu, scale)
            x[i] = x0 - h; lm = _loss(oracle, q, k, v, do, cu, scale)
            x[i] = x0
            fd = (lp - lm) / (2 * h)
            assert abs(fd - grad[i]) <= 2e-7 * max(1.0, abs(grad[i])), (name, i, fd, grad[i])


def test_finite_differences_sampled_on_tiny_config(oracle):
    """64 random coordinates of the 2048-token tiny configuration (bf16-valued inputs)."""
    from paper_2605_06374_amd import workloads as W
    w = W.config(1)
    vals = {n: W.bf16_bits_to_f32(b).astype(np.float64) for n, b in w.values().items()}
    q, k, v, do, cu, scale = vals["q"], vals["k"], vals["v"], vals["do"], w.cu_seqlens, w.softmax_scale
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, scale)
    rng = np.random.default_rng(17)
    doc = oplan.doc_of_token(cu)
    for trial in range(64):
        name = ("q", "k", "v")[trial % 3]
        x, grad = {"q": (q, dq), "k": (k, dk), "v": (v, dv)}[name]
        i = tuple(int(rng.integers(0, s)) for s in x.shape)
        b = doc[i[0]]
        rows = np.arange(cu[b], cu[b + 1], dtype=np.int32)   # only this document can change

        def partial_loss():
            o, _ = oracle.fwd(q, k, v, cu, scale, rows=rows)
            return float((o * do[rows]).sum())

        x0 = x[i]
        h = 1e-5 * max(1.0, abs(x0))
        x[i] = x0 + h; lp = partial_loss()
        x[i] = x0 - h; lm = partial_loss()
        x[i] = x0
        fd = (lp - lm) / (2 * h)
        assert abs(fd - grad[i]) <= 1e-6 * max(1.0, abs(grad[i])), (name, i, fd, grad[i])


def test_length_one_document_closed_form(oracle):
    rng = np.random.default_rng(18)
    hq, hkv, d = 4, 2, 8
    q, k, v, do, cu = rand_problem(rng, [6, 1, 5], hq, hkv, d)
    scale = 0.3
    o, lse = oracle.fwd(q, k, v, cu, scale)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, scale)
    t = 6
    for h in range(hq):
        kap = h // 2
        assert np.array_equal(o[t, h], v[t, kap])
        assert abs(lse[h, t] - scale * q[t, h] @ k[t, kap]) < 1e-14
        assert np.abs(dq[t, h]).max() < 1e-15
    for kap in range(hkv):
        assert np.abs(dk[t, kap]).max() < 1e-15
        np.testing.assert_allclose(dv[t, kap], do[t, 2 * kap] + do[t, 2 * kap + 1], rtol=1e-15)


def test_equal_keys_give_running_mean(oracle):
    """All keys of a document equal: P is uniform over the allowed keys."""
    rng = np.random.default_rng(19)
    hq, hkv, d = 2, 1, 8
    lengths = [9, 14]
    q, k, v, do, cu = rand_problem(rng, lengths, hq, hkv, d)
    for b in range(2):
        k[cu[b]:cu[b + 1]] = k[cu[b]]
    scale = 0.7
    o, lse = oracle.fwd(q, k, v, cu, scale)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, scale)
    for b in range(2):
        for t in range(cu[b], cu[b + 1]):
            cnt = t - cu[b] + 1
            for h in range(hq):
                np.testing.assert_allclose(o[t, h], v[cu[b]:t + 1, 0].mean(axis=0), rtol=1e-13)
                assert abs(lse[h, t] - (scale * q[t, h] @ k[t, 0] + math.log(cnt))) < 1e-13
        for j in range(cu[b], cu[b + 1]):
            want = sum(do[t, h] / (t - cu[b] + 1) for t in range(j, cu[b + 1]) for h in range(hq))
            np.testing.assert_allclose(dv[j, 0], want, rtol=1e-12, atol=1e-14)
    # with equal keys every dS row sums to zero against identical K rows: dQ vanishes
    assert np.abs(dq).max() < 1e-13


def test_gradient_invariants(oracle):
    """sum_j dK[j] = 0 per document (a constant shift of all keys of a document leaves every
    softmax row unchanged) and sum_j dV[j] = sum_{t,h} dO[t,h] (rows of P sum to one)."""
    rng = np.random.default_rng(20)
    lengths, hq, hkv, d = [31, 2, 57], 4, 2, 16
    q, k, v, do, cu = rand_problem(rng, lengths, hq, hkv, d)
    scale = 0.25
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, scale)
    for b in range(len(lengths)):
        sl = slice(cu[b], cu[b + 1])
        assert np.abs(dk[sl].sum(axis=0)).max() < 1e-12
        want = do[sl].reshape(-1, hkv, hq // hkv, d).sum(axis=(0, 2))
        np.testing.assert_allclose(dv[sl].sum(axis=0), want, rtol=1e-12, atol=1e-12)


def test_row_subsets_match_full(oracle):
    rng = np.random.default_rng(21)
    lengths, hq, hkv, d = [19, 5, 40], 4, 2, 8
    q, k, v, do, cu = rand_problem(rng, lengths, hq, hkv, d)
    scale = 0.4
    o, lse = oracle.fwd(q, k, v, cu, scale)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, scale)
    rows = np.array([0, 18, 19, 23, 24, 63, 40], dtype=np.int32)
    o_r, lse_r = oracle.fwd(q, k, v, cu, scale, rows=rows)
    dq_r, d_r = oracle.dq_rows(q, k, v, do, cu, scale, rows=rows)
    _, d_full = oracle.dq_rows(q, k, v, do, cu, scale)
    dk_r, dv_r = oracle.dkv_rows(q, k, v, do, lse, d_full, cu, scale, rows=rows)
    assert np.array_equal(o_r, o[rows]) and np.array_equal(lse_r, lse[:, rows])
    assert np.array_equal(dq_r, dq[rows]) and np.array_equal(d_r, d_full[:, rows])
    assert np.array_equal(dk_r, dk[rows]) and np.array_equal(dv_r, dv[rows])
    np.testing.assert_allclose(d_full, np.einsum("thc,thc->ht", do, o), rtol=1e-13, atol=1e-14)


def test_bad_cu_seqlens_rejected(oracle):
    rng = np.random.default_rng(22)
    q, k, v, do, cu = rand_problem(rng, [4, 4], 1, 1, 4)
    for bad in ([1, 4, 8], [0, 5, 4, 8], [0, 4, 7]):
        with pytest.raises(ValueError):
            oracle.fwd(q, k, v, np.array(bad, dtype=np.int32), 1.0)


# ---------------------------------------------------------------- integers and printed values
def _golden(name):
    rows = []
    with open(os.path.join(HERE, "golden", name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([c.strip() for c in line.split("|")])
    return rows


def test_paper_cost_ratio():
    for a, b, ratio, tol in _golden("packed_cost_ratio.txt"):
        la, lb = [int(x) for x in a.split()], [int(x) for x in b.split()]
        cua, cub = np.cumsum([0] + la), np.cumsum([0] + lb)
        # the paper's proportionality (sum of squares) and the exact causal pair count agree
        r_sq = sum(l * l for l in la) / sum(l * l for l in lb)
        r_pairs = oplan.pairs(cua) / oplan.pairs(cub)
        assert abs(r_sq - float(ratio)) <= float(tol)
        assert abs(r_pairs - float(ratio)) <= float(tol)
        assert oplan.pairs(cua) == 8390656 and oplan.pairs(cub) == 2099200


def test_workload_generator_matches_golden_lengths():
    from paper_2605_06374_amd import workloads as W
    get = {"cfg1": lambda: W.config(1), "cfg2": lambda: W.config(2), "cfg3": lambda: W.config(3),
           "cfg4": lambda: W.config(4), "cfg5_mb0": lambda: W.config(5, microbatch=0),
           "cfg5_mb5": lambda: W.config(5, microbatch=5)}
    for name, lengths, pairs in _golden("workload_lengths.txt"):
        w = get[name]()
        assert w.lengths == [int(x) for x in lengths.split()]
        assert w.pairs == int(pairs) == oplan.pairs(w.cu_seqlens)
        assert sum(w.lengths) == w.n_tokens
        assert w.flops_fwd_bwd == oplan.flops_fwd_bwd(w.cu_seqlens, w.n_q_heads, w.head_dim)
    assert sum(W.config(5, microbatch=i).pairs for i in range(64)) == 159302466


def test_plan_integers():
    cu = [0, 5, 5, 300, 301, 1000]
    doc = oplan.doc_of_token(cu)
    assert len(doc) == 1000 and doc[0] == 0 and doc[4] == 0 and doc[5] == 2 and doc[299] == 2
    assert doc[300] == 3 and doc[301] == 4
    tiles = oplan.row_tiles(cu, 128)
    assert tiles == [(0, 0, 0, 5), (2, 0, 5, 128), (2, 1, 133, 128), (2, 2, 261, 39), (3, 0, 300, 1),
                     (4, 0, 301, 128), (4, 1, 429, 128), (4, 2, 557, 128), (4, 3, 685, 128),
                     (4, 4, 813, 128), (4, 5, 941, 59)]
    # brute-force count of non-empty (q tile, kv tile) pairs
    bq, bk = 128, 64
    want = 0
    for b in range(len(cu) - 1):
        l = cu[b + 1] - cu[b]
        seen = set()
        for t in range(l):
            for j in range(0, t + 1, 1 if l < 200 else 7):
                seen.add((t // bq, j // bk))
            seen.add((t // bq, t // bk))
        want += len(seen)
    assert oplan.causal_tile_pairs(cu, bq, bk) == want


def test_bf16_rounding_helpers():
    from paper_2605_06374_amd import workloads as W
    torch = pytest.importorskip("torch")
    x = np.random.default_rng(3).standard_normal(10000).astype(np.float32) * 3
    x[:4] = [1.00390625, 1.01171875, -0.0, 65504.0]     # ties: to even
    bits = W.f32_to_bf16_bits(x)
    ref = torch.tensor(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    assert np.array_equal(W.bf16_bits_to_f32(bits), ref.float().numpy())


# ------------------------------------------------------------------ chains of the plan
@pytest.mark.parametrize("tile,step", [(128, 64), (8, 4), (6, 3), (4, 4)])
def test_chain_steps_against_brute_force_over_the_mask(tile, step):
    """row_chain_steps / col_chain_steps against a count over the explicit mask: for every
    tile, the steps (of `step` keys counted from the document start, resp. `step` queries
    counted from the tile's first row) that hold at least one allowed (t, j)."""
    from oracle import plan as oplan
    rng = np.random.default_rng(tile * 100 + step)
    cases = [[0], [1], [0, 0, 1, 0], [step, step + 1, tile, tile + 1, tile - 1, 1, 0, 2 * tile + 1],
             [3 * tile + step + 1]]
    for _ in range(12):
        cases.append([int(x) for x in rng.integers(0, 3 * tile + 2, size=int(rng.integers(1, 7)))])
    for lengths in cases:
        cu = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
        n = int(cu[-1])
        doc = np.array(oplan.doc_of_token(cu), dtype=np.int64)
        t_idx, j_idx = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
        allowed = (doc[t_idx] == doc[j_idx]) & (j_idx <= t_idx) if n else np.zeros((0, 0), bool)
        want_row, want_col = {}, {}
        for b in range(len(lengths)):
            s, e = int(cu[b]), int(cu[b + 1])
            for r0 in range(s, e, tile):
                r1 = min(r0 + tile, e)
                # keys seen by some query of the tile, in steps from the document start
                keys = np.nonzero(allowed[r0:r1].any(axis=0))[0]
                want_row[(r0, s, e)] = len(set(int((j - s) // step) for j in keys))
                # queries that see some key of the tile, in steps from the tile's first row
                queries = np.nonzero(allowed[:, r0:r1].any(axis=1))[0]
                want_col[(r0, s, e)] = len(set(int((t - r0) // step) for t in queries))
                # both sets are gap-free ranges starting at step 0
                assert set(int((j - s) // step) for j in keys) == set(range(want_row[(r0, s, e)]))
                assert set(int((t - r0) // step) for t in queries) == set(range(want_col[(r0, s, e)]))
        assert oplan.row_chain_steps(cu, tile, step) == want_row, lengths
        assert oplan.col_chain_steps(cu, tile, step) == want_col, lengths
