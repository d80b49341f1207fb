"""varlen_attn_fwd_static (the forward for callers that cannot allocate: its workspace is a
fixed device array inside the library) against varlen_attn_fwd, through the C ABI: bit-identical
O and LSE on two calls in a row, the second on a smaller input, then a larger one again; the
size limit and the status word."""
import numpy as np
import pytest

from paper_2605_06374_amd import workloads as W

pytestmark = pytest.mark.gpu


def _static_forward(binding, prob, status=None):
    import torch
    o = torch.empty_like(prob.o)
    lse = torch.empty_like(prob.lse)
    o.view(torch.int16).fill_(0x7FC0)
    lse.fill_(float("nan"))
    binding.check(binding.varlen_attn_fwd_static(prob.params, prob.q, prob.k, prob.v, prob.cu, o,
                                                 lse, status))
    torch.cuda.synchronize()
    return (o.view(torch.int16).cpu().numpy().view(np.uint16), lse.cpu().numpy().view(np.uint32))


def test_static_workspace_forward_matches_the_workspace_forward():
    import torch
    from paper_2605_06374_amd import binding, runner
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.lib()
    status = torch.full((1,), -99, dtype=torch.int32, device="cuda:0")
    # large first (cut chains: partial results in the static array), then smaller, then the
    # 7B-shard configuration again: the array keeps the previous call's contents in between
    cases = [W.config(2), W.custom("small_after_large", [300, 1, 77], 4, 2, 128, seed=11),
             W.config(1), W.config(2)]
    for w in cases:
        print("case", w.name, flush=True)
        prob = runner.DeviceProblem(w)
        prob.poison_outputs()
        prob.forward()
        assert binding.varlen_attn_check(prob.workspace) == binding.OK
        want = prob.result_bits()
        status.fill_(-99)
        got_o, got_lse = _static_forward(binding, prob, status)
        assert int(status.item()) == binding.OK
        assert np.array_equal(got_o, want["o"]), w.name
        assert np.array_equal(got_lse, want["lse"]), w.name


def test_static_workspace_forward_reports_errors():
    import torch
    from paper_2605_06374_amd import binding, runner
    w = W.custom("bad", [100, 200, 84], 2, 2, 128, seed=3)
    prob = runner.DeviceProblem(w)
    status = torch.full((1,), -99, dtype=torch.int32, device="cuda:0")
    prob.cu.copy_(torch.tensor([0, 250, 200, 384], dtype=torch.int32))
    _static_forward(binding, prob, status)
    assert int(status.item()) == binding.BAD_CU_SEQLENS
    # a problem whose forward workspace exceeds the static array is refused on the host
    big = binding.make_params(1 << 20, 4, 64, 64, 128, 0.1)
    L = binding.varlen_attn_workspace_regions(big)
    assert L.col_partials_offset > binding.STATIC_SCRATCH_BYTES
    rc = binding.varlen_attn_fwd_static(big, prob.q, prob.k, prob.v, prob.cu, prob.o, prob.lse, None)
    assert rc == binding.STATIC_TOO_LARGE
    assert "static" in binding.varlen_attn_status_string(rc)
    assert binding.varlen_attn_fwd_static(prob.params, None, prob.k, prob.v, prob.cu, prob.o,
                                          prob.lse, None) == binding.INVALID_ARG
