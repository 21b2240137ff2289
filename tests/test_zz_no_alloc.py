"""GPU test of zo2_op_lm_head_ce_static, the LM head + cross-entropy entry point that allocates nothing: through the
C ABI, against zo2_op_lm_head_ce (caller-supplied workspace), bit for bit, on two calls in a row of which the second
is smaller (the built-in buffer then still holds the first call's partials), then a larger one again; and the
refusal of shapes beyond the buffer."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def _b():
    from paper_2503_12668_amd import binding
    return binding


def _case(M, N, K, dtype, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    X = torch.randn(M, K, device="cuda", generator=g).to(dtype)
    W = (torch.randn(N, K, device="cuda", generator=g) * 0.2).to(dtype)
    lab = torch.randint(0, N, (M,), device="cuda", generator=g, dtype=torch.int32)
    lab[3] = -100
    lab[4], lab[5] = 0, N - 1
    return X, W, lab


def test_static_scratch_entry_point_matches_workspace_entry_point():
    b = _b()
    torch.cuda.synchronize()
    for i, (M, N, K, dtype) in enumerate([(1024, 5000, 256, torch.bfloat16),      # 20 spans of 256 columns, ragged last
                                          (300, 520, 128, torch.float16),         # smaller: ragged rows and columns
                                          (2048, 50272, 128, torch.bfloat16)]):   # close to the buffer's limit
        X, W, lab = _case(M, N, K, dtype, 7 + i)
        want = b.op_lm_head_ce(X, W, lab)
        out = torch.full((M,), float("nan"), dtype=torch.float32, device="cuda")
        got = b.op_lm_head_ce_static(X, W, lab, out=out)
        torch.cuda.synchronize()
        assert torch.isfinite(want).all() and float(want[3]) == 0.0
        assert torch.equal(got, want), (M, N, K)
    assert b.lib().zo2_op_lm_head_ce_workspace_bytes(2048, 50272) <= 16 << 20
    # beyond the buffer: refused, with a message that names the other entry point
    X, W, lab = _case(4096, 50272, 128, torch.bfloat16, 1)
    with pytest.raises(b.Zo2Error) as e:
        b.op_lm_head_ce_static(X, W, lab)
    assert e.value.status == 1 and "zo2_op_lm_head_ce" in str(e.value)
    # the shape checks of the workspace variant hold here too
    with pytest.raises(b.Zo2Error):
        b.op_lm_head_ce_static(X[:100], W, lab[:100])
