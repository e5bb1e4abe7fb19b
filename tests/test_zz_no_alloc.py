"""The entry point that allocates nothing, mllm_op_colsum_static, against mllm_op_colsum (same
kernels, partial sums in the library's static device array instead of a caller's buffer): two calls
in a row, the second on a smaller input, must equal the existing entry point bit for bit; both are
also held to the fp32-output tolerance against the plain fp64 column sum."""
import numpy as np
import pytest

import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from tests.gpu_util import dev_bf16, host_f64, nmax_err, scratch  # noqa: E402


@pytest.fixture(scope="module")
def B():
    from paper_2603_25120_amd import binding
    binding.lib()
    return binding


def _both(B, x_np, accumulate, seed_out):
    t, n = x_np.shape
    x = dev_bf16(x_np)
    base = torch.linspace(-1.0, 1.0, n, device="cuda", dtype=torch.float32) * seed_out
    ref, got = base.clone(), base.clone()
    partial = scratch(B.mllm_op_colsum_partial_bytes(t, n))
    B.mllm_op_colsum(x, ref, accumulate, partial, t, n)
    # cumulative count of the allocator's requests: unlike the bytes in use it cannot drop when the
    # garbage collector frees an earlier test's tensors in the middle of the call
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    B.mllm_op_colsum_static(x, got, accumulate, t, n)
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    torch.cuda.synchronize()
    return host_f64(base), ref, got


def test_static_scratch_column_sum_two_calls_in_a_row(B):
    assert B.mllm_op_colsum_static_max_bytes() == 8 << 20
    big = W.draw_tensor(61, 5000, 4096)          # 512 row chunks x 4096 columns: the whole 8 MiB array
    small = W.draw_tensor(62, 37, 264)           # 9 row chunks, a ragged last block of columns
    for x_np, accumulate, seed_out in ((big, 0, 1.0), (small, 0, 2.0), (small, 1, 3.0), (big, 1, 0.5)):
        base, ref, got = _both(B, x_np, accumulate, seed_out)
        assert torch.equal(ref, got), (x_np.shape, accumulate)
        want = x_np.astype(np.float64).sum(axis=0) + (base if accumulate else 0.0)
        assert nmax_err(host_f64(got), want) < 2e-3, (x_np.shape, accumulate)


def test_static_scratch_rejects_what_does_not_fit(B):
    x = torch.zeros(4096, 8192, dtype=torch.bfloat16, device="cuda")      # 512 x 8192 x 4 B = 16 MiB of partial sums
    out = torch.full((8192,), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(B.MllmError) as e:
        B.mllm_op_colsum_static(x, out, 0, 4096, 8192)
    assert e.value.status == 7 and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())                                       # nothing was launched
    with pytest.raises(B.MllmError):
        B.mllm_op_colsum_static(None, out, 0, 16, 64)
