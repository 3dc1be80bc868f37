"""The allocation-free entry point (qadam_quantize_segment_noalloc) against qadam_worker_quantize.

Collected last (file name), so a failure here cannot hide the other GPU tests; passes alone in a
fresh process as well as after the others.  Two calls in a row share the library's static device
array; the second is smaller, so stale maxima of the first call's extra tiles must not leak into it.
"""
import numpy as np
import pytest
import torch

from paper_2004_14180_amd import QAdam, QAdamConfig
from paper_2004_14180_amd.binding import QADAM_NOALLOC_MAX_ELEMS, QAdamError, quantize_segment_noalloc

pytestmark = pytest.mark.gpu


def _reference(k_g, grad, err):
    """qadam_worker_quantize on a handle with the single segment [0, n)."""
    n = grad.numel()
    q = QAdam(QAdamConfig(k_g=k_g, k_x=6, rounding=0), [0, n], 1)
    codes = torch.full((max(q.grad_code_bytes() // 4, 1),), -1, dtype=torch.int32, device="cuda")
    scale = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    e = err.clone()
    q.worker_quantize(0, 1, grad, e, codes, scale)
    torch.cuda.synchronize()
    assert q.get_status() == 0
    nbytes = q.grad_code_bytes()
    q.close()
    return codes[: nbytes // 4], e, scale


def _inputs(n, seed, scale):
    g = torch.Generator(device="cuda").manual_seed(seed)
    grad = torch.randn(n, generator=g, device="cuda") * scale
    err = torch.randn(n, generator=g, device="cuda") * (0.2 * scale)
    return grad, err


@pytest.mark.parametrize("k_g", [2, 0, 5])
def test_two_calls_in_a_row_second_smaller(k_g):
    # first: many tiles with a ragged tail and a large maximum; second: fewer tiles, much smaller values
    for n, seed, scale in [(3 * 4096 * 37 + 1001, 11, 5.0), (4096 * 5 + 77, 12, 1e-3)]:
        grad, err = _inputs(n, seed, scale)
        want_codes, want_err, want_scale = _reference(k_g, grad, err)
        codes = torch.full_like(want_codes, -1)
        scale_out = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
        e = err.clone()
        quantize_segment_noalloc(k_g, n, grad, e, codes, scale_out)
        torch.cuda.synchronize()
        assert torch.equal(scale_out.view(torch.int32), want_scale.view(torch.int32)), (n, k_g)
        assert torch.equal(codes, want_codes), (n, k_g)
        assert torch.equal(e.view(torch.int32), want_err.view(torch.int32)), (n, k_g)


def test_against_the_oracle_and_edge_sizes():
    from oracle import qadam_oracle as oracle
    ocfg = oracle.OracleConfig(k_g=2, k_x=6)
    for n in [1, 31, 4096, 4097, 0]:
        grad, err = _inputs(max(n, 1), 100 + n, 0.01)
        grad, err = grad[:n].contiguous(), err[:n].contiguous()
        words = (n + 31) // 32 * 3
        codes = torch.full(((words + 3) // 4 * 4 + 4,), -1, dtype=torch.int32, device="cuda")
        scale_out = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
        e = err.clone()
        quantize_segment_noalloc(2, n, grad, e, codes, scale_out)
        torch.cuda.synchronize()
        he = err.cpu().numpy().copy()
        out = oracle.worker_quantize(ocfg, [0, n], 0, 1, grad.cpu().numpy(), he)
        nw = len(out["words"])
        assert np.array_equal(codes[:nw].cpu().numpy().view(np.uint32), out["words"]), n
        assert (codes[nw:] == -1).all(), "wrote past the segment's code words"
        assert np.array_equal(e.cpu().numpy().view(np.uint32), he.view(np.uint32)), n
        assert np.float32(scale_out.cpu().numpy()[0]).view(np.uint32) == out["scales"][0].view(np.uint32), n


def test_size_limit_and_arguments_are_checked_on_the_host():
    one = torch.zeros(4, device="cuda")
    with pytest.raises(QAdamError) as ei:
        quantize_segment_noalloc(2, QADAM_NOALLOC_MAX_ELEMS + 1, one, one, one, one)
    assert ei.value.code == -3
    with pytest.raises(QAdamError) as ei:
        quantize_segment_noalloc(7, 4, one, one, one, one)
    assert ei.value.code == -1
    with pytest.raises(QAdamError) as ei:
        quantize_segment_noalloc(2, 4, one, one[1:], one, one)     # misaligned pointer
    assert ei.value.code == -2
