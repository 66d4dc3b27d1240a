"""GPU parity of the parameter-free visual token compressors against the oracle.

Pruning is a bit copy: exact.  Pooling sums at most `ratio` (<= 30) bf16/fp32 values of size ~1 in
fp32, multiplies by 1/count and rounds once to the tensor's type: against the fp64 mean the error
is at most the output rounding (2^-9 relative for bf16, 2^-24 for fp32) plus ~ratio * 2^-24 of the
sum, so |got - ref| <= 2^-8 |ref| + 1e-6 (bf16) and <= 1e-6 (fp32, values of size <= ~4)."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sv():
    import paper_2509_11815_amd as sv
    sv.load_library()
    return sv


def _close(got, ref, dtype):
    err = np.abs(got - ref)
    tol = (2.0 ** -8) * np.abs(ref) + 1e-6 if dtype == "bf16" else 1e-6
    assert np.all(err <= tol), err.max()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,T,E,ratio", [
    (1, 576, 4096, 2), (1, 576, 4096, 3), (1, 577, 4096, 5), (2, 2880, 4096, 20), (1, 2880, 5120, 30),
    (3, 100, 64, 7), (1, 5, 8, 10), (1, 4608, 1024, 1)])
def test_pool_matches_oracle(sv, oracle, dtype, B, T, E, ratio):
    from gpu_util import i32, to_dev, to_host_f64
    rng = np.random.default_rng(T * 31 + ratio)
    x = W.normal(rng, (B, T, E), 1.0, dtype)
    nt = rng.integers(0, T + 1, size=B).astype(np.int32)
    nt[0] = T
    y, out_tokens = sv.specvlm_visual_pool(to_dev(x), ratio, num_tokens=i32(nt))
    ref, r_tokens = oracle.visual_pool(x, ratio, nt)
    assert np.array_equal(out_tokens.cpu().numpy(), r_tokens)
    got = to_host_f64(y)
    for b in range(B):
        _close(got[b, :r_tokens[b]], ref[b, :r_tokens[b]], dtype)
        assert np.all(got[b, r_tokens[b]:] == 0)                     # rows past the pooled length: untouched (zero-initialised)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_prune_matches_oracle_and_views(sv, oracle, dtype):
    from gpu_util import i32, to_dev, to_host_bits
    rng = np.random.default_rng(11)
    B, T, E = 2, 2880, 4096
    keep_n = -(-T // 20)
    big = W.normal(rng, (B, T, 2 * E), 1.0, dtype)                   # features inside a wider buffer
    keep = np.stack([np.sort(rng.choice(T, keep_n, replace=False)) for _ in range(B)]).astype(np.int32)
    keep[1, -7:] = -1
    keep[0, :3] = [T - 1, 0, T - 1]
    xd = to_dev(big)
    out = torch.full((B, keep_n, E + 8), 3.0, dtype=xd.dtype, device="cuda")
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    sv.specvlm_visual_prune(xd[:, :, E:], i32(keep), out=out[:, :, :E], err_flag=err)
    ref = oracle.visual_prune(np.ascontiguousarray(big[:, :, E:]), keep)
    got = to_host_bits(out)
    real = keep >= 0
    assert np.array_equal(got[:, :, :E][real], ref[real])
    assert np.all(to_host_bits(out[:, :, E:]) == to_host_bits(torch.full((1,), 3.0, dtype=xd.dtype, device="cuda"))[0])
    assert np.all(got[1, -7:, :E] == got[1, -1, E])                 # padding rows untouched
    assert int(err.item()) == 0
    bad = keep.copy()
    bad[0, 5] = T
    sv.specvlm_visual_prune(xd[:, :, E:], i32(bad), out=out[:, :, :E], err_flag=err)
    assert int(err.item()) == 4


def test_pool_error_flag_and_argument_checks(sv):
    from gpu_util import i32
    x = torch.randn((2, 40, 64), device="cuda").to(torch.bfloat16)
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    _, nt = sv.specvlm_visual_pool(x, 4, num_tokens=i32([41, -3]), err_flag=err)
    assert int(err.item()) == 4 and nt.cpu().tolist() == [10, 0]
    with pytest.raises(sv.SpecvlmError, match="INVALID_ARG"):
        sv.specvlm_visual_pool(x[:, :, :60], 4)                     # 120-byte rows
    with pytest.raises(sv.SpecvlmError, match="INVALID_ARG"):
        sv.specvlm_visual_pool(x, 0)
