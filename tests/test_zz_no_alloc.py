"""GPU test of intattn_forward_noalloc (the forward whose workspace is the library's static device
array): same bytes as intattn_forward, on two calls in a row, the second with a smaller input; plus
the rejection of a problem whose workspace exceeds the array.  Collected last (file name), so that
a failure here hides no other test under `pytest -x`."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    import torch

    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a visible MI355X (torch.cuda.is_available() is False)")
    return torch


def _both(torch, ia, p, s_o):
    dev = torch.device("cuda:0")
    q, k, v = (torch.from_numpy(x).to(dev) for x in (p.q, p.k, p.v))
    stream = torch.cuda.current_stream(dev).cuda_stream
    want = torch.empty_like(q)
    args, keep = ia.make_args(q, k, v, want, p.s_q, p.s_k, p.s_v, s_o, causal=p.causal, per_head=p.per_head)
    ia.forward_args(args, stream)
    got = torch.full_like(q, 77)
    args2, keep2 = ia.make_args(q, k, v, got, p.s_q, p.s_k, p.s_v, s_o, causal=p.causal, per_head=p.per_head)
    ia.forward_noalloc_args(args2, stream)
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy()


@pytest.mark.parametrize("variant", [0, 5, 9])
def test_noalloc_forward_matches_forward_twice(torch_mod, oracle, variant):
    from paper_2511_21513_amd import binding

    ia = binding.IntAttn(device=0, variant=variant)
    # first call: per-head scales (table in the static array), two-launch path under variant 5
    big = workloads.random_problem(91, 2, 4, 2, 700, 128, True, per_head=True, spread=1.3)
    got, want = _both(torch_mod, ia, big, workloads.calibrated_out_scale(big))
    assert int((got != want).sum()) == 0
    ref = oracle.forward(big.q, big.k, big.v, big.s_q, big.s_k, big.s_v, workloads.calibrated_out_scale(big), causal=True,
                         per_head=True, threads=8)["out"]
    assert int((got != ref).sum()) == 0
    # second call, smaller and of another shape: whatever the first left in the array must not matter
    small = workloads.random_problem(92, 1, 2, 1, 133, 64, False, spread=0.8)
    got, want = _both(torch_mod, ia, small, None)
    assert int((got != want).sum()) == 0
    # a decoded token (split-key kernels under variants 0 and 9: partial results in the array)
    dec = workloads.random_problem(93, 2, 4, 1, 1500, 128, True)
    dec.q = np.ascontiguousarray(dec.q[:, :, -1:])
    dec.L = 1
    got, want = _both(torch_mod, ia, dec, None)
    assert int((got != want).sum()) == 0
    ia.close()


def test_noalloc_rejects_what_does_not_fit(torch_mod):
    from paper_2511_21513_amd import binding

    torch = torch_mod
    dev = torch.device("cuda:0")
    ia = binding.IntAttn(device=0, variant=5)
    # 8 bytes per query row: 64 heads x 16384 rows = 8 MiB > the 4 MiB array
    q = torch.zeros((1, 64, 16384, 64), dtype=torch.int8, device=dev)
    k = torch.zeros((1, 8, 16384, 64), dtype=torch.int8, device=dev)
    out = torch.empty_like(q)
    one = np.asarray([0.01], dtype=np.float32)
    args, keep = ia.make_args(q, k, k, out, one, one, one, None, causal=True)
    with pytest.raises(binding.IntAttnError) as e:
        ia.forward_noalloc_args(args, torch.cuda.current_stream(dev).cuda_stream)
    assert e.value.code == binding.ERR_UNSUPPORTED and "static array" in str(e.value)
    ia.forward_args(args, torch.cuda.current_stream(dev).cuda_stream)  # the allocating entry point takes it
    torch.cuda.synchronize()
    ia.close()
