"""GPU parity at the full benchmark sizes, every byte: the headline configuration (long-context
GQA prefill) over all of its heads, and whole (batch, head) pairs of the batched prefill
configuration spread over its batch entries and heads.  Automatic kernel choice, i.e. exactly the
launch configuration `bench.py` times, with the calibrated output scale so that the bytes carry
information.  The oracle runs every row of every compared head (heads fanned over host threads)."""
from concurrent.futures import ThreadPoolExecutor

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


def _gpu_out(torch, p, s_o, variant=0):
    from paper_2511_21513_amd import binding

    dev = torch.device("cuda:0")
    ia = binding.IntAttn(device=0, variant=variant)
    q, k, v = (torch.from_numpy(x).to(dev) for x in (p.q, p.k, p.v))
    out = ia.forward(q, k, v, p.s_q, p.s_k, p.s_v, s_o, causal=p.causal, per_head=p.per_head)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    ia.close()
    return got


def test_config4_every_output_byte(torch_mod, oracle):
    p = workloads.make_problem("c4_gqa_prefill_8k")
    s_o = workloads.calibrated_out_scale(p, sample_rows=16)
    print("c4: GPU forward", flush=True)
    got = _gpu_out(torch_mod, p, s_o)
    print("c4: oracle over all 32 heads", flush=True)
    want = oracle.forward(p.q, p.k, p.v, p.s_q, p.s_k, p.s_v, s_o, causal=True, per_head=False, threads=16)["out"]
    assert got.shape == want.shape == (1, 32, 8192, 128)
    bad = int((got != want).sum())
    assert bad == 0, f"c4: {bad} of {want.size} output bytes differ from the oracle"
    assert int(np.abs(want).max()) > 20  # the calibrated scale makes the bytes informative


def test_config5_whole_heads_over_all_groups(torch_mod, oracle):
    """64 of the 512 (batch, head) pairs in full: four heads of every batch entry, chosen so that all
    32 head indices (= all 32 per-head parameter sets) are covered twice."""
    p = workloads.make_problem("c5_batched_prefill_4k")
    s_o = workloads.calibrated_out_scale(p, sample_rows=8)
    print("c5: GPU forward", flush=True)
    got = _gpu_out(torch_mod, p, s_o)
    pairs = [(b, (8 * j + b // 2 + 4 * (b % 2)) % 32) for b in range(16) for j in range(4)]
    assert len(set(pairs)) == 64 and {h for _, h in pairs} == set(range(32))
    # each chosen pair as a single-head problem with that head's own scales, 16 at a time over host threads
    def one(pair):
        b, h = pair
        sel = lambda x: np.ascontiguousarray(x[b:b + 1, h:h + 1])
        want = oracle.forward(sel(p.q), sel(p.k), sel(p.v), p.s_q[h:h + 1], p.s_k[h:h + 1], p.s_v[h:h + 1],
                              s_o[h:h + 1], causal=True, per_head=False)["out"][0, 0]
        return int((got[b, h] != want).sum())

    print("c5: oracle over 64 whole heads", flush=True)
    with ThreadPoolExecutor(max_workers=16) as ex:
        bad = sum(ex.map(one, pairs))
    assert bad == 0, f"c5: {bad} output bytes differ from the oracle on 64 whole (batch, head) pairs"
