"""GPU tests of the entry points under HIP graph capture: a forward is captured once (after a first, eager call
has allocated what the context needs and uploaded the head table) and replayed several times, with eager work of
the same library and synchronizations between the replays; every replay must reproduce the eager call's bytes,
which are the oracle's.  Covers the paths that keep state between their kernels: the two-launch tiled path (row
maxima and sums in the workspace), the one-launch split-key path (counters in device memory that every launch must
leave at zero), the device-scale entry (parameters derived by a kernel) and the entry that allocates nothing."""
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


def _capture_and_replay(torch, enqueue, out, want, eager_between, replays=3):
    """enqueue(stream_handle) enqueues the work on a raw stream; out is the tensor it writes."""
    side = torch.cuda.Stream()  # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue(side.cuda_stream)  # eager: allocations and uploads happen here, outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert int((out.cpu().numpy() != want).sum()) == 0, "eager call"
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue(torch.cuda.current_stream().cuda_stream)
    for rep in range(replays):
        out.fill_(55)
        eager_between()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int((out.cpu().numpy() != want).sum()) == 0, f"replay {rep}"


CASES = [
    # name, variant, entry, B, Hq, Hkv, Lq, Lk, d, per_head
    ("two launches, per-head scales", 5, "forward", 2, 4, 2, 700, 700, 128, True),
    ("split-key single launch", 3, "forward", 1, 4, 4, 300, 300, 64, False),
    ("one decoded token, one launch with counters", 9, "forward", 3, 8, 2, 1, 3000, 128, True),
    ("one decoded token, device scales", 9, "dynamic", 3, 8, 2, 1, 3000, 128, True),
    ("prefill, device scales", 0, "dynamic", 1, 4, 2, 520, 520, 128, True),
    ("entry that allocates nothing, per-tensor scales", 5, "noalloc", 2, 4, 2, 700, 700, 128, False),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: c[0].replace(" ", "_").replace(",", ""))
def test_captured_forward_replays_bit_exact(torch_mod, oracle, case):
    from paper_2511_21513_amd import binding

    torch = torch_mod
    name, variant, entry, B, Hq, Hkv, lq, lk, d, per_head = case
    print(f"case {case}", flush=True)
    p = workloads.random_problem(len(name), B, Hq, Hkv, lk, d, True, per_head=per_head, spread=1.2)
    qh = np.ascontiguousarray(p.q[:, :, lk - lq:])
    want = oracle.forward(qh, p.k, p.v, p.s_q, p.s_k, p.s_v, None, causal=True, per_head=per_head, threads=8)["out"]
    dev = torch.device("cuda:0")
    q, k, v = (torch.from_numpy(x).to(dev) for x in (qh, p.k, p.v))
    out = torch.empty_like(q)
    ia = binding.IntAttn(device=0, variant=variant)
    if entry == "dynamic":
        sc = [torch.from_numpy(np.asarray(x, dtype=np.float32)).to(dev) for x in (p.s_q, p.s_k, p.s_v)]
        args, keep = ia.make_args(q, k, v, out, sc[0], sc[1], sc[2], None, causal=True, per_head=per_head, device_scales=True)
        enqueue = lambda st: ia.forward_dynamic_args(args, st)
    else:
        args, keep = ia.make_args(q, k, v, out, p.s_q, p.s_k, p.s_v, None, causal=True, per_head=per_head)
        enqueue = (lambda st: ia.forward_noalloc_args(args, st)) if entry == "noalloc" else (lambda st: ia.forward_args(args, st))
    # eager work between the replays: another problem through a context of its own
    other = workloads.random_problem(7, 1, 2, 1, 200, 64, False, spread=0.9)
    ib = binding.IntAttn(device=0, variant=0)
    oq, ok_, ov = (torch.from_numpy(x).to(dev) for x in (other.q, other.k, other.v))

    def eager_between():
        ib.forward(oq, ok_, ov, other.s_q, other.s_k, other.s_v, None, causal=False)

    _capture_and_replay(torch, enqueue, out, want, eager_between)
    if entry == "dynamic":
        assert ia.dynamic_status() == 0
    ia.close()
    ib.close()
