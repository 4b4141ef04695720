#!/usr/bin/env python3
"""Benchmark of the fused integer attention path on one MI355X.

A step is one pass of the whole hot path (INT8 Q.K^T, IndexSoftmax, UINT8 P times INT8 V,
INT8 requantization) over one batch of synthetic input already resident in HBM.  The default
workload is the configuration the headline metric is quoted on: long-context causal prefill
with grouped-query attention, B=1, 32 query heads over 8 KV heads, L=8192, d=128.

Prints ONE JSON line.  `value` is int8 attention TOPS counting the two contractions only
(4*d*pairs*B*Hq operations, pairs = L(L+1)/2 under the causal mask); recomputation sweeps and
masked halves of diagonal tiles are executed but not counted.

Other modes, each with its own JSON line against the HBM roofline: --quantizer (Eq. quant on fp16
Q, K, V, and the chains quantizer -> attention on device-resident scales), --decode (one token
per sequence through the split-key kernels), --softmax (IndexSoftmax as an operator on INT32
logits).  --workload / --batch select another configuration for the default mode.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0  # MI355X dense int8 matrix peak, 5.0 POP/s
HBM_PEAK_GBS = 8000.0
# Lane operations the vector ALUs can issue: 64 per clock and compute unit (four SIMDs, each a 64-wide wave
# instruction over four clocks), 256 compute units, 2.4 GHz peak engine clock.
VALU_PEAK_LANE_OPS = 64 * 256 * 2.4e9
CSRC = os.path.join(ROOT, "paper_2511_21513_amd", "csrc")


def kernel_source_hash(names):
    """SHA-256 over the named kernel sources (in the order given): what a stored counter reading is valid for."""
    import hashlib

    h = hashlib.sha256()
    for fn in names:
        with open(os.path.join(CSRC, fn), "rb") as f:
            h.update(fn.encode() + b"\0" + f.read())
    return h.hexdigest()


def stored_counters(tag):
    """`key: value` lines of profiles/counters_<tag>.md (rocprofv3 --pmc readings that a timing run
    cannot take itself), or {} when there is no such file or the kernel sources it names
    (`kernel_sources:`) no longer hash to its `kernel_source_sha256:`."""
    path = os.path.join(ROOT, "profiles", f"counters_{tag}.md")
    if not os.path.exists(path):
        return {}
    vals = {}
    with open(path) as f:
        for line in f:
            key, sep, val = line.strip().lstrip("-* ").partition(":")
            if sep and key and " " not in key:
                vals[key] = val.strip()
    try:
        if vals.get("kernel_source_sha256") != kernel_source_hash(vals.get("kernel_sources", "").split()):
            return {}
    except OSError:
        return {}
    out = {"source": f"profiles/counters_{tag}.md"}
    for key, val in vals.items():
        try:
            out[key] = float(val)
        except ValueError:
            out[key] = val
    return out


def host_cpu():
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return {"model": model, "nproc": os.cpu_count() or 1, "usable": usable}


ALIASES = {"c1": "c1_single_head", "c2": "c2_vit_b16", "c3": "c3_llm_prefill_2k",
           "c4": "c4_gqa_prefill_8k", "c5": "c5_batched_prefill_4k"}


def cpu_baseline(p, s_o, budget_heads, gpu_out=None):
    """The oracle as it stands on this host's cores, over whole heads of the same workload with the
    same output scale; its bytes are compared with the timed GPU output where one is given."""
    import numpy as np

    import oracle

    cpu = host_cpu()
    n_heads = min(p.B * p.Hq, budget_heads)
    # the first batch entries' first n_heads query heads (with their KV heads), all rows
    b_cnt = (n_heads + p.Hq - 1) // p.Hq
    hq_cnt = min(n_heads, p.Hq)
    g = p.Hq // p.Hkv
    kv_cnt = (hq_cnt + g - 1) // g
    if hq_cnt % kv_cnt != 0:  # keep the group structure intact
        return None
    threads = max(1, min(16, cpu["usable"], b_cnt * hq_cnt))  # the oracle fans (batch, head) pairs over threads
    q = np.ascontiguousarray(p.q[:b_cnt, :hq_cnt])
    k = np.ascontiguousarray(p.k[:b_cnt, :kv_cnt])
    v = np.ascontiguousarray(p.v[:b_cnt, :kv_cnt])
    sq = p.s_q[:hq_cnt] if p.per_head else p.s_q
    sk = p.s_k[:kv_cnt] if p.per_head else p.s_k
    sv = p.s_v[:kv_cnt] if p.per_head else p.s_v
    so = s_o[:hq_cnt] if (p.per_head and s_o is not None) else s_o
    t0 = time.perf_counter()
    want = oracle.forward(q, k, v, sq, sk, sv, so, causal=p.causal, per_head=p.per_head, threads=threads)["out"]
    dt = time.perf_counter() - t0
    ops = 4 * p.d * p.pairs * b_cnt * hq_cnt
    res = {"value": ops / dt / 1e12, "unit": "TOPS", "cores": threads, "kind": "oracle",
           "sample": f"{b_cnt * hq_cnt} of {p.B * p.Hq} (batch, head) pairs, all rows, {dt:.1f} s",
           "seconds": dt, "host_cpu": cpu["model"], "host_nproc": cpu["nproc"], "host_usable_cores": cpu["usable"]}
    if gpu_out is not None:
        got = gpu_out[:b_cnt, :hq_cnt].cpu().numpy()
        res["bytes_compared_with_timed_output"] = int(want.size)
        res["parity_mismatching_bytes"] = int((got != want).sum())
    return res


def quantizer_bench(a, name, dev):
    """One step = Eq. quant on fp16 Q, K and V of the workload's shape (one batched call, per-tensor
    scales).  Two passes over the input are inherent (the scale needs the global max first), so
    the algorithmic bytes per element are 2 reads of 2 bytes and 1 write of 1 byte."""
    import numpy as np
    import torch

    import oracle
    import workloads as inputs
    from paper_2511_21513_amd import binding

    B, Hq, Hkv, L, d = inputs.CONFIGS[name][:5]
    g = torch.Generator(device=dev).manual_seed(0)
    xs = [torch.randn((B, h, L, d), device=dev, generator=g, dtype=torch.float32).half() for h in (Hq, Hkv, Hkv)]
    ia = binding.IntAttn(device=0)
    outs = [torch.empty(x.shape, dtype=torch.int8, device=dev) for x in xs]
    scs = [torch.empty(1, dtype=torch.float32, device=dev) for _ in xs]
    stream = torch.cuda.current_stream(dev).cuda_stream

    def step():
        ia.quantize_batch(xs, False, outs=outs, scales=scs, stream=stream)

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(a.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / a.steps
    n = sum(x.numel() for x in xs)
    alg_bytes = n * (2 * 2 + 1)
    gbps = alg_bytes / (ms * 1e-3) / 1e9
    # parity of the timed outputs on the smallest tensor, and the oracle's own rate beside it
    t0 = time.perf_counter()
    want_q, want_s = oracle.quantize(xs[1].float().cpu().numpy())
    cpu_s = time.perf_counter() - t0
    mism = int((outs[1].cpu().numpy() != want_q).sum()) + int(scs[1].cpu().numpy()[0] != want_s[0])
    res = {"metric": "dynamic INT8 quantizer (Eq. quant), algorithmic GB/s", "value": gbps, "unit": "GB/s", "n_gpus": 1,
           "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": name + " (fp16 Q, K, V -> INT8, per-tensor scales)", "elements": n},
           "parity_mismatches": mism,
           "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBS,
                        "traffic": None, "kernel": "absmax_kernel + quantize_kernel (one launch each for Q, K, V together)",
                        "algorithmic_bytes_per_step": alg_bytes},
           "cpu_baseline": {"value": xs[1].numel() * 5 / cpu_s / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                            "sample": f"the K tensor ({xs[1].numel()} elements), {cpu_s:.2f} s"}}
    # quantizer and attention back to back, nothing read by the host in between
    causal = bool(inputs.CONFIGS[name][5])
    att_out = torch.empty_like(outs[0])
    dargs, dkeep = ia.make_args(outs[0], outs[1], outs[2], att_out, scs[0], scs[1], scs[2], None, causal=causal,
                                per_head=False, device_scales=True)

    def chain():
        step()
        ia.forward_dynamic_args(dargs, stream)

    for _ in range(2):
        chain()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(a.steps):
        chain()
    e1.record()
    torch.cuda.synchronize()
    res["chain_fp16_to_int8_attention"] = {"entries": "intattn_quantize_batch (Q, K, V) + intattn_forward_dynamic",
                                           "ms_per_step": e0.elapsed_time(e1) / a.steps,
                                           "status": ia.dynamic_status()}
    # the same chain with Q quantized per token (finer groups over the query rows, Sec. 3.3)
    tok_scales = torch.empty((B, Hq, L), dtype=torch.float32, device=dev)
    hk, hv = (torch.empty(Hkv, dtype=torch.float32, device=dev) for _ in range(2))
    targs, tkeep = ia.make_args(outs[0], outs[1], outs[2], att_out, tok_scales, hk, hv, None, causal=causal,
                                device_scales=True, q_block=1)

    def chain_tok():
        ia.quantize(xs[0], out=outs[0], scales=tok_scales, stream=stream, q_block=1)
        ia.quantize(xs[1], True, out=outs[1], scales=hk, stream=stream)
        ia.quantize(xs[2], True, out=outs[2], scales=hv, stream=stream)
        ia.forward_dynamic_args(targs, stream)

    for _ in range(2):
        chain_tok()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(a.steps):
        chain_tok()
    e1.record()
    torch.cuda.synchronize()
    res["chain_per_token_q"] = {"entries": "intattn_quantize (Q, q_block 1) + 2 x intattn_quantize (K, V per head) + intattn_forward_dynamic (scale_mode 2)",
                                "ms_per_step": e0.elapsed_time(e1) / a.steps, "status": ia.dynamic_status()}
    ia.close()
    print(json.dumps(res))


def softmax_bench(a, name, dev):
    """One step = IndexSoftmax as an operator on INT32 logits of --softmax-heads heads of the
    workload ([heads * L, L], no mask).  HBM-bound: 4 bytes in and 1 byte out per element."""
    import numpy as np
    import torch

    import oracle
    import workloads as inputs
    from paper_2511_21513_amd import binding

    L = inputs.CONFIGS[name][3]
    rows, cols = a.softmax_heads * L, L
    g = torch.Generator(device=dev).manual_seed(0)
    c_int = 5203  # the workload's threshold
    logits = torch.randint(-4 * c_int, 4 * c_int, (rows, cols), device=dev, dtype=torch.int32, generator=g)
    prob = torch.empty((rows, cols), dtype=torch.uint8, device=dev)
    ia = binding.IntAttn(device=0)
    stream = torch.cuda.current_stream(dev).cuda_stream
    for _ in range(a.warmup):
        ia.index_softmax(logits, c_int, out=prob, stream=stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(a.steps):
        ia.index_softmax(logits, c_int, out=prob, stream=stream)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / a.steps
    alg_bytes = rows * cols * 5
    gbps = alg_bytes / (ms * 1e-3) / 1e9
    sample = np.unique(np.concatenate([[0, rows - 1], np.random.default_rng(0).integers(0, rows, 254)]))
    t0 = time.perf_counter()
    want = oracle.index_softmax(logits[sample].cpu().numpy(), c_int)
    cpu_s = time.perf_counter() - t0
    mism = int((prob[sample].cpu().numpy() != want).sum())
    res = {"metric": "IndexSoftmax operator (INT32 logits -> UINT8 probabilities), algorithmic GB/s", "value": gbps,
           "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
           "config": {"workload": f"logits of {a.softmax_heads} heads of {name}", "rows": rows, "cols": cols, "c_int": c_int},
           "parity_mismatching_bytes": mism,
           "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBS,
                        "traffic": None, "kernel": "index_softmax_kernel", "algorithmic_bytes_per_step": alg_bytes},
           "cpu_baseline": {"value": sample.size * cols * 5 / cpu_s / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                            "sample": f"{sample.size} of {rows} rows, {cpu_s:.2f} s"}}
    ia.close()
    print(json.dumps(res))


def decode_bench(a, name, dev):
    """One step = one decoded token for each of --decode-batch sequences: L = 1 query row per head
    against the workload's key/value length, heads and head dimension, causal (the token sees every
    key).  HBM-bound: K and V are read once; algorithmic bytes = K + V + Q + out."""
    import numpy as np
    import torch

    import oracle
    import workloads as inputs
    from paper_2511_21513_amd import binding

    _, Hq, Hkv, Lk, d = inputs.CONFIGS[name][:5]
    B = a.decode_batch
    g = torch.Generator(device=dev).manual_seed(0)
    # the recipe's value range: symmetric INT8 with the extremes present
    q = torch.randint(-127, 128, (B, Hq, 1, d), device=dev, dtype=torch.int8, generator=g)
    k = torch.randint(-127, 128, (B, Hkv, Lk, d), device=dev, dtype=torch.int8, generator=g)
    v = torch.randint(-127, 128, (B, Hkv, Lk, d), device=dev, dtype=torch.int8, generator=g)
    out = torch.empty_like(q)
    # scales of the size the workload's own quantizer finds (c4: max|Q| about 5, one K channel times ten), so the
    # clip thresholds are those of the prefill workload, about 5200
    s_q = np.linspace(0.035, 0.045, Hq).astype(np.float32)
    s_k = np.linspace(0.33, 0.39, Hkv).astype(np.float32)
    s_v = np.linspace(0.02, 0.03, Hkv).astype(np.float32)
    ia = binding.IntAttn(device=0, variant=a.variant)
    args, keep = ia.make_args(q, k, v, out, s_q, s_k, s_v, None, causal=True, per_head=True)
    stream = torch.cuda.current_stream(dev).cuda_stream
    for _ in range(a.warmup):
        ia.forward_args(args, stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(a.steps):
        ia.forward_args(args, stream)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / a.steps
    alg_bytes = k.numel() + v.numel() + q.numel() + out.numel()
    gbps = alg_bytes / (ms * 1e-3) / 1e9
    # parity of the timed output on two sequences, and the oracle's own rate beside it
    bs = sorted(set([0, B - 1] + list(range(0, B, max(1, B // 6)))))
    qs, ks, vs = (x[bs].cpu().numpy() for x in (q, k, v))
    t0 = time.perf_counter()
    cpu = host_cpu()
    threads = max(1, min(16, cpu["usable"], len(bs) * Hq))
    want = oracle.forward(qs, ks, vs, s_q, s_k, s_v, None, causal=True, per_head=True, threads=threads)["out"]
    cpu_s = time.perf_counter() - t0
    mism = int((out[bs].cpu().numpy() != want).sum())
    res = {"metric": "decode attention (one token per sequence), algorithmic GB/s", "value": gbps, "unit": "GB/s",
           "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
           "config": {"workload": f"decode on the shape of {name}", "B": B, "Hq": Hq, "Hkv": Hkv, "L": 1, "Lkv": Lk, "d": d,
                      "causal": True, "scales": "per-head", "variant": a.variant},
           "tokens_per_s": B / (ms * 1e-3),
           "parity_mismatching_bytes": mism,
           "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbps / HBM_PEAK_GBS,
                        "traffic": stored_counters(f"decode_{name}_b{B}").get("step_hbm_bytes"),
                        "kernel": "decode_fused_kernel (one launch; variant 10: decode_scores_kernel + decode_lookup_kernel + decode_pv_kernel + decode_finish_kernel)",
                        "algorithmic_bytes_per_step": alg_bytes},
           "cpu_baseline": {"value": (ks.nbytes + vs.nbytes + 2 * qs.nbytes) / cpu_s / 1e9, "unit": "GB/s",
                            "cores": threads, "kind": "oracle", "host_cpu": cpu["model"], "host_nproc": cpu["nproc"],
                            "sample": f"{len(bs)} of {B} sequences, all heads, {cpu_s:.2f} s"}}
    ia.close()
    print(json.dumps(res))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--preheat", type=int, default=100,
                    help="forward calls issued before the warm-up steps, so that the timed steps see the GPU at its "
                         "working clocks rather than waking up from idle (the first 10-20 ms after idle run several "
                         "percent slower); 0 switches it off")
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-comparator", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="instead of the benchmark, run a plain device copy of this many MiB three times "
                         "(the known-size reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--cpu-heads", type=int, default=32)
    ap.add_argument("--batch", type=int, default=None,
                    help="override the workload's batch size (e.g. --workload c2 --batch 512 shows the bandwidth the "
                         "kernel reaches on short sequences once the GPU is filled)")
    ap.add_argument("--softmax", action="store_true",
                    help="instead of the attention benchmark, time IndexSoftmax as an operator on INT32 logits of "
                         "the workload's length (HBM-bound)")
    ap.add_argument("--softmax-heads", type=int, default=8)
    ap.add_argument("--decode", action="store_true",
                    help="instead of the prefill benchmark, time one decoded token per sequence against the "
                         "workload's key/value length (split-key kernels, HBM-bound)")
    ap.add_argument("--decode-batch", type=int, default=32)
    ap.add_argument("--quantizer", action="store_true",
                    help="instead of the attention benchmark, time the dynamic quantizer in front of it: "
                         "fp16 Q, K, V of the workload's shape to INT8 with per-tensor scales (HBM-bound)")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (heads are independent; nothing is sharded "
              "or exchanged); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    if a.copy_calibration > 0:
        n = a.copy_calibration << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n, "launches": 3}))
        return

    import workloads as inputs
    from paper_2511_21513_amd import binding

    name = ALIASES.get(a.workload, a.workload)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if a.quantizer:
        return quantizer_bench(a, name, dev)
    if a.decode:
        return decode_bench(a, name, dev)
    if a.softmax:
        return softmax_bench(a, name, dev)
    p = inputs.make_problem(name, B=a.batch)  # --batch: a scaled-batch variant of a short workload (not the headline line)
    ia = binding.IntAttn(device=0, variant=a.variant)
    q, k, v = (torch.from_numpy(x).to(dev) for x in (p.q, p.k, p.v))
    out = torch.empty_like(q)
    s_o = inputs.calibrated_out_scale(p, sample_rows=16)
    args, keep = ia.make_args(q, k, v, out, p.s_q, p.s_k, p.s_v, s_o, causal=p.causal, per_head=p.per_head)
    stream = torch.cuda.current_stream(dev).cuda_stream

    def timed(fn, steps, warmup):
        """`steps` back-to-back calls between two synchronizations, an event before each and one after
        the last: (mean ms per step over the whole bracket, wall-clock ms per step, median ms of a step)."""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t0 = time.perf_counter()
        for i in range(steps):
            evs[i].record()
            fn()
        evs[steps].record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        each = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(steps))
        median = each[steps // 2] if steps % 2 else 0.5 * (each[steps // 2 - 1] + each[steps // 2])
        return evs[0].elapsed_time(evs[steps]) / steps, wall_ms, median

    for _ in range(a.preheat):  # not steps of the measurement: see --preheat
        ia.forward_args(args, stream)
    torch.cuda.synchronize()
    ms, wall_ms, median_ms = timed(lambda: ia.forward_args(args, stream), a.steps, a.warmup)
    tops = p.ops / (ms * 1e-3) / 1e12
    out_timed = out.clone()  # later calls (stages, comparator) write `out` again

    # The step is up to three kernels on one stream: V column sums, sweeps A+B, sweep C.  Sweep C is
    # the dominant one and executes every counted operation (it recomputes Q.K^T and does P.V), so
    # the roofline object is its: timed alone through the staged entry point, same HIP events.
    try:
        ia.forward_stage(args, 1, stream)
        ab_ms = timed(lambda: ia.forward_stage(args, 1, stream), a.steps, 1)[0]
        c_ms = timed(lambda: ia.forward_stage(args, 2, stream), a.steps, 1)[0]
        kernels = {"colsum_kernel+sweeps_a_b": ab_ms, "sweep_c_kernel": c_ms}
        dom_name, dom_ms = "sweep_c_kernel", c_ms
    except binding.IntAttnError:
        kernels = {"fwd_kernel (colsum_kernel included)": ms}  # single launch for this problem size
        dom_name, dom_ms = "fwd_kernel", ms
    dom_tops = p.ops / (dom_ms * 1e-3) / 1e12

    # sampled parity against the oracle on the benchmarked launch
    import oracle

    rows = np.asarray([0, 1, p.L // 2, p.L - 1], dtype=np.int32)
    want = oracle.rows(p.q, p.k, p.v, p.s_q, p.s_k, p.s_v, s_o, b=p.B - 1, hq=p.Hq - 1, rows=rows, causal=p.causal,
                       per_head=p.per_head)["out"]
    mism = int((out_timed[p.B - 1, p.Hq - 1].cpu().numpy()[rows] != want).sum())

    # Readings a timing run cannot take itself (rocprofv3 --pmc), stored with the hash of the kernel
    # sources they were taken on; absent or stale -> null.
    ctr = stored_counters(name) if (a.variant == 0 and not a.batch) else {}
    traffic = None
    if "sweep_c_fetch_bytes_per_launch" in ctr and dom_name == "sweep_c_kernel":
        traffic = ctr["sweep_c_fetch_bytes_per_launch"] + ctr["sweep_c_write_bytes_per_launch"]
    # The IndexSoftmax stage is element-wise integer work on the vector ALUs: its roofline is the lane
    # operations per second the chip can issue.  Lane operations = 64 x vector instructions issued
    # (SQ_INSTS_VALU, matrix instructions excluded), per score element of the causal triangle.
    score_elems = p.pairs * p.B * p.Hq
    valu = {"bound": "alu", "peak": VALU_PEAK_LANE_OPS / 1e12, "unit": "T lane-op/s", "score_elements_per_step": score_elems,
            "lane_ops_per_score": None, "achieved": None, "frac": None}
    if "step_valu_insts" in ctr:
        lane_ops = 64.0 * ctr["step_valu_insts"]
        valu.update({"lane_ops_per_score": lane_ops / score_elems,
                     "lane_ops_per_score_by_kernel": {k[:-len("_valu_insts")]: 64.0 * v / score_elems for k, v in ctr.items()
                                                      if k.endswith("_valu_insts") and k != "step_valu_insts"},
                     "achieved": lane_ops / (ms * 1e-3) / 1e12, "frac": lane_ops / (ms * 1e-3) / VALU_PEAK_LANE_OPS})

    res = {
        "metric": "int8 attention TOPS (QK^T+PV) + % of int8 MFMA peak at L=8192",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": name + (f" (batch scaled to {a.batch})" if a.batch else ""), "B": p.B, "Hq": p.Hq, "Hkv": p.Hkv, "L": p.L, "d": p.d,
                   "causal": p.causal, "scales": "per-head" if p.per_head else "per-tensor",
                   "lut_bits": 5, "clip": 6.6, "variant": a.variant},
        "pct_of_int8_mfma_peak": 100.0 * tops / INT8_MFMA_PEAK_TOPS,
        "wall_ms_per_step": wall_ms,
        "preheat_calls_before_warmup": a.preheat,
        "median_ms_per_step": median_ms, "value_at_median": p.ops / (median_ms * 1e-3) / 1e12,
        "sampled_parity_mismatching_bytes": mism,
        "roofline": {"bound": "mfma", "achieved": dom_tops, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": dom_tops / INT8_MFMA_PEAK_TOPS, "traffic": traffic,
                     "kernel": dom_name, "kernel_ms_per_launch": dom_ms, "counted_ops_per_launch": p.ops,
                     "whole_step_frac": tops / INT8_MFMA_PEAK_TOPS, "kernels_ms": kernels,
                     "hbm_algorithmic_bytes_per_launch": p.algorithmic_bytes,
                     "hbm_algorithmic_GBps": p.algorithmic_bytes / (ms * 1e-3) / 1e9,
                     "counters_from": ctr.get("source")},
        "valu_roofline": valu,
    }
    # the same step with the scales in device memory (parameters derived by a kernel, no host read)
    dscales = [torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(dev) for x in (p.s_q, p.s_k, p.s_v, s_o)]
    out_d = torch.empty_like(q)
    dargs, dkeep = ia.make_args(q, k, v, out_d, *dscales, causal=p.causal, per_head=p.per_head, device_scales=True)
    dms = timed(lambda: ia.forward_dynamic_args(dargs, stream), a.steps, 2)[0]
    res["device_scales"] = {"entry": "intattn_forward_dynamic", "ms_per_step": dms, "TOPS": p.ops / (dms * 1e-3) / 1e12,
                            "bytes_differing_from_host_scale_output": int((out_d != out_timed).sum().item()),
                            "status": ia.dynamic_status()}
    if not a.no_comparator:
        try:
            cms = timed(lambda: ia.forward_args(args, stream, quantonly=True), max(3, a.steps // 3), 2)[0]
            res["comparator"] = {"kind": "fused conventional INT8 pipeline (dequant -> fp32 softmax -> requant)",
                                 "ms_per_step": cms, "speedup_of_intattention": cms / ms}
        except binding.IntAttnError as e:
            res["comparator"] = {"error": str(e)}
    if not a.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(p, s_o, a.cpu_heads, gpu_out=out_timed)
        if res["cpu_baseline"] and "parity_mismatching_bytes" in res["cpu_baseline"]:
            res["parity_mismatching_bytes"] = res["cpu_baseline"]["parity_mismatching_bytes"]
            res["parity_bytes_compared"] = res["cpu_baseline"]["bytes_compared_with_timed_output"]
    ia.close()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
