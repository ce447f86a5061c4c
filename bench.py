#!/usr/bin/env python3
"""Benchmark of the VeLoRA hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input
for one linear layer: compress(X, v) -> S, then weight_grad(G, S, v) -> dW
(init_v is a one-off and is not part of the steady-state step).  Inputs are
resident in HBM before the timed region starts; the step rotates through a ring
of distinct buffer sets larger than the 256 MB last-level cache so that no
re-read is served from cache.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

prints ONE JSON line.  `value` is the whole step's algorithmic bytes per second;
`roofline` prices the dominant kernel (compress) against the HBM peak from HIP
event timings taken inside the timed region (mean, median and minimum), and
against streaming ceilings measured in the same run with the library's own
plainest kernels (`measured_ceilings`, `frac_of_measured`); `roofline.weight_grad`
does the same for the gradient kernels; `warm_cache` is the same step without
buffer rotation (labelled: it is not an HBM figure); `vit_block_sequence` times
configuration 2 as twelve launches on twelve buffers; `shapes` lists every
layer shape of the configurations; `cpu_baseline` is the CPU oracle timed on
this machine's host cores, single-threaded and on all cores it may use, on a stated
sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 MFMA peak
RING_BYTES = 1 << 30            # rotate through at least this much distinct memory
DEFAULT_WORKLOAD = "cfg4_down"  # LLaMA-7B-like MLP down projection (D=11008 -> O=4096, d=256)
METRIC = "compress GB/s (% HBM peak); weight-grad TFLOP/s (% MFMA peak), 1 MI355X"


def _parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--dw-dtype", choices=["f32", "bf16"], default="f32")
    ap.add_argument("--no-shapes", action="store_true", help="skip the per-shape sweep")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the streaming probes and the step's two entry points on the headline workload "
                         "(no warm-cache leg, no other records, no shape sweep): under rocprofv3 every launch of "
                         "a hot-path kernel then has the headline shape and cold buffers")
    ap.add_argument("--shape-steps", type=int, default=100)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 256 MiB device-to-device copies (a kernel of known traffic, "
                         "used to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


class Ring:
    """R distinct (X, G, S, dW) buffer sets for one layer shape."""

    def __init__(self, vl, torch, sh, X0, G0, v, dw_dtype):
        import workloads as wl
        dw_b = 2 if dw_dtype == torch.bfloat16 else 4
        set_bytes = (sh.N * sh.D + sh.N * sh.O + sh.N * sh.M) * sh.elem_bytes + sh.O * sh.D * dw_b
        self.R = max(2, -(-RING_BYTES // set_bytes))
        self.sh, self.v, self.vl = sh, v, vl
        self.X = [X0] + [X0.clone() for _ in range(self.R - 1)]
        self.G = [G0] + [G0.clone() for _ in range(self.R - 1)]
        self.S = [torch.empty((sh.N, sh.M), dtype=X0.dtype, device=X0.device) for _ in range(self.R)]
        self.dW = [torch.empty((sh.O, sh.D), dtype=dw_dtype, device=X0.device) for _ in range(self.R)]
        in_dt = vl.BF16 if sh.dtype == wl.BF16 else vl.F32
        need = vl.velora_workspace_bytes(vl.OP_WEIGHT_GRAD, sh.N, sh.D, sh.O, sh.M, in_dt)
        self.ws = torch.empty(max(need, 16), dtype=torch.uint8, device=X0.device)
        self.ws_bytes = need

    def compress(self, i):
        r = i % self.R
        self.vl.velora_compress(self.X[r], self.v, self.sh.M, S=self.S[r])

    def wgrad(self, i):
        r = i % self.R
        self.vl.velora_weight_grad(self.G[r], self.S[r], self.v, self.sh.D, dW=self.dW[r], ws=self.ws)

    def step(self, i):
        self.compress(i)
        self.wgrad(i)


EVENT_BATCH = 10   # launches between two HIP events


def _stats(samples):
    """mean / median / min of per-launch microseconds (each sample = one event pair around EVENT_BATCH launches)."""
    xs = sorted(samples)
    n = len(xs)
    med = xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])
    return {"mean": sum(xs) / n, "median": med, "min": xs[0], "samples": n}


def _time_steps(torch, ring, steps, warmup, with_events, rotate=True):
    """-> (seconds for `steps` steps, compress per-launch us samples, wgrad per-launch us samples).

    Without events: `steps` steps back to back, wall clock around a
    synchronise on both sides (this is what `value` is computed from).
    With events: the same launches, grouped so that HIP events on the launch
    stream (torch's current stream, the one the binding launches on) bracket
    EVENT_BATCH launches of one entry point at a time; an event pair around a
    single 20-100 us kernel would add its own few us of dispatch latency to
    every sample.  rotate=False keeps every launch on buffer set 0 (warm cache)."""
    pick = (lambda i: i) if rotate else (lambda i: 0)
    for i in range(warmup):
        ring.step(pick(i))
    torch.cuda.synchronize()
    if not with_events:
        t0 = time.perf_counter()
        for i in range(steps):
            ring.step(pick(warmup + i))
        torch.cuda.synchronize()
        return time.perf_counter() - t0, None, None
    n_batches = max(1, steps // EVENT_BATCH)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_batches)]
    t0 = time.perf_counter()
    for b in range(n_batches):
        i0 = warmup + b * EVENT_BATCH
        ev[b][0].record()
        for i in range(EVENT_BATCH):
            ring.compress(pick(i0 + i))
        ev[b][1].record()
        for i in range(EVENT_BATCH):
            ring.wgrad(pick(i0 + i))
        ev[b][2].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    c = [e[0].elapsed_time(e[1]) / EVENT_BATCH * 1e3 for e in ev]
    w = [e[1].elapsed_time(e[2]) / EVENT_BATCH * 1e3 for e in ev]
    return dt, c, w


def _settle(torch, ring, ms=30.0):
    """Steps of the ring's own workload until `ms` of them have run: the same protection against the chip's
    power-management transient as the headline's 100 warm-up steps (a fixed count would be 3 ms of a small
    layer and 20 ms of a large one)."""
    t0 = time.perf_counter()
    i = 0
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(20):
            ring.step(i)
            i += 1
        torch.cuda.synchronize()


def _event_samples_us(torch, fn, launches):
    """Per-launch microseconds of fn(i), one sample per event pair around EVENT_BATCH launches."""
    # at least 20 ms of the same launches first (see _settle)
    t0, k = time.perf_counter(), 0
    while k < 3 or (time.perf_counter() - t0) * 1e3 < 20.0:
        for _ in range(5):
            fn(k)
            k += 1
        torch.cuda.synchronize()
    n_batches = max(1, launches // EVENT_BATCH)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n_batches)]
    for b in range(n_batches):
        ev[b][0].record()
        for i in range(EVENT_BATCH):
            fn(k + b * EVENT_BATCH + i)
        ev[b][1].record()
    torch.cuda.synchronize()
    return [e[0].elapsed_time(e[1]) / EVENT_BATCH * 1e3 for e in ev]


def _event_avg_us(torch, fn, launches):
    """Mean microseconds per launch of fn(i), EVENT_BATCH launches between two events."""
    xs = _event_samples_us(torch, fn, launches)
    return sum(xs) / len(xs)


def _measured_ceilings(vl, torch, dev, launches):
    """What the memory system gives the library's plainest streaming kernels on this machine, in this run:
    read-only, write-only and copy over a ring of buffers larger than the last-level cache (GB/s,
    from the median launch)."""
    nbytes = 384 << 20
    sets = 4
    bufs = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(sets)]
    for b in bufs:
        b.zero_()
    sink = torch.zeros(64, dtype=torch.int32, device=dev)
    out = {}
    for kind in ("read", "write", "copy"):
        if kind == "read":
            fn = lambda i: vl.velora_bandwidth_probe("read", src=bufs[i % sets], sink=sink)
        elif kind == "write":
            fn = lambda i: vl.velora_bandwidth_probe("write", dst=bufs[i % sets])
        else:
            fn = lambda i: vl.velora_bandwidth_probe("copy", src=bufs[i % sets], dst=bufs[(i + 2) % sets])
        st = _stats(_event_samples_us(torch, fn, launches))
        moved = nbytes * (2 if kind == "copy" else 1)
        out[kind + "_GBps"] = round(moved / st["median"] * 1e-3, 1)
    out["note"] = ("velora_bandwidth_probe: one block per compute unit, eight non-temporal 16-byte accesses in flight "
                   f"per thread, {nbytes >> 20} MiB per launch over {sets} buffers; copy counts bytes read + written")
    del bufs
    return out


def _vit_sequence_record(vl, torch, wl, dev, reps):
    """Configuration 2 the way a ViT-B runs it: twelve blocks, i.e. twelve compress launches (and twelve
    weight gradients) back to back on twelve distinct buffer sets, because one 3-20 us launch cannot show
    a bandwidth through its own launch overhead."""
    sh = wl.shape_by_name("cfg2_vit_fc1")
    blocks = 12
    Xs, Gs = _device_inputs(torch, sh, dev)
    v = vl.velora_init_v(Xs, sh.M, allow_degenerate=True)
    X = [Xs] + [Xs.clone() for _ in range(blocks - 1)]
    G = [Gs] + [Gs.clone() for _ in range(blocks - 1)]
    S = [torch.empty((sh.N, sh.M), dtype=Xs.dtype, device=dev) for _ in range(blocks)]
    dW = [torch.empty((sh.O, sh.D), dtype=torch.float32, device=dev) for _ in range(blocks)]
    need = vl.velora_workspace_bytes(vl.OP_WEIGHT_GRAD, sh.N, sh.D, sh.O, sh.M, vl.BF16)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)

    def seq(which):
        for b in range(blocks):
            if which == "compress":
                vl.velora_compress(X[b], v, sh.M, S=S[b])
            else:
                vl.velora_weight_grad(G[b], S[b], v, sh.D, dW=dW[b], ws=ws)

    rec = {"workload": sh.name, "launches_per_sequence": blocks}
    for which, nbytes in (("compress", sh.compress_bytes()), ("weight_grad", sh.wgrad_bytes(4))):
        for _ in range(2):
            seq(which)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(reps)]
        for r in range(reps):
            ev[r][0].record()
            seq(which)
            ev[r][1].record()
        torch.cuda.synchronize()
        st = _stats([e[0].elapsed_time(e[1]) / blocks * 1e3 for e in ev])
        rec[which] = {"us_per_launch_median": round(st["median"], 2), "us_per_launch_min": round(st["min"], 2),
                      "GBps": round(nbytes / st["median"] * 1e-3, 1),
                      "frac": round(nbytes / st["median"] * 1e-3 / HBM_PEAK_GBPS, 4)}
    rec["note"] = ("the twelve buffer sets hold 1.2 GB, so nothing is served from cache; what keeps these launches "
                   "below the large layers' rates is launch ramp-up and drain, a few us per launch")
    return rec


def _graph_step_us(torch, ring, steps):
    """The same step replayed from a captured HIP graph (one graph holding one
    step per ring set): what remains when the host's launch work is taken out."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for r in range(ring.R):
            ring.step(r)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for r in range(ring.R):
            ring.step(r)
    reps = max(1, steps // ring.R)
    for _ in range(2):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / (reps * ring.R) * 1e6


def _other_steps_record(vl, torch, sh, ring, launches):
    """The remaining steps of the path, each on its own: init_v (one-off per
    layer), the per-batch-v variants, and the materialising reconstruct."""
    R = ring.R
    eb = sh.elem_bytes
    x_bytes = sh.N * sh.D * eb
    s_bytes = sh.N * sh.M * eb
    need = vl.velora_workspace_bytes(vl.OP_INIT_V, sh.N, sh.D, 0, sh.M, vl.BF16 if sh.dtype == "bf16" else vl.F32)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=ring.X[0].device)
    vbuf = torch.empty(sh.d, dtype=torch.float32, device=ring.X[0].device)
    state = torch.zeros(sh.d, dtype=torch.float32, device=ring.X[0].device)
    out = {}
    t = _event_avg_us(torch, lambda i: vl.velora_update_v(ring.X[i % R], sh.M, v=vbuf, ws=ws), launches)
    out["init_v"] = {"avg_us": round(t, 2), "algorithmic_bytes": x_bytes,
                     "frac": round(x_bytes / t * 1e-3 / HBM_PEAK_GBPS, 4),
                     "note": "velora_update_v without a state: the same kernels as velora_init_v, minus its final synchronise"}
    t = _event_avg_us(torch, lambda i: vl.velora_compress_update(ring.X[i % R], ring.v, sh.M, mean_state=state, beta=0.9,
                                                                 S=ring.S[i % R], v_out=vbuf, ws=ws), launches)
    out["compress_update"] = {"avg_us": round(t, 2), "algorithmic_bytes": x_bytes + s_bytes,
                              "frac": round((x_bytes + s_bytes) / t * 1e-3 / HBM_PEAK_GBPS, 4)}
    Xhat = torch.empty_like(ring.X[0])
    t = _event_avg_us(torch, lambda i: vl.velora_reconstruct(ring.S[i % R], ring.v, sh.D, Xhat=Xhat), launches)
    out["reconstruct"] = {"avg_us": round(t, 2), "algorithmic_bytes": x_bytes + s_bytes,
                          "frac": round((x_bytes + s_bytes) / t * 1e-3 / HBM_PEAK_GBPS, 4)}
    return out


def _swiglu_record(vl, torch, sh, v, dev, launches):
    """Producer-side fusion: X = silu(gate) * up written and compressed in one pass
    (not part of `value`).  Bytes: gate and up in, X and S out."""
    sets = 2
    gate = [torch.randn((sh.N, sh.D), device=dev).mul_(2.0).to(torch.bfloat16) for _ in range(sets)]
    up = [torch.randn((sh.N, sh.D), device=dev).to(torch.bfloat16) for _ in range(sets)]
    X = [torch.empty((sh.N, sh.D), device=dev, dtype=torch.bfloat16) for _ in range(sets)]
    S = torch.empty((sh.N, sh.M), device=dev, dtype=torch.bfloat16)
    us = _event_avg_us(torch, lambda i: vl.velora_swiglu_compress(gate[i % sets], up[i % sets], v, sh.M,
                                                                  X=X[i % sets], S=S), launches)
    nbytes = 3 * sh.N * sh.D * 2 + sh.N * sh.M * 2 + sh.d * 4
    return {"kernel": "swiglu_compress_vec_kernel", "bound": "hbm", "avg_us": round(us, 2), "algorithmic_bytes": nbytes,
            "achieved": round(nbytes / us * 1e-3, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(nbytes / us * 1e-3 / HBM_PEAK_GBPS, 4)}


def _linear_record(vl, torch, sh, v, dev, launches):
    """The layer's forward with compress inside the GEMM (not part of `value`):
    Y = X W^T as a bf16 MFMA kernel that also forms S from its tiles of X.  Next
    to it, for scale only, the vendor GEMM followed by velora_compress."""
    launches = max(5, min(launches, 40))
    X = torch.randn((sh.N, sh.D), device=dev).to(torch.bfloat16)
    W = (torch.randn((sh.O, sh.D), device=dev) * sh.D ** -0.5).to(torch.bfloat16)
    Y = torch.empty((sh.N, sh.O), device=dev, dtype=torch.bfloat16)
    S = torch.empty((sh.N, sh.M), device=dev, dtype=torch.bfloat16)
    us = _event_avg_us(torch, lambda i: vl.velora_linear_compress(X, W, v, sh.M, Y=Y, S=S), launches)
    Wt = W.t()
    ref = _event_avg_us(torch, lambda i: (torch.matmul(X, Wt, out=Y), vl.velora_compress(X, v, sh.M, S=S)), launches)
    flops = 2.0 * sh.N * sh.O * sh.D + 2.0 * sh.N * sh.D
    rec = {"kernel": "linear_mfma_kernel<fused S>", "bound": "mfma", "avg_us": round(us, 1), "algorithmic_flops": flops,
           "achieved": round(flops / us * 1e-6, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
           "frac": round(flops / us * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
           "vendor_gemm_plus_compress_us": round(ref, 1)}
    # the input gradient of the same layer: dX = G W, W read in its own [O, D] layout
    G = (torch.randn((sh.N, sh.O), device=dev) * 0.05).to(torch.bfloat16)
    dX = torch.empty((sh.N, sh.D), device=dev, dtype=torch.bfloat16)
    us2 = _event_avg_us(torch, lambda i: vl.velora_grad_input(G, W, dX=dX), launches)
    ref2 = _event_avg_us(torch, lambda i: torch.matmul(G, W, out=dX), launches)
    fl2 = 2.0 * sh.N * sh.O * sh.D
    rec["grad_input"] = {"kernel": "linear_mfma_kernel<W as stored>", "avg_us": round(us2, 1),
                         "achieved": round(fl2 / us2 * 1e-6, 1), "unit": "TFLOP/s",
                         "frac": round(fl2 / us2 * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4), "vendor_gemm_us": round(ref2, 1)}
    return rec


def _dense_form_record(vl, torch, sh, v, dev, launches):
    """The backward of paper Listing 1 as printed, for comparison with the factored weight gradient (not part
    of `value`): Xhat = reconstruct(S, v) materialised by velora_reconstruct, then the dense product
    dW = G^T Xhat in the vendor GEMM (bf16 in, bf16 out).  `gemm_only_us` is what any kernel that builds the
    tiles of Xhat on the fly instead would still have to spend at the vendor GEMM's rate on this shape: d times
    the flops of the factored form."""
    launches = max(5, min(launches, 20))
    G = (torch.randn((sh.N, sh.O), device=dev) * 0.05).to(torch.bfloat16)
    S = torch.randn((sh.N, sh.M), device=dev).to(torch.bfloat16)
    Xhat = torch.empty((sh.N, sh.D), device=dev, dtype=torch.bfloat16)
    dWd = torch.empty((sh.O, sh.D), device=dev, dtype=torch.bfloat16)
    Gt = G.t()
    vl.velora_reconstruct(S, v, sh.D, Xhat=Xhat)
    gemm = _event_avg_us(torch, lambda i: torch.matmul(Gt, Xhat, out=dWd), launches)
    both = _event_avg_us(torch, lambda i: (vl.velora_reconstruct(S, v, sh.D, Xhat=Xhat),
                                           torch.matmul(Gt, Xhat, out=dWd)), launches)
    flops = sh.wgrad_flops_dense()
    return {"what": "velora_reconstruct + vendor GEMM G^T Xhat (bf16 out)", "reconstruct_plus_gemm_us": round(both, 1),
            "gemm_only_us": round(gemm, 1), "gemm_TFLOPs": round(flops / gemm * 1e-6, 1),
            "gemm_frac_mfma": round(flops / gemm * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
            "gemm_time_at_mfma_peak_us": round(flops / MFMA_BF16_PEAK_TFLOPS * 1e-6, 1),
            "materialised_MB": round(sh.N * sh.D * 2 / 1e6, 1)}


def _mlp_block_record(torch, dev):
    """A whole LLaMA-7B-like gated MLP block (hidden 4096, intermediate 11008, 16384 tokens, bf16), forward +
    backward through autograd: the plain block against the same block with VeLoRA on its three projections
    (paper Sec. 5.5, "Comparison with gradient checkpointing", Table 7: what the method costs in time and what
    it frees in memory).  Memory = what stays allocated
    between the end of the forward and the start of the backward, beyond weights, input and output.
    Not part of `value`."""
    from paper_2405_17991_amd import autograd as va
    N, H, F, d_h, d_f = 16384, 4096, 11008, 256, 256
    torch.manual_seed(0)
    blk = va.VeLoRALlamaMLP(H, F, d_h, d_f, device=dev, dtype=torch.bfloat16)
    h0 = torch.randn((N, H), device=dev).to(torch.bfloat16)
    blk.init_v(h0)
    gout = (torch.randn((N, H), device=dev) * 0.05).to(torch.bfloat16)

    def plain(h):
        gate = torch.nn.functional.linear(h, blk.w_gate)
        up = torch.nn.functional.linear(h, blk.w_up)
        return torch.nn.functional.linear(torch.nn.functional.silu(gate) * up, blk.w_down)

    def run(fn, reps=6):
        held, times = 0, []
        for r in range(reps + 2):
            for p in blk.parameters():
                p.grad = None
            h = h0.clone().requires_grad_(True)
            torch.cuda.synchronize()
            base = torch.cuda.memory_allocated()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            y = fn(h)
            torch.cuda.synchronize()
            held = torch.cuda.memory_allocated() - base - y.numel() * y.element_size()
            y.backward(gout)
            e1.record()
            torch.cuda.synchronize()
            if r >= 2:
                times.append(e0.elapsed_time(e1))
            del y, h
        return sum(times) / len(times), held

    t_plain, m_plain = run(plain)
    t_velora, m_velora = run(blk)
    return {"workload": "LLaMA-7B-like MLP block, N=16384, 4096 -> 11008 -> 4096, d=256, bf16, forward + backward",
            "plain_ms": round(t_plain, 3), "velora_ms": round(t_velora, 3),
            "time_ratio": round(t_velora / t_plain, 4),
            "plain_saved_MB": round(m_plain / 1e6, 1), "velora_saved_MB": round(m_velora / 1e6, 1),
            "note": "the three dense products and their input gradients run in the vendor GEMM in both columns; "
                    "the VeLoRA column keeps gate and up (the activation's own backward needs them) but neither "
                    "the block input nor the down projection's input"}


def _rmsnorm_record(vl, torch, wl, dev, launches):
    """Producer-side fusion for the attention projections' input (LLaMA-7B-like:
    N=16384, D=4096, d=256): X = RMSNorm(H) written and compressed in one pass."""
    sh = wl.shape_by_name("cfg4_attn")
    sets = 4
    H = [torch.randn((sh.N, sh.D), device=dev).to(torch.bfloat16) for _ in range(sets)]
    X = [torch.empty((sh.N, sh.D), device=dev, dtype=torch.bfloat16) for _ in range(sets)]
    S = torch.empty((sh.N, sh.M), device=dev, dtype=torch.bfloat16)
    gamma = torch.ones(sh.D, device=dev)
    v = torch.nn.functional.normalize(torch.randn(sh.d, device=dev), dim=0)
    us = _event_avg_us(torch, lambda i: vl.velora_rmsnorm_compress(H[i % sets], gamma, 1e-5, v, sh.M, X=X[i % sets], S=S),
                       launches)
    nbytes = 2 * sh.N * sh.D * 2 + sh.N * sh.M * 2 + sh.D * 4 + sh.d * 4
    return {"kernel": "rmsnorm_compress_row_kernel", "workload": sh.name, "bound": "hbm", "avg_us": round(us, 2),
            "algorithmic_bytes": nbytes, "achieved": round(nbytes / us * 1e-3, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(nbytes / us * 1e-3 / HBM_PEAK_GBPS, 4)}


def _adamw_record(vl, torch, sh, v, dev, steps):
    """The optimiser step fed by the factored gradient (not part of `value`): W
    and both moments in float32 stream through HBM once, dW is never formed."""
    sets = max(2, -(-RING_BYTES // (sh.O * sh.D * 12)))
    W = [torch.randn((sh.O, sh.D), device=dev) * 0.05 for _ in range(sets)]
    m = [torch.zeros((sh.O, sh.D), device=dev) for _ in range(sets)]
    u = [torch.zeros((sh.O, sh.D), device=dev) for _ in range(sets)]
    T = torch.randn((sh.O, sh.M), device=dev) * 0.02

    def run(i):
        r = i % sets
        vl.velora_adamw_step_factor(T, v, W[r], m[r], u[r], lr=1e-3, step=1 + i // sets)

    for i in range(3):
        run(i)
    n_batches = max(1, steps // EVENT_BATCH)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n_batches)]
    for b in range(n_batches):
        ev[b][0].record()
        for i in range(EVENT_BATCH):
            run(3 + b * EVENT_BATCH + i)
        ev[b][1].record()
    torch.cuda.synchronize()
    us = sum(e[0].elapsed_time(e[1]) for e in ev) / (n_batches * EVENT_BATCH) * 1e3
    nbytes = sh.O * sh.D * 24 + sh.O * sh.M * 4 + sh.d * 4
    return {"kernel": "adamw_factor_vec_kernel", "bound": "hbm", "avg_us": round(us, 2), "algorithmic_bytes": nbytes,
            "achieved": round(nbytes / us * 1e-3, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(nbytes / us * 1e-3 / HBM_PEAK_GBPS, 4), "W_dtype": "f32", "ring_sets": sets}


def _device_inputs(torch, sh, dev):
    """Synthetic layer inputs drawn on the device (sweep only: the kernels have
    no data-dependent control flow, so timing needs the shape and dtype, and
    roughly the distribution; parity is established by the tests on the
    host-generated inputs)."""
    import workloads as wl
    g = torch.Generator(device=dev)
    g.manual_seed(sh.seed)
    dt = torch.float32 if sh.dtype == wl.F32 else torch.bfloat16
    X = torch.randn((sh.N, sh.D), generator=g, device=dev, dtype=torch.float32)
    if sh.x_dist == "chan_scale":
        X *= torch.empty(sh.D, device=dev).uniform_(0.5, 2.0, generator=g)
    elif sh.x_dist == "student_t4":
        chi = torch.randn((4, sh.N, sh.D), generator=g, device=dev).square_().sum(0)
        X = X / torch.sqrt(chi / 4.0) / (2.0 ** 0.5)
        del chi
    elif sh.x_dist == "outlier_chan":
        idx = torch.randperm(sh.D, generator=g, device=dev)[: int(round(0.01 * sh.D))]
        X[:, idx] *= 20.0
    G = torch.randn((sh.N, sh.O), generator=g, device=dev, dtype=torch.float32) * sh.g_sigma
    return X.to(dt), G.to(dt)


def _shape_record(sh, c_us, w_us, dw_b, ws_bytes):
    cb, wb = sh.compress_bytes(), sh.wgrad_bytes(dw_b)
    rec = {
        "shape": sh.name, "cfg": sh.cfg, "N": sh.N, "D": sh.D, "O": sh.O, "d": sh.d, "M": sh.M,
        "compress_us": round(c_us, 2), "compress_GBps": round(cb / c_us * 1e-3, 1),
        "compress_frac_hbm": round(cb / c_us * 1e-3 / HBM_PEAK_GBPS, 4),
        "wgrad_us": round(w_us, 2), "wgrad_GBps": round(wb / w_us * 1e-3, 1),
        "wgrad_frac_hbm": round(wb / w_us * 1e-3 / HBM_PEAK_GBPS, 4),
        "wgrad_TFLOPs_factored": round(sh.wgrad_flops_factored() / w_us * 1e-6, 2),
        "wgrad_TFLOPs_dense_equiv": round(sh.wgrad_flops_dense() / w_us * 1e-6, 1),
        "wgrad_ws_MB": round(ws_bytes / 1e6, 2),
    }
    return rec


def _best_of(fn, reps=3):
    best = None
    for _ in range(reps):
        t0 = time.perf_counter()
        out = fn()
        dt = time.perf_counter() - t0
        best = dt if best is None or dt < best else best
    return best, out


def _cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _cpu_baseline(sh, Xh, Gh, v_ref):
    """The oracle as it stands, on this machine's host cores, on a bounded sample of
    the same workload: compress over all tokens; the factored weight gradient
    over a prefix of the output features sized to a few GFLOP (scaled linearly
    in O); and, for reference, the literal form of the paper's backward
    (materialised reconstruction + dense product) on 16 output rows, scaled.
    Timed twice: with one thread, and with every core this process may run on
    (sched_getaffinity, capped by OMP_NUM_THREADS where the box exports its CPU
    share there)."""
    import numpy as np
    import oracle
    try:
        affinity = len(os.sched_getaffinity(0))
    except AttributeError:
        affinity = os.cpu_count() or 1
    threads = oracle.default_threads()
    budget_flops = 6e9
    o_s = int(min(sh.O, max(16, budget_flops // (2 * sh.N * sh.M))))
    Gs = np.ascontiguousarray(Gh[:, :o_s])
    bytes_step = sh.compress_bytes() + sh.wgrad_bytes(4)
    runs = {}
    S_store = None
    for label, nt in (("all_cores", threads), ("one_thread", 1)):
        reps = 3 if nt > 1 else 1
        t_c, (_, S_store) = _best_of(lambda: oracle.compress(Xh, v_ref, sh.M, threads=nt), reps=reps)
        t_w, _ = _best_of(lambda: oracle.weight_grad_factored(Gs, S_store, v_ref, sh.D, threads=nt), reps=reps)
        t_w *= sh.O / o_s
        runs[label] = {"threads": nt, "GBps": round(bytes_step / (t_c + t_w) * 1e-9, 3),
                       "compress_s": round(t_c, 4), "compress_GBps": round(sh.compress_bytes() / t_c * 1e-9, 3),
                       "wgrad_s_scaled": round(t_w, 4), "wgrad_GBps": round(sh.wgrad_bytes(4) / t_w * 1e-9, 3)}
    rows = list(range(0, sh.O, max(1, sh.O // 16)))[:16]
    t_b, _ = _best_of(lambda: oracle.weight_grad_bruteforce_rows(Gh, S_store, v_ref, sh.D, rows, threads=threads), reps=1)
    t_b *= sh.O / len(rows)
    a = runs["all_cores"]
    return {
        "value": a["GBps"], "unit": "GB/s", "cores": threads, "kind": "oracle",
        "sample": (f"oracle.compress on all {sh.N} tokens + oracle.weight_grad_factored on the first {o_s} of {sh.O} "
                   f"output features, time scaled by {sh.O / o_s:.2f}; best of 3 with {threads} threads, one run with "
                   "1 thread; plain C++ -O2 double precision, std::thread, no BLAS, not tuned"),
        "cpu_model": _cpu_model(), "affinity_cores": affinity, "os_cpu_count": os.cpu_count(),
        "all_cores": a, "one_thread": runs["one_thread"],
        "compress_GBps": a["compress_GBps"], "wgrad_GBps": a["wgrad_GBps"],
        "wgrad_bruteforce_s_extrapolated": round(t_b, 2),
        "wgrad_bruteforce_sample": f"{len(rows)} of {sh.O} output rows, scaled by {sh.O / len(rows):.0f}",
    }


def _traffic(workload):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if any."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    if os.path.exists(path):
        try:
            with open(path) as f:
                return json.load(f)
        except Exception:
            return None
    return None


def main():
    args = _parse()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (one GPU per box, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import __graft_entry__ as ge
    ge.ensure_built()
    import paper_2405_17991_amd as vl
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    dw_dtype = torch.float32 if args.dw_dtype == "f32" else torch.bfloat16
    dw_b = 4 if args.dw_dtype == "f32" else 2

    if args.calibrate_copy:
        src = torch.empty(1 << 26, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------- headline workload: host-generated inputs (same as the parity tests)
    sh = wl.shape_by_name(args.workload)
    Xh, Gh = wl.make_X(sh), wl.make_G(sh)
    tdt = torch.float32 if sh.dtype == wl.F32 else torch.bfloat16
    X0 = torch.from_numpy(Xh).view(tdt).to(dev) if sh.dtype == wl.BF16 else torch.from_numpy(Xh).to(dev)
    G0 = torch.from_numpy(Gh).view(tdt).to(dev) if sh.dtype == wl.BF16 else torch.from_numpy(Gh).to(dev)
    v = vl.velora_init_v(X0, sh.M)           # first batch = this batch (one-off, untimed)
    ring = Ring(vl, torch, sh, X0, G0, v, dw_dtype)

    # Order of the regions: streaming ceilings, then the per-kernel event timings (at least 100 launches
    # of each entry point after 100 warm-up steps, whatever K is), then the contract's region (W warm-up
    # steps, exactly K timed steps, wall clock), back to back.  After any idle stretch this chip's power
    # management takes about 15 ms of load to settle (the gradient kernels run 5-15 % slower
    # meanwhile); this order keeps that transient out of all three.
    ceilings = _measured_ceilings(vl, torch, dev, 100)
    _, c_samples, w_samples = _time_steps(torch, ring, max(args.steps, 100), 100, with_events=True)
    dt, _, _ = _time_steps(torch, ring, args.steps, args.warmup, with_events=False)
    c_st, w_st = _stats(c_samples), _stats(w_samples)
    c_us, w_us = c_st["mean"], w_st["mean"]
    ms_per_step = dt / args.steps * 1e3
    step_bytes = sh.compress_bytes() + sh.wgrad_bytes(dw_b)
    value = step_bytes / (dt / args.steps) * 1e-9

    # the same step without rotation: every launch on buffer set 0, so whatever fits stays in the
    # 256 MB last-level cache (labelled as such; not an HBM figure)
    warm_steps = max(EVENT_BATCH, min(args.steps, 100))
    if args.headline_only:
        cw_samples, ww_samples = c_samples, w_samples      # placeholder, not reported
    else:
        _, cw_samples, ww_samples = _time_steps(torch, ring, warm_steps, 2, with_events=True, rotate=False)

    cb, wb = sh.compress_bytes(), sh.wgrad_bytes(dw_b)
    c_gbps, w_gbps = cb / c_us * 1e-3, wb / w_us * 1e-3
    traffic = _traffic(args.workload) if args.dw_dtype == "f32" else None   # the committed counters are for fp32 dW
    traffic_source = (f"profiles/traffic_{args.workload}.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier "
                      "run of this command, scaled by what the same counters read for the 384 MiB copy probe it "
                      "launches; valid for this workload with float32 dW only)") if traffic else None

    def _us(st):
        return {"avg_us": round(st["mean"], 2), "median_us": round(st["median"], 2), "min_us": round(st["min"], 2),
                "event_pairs": st["samples"], "launches_per_event_pair": EVENT_BATCH}

    # weight_grad's ceiling: its bytes are read (G, S) and written (dW) in two phases, so the measured
    # ceiling is the time the two probes need for the same bytes
    w_read = sh.N * sh.O * sh.elem_bytes + sh.N * sh.M * sh.elem_bytes
    w_write = sh.O * sh.D * dw_b
    w_ceiling_us = (w_read / ceilings["read_GBps"] + w_write / ceilings["write_GBps"]) * 1e-3
    wg = {"kernels": "wgrad_partial + wgrad_expand", "bound": "hbm", "achieved": round(w_gbps, 1),
          "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(w_gbps / HBM_PEAK_GBPS, 4),
          "achieved_median": round(wb / w_st["median"] * 1e-3, 1),
          "frac_of_measured": round(w_ceiling_us / w_st["median"], 4),
          "measured_ceiling_us": round(w_ceiling_us, 2),
          "traffic": (traffic or {}).get("weight_grad"), "traffic_source": traffic_source,
          "algorithmic_bytes": wb,
          "TFLOPs_factored": round(sh.wgrad_flops_factored() / w_us * 1e-6, 2),
          "TFLOPs_dense_equiv": round(sh.wgrad_flops_dense() / w_us * 1e-6, 1),
          "frac_mfma_dense_equiv": round(sh.wgrad_flops_dense() / w_us * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
          "workspace_MB": round(ring.ws_bytes / 1e6, 2)}
    wg.update(_us(w_st))
    roof = {"kernel": "compress", "bound": "hbm", "achieved": round(c_gbps, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(c_gbps / HBM_PEAK_GBPS, 4),
            "achieved_median": round(cb / c_st["median"] * 1e-3, 1),
            "frac_of_measured": round(cb / c_st["median"] * 1e-3 / ceilings["read_GBps"], 4),
            "traffic": (traffic or {}).get("compress"), "traffic_source": traffic_source,
            "algorithmic_bytes": cb, "measured_ceilings": ceilings, "weight_grad": wg}
    roof.update(_us(c_st))
    cw_st, ww_st = _stats(cw_samples), _stats(ww_samples)
    out = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if sh.dtype == wl.BF16 else "f32", "data": "synthetic",
        "config": {"workload": sh.name, "N": sh.N, "D": sh.D, "O": sh.O, "d": sh.d, "M": sh.M,
                   "x_dist": sh.x_dist, "dW_dtype": args.dw_dtype, "ring_sets": ring.R,
                   "step": "compress + weight_grad (2 kernels)"},
        "roofline": roof,
        "weight_grad": wg,
        "warm_cache": {"label": "NOT an HBM figure: every launch on the same buffer set, re-reads may come from the "
                                "256 MB last-level cache", "steps": warm_steps,
                       "compress_median_us": round(cw_st["median"], 2),
                       "compress_GBps": round(cb / cw_st["median"] * 1e-3, 1),
                       "weight_grad_median_us": round(ww_st["median"], 2),
                       "weight_grad_GBps": round(wb / ww_st["median"] * 1e-3, 1)},
    }
    v_host = v.cpu().numpy()
    if args.headline_only:
        del out["warm_cache"]
        print(json.dumps(out))
        return
    out["graph_replay_us_per_step"] = round(_graph_step_us(torch, ring, args.steps), 2)
    out["other_steps"] = _other_steps_record(vl, torch, sh, ring, args.steps)
    del ring, X0, G0
    torch.cuda.empty_cache()
    out["adamw_step_factor"] = _adamw_record(vl, torch, sh, v, dev, args.steps)
    torch.cuda.empty_cache()
    if sh.dtype == wl.BF16:
        out["swiglu_compress"] = _swiglu_record(vl, torch, sh, v, dev, args.steps)
        torch.cuda.empty_cache()
        out["rmsnorm_compress"] = _rmsnorm_record(vl, torch, wl, dev, args.steps)
        torch.cuda.empty_cache()
        out["linear_compress"] = _linear_record(vl, torch, sh, v, dev, args.steps)
        torch.cuda.empty_cache()
        out["weight_grad"]["dense_form"] = _dense_form_record(vl, torch, sh, v, dev, args.steps)
        torch.cuda.empty_cache()
        out["mlp_block"] = _mlp_block_record(torch, dev)
    torch.cuda.empty_cache()

    if sh.dtype == wl.BF16:
        out["vit_block_sequence"] = _vit_sequence_record(vl, torch, wl, dev, 10)
        torch.cuda.empty_cache()

    # ---------------- every layer shape of the five configurations
    if not args.no_shapes:
        recs = []
        for s in wl.valid_shapes():
            Xs, Gs = _device_inputs(torch, s, dev)
            vs = vl.velora_init_v(Xs, s.M, allow_degenerate=True)
            r = Ring(vl, torch, s, Xs, Gs, vs, dw_dtype)
            _settle(torch, r)
            _, cs, wsmp = _time_steps(torch, r, args.shape_steps, 40, with_events=True)
            cst, wst = _stats(cs), _stats(wsmp)
            rec = _shape_record(s, cst["mean"], wst["mean"], dw_b, r.ws_bytes)
            rec["compress_min_us"], rec["wgrad_min_us"] = round(cst["min"], 2), round(wst["min"], 2)
            dt_s, _, _ = _time_steps(torch, r, args.shape_steps, 3, with_events=False)
            rec["step_us"] = round(dt_s / args.shape_steps * 1e6, 2)
            recs.append(rec)
            del r, Xs, Gs
            torch.cuda.empty_cache()
        out["shapes"] = recs

    # ---------------- CPU oracle on the same workload
    if not args.no_cpu_baseline:
        import oracle
        v_ref, _, _ = oracle.init_v(Xh, sh.M)
        out["cpu_baseline"] = _cpu_baseline(sh, Xh, Gh, v_ref)
        out["cpu_baseline"]["init_v_l2_diff_gpu_vs_oracle"] = float(
            np.linalg.norm(v_host.astype(np.float64) - v_ref.astype(np.float64)))

    print(json.dumps(out))


if __name__ == "__main__":
    main()
