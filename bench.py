#!/usr/bin/env python3
"""Benchmark of the fused SOLO AdamW step on one MI355X.

One "step" is one call of solo_adamw_step over the whole flat buffer of a workload:
dequantize both moments, both EMAs, the parameter update, block statistics, re-quantize,
re-pack, with every input already resident in HBM.  Default workload: the LLaMA-7B-shaped
tensor set (6,738,415,616 fp32 parameters, bf16 gradients, 2-bit m, 3-bit log v, block 128).

Prints ONE JSON line: updated parameters per second, the HBM roofline of the step kernel
(algorithmic bytes / HIP-event duration of the launches on their own stream), and the CPU
oracle timed on the host cores of this machine on a bounded sample of the same workload.
"""
import argparse
import contextlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X: 8 TB/s HBM3E

# HBM bytes per launch of the step kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each
# scaled by what the same counter reads for a plain copy of known size (see profiles/).
MEASURED_TRAFFIC = {"c5_llama7b_2bit_3bit": 77.408e9,    # profiles/step_kernel_c5_llama7b_traffic.txt
                    "c5_llama7b_block2048": 77.78e9}     # profiles/big_wide_kernel_c5_block2048.txt


def bytes_per_param(w):
    """Algorithmic HBM bytes per parameter and step: read p, g, both code streams and three
    block scalars; write p, both code streams and three block scalars.  A 3-bit code costs
    3.2 bits (ten per 32-bit word)."""
    stored = {2: 2.0, 3: 3.2, 4: 4.0}
    g = 2 if w.grad_dtype == "bf16" else 4
    codes = (stored[w.bits_m] + stored[w.bits_v]) / 8.0
    scales = 12.0 / w.block_size
    return (4 + g + codes + scales) + (4 + codes + scales)


def device_grads(torch, n, kind, std, seed, dtype, sparse_rows=None):
    """Seeded synthetic gradients generated on the device, chunk by chunk (same recipe as
    synth.make_grads: N(0, std^2), Student-t(3) * std, or normal with 1 % of entries x100).
    sparse_rows = (first element, rows, row length, zero fraction): that many rows of that
    matrix, drawn afresh with the same seed, are set to zero (the embedding rows of tokens that
    do not occur in a batch)."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    out = torch.empty(n, dtype=dtype, device="cuda")
    chunk = 1 << 27
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        x = torch.randn(b - a, device="cuda", generator=gen)
        if kind == "normal_outliers":
            mask = torch.rand(b - a, device="cuda", generator=gen) < 0.01
            x = torch.where(mask, x * 100.0, x)
        elif kind == "student_t3":
            chi = torch.randn(3, b - a, device="cuda", generator=gen).square_().sum(0).div_(3.0).sqrt_()
            x = x / chi
        out[a:b] = (x * std).to(dtype)
    if sparse_rows is not None:
        first, rows, row_len, zero_frac = sparse_rows
        idle = torch.rand(rows, device="cuda", generator=gen) < zero_frac
        out[first:first + rows * row_len].view(rows, row_len)[idle] = 0
    return out


def sparse_rows_of(w):
    """The sparse_rows argument of device_grads for a workload (None: dense gradients)."""
    sp = w.extra.get("sparse_rows")
    if not sp:
        return None
    first = sum(t[1] for t in w.tensors[:sp["tensor"]])
    numel = w.tensors[sp["tensor"]][1]
    return (first, numel // sp["row_len"], sp["row_len"], sp["zero_frac"])


def device_params(torch, w, seed):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    p = torch.empty(w.n, dtype=torch.float32, device="cuda")
    pos = 0
    chunk = 1 << 27
    for _, numel, kind in w.tensors:
        if kind == "ones":
            p[pos:pos + numel] = 1.0
        elif kind == "zeros":
            p[pos:pos + numel] = 0.0
        else:
            for a in range(pos, pos + numel, chunk):
                b = min(pos + numel, a + chunk)
                p[a:b] = torch.randn(b - a, device="cuda", generator=gen) * 0.02
        pos += numel
    return p


def cpu_baseline(w, sample, steps=5):
    """The CPU oracle, as it stands, on the first `sample` elements of the workload's first
    tensor: with all host threads (median of the timed steps), and with one thread on an eighth
    of that sample."""
    import numpy as np
    from oracle import solo_oracle as so
    from paper_2505_00347_amd import synth
    threads = min(so.max_threads(), int(os.environ.get("OMP_NUM_THREADS", "1000")))
    cfg = so.make_config(bits_m=w.bits_m, bits_v=w.bits_v, block_size=w.block_size, beta1=w.beta1,
                         beta2=w.beta2, lr=w.lr, eps=w.eps, weight_decay=w.weight_decay,
                         quantile_p=w.quantile_p, seed=synth.SEED_XI,
                         m_codebook=1 if w.m_codebook == "de" else 0)

    def rate(count, nthreads):
        p = synth.make_params(count)
        st = so.State(count, cfg)
        times = []
        for step in range(1, steps + 1):
            g = synth.make_grads(count, w.grad_kind, w.grad_std, synth.seed_grad(w.config_id, step))
            if w.grad_dtype == "bf16":
                g = synth.round_to_bf16(g)[1]
            t0 = time.perf_counter()
            so.step_packed(p, g, st, step, cfg, threads=nthreads)
            times.append(time.perf_counter() - t0)
        t = float(np.median(times[1:])) if len(times) > 1 else times[0]
        return count / t

    what = (f"first %d elements of the workload (one contiguous slice, packed states, {steps} steps, "
            f"median of steps 2..{steps}); the step is block-local, so the rate carries over to the "
            "full tensor set")
    small = max(sample // 8, min(sample, 1 << 20))
    return {"value": rate(sample, threads), "unit": "params/s", "cores": threads, "kind": "oracle",
            "sample": what % sample,
            "single_thread": {"value": rate(small, 1), "unit": "params/s", "cores": 1, "sample": what % small}}


def stream_probe(n):
    """Runs the stand-alone memory-ceiling probe (paper_2505_00347_amd/csrc/stream_probe.hip) as a
    child process before this process touches the GPU, and returns its GB/s figures: what HBM
    delivers on this machine for pure reads, pure writes, a copy and the step's own access pattern
    without arithmetic.  None if the probe is not built."""
    import re
    import subprocess
    exe = os.path.join(ROOT, "paper_2505_00347_amd", "lib", "stream_probe")
    if not os.path.exists(exe):
        return None
    try:
        out = subprocess.run([exe, str(n)], capture_output=True, text=True, timeout=120).stdout
    except Exception:
        return None
    res = {}
    for key, label in (("read_gbs", "read only"), ("write_gbs", "write only"), ("copy_gbs", "copy"),
                       ("step_shaped_gbs", "step-shaped")):
        m = re.search(re.escape(label) + r".*?([0-9.]+) GB/s", out)
        if m:
            res[key] = float(m.group(1))
    return res or None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c5_llama7b_2bit_3bit")
    ap.add_argument("--cpu-sample", type=int, default=1 << 26)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stream-probe", action="store_true",
                    help="skip the memory-ceiling probe (read / write / copy / step-shaped streams)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="after the timed steps, copy the parameter buffer once (a plain copy of "
                         "known size that calibrates rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--variant", default="adamw",
                    choices=("adamw", "adam_l2", "adabelief", "adamw_mp", "adabelief_mp"),
                    help="step variant: coupled decay, AdaBelief; *_mp adds the bf16 weight copy and "
                         "a gradient scale read from device memory (the default, adamw, is the metric)")
    ap.add_argument("--eps", type=float, default=None,
                    help="eps of the optimizer (default: the workload's 1e-8; AdaBelief variants 1e-16)")
    ap.add_argument("--launch", default="flat", choices=("flat", "multi", "per_tensor"),
                    help="flat: one call over the whole flat buffer (the metric); multi: the workload's "
                         "tensors as separate buffers in one solo_adamw_step_multi launch; per_tensor: one "
                         "solo_adamw_step call per tensor")
    ap.add_argument("--placements", type=int, default=5,
                    help="allocate the workload this many times, time the warm-up steps on each and "
                         "measure on the one --placement-policy picks (1: the first allocation as it comes)")
    ap.add_argument("--placement-policy", default="median", choices=("median", "best", "first"),
                    help="which of the allocations the timed steps run on: the one whose warm-up "
                         "time is the median of all (the default: what a caller gets on a typical "
                         "allocation), the fastest, or the first")
    ap.add_argument("--no-state-apart", dest="state_apart", action="store_false",
                    help="allocate parameters, gradients and state one behind the other.  By default the "
                         "packed state is allocated behind a spacer that ends 96 GiB after the start of "
                         "the parameters (freed again at once), the library's allocation rule for "
                         "MI355X: the state must not share a third of HBM with the parameters (see "
                         "include/solo.h and paper_2505_00347_amd/hbm_regions.py).  With more than one "
                         "placement the first allocation is made without the spacer and reported as "
                         "frac_first")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the step is block-local and this build has no "
                 "multi-GPU path (run with --gpus 1)")

    from paper_2505_00347_amd import solo, synth
    probe = None if args.no_stream_probe else stream_probe(synth.workload(args.workload).n)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    solo.lib()
    w = synth.workload(args.workload)
    n = w.n
    cfg = solo.make_config(w.bits_m, w.bits_v, w.block_size,
                           solo.SOLO_GRAD_BF16 if w.grad_dtype == "bf16" else solo.SOLO_GRAD_FP32,
                           lr=w.lr, beta1=w.beta1, beta2=w.beta2,
                           # AdaBelief adds eps to the 2nd EMA itself; its published default is 1e-16
                           # (1e-8 would swamp the squared residuals of these gradients and make
                           # every block constant)
                           eps=args.eps if args.eps is not None else
                           (1e-16 if args.variant.startswith("adabelief") else w.eps),
                           weight_decay=w.weight_decay, quantile_p=w.quantile_p, seed=synth.SEED_XI,
                           flags=solo.SOLO_FLAG_STOCHASTIC
                           | (solo.SOLO_FLAG_M_DYNAMIC_EXPONENT if w.m_codebook == "de" else 0)
                           | (solo.SOLO_FLAG_ADABELIEF if args.variant.startswith("adabelief") else 0)
                           | (solo.SOLO_FLAG_COUPLED_DECAY if args.variant == "adam_l2" else 0))
    mp = args.variant.endswith("_mp")
    gdtype = torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32

    class Resident:
        """One set of device buffers of the workload (parameters, two gradient buffers that the
        steps alternate between, the packed state), and the steps run on it so far."""

        def __init__(self, apart=False):
            self.p = device_params(torch, w, synth.SEED_PARAM)
            self.grads = [device_grads(torch, n, w.grad_kind, w.grad_std,
                                       synth.seed_grad(w.config_id, k), gdtype, sparse_rows_of(w)) for k in (1, 2)]
            self.extras = {}
            if mp:
                self.extras = {"param_bf16": torch.empty(n, dtype=torch.bfloat16, device="cuda"),
                               "grad_scale": torch.tensor([0.5], dtype=torch.float32, device="cuda")}
            self.step = 0
            # (smaller buffers run the kernels that show no placement effect)
            used = 4 * n + 2 * (2 if w.grad_dtype == "bf16" else 4) * n + (2 * n if mp else 0)
            with (solo.state_region(used) if apart and n >= (1 << 28) else contextlib.nullcontext()):
                self.allocate_state()
            torch.cuda.synchronize()

        def allocate_state(self):
            if args.launch == "flat":
                self.state = solo.SoloState(n, cfg)
            else:
                # every tensor of the workload with buffers of its own: slices of p and g (tensor
                # sizes are multiples of 8, so the slices stay 16-byte aligned) and its own state
                self.tensors, pos = [], 0
                for _, numel, _ in w.tensors:
                    assert numel % 8 == 0
                    st = solo.SoloState(numel, cfg)
                    h = self.extras["param_bf16"][pos:pos + numel] if mp else None
                    self.tensors.append((self.p[pos:pos + numel], [g[pos:pos + numel] for g in self.grads], st, h))
                    pos += numel
                if args.launch == "multi":
                    self.tables = [solo.SoloMultiTable([(t[0], t[1][k], t[2], t[3]) for t in self.tensors], cfg)
                                   for k in (0, 1)]

        def one_step(self):
            self.step += 1
            k = self.step & 1
            if args.launch == "flat":
                self.state.step(self.p, self.grads[k], self.step, **self.extras)
            elif args.launch == "multi":
                self.tables[k].step(self.step, grad_scale=self.extras.get("grad_scale"))
            else:
                for pt, gt, st, h in self.tensors:
                    st.step(pt, gt[k], self.step, param_bf16=h, grad_scale=self.extras.get("grad_scale"))

        def run(self, count):
            """`count` steps; returns the HIP-event duration of each launch in ms (events on the
            stream of the launch, which is torch's current one)."""
            starts = [torch.cuda.Event(enable_timing=True) for _ in range(count)]
            ends = [torch.cuda.Event(enable_timing=True) for _ in range(count)]
            for k in range(count):
                starts[k].record()
                self.one_step()
                ends[k].record()
            torch.cuda.synchronize()
            return [s.elapsed_time(e) for s, e in zip(starts, ends)]

    # Where the buffers land in physical HBM changes the rate this machine delivers for identical code
    # by 8 %: the step is slower when the code words of the state lie in the same third of HBM
    # (96 GiB) as the parameters.  The candidates are therefore allocated by the library's rule
    # (state apart, see --no-state-apart).  What a caller who allocates everything one behind the
    # other gets is measured first, on an allocation of its own, and reported as frac_first.
    # Up to --placements candidates are allocated (every one held until the choice is made), each
    # is warmed up and timed, and the timed steps run on the one whose time is the median of the
    # candidates (policy "median", the headline: a typical allocation); the times of all candidates,
    # and the roofline fractions of the first and of the fastest, are reported beside it.
    cands, trial_ms = [], []
    trials = max(args.warmup, 2) if args.placements > 1 else args.warmup
    naive_ms = None
    if args.state_apart and args.placements > 1:
        r = Resident(apart=False)
        ms = r.run(trials)
        naive_ms = sorted(ms[-2:])[0] if ms else None
        del r
        torch.cuda.empty_cache()
    for k in range(max(1, args.placements)):
        if k:                                    # every candidate stays allocated until the choice is made
            free_b, total_b = torch.cuda.mem_get_info()
            if free_b < (total_b - free_b) / k + (8 << 30):
                break
        r = Resident(apart=args.state_apart)
        ms = r.run(trials)
        cands.append(r)
        trial_ms.append(sorted(ms[-2:])[0] if ms else None)
    order = list(range(len(cands))) if trial_ms[0] is None else sorted(range(len(cands)), key=lambda k: trial_ms[k])
    chosen = {"median": order[(len(order) - 1) // 2], "best": order[0], "first": 0}[args.placement_policy]
    res = cands[chosen]
    del cands, r
    torch.cuda.empty_cache()
    if args.placements > 1:
        res.run(trials)                          # back to a steady state after the idle gap of the frees

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    kernel_ms = res.run(args.steps)
    wall = time.perf_counter() - t0
    avg_kernel_s = sum(kernel_ms) / len(kernel_ms) / 1e3
    p = res.p
    assert bool(torch.isfinite(p[:1 << 20]).all())
    if args.copy_probe:
        p_copy = torch.empty_like(p)
        p_copy.copy_(p)                          # reads 4n bytes, writes 4n bytes
        torch.cuda.synchronize()
        del p_copy

    ms_per_step = wall / args.steps * 1e3
    bpp = bytes_per_param(w) + (2.0 if mp else 0.0)      # the bf16 copy is two more bytes written
    achieved = bpp * n / avg_kernel_s / 1e9

    def frac_of(ms):
        return (bpp * n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS) if ms else None

    # the kernel that takes the time (the library picks it from the format, the size and the launch)
    if w.block_size == 2048:
        kernel_name = "solo::multi_big_wide_kernel" if args.launch == "multi" else "solo::big_wide_kernel"
    elif args.launch == "multi":
        kernel_name = "solo::multi_chunk_kernel" if (w.grad_dtype == "fp32" and w.m_codebook == "linear") else "solo::multi_kernel"
    else:
        kernel_name = "solo::step_kernel"
    out = {
        "metric": "updated_params_per_sec", "value": n / (wall / args.steps), "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "params": n, "bits_m": w.bits_m, "bits_v": w.bits_v,
                   "block_size": w.block_size, "grad_dtype": w.grad_dtype, "beta1": w.beta1,
                   "m_codebook": w.m_codebook, "variant": args.variant, "launch": args.launch,
                   "tensors": len(w.tensors),
                   "bytes_per_param": bpp},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC.get(w.name) if (args.variant, args.launch) == ("adamw", "flat") else None,
                     "kernel": kernel_name, "kernel_ms": avg_kernel_s * 1e3,
                     "stream_probe": probe},
        # the warm-up time of every allocation that was tried, which one the timed steps ran on, and
        # the roofline fraction the warm-up steps gave on the first and on the fastest of them
        "placement": {"policy": (args.placement_policy if len(trial_ms) > 1 else "first")
                      + (", state apart" if args.state_apart else ", buffers one behind the other"),
                      "candidates_ms": trial_ms, "chosen": chosen,
                      "first_ms": naive_ms if naive_ms is not None else trial_ms[0],
                      "frac_first": frac_of(naive_ms if naive_ms is not None else trial_ms[0]),
                      "frac_best": frac_of(trial_ms[order[0]]),
                      "frac_median": frac_of(trial_ms[order[(len(order) - 1) // 2]])},
    }
    del res, p
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, min(args.cpu_sample, n))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
