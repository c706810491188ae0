#!/usr/bin/env python3
"""Benchmark of the fused RTPrune operator on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 5]

A step is one pass of the whole hot path (``rtprune_prune``: norms, ratio,
selection, scores, Sinkhorn, pairing, merge + compaction) over one synthetic
batch that is already resident in HBM.  Prints ONE JSON line: whole-job
throughput in images/s (tokens/s alongside), the roofline position of the
kernel that dominates the step (timed with HIP events inside the timed
region), and the CPU oracle timed on a bounded sample of the same workload as
a baseline.
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

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
FP64_VECTOR_TFLOPS = 78.6      # 256 CU x 2.4 GHz x 128 flop/clk
FP32_VECTOR_TFLOPS = 157.3     # fp32 vector peak
BF16_MFMA_TFLOPS = 2500.0      # dense bf16 matrix-core peak
COMPUTE_UNITS = 256


def generate(cfg: int, workers: int):
    """Draw the workload on the host (worker processes only speed the drawing up)."""
    from paper_2605_00392_amd import synth
    return synth.gen_batch_parallel(cfg, max(1, min(workers, 16, (os.cpu_count() or 1))))


def _oracle_worker(job):
    """One worker of the all-cores oracle timing: draws its images (untimed), then times the
    single-threaded oracle over them.  Runs in a fresh process; touches no GPU."""
    cfg, images = job
    from threadpoolctl import threadpool_limits
    from oracle import rtprune_oracle as orc
    from paper_2605_00392_amd import synth
    sub = synth.gen_batch(cfg, images=images)
    op = orc.Params.from_dict(sub.params)
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        orc.prune_batch(sub.tokens, sub.dtype, sub.offsets, sub.density, op)
        return len(images), time.perf_counter() - t0


def oracle_fanout(cfg: int, k: int, workers: int):
    """The oracle on the first ``k`` images of a workload, one single-threaded worker process per
    host core (at most 16), each on its share of the images: images/s = k / the slowest worker's time."""
    import multiprocessing as mp
    workers = max(1, min(workers, k))
    shares = [list(range(i, k, workers)) for i in range(workers)]
    with mp.get_context("spawn").Pool(workers) as pool:
        done = pool.map(_oracle_worker, [(cfg, sh) for sh in shares])
    slowest = max(t for _, t in done)
    return dict(value=round(sum(n for n, _ in done) / slowest, 3), unit="images/s", cores=workers,
                sample=f"the same {k} images dealt to {workers} single-threaded worker processes, slowest {slowest:.2f} s")


def kernel_work(kernel: str, n: np.ndarray, m: np.ndarray, d: int, elt: int, iters: int,
                eps: float = 0.05, z: float = 0.2):
    """Algorithmic work of one launch of a kernel over the batch: (bound, amount, unit, peak).

    Bytes are the unavoidable HBM traffic of the step the kernel performs
    (inputs read once, outputs written once); flops count useful arithmetic.
    """
    r = n - m
    tok_bytes = float(n.sum()) * d * elt
    if kernel == "k_norms":
        # every token row read once; 4-byte score + 8-byte squared norm written
        return "hbm", tok_bytes + 12.0 * n.sum(), "GB/s", HBM_PEAK_GBS
    if kernel == "k_merge":
        # kept and pruned rows read once, merged kept rows written once, plan read;
        # one fp32 multiply-add per (kept, pruned, d)
        nbytes = tok_bytes + float(m.sum()) * d * elt + 4.0 * float((m * r).sum())
        flops = 2.0 * float((m * r).sum()) * d
        # Which unit does the multiply-adds: pruned sets of more than 64 go to the matrix
        # cores (bf16, width a multiple of 128), and so do those of 17 to 64 (width a
        # multiple of 64) when the batch holds enough of them to fill the chip (four
        # 128-row tiles per compute unit); the rest runs on the fp32 vector units.
        on_mfma = np.zeros(len(n), bool)
        if elt == 2 and d % 128 == 0:
            on_mfma |= r > 64
        mid = (r > 16) & (r <= 64)
        tiles = max(1, -(-int(n.max(initial=1)) // 128))
        if elt == 2 and d % 64 == 0 and mid.sum() >= max(1, -(-4 * COMPUTE_UNITS // tiles)):
            on_mfma |= mid
        mfma_share = float((m * r)[on_mfma].sum()) / max(1.0, float((m * r).sum()))
        if mfma_share > 0.5:
            # (useful flops: the plan's two bf16 terms double the executed ones)
            if flops / nbytes > BF16_MFMA_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
                return "mfma", flops, "TFLOP/s", BF16_MFMA_TFLOPS
            if r.max(initial=0) > 64:
                # the LDS-tiled kernel re-reads its operands per tile: priced as a contraction
                return "mfma", flops, "TFLOP/s", BF16_MFMA_TFLOPS
            return "hbm", nbytes, "GB/s", HBM_PEAK_GBS
        # vector units: with many pruned tokens per image the arithmetic outweighs the
        # traffic (ridge of the fp32 vector units: 20 flop/B)
        if flops / nbytes > FP32_VECTOR_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
            return "alu", flops, "TFLOP/s", FP32_VECTOR_TFLOPS
        return "hbm", nbytes, "GB/s", HBM_PEAK_GBS
    if kernel == "k_scores":
        flops = 2.0 * float((m * r).sum()) * d          # one multiply-add per (kept, pruned, d)
        if elt == 2 and d % 128 == 0:
            # bf16 matrix cores.  Every token row read once, the kernel matrix written once
            # (8 bytes per entry): below the ridge of the matrix cores (312 flop/B) the pass
            # is a stream over the tokens.  Pruned sets of more than 64 take the LDS-tiled
            # kernel, priced as a contraction.
            nbytes = tok_bytes + 8.0 * float((m * r).sum())
            if r.max(initial=0) <= 64 and flops / nbytes < BF16_MFMA_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
                return "hbm", nbytes, "GB/s", HBM_PEAK_GBS
            return "mfma", flops, "TFLOP/s", BF16_MFMA_TFLOPS
        return "alu", flops, "TFLOP/s", FP64_VECTOR_TFLOPS
    if kernel in ("k_sinkhorn", "k_sinkhorn_regs", "k_sinkhorn_c32", "k_sinkhorn_tall"):
        # Sinkhorn is arithmetic on the augmented matrix wherever that matrix lives: two sweeps
        # of multiply-adds per iteration, counted over the whole batch and priced against the
        # fp64 vector peak.  (What the multi-workgroup kernels of the large pages stream from
        # memory per iteration is reported beside it, as `streamed`, not as the roofline.)
        return "alu", 2.0 * 2.0 * iters * float(((m + 1) * (r + 1)).sum()), "TFLOP/s", FP64_VECTOR_TFLOPS
    return "hbm", 0.0, "GB/s", HBM_PEAK_GBS


def sinkhorn_streamed_bytes(n: np.ndarray, m: np.ndarray, iters: int, eps: float, z: float) -> float:
    """Bytes the multi-workgroup Sinkhorn kernels read per call: images beyond the
    register-resident shapes (batches with images above 512 tokens only) have their kernel
    matrix streamed once per iteration, in fp32 when exp's range allows."""
    r = n - m
    if n.max(initial=0) <= 512:
        return 0.0
    big = ((m + 1 > 512) | (r > 64)) & (r > 0) & (r <= 2048)
    kbytes = 4.0 if (max(1.0, z) - min(-1.0, z)) / eps <= 80.0 else 8.0
    return kbytes * iters * float((m * r)[big].sum())


def bench_density(rt, torch, steps: int, unique: int = 16, copies: int = 16):
    """Time rtprune_text_density on `unique * copies` large-mode pages (1280 x 1280 RGB)."""
    from paper_2605_00392_amd import synth
    side, patch = synth.PAGE_MODES["large"], synth.PATCH_PIXELS
    pages = synth.gen_pages(unique, side)
    dev = "cuda:0"
    B = unique * copies
    pix = torch.from_numpy(pages).to(dev).repeat(copies, 1, 1, 1).contiguous()
    per = side * side * 3
    poff = torch.arange(B + 1, dtype=torch.int64, device=dev) * per
    hs = torch.full((B,), side, dtype=torch.int32, device=dev)
    npatch = (side // patch) ** 2
    pto = torch.arange(B + 1, dtype=torch.int32, device=dev) * npatch
    rc, nbytes = rt.rtprune_text_density_workspace_bytes(B, side, side, patch, patch)
    rt.check(rc)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    rho = torch.empty(B, dtype=torch.float32, device=dev)
    rho_k = torch.empty(B * npatch, dtype=torch.float32, device=dev)

    def run():
        rt.check(rt.rtprune_text_density(pix, poff, hs, hs, B, side, side, patch, patch, 0.2, rho, rho_k, pto, ws))

    for _ in range(2):
        run()
    torch.cuda.synchronize()
    rt.rtprune_profile_enable(1)
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    rc, prof = rt.rtprune_profile_summary()
    rt.rtprune_profile_enable(0)
    rt.check(rc)
    ms = (t1 - t0) * 1e3 / steps
    sobel = next((r["total_ms"] / r["launches"] for r in prof if r["kernel"] == "k_density_sobel"), None)
    from oracle import rtprune_oracle as orc
    c0 = time.perf_counter()
    want = [orc.text_density(pages[i], patch, patch, 0.2)[0] for i in range(min(unique, 8))]
    c1 = time.perf_counter()
    got = rho.cpu().numpy()
    assert all(got[i] == want[i] for i in range(len(want))), "text density differs from the oracle"
    return {"pages": B, "page": f"{side}x{side}x3 u8", "ms_per_call": round(ms, 4),
            "pages_per_s": round(B / (ms * 1e-3), 1),
            "kernel": "k_density_rows (timed under the name k_density_sobel, which covers both density kernels)", "kernel_ms": None if sobel is None else round(sobel, 4),
            "bound": "hbm", "achieved_GBs": None if sobel is None else round(B * per / (sobel * 1e-3) / 1e9, 1),
            "peak_GBs": HBM_PEAK_GBS,
            "frac": None if sobel is None else round(B * per / (sobel * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "cpu_oracle_pages_per_s": round(len(want) / (c1 - c0), 2), "bit_exact_vs_oracle": True}


def bench_side(rt, torch, synth, steps: int, cfg: int, batch=None, rooflines: bool = True):
    """Time the fused call on another workload: the other benchmark workloads (1-4), the
    largest page size of the paper's other OCR models (Table 6: 4512 -> 2783 tokens, the
    shapes whose Sinkhorn matrix does not fit a workgroup and whose similarity product is a
    real GEMM), the benchmark's pages at the paper's own retention."""
    if batch is None:
        batch = synth.gen_batch(cfg)
    w = synth.WORKLOADS[cfg]
    dev = "cuda:0"
    p = rt.make_params(batch.params)
    db = rt.upload(batch, dev)
    ws = rt.alloc_workspace(db, p)
    B, total, D = db.B, db.total_tokens, db.D
    out = torch.empty((total, D), dtype=db.tokens.dtype, device=dev)
    out_off = torch.empty(B + 1, dtype=torch.int32, device=dev)
    keep = torch.empty(B, dtype=torch.int32, device=dev)
    pair = torch.empty(total, dtype=torch.int32, device=dev)
    dens = torch.from_numpy(np.ascontiguousarray(batch.density, dtype=np.float32)).to(dev)

    def step():
        rt.check(rt.rtprune_prune(db, dens, p, out, out_off, keep, None, pair, None, ws))

    for _ in range(2):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    rt.rtprune_profile_enable(1)             # per-kernel durations from steps of their own
    for _ in range(max(2, min(5, steps))):
        step()
    torch.cuda.synchronize()
    rc, prof = rt.rtprune_profile_summary()
    rt.rtprune_profile_enable(0)
    rt.check(rc)
    ms = (t2 - t1) * 1e3 / steps
    kernels = {r_["kernel"]: r_["total_ms"] / max(1, r_["launches"]) for r_ in prof}
    n_h = np.diff(batch.offsets).astype(np.int64)
    keep_h = keep.cpu().numpy().astype(np.int64)
    elt = 2 if batch.dtype == "bf16" else 4
    iters, eps, z = int(batch.params["iters"]), float(batch.params["eps"]), float(batch.params["z"])
    res = dict(workload=w.name, images=B, total_tokens=int(total), kept_tokens=int(keep_h.sum()),
               ms_per_step=round(ms, 4), images_per_s=round(B / (ms * 1e-3), 1),
               tokens_per_s=round(total / (ms * 1e-3), 1),
               step_hbm_floor_frac=round((float(n_h.sum()) + float(keep_h.sum())) * D * elt
                                         / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 5),
               kernels_ms={k_: round(v, 4) for k_, v in kernels.items()})
    if rooflines:
        roof = {}
        for k_ in ("k_norms", "k_sinkhorn_regs", "k_sinkhorn_c32", "k_sinkhorn_tall", "k_sinkhorn", "k_scores", "k_merge"):
            if kernels.get(k_, 0.0) < 0.02 * ms:      # a kernel that has nothing to do on this workload
                continue
            bound, amount, unit, peak = kernel_work(k_, n_h, keep_h, D, elt, iters, eps, z)
            ach = amount / (kernels[k_] * 1e-3) / (1e9 if unit == "GB/s" else 1e12)
            roof[k_] = dict(bound=bound, achieved=round(ach, 2), peak=peak, unit=unit, frac=round(ach / peak, 4))
            if k_ == "k_sinkhorn":
                streamed = sinkhorn_streamed_bytes(n_h, keep_h, iters, eps, z)
                if streamed > 0:
                    roof[k_]["streamed"] = dict(bytes_per_call=streamed, unit="GB/s",
                                                rate=round(streamed / (kernels[k_] * 1e-3) / 1e9, 1))
        res["roofline"] = roof
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=5, help="synthetic workload 1..9 (5 = 1024 x 400 tokens, the default; 6-8 = 1083/2137/4512-token pages; 9 = workload 5's pages at retention 337/400)")
    ap.add_argument("--cpu-images", type=int, default=384, help="images the CPU oracle is timed on")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--lib", default=None, help="path of an alternative build of librtprune.so")
    ap.add_argument("--no-density", action="store_true", help="skip the textual-density side measurement")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the side measurements on benchmark workloads 1-4")
    ap.add_argument("--no-large-pages", action="store_true",
                    help="skip the side measurement on 4512-token pages")
    ap.add_argument("--gen-workers", type=int, default=16,
                    help="processes drawing the synthetic batch (1: in-process, for runs under a profiler)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this operator runs on ONE GPU (images are independent; there is no "
              "multi-GPU path in this build). Re-run with --gpus 1.", file=sys.stderr)
        return 2

    from paper_2605_00392_amd import rtprune as rt
    from paper_2605_00392_amd import synth

    t0 = time.time()
    batch = generate(args.workload, args.gen_workers)   # before the GPU is touched (fork)
    side9 = None
    if not args.no_large_pages and args.workload == 5:
        side9 = generate(9, args.gen_workers)              # the paper-retention side workload, likewise
    others_h = {}
    if not args.no_other_workloads and args.workload == 5:
        others_h = {c: generate(c, args.gen_workers) for c in (1, 2, 3, 4)}
    gen_s = time.time() - t0

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    if args.lib:
        rt._lib = rt.load_library(args.lib)
    rt.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload]
    p = rt.make_params(batch.params)
    db = rt.upload(batch, dev)
    ws = rt.alloc_workspace(db, p)               # sized for these parameters
    B, total, D = db.B, db.total_tokens, db.D
    out = torch.empty((total, D), dtype=db.tokens.dtype, device=dev)
    out_off = torch.empty(B + 1, dtype=torch.int32, device=dev)
    keep = torch.empty(B, dtype=torch.int32, device=dev)
    sel = torch.empty(total, dtype=torch.int32, device=dev)
    pair = torch.empty(total, dtype=torch.int32, device=dev)
    ratio = torch.empty(B, dtype=torch.float32, device=dev)
    dens = torch.from_numpy(batch.density).to(dev)

    def step():
        rt.check(rt.rtprune_prune(db, dens, p, out, out_off, keep, sel, pair, ratio, ws))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Every kernel's duration, from a few steps before the timed region (an event pair
    # per launch costs a few microseconds of stream time each, ten and more per step);
    # the timed region then records the slowest kernel alone.
    rt.rtprune_profile_only(None)
    rt.rtprune_profile_enable(1)
    pre_steps = max(2, min(5, args.steps))
    for _ in range(pre_steps):
        step()
    torch.cuda.synchronize()
    rc, pre = rt.rtprune_profile_summary()
    rt.rtprune_profile_enable(0)
    rt.check(rc)
    kernels_pre = {r_["kernel"]: r_["total_ms"] / max(1, r_["launches"]) for r_ in pre}
    dominant_pre = max(kernels_pre, key=kernels_pre.get) if kernels_pre else None
    rt.check(rt.rtprune_profile_only(dominant_pre))
    rt.rtprune_profile_enable(1)
    # one event pair per step on the launch stream (torch's current stream): median and
    # minimum of the steps beside the wall-clock mean
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    rc, prof = rt.rtprune_profile_summary()
    rt.rtprune_profile_enable(0)
    rt.rtprune_profile_only(None)
    rt.check(rc)
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    status = int(ws[:4].view(torch.int32).item())
    assert status == 0, f"device status {status}"
    # one plain copy of the input's size, outside the timed region: the
    # calibration point for hardware traffic counters in profiled runs
    nbytes = db.tokens.numel() * db.tokens.element_size() // 16 * 16
    rt.check(rt.rtprune_copy_bytes(out, db.tokens, nbytes))
    torch.cuda.synchronize()
    step()                                   # restore `out`
    torch.cuda.synchronize()

    ms_per_step = (t2 - t1) * 1e3 / args.steps
    images_per_s = B / (ms_per_step * 1e-3)
    tokens_per_s = total / (ms_per_step * 1e-3)
    keep_h = keep.cpu().numpy().astype(np.int64)
    n_h = np.diff(batch.offsets).astype(np.int64)
    elt = 2 if batch.dtype == "bf16" else 4

    kernels = dict(kernels_pre)
    for rec in prof:                         # the slowest kernel: as measured inside the timed region
        kernels[rec["kernel"]] = rec["total_ms"] / max(1, rec["launches"])
    dominant = dominant_pre
    roofline = None
    if dominant:
        bound, amount, unit, peak = kernel_work(dominant, n_h, keep_h, D, elt, int(batch.params["iters"]),
                                                 float(batch.params["eps"]), float(batch.params["z"]))
        dur_s = kernels[dominant] * 1e-3
        achieved = amount / dur_s / (1e9 if unit == "GB/s" else 1e12)
        traffic = None
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
        if os.path.exists(tpath):
            try:
                tmap = json.load(open(tpath)).get(w.name, {})
                traffic = next((v for k_, v in tmap.items() if k_.startswith(dominant)), None)
            except Exception:
                traffic = None
        roofline = dict(kernel=dominant, bound=bound, achieved=round(achieved, 3), peak=peak, unit=unit,
                        frac=round(achieved / peak, 5), traffic=traffic,
                        avg_launch_ms=round(kernels[dominant], 5),
                        algorithmic_per_launch=amount)
    # whole-step HBM floor: every token read once, every kept token written once
    floor_bytes = float(n_h.sum()) * D * elt + float(keep_h.sum()) * D * elt
    step_hbm_frac = floor_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import rtprune_oracle as orc
        from tests import harness
        from threadpoolctl import threadpool_limits
        k = min(args.cpu_images, B)
        sub = synth.subset(batch, list(range(k)))
        op = orc.Params.from_dict(batch.params)
        # primary number: the oracle as it stands on ONE thread (numpy's BLAS capped for the timed block)
        with threadpool_limits(limits=1):
            c0 = time.perf_counter()
            res = orc.prune_batch(sub.tokens, sub.dtype, sub.offsets, sub.density, op)
            c1 = time.perf_counter()
        del res
        # the timed device outputs are checked against the oracle on a spread of the same images
        gpu = dict(keep=keep_h, out_offsets=out_off.cpu().numpy(), sel=sel.cpu().numpy(),
                   pair=pair.cpu().numpy(), ratio=ratio.cpu().numpy(), out=harness._np(out))
        rep = harness.compare_batch(batch, gpu, images=list(range(0, k, max(1, k // 24))))
        # secondary: the same single-threaded function, the images dealt to one worker process per host core
        fan = oracle_fanout(args.workload, k, harness.host_workers())
        cpu = dict(value=round(k / (c1 - c0), 3), unit="images/s", cores=1, kind="oracle",
                   sample=f"first {k} images of {w.name}, float64 numpy oracle on one thread, {c1 - c0:.2f} s",
                   all_cores=fan, host_cpu_count=os.cpu_count(),
                   parity_checked_images=rep.images,
                   near_ties=rep.selection_near_ties + rep.pairing_near_ties)

    density = None
    if not args.no_density:
        del out, ws
        torch.cuda.empty_cache()
        density = bench_density(rt, torch, max(3, args.steps // 2))

    # the other four benchmark workloads: a few steps each, outside the headline's timed region
    other = None
    if not args.no_other_workloads and args.workload == 5:
        other = {}
        for cfg_o in (1, 2, 3, 4):
            other[f"c{cfg_o}"] = bench_side(rt, torch, synth, 10, cfg_o, batch=others_h.get(cfg_o), rooflines=False)
            torch.cuda.empty_cache()

    large = paper_ret = large_other = None
    if not args.no_large_pages and args.workload == 5:
        del db
        torch.cuda.empty_cache()
        large = bench_side(rt, torch, synth, 3, 8)
        torch.cuda.empty_cache()
        # the two smaller page sizes of the same table (1083 -> 560 and 2137 -> 1238 tokens)
        large_other = {f"c{c}": bench_side(rt, torch, synth, 3, c, rooflines=False) for c in (6, 7)}
        torch.cuda.empty_cache()
        # the benchmark's pages at the paper's own average retention (337 of 400 kept)
        paper_ret = bench_side(rt, torch, synth, 5, 9, batch=side9)

    line = {
        "metric": "images/s pruned (fused rtprune_prune, 400-token 1280-d bf16 pages)",
        "value": round(images_per_s, 2),
        "unit": "images/s",
        "tokens_per_s": round(tokens_per_s, 1),
        "kept_tokens": int(keep_h.sum()),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(per_step[len(per_step) // 2], 4) if per_step else None,
        "ms_per_step_min": round(per_step[0], 4) if per_step else None,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": batch.dtype, "data": "synthetic",
        "config": {"workload": w.name, "images": B, "total_tokens": int(total), "D": D,
                   "iters": int(batch.params["iters"]), "eps": batch.params["eps"],
                   "dynamic": int(batch.params["dynamic"]), "gen_s": round(gen_s, 1)},
        "kernels_ms": {k_: round(v, 5) for k_, v in kernels.items()},
        "kernels_ms_from": f"{pre_steps} profiled steps before the timed region; {dominant} from the timed region",
        "step_hbm_floor_frac": round(step_hbm_frac, 5),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "other_workloads": other,
        "text_density": density,
        "large_pages": large,
        "large_pages_other_sizes": large_other,
        "paper_retention_pages": paper_ret,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
