"""Test harness: drive the HIP library through its binding and compare with the oracle.

The device side is called only through ``paper_2605_00392_amd.rtprune`` (the
C ABI); the oracle side only through ``oracle.rtprune_oracle``.  The two meet
here and nowhere else.
"""
from __future__ import annotations

import os
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

from oracle import rtprune_oracle as orc
from paper_2605_00392_amd import rtprune as rt
from paper_2605_00392_amd import synth

# Parity bars
NEAR_TIE = 1e-6            # relative gap below which an index disagreement is a counted near-tie
MERGE_RTOL, MERGE_ATOL = 2e-3, 1e-3     # bf16 merged features, elementwise
MERGE_ROW_REL = 3e-3       # per-token ||g - o|| / ||o||; bf16 rounding alone gives about 2^-8 / sqrt(3) = 2.3e-3
MERGE_F32_REL = 1e-5       # fp32 in/out
PLAN_REL = 1e-4            # plan entries above 1e-6
SCORE_ATOL = 5e-8          # cosine scores: 32- or 128-term fp32 partial sums on the matrix cores, added in fp64
RATIO_TOL = 1e-5


def _np(t):
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def device_status(ws) -> int:
    return int(ws[:4].view(__import__("torch").int32).item())


def run_prune(batch: synth.Batch, params: Optional[Dict] = None, device="cuda:0"):
    """The fused entry point on a host batch; returns numpy outputs."""
    import torch
    p = rt.make_params(batch.params if params is None else params)
    db = rt.upload(batch, device)
    ws = rt.alloc_workspace(db)
    ws.fill_(0xFF)     # the workspace is scratch: a value read before it is written must not be a plausible one
    B, total = db.B, db.total_tokens
    out = torch.zeros((max(total, 1), db.D), dtype=db.tokens.dtype, device=device)
    out_off = torch.full((B + 1,), -7, dtype=torch.int32, device=device)
    keep = torch.full((max(B, 1),), -7, dtype=torch.int32, device=device)
    sel = torch.full((max(total, 1),), -7, dtype=torch.int32, device=device)
    pair = torch.full((max(total, 1),), -7, dtype=torch.int32, device=device)
    ratio = torch.full((max(B, 1),), -7.0, dtype=torch.float32, device=device)
    dens = torch.from_numpy(np.ascontiguousarray(batch.density, dtype=np.float32)).to(device)
    if dens.numel() == 0:
        dens = torch.zeros(1, dtype=torch.float32, device=device)
    rc = rt.rtprune_prune(db, dens, p, out, out_off, keep, sel, pair, ratio, ws)
    torch.cuda.synchronize()
    return dict(rc=rc, status=device_status(ws) if rc == 0 else None, out=_np(out), out_offsets=_np(out_off),
                keep=_np(keep)[:B], sel=_np(sel)[:total], pair=_np(pair)[:total], ratio=_np(ratio)[:B])


def run_staged(batch: synth.Batch, params: Optional[Dict] = None, keep_counts_in=None, device="cuda:0"):
    """ratio -> norms_topk -> ot_pair -> merge through the four staged entry points."""
    import torch
    pd = dict(batch.params if params is None else params)
    p = rt.make_params(pd)
    db = rt.upload(batch, device)
    ws = rt.alloc_workspace(db)
    ws.fill_(0xFF)     # the workspace is scratch: a value read before it is written must not be a plausible one
    B, total = db.B, db.total_tokens
    i32 = dict(dtype=torch.int32, device=device)
    f32 = dict(dtype=torch.float32, device=device)
    res = {}
    keep_in = None
    if pd.get("dynamic"):
        dens = torch.from_numpy(np.ascontiguousarray(batch.density, dtype=np.float32)).to(device)
        phi = torch.zeros(max(B, 1), **f32)
        ratio = torch.zeros(max(B, 1), **f32)
        keep_dyn = torch.zeros(max(B, 1), **i32)
        rc = rt.rtprune_dynamic_ratio(db, dens, p, phi, ratio, keep_dyn, ws)
        rt.check(rc)
        torch.cuda.synchronize()
        res.update(phi=_np(phi)[:B], ratio=_np(ratio)[:B], keep_dyn=_np(keep_dyn)[:B])
        keep_in = keep_dyn
    if keep_counts_in is not None:
        keep_in = torch.from_numpy(np.asarray(keep_counts_in, dtype=np.int32)).to(device)
    norms = torch.zeros(max(total, 1), **f32)
    sel = torch.full((max(total, 1),), -7, **i32)
    keep = torch.zeros(max(B, 1), **i32)
    out_off = torch.zeros(B + 1, **i32)
    plan_off = torch.zeros(B + 1, dtype=torch.int64, device=device)
    rt.check(rt.rtprune_norms_topk(db, keep_in, p, norms, sel, keep, out_off, plan_off, ws))
    torch.cuda.synchronize()
    n_plan = int(plan_off[-1].item())
    n_out = int(out_off[-1].item())
    scores = torch.zeros(max(n_plan, 1), dtype=torch.float64, device=device)
    plan = torch.zeros(max(n_plan, 1), **f32)
    pair = torch.full((max(total, 1),), -7, **i32)
    rt.check(rt.rtprune_ot_pair(db, sel, keep, plan_off, p, scores, plan, pair, ws))
    torch.cuda.synchronize()
    out = torch.zeros((max(n_out, 1), db.D), dtype=db.tokens.dtype, device=device)
    rt.check(rt.rtprune_merge(db, sel, keep, out_off, plan, plan_off, p, out, ws))
    torch.cuda.synchronize()
    res.update(status=device_status(ws), norms=_np(norms)[:total], sel=_np(sel)[:total], keep=_np(keep)[:B],
               out_offsets=_np(out_off), plan_offsets=_np(plan_off), scores=_np(scores)[:n_plan],
               plan=_np(plan)[:n_plan], pair=_np(pair)[:total], out=_np(out)[:n_out])
    return res


# ---------------------------------------------------------------------------
# comparison with the oracle
# ---------------------------------------------------------------------------
@dataclass
class Report:
    images: int = 0
    ratio_boundary: int = 0          # images whose kept count differs by a ceil() boundary effect
    selection_near_ties: int = 0     # images whose kept set differs inside the near-tie band
    pairing_near_ties: int = 0       # pruned tokens whose partner differs inside the band
    pairs_checked: int = 0
    max_ratio_err: float = 0.0
    max_merge_row_rel: float = 0.0
    max_plan_rel: float = 0.0
    max_score_abs: float = 0.0
    notes: List[str] = field(default_factory=list)


def compare_image(b: int, batch: synth.Batch, gpu: Dict, p: orc.Params, rep: Report,
                  staged: bool = False, keep_count: Optional[int] = None) -> None:
    """Compare image ``b`` of a device result with the oracle; raises AssertionError.
    ``keep_count``: the kept count the caller gave the staged calls for this image."""
    lo, hi = int(batch.offsets[b]), int(batch.offsets[b + 1])
    n = hi - lo
    X = orc.widen(batch.tokens[lo:hi], batch.dtype)
    rho = float(batch.density[b]) if len(batch.density) else 0.0
    ref = orc.prune_image(X, rho, p, keep_count=keep_count)
    rep.images += 1
    m_gpu = int(gpu["keep"][b])
    if keep_count is not None:
        assert m_gpu == min(max(keep_count, 0), n), (b, m_gpu, keep_count)
    elif p.dynamic:
        err = abs(float(gpu["ratio"][b]) - float(ref.retention))
        rep.max_ratio_err = max(rep.max_ratio_err, err)
        assert err <= RATIO_TOL, (b, gpu["ratio"][b], ref.retention)
        if staged and "phi" in gpu:
            assert abs(float(gpu["phi"][b]) - ref.phi) <= RATIO_TOL
    if m_gpu != ref.m:
        # only legitimate when the two retentions straddle a ceil boundary
        frac = float(np.float32(ref.retention)) * n - orc.COUNT_SLACK
        assert abs(m_gpu - ref.m) == 1 and abs(frac - round(frac)) < 1e-3, (b, m_gpu, ref.m, frac)
        rep.ratio_boundary += 1
        ref = orc.prune_image(X, rho, p, keep_count=m_gpu)
    m, r = ref.m, n - ref.m
    assert int(gpu["out_offsets"][b + 1]) - int(gpu["out_offsets"][b]) == m
    sel = gpu["sel"][lo:hi]
    kept_g, prop_g = sel[:m], sel[m:]
    assert list(kept_g) == sorted(kept_g) and list(prop_g) == sorted(prop_g)
    assert sorted(list(kept_g) + list(prop_g)) == list(range(n)), "sel_idx is not a permutation"
    if staged and "norms" in gpu:
        np.testing.assert_allclose(gpu["norms"][lo:hi], np.sqrt(ref.sqnorm), rtol=2e-7)
    if not np.array_equal(kept_g, ref.kept):
        gap = orc.selection_gap(ref.score, m)
        assert gap < NEAR_TIE, (b, "kept set differs outside the near-tie band", gap)
        rep.selection_near_ties += 1
        rep.notes.append(f"image {b}: kept set differs at a near-tie (gap {gap:.2e}); stage 2 not compared")
        return
    o0 = int(gpu["out_offsets"][b])
    out_g = gpu["out"][o0:o0 + m]
    if batch.dtype == "bf16":
        out_g = synth.bf16_bits_to_f32(out_g).astype(np.float64)
    else:
        out_g = out_g.astype(np.float64)
    # pairing
    pair_g = gpu["pair"][lo:hi]
    assert list(pair_g[:m]) == list(range(m))
    if r > 0:
        gaps = orc.pairing_gaps(ref.P_bar)
        diff = np.nonzero(pair_g[m:] != ref.pair)[0]
        rep.pairs_checked += r
        for j in diff:
            assert gaps[j] < NEAR_TIE, (b, int(j), "partner differs outside the near-tie band",
                                        float(gaps[j]), int(pair_g[m + j]), int(ref.pair[j]))
            rep.pairing_near_ties += 1
        if staged:
            po = int(gpu["plan_offsets"][b])
            S_g = gpu["scores"][po:po + m * r].reshape(m, r)
            rep.max_score_abs = max(rep.max_score_abs, float(np.abs(S_g - ref.S).max()))
            assert np.abs(S_g - ref.S).max() <= SCORE_ATOL, (b, float(np.abs(S_g - ref.S).max()))
            P_g = gpu["plan"][po:po + m * r].reshape(m, r).astype(np.float64)
            P_o = ref.P
            big = P_o > 1e-6
            if big.any():
                rel = float((np.abs(P_g - P_o)[big] / P_o[big]).max())
                rep.max_plan_rel = max(rep.max_plan_rel, rel)
                assert rel <= PLAN_REL, (b, rel)
            assert np.abs(P_g - P_o)[~big].max(initial=0.0) <= 1e-9
    # merged features against the oracle's unrounded rows
    o = ref.merged
    err = np.abs(out_g - o)
    # fp32 accumulation noise of the merge sum, per kept row
    floor = 4e-6 * np.abs(o).max(axis=1, keepdims=True)
    if r > 0:
        spread = p.f32("alpha") * ref.P.sum(axis=1) * np.abs(X[ref.prop]).max()
        floor = np.maximum(floor, 4e-6 * spread[:, None])
    if batch.dtype == "bf16":
        # the stated bar; bf16 spacing lets any output meet it only up to |o| = 0.5
        # (half an ulp at 0.5 is 1.95e-3), which covers the five workloads' values
        small = np.abs(o) <= 0.5
        assert (err[small] <= MERGE_ATOL + MERGE_RTOL * np.abs(o[small])).all(), (b, float(err[small].max()))
        # at every magnitude: correctly rounded up to the accumulation noise
        ulp = np.ldexp(1.0, np.maximum(np.frexp(np.maximum(np.abs(o), 1e-300))[1] - 1, -126) - 7)
        assert (err <= 0.5 * ulp + floor).all(), (b, float(((err - floor) / ulp).max()))
    else:
        assert (err <= MERGE_F32_REL * np.abs(o) + floor).all(), (b, float(err.max()))
    row = np.linalg.norm(out_g - o, axis=1) / np.maximum(np.linalg.norm(o, axis=1), 1e-300)
    rep.max_merge_row_rel = max(rep.max_merge_row_rel, float(row.max(initial=0.0)))
    assert (row <= MERGE_ROW_REL).all(), (b, float(row.max()))
    # the merge must actually have happened: the device output is closer to the
    # oracle's merged rows than the unmerged kept rows are, whenever they differ visibly
    if r > 0 and p.f32("alpha") != 0.0:
        moved = np.linalg.norm(o - X[ref.kept], axis=1)
        resid = np.linalg.norm(out_g - o, axis=1)
        vis = moved > 8 * np.linalg.norm(o, axis=1) * 2.0 ** -8
        assert (resid[vis] < 0.5 * moved[vis]).all(), (b, "merge delta missing")


def compare_batch(batch: synth.Batch, gpu: Dict, params: Optional[Dict] = None,
                  images: Optional[List[int]] = None, staged: bool = False,
                  keep_counts: Optional[List[int]] = None) -> Report:
    p = orc.Params.from_dict(batch.params if params is None else params)
    rep = Report()
    for b in (range(batch.batch) if images is None else images):
        compare_image(b, batch, gpu, p, rep, staged=staged,
                      keep_count=None if keep_counts is None else int(keep_counts[b]))
    return rep


# ---------------------------------------------------------------------------
# whole large batches: the oracle fanned out over host processes
# ---------------------------------------------------------------------------
def host_workers() -> int:
    """Worker processes for the oracle: the host's cores, at most 16."""
    return max(1, min(16, os.cpu_count() or 1))


def _merge_reports(into: Report, rep: Report) -> None:
    into.images += rep.images
    into.ratio_boundary += rep.ratio_boundary
    into.selection_near_ties += rep.selection_near_ties
    into.pairing_near_ties += rep.pairing_near_ties
    into.pairs_checked += rep.pairs_checked
    for k in ("max_ratio_err", "max_merge_row_rel", "max_plan_rel", "max_score_abs"):
        setattr(into, k, max(getattr(into, k), getattr(rep, k)))
    into.notes.extend(rep.notes)


def _slice_images(batch: synth.Batch, gpu: Dict, b0: int, b1: int):
    """Images b0..b1-1 of a batch and of a fused result, re-based to start at zero."""
    lo, hi = int(batch.offsets[b0]), int(batch.offsets[b1])
    sub = synth.Batch(batch.cfg, batch.dtype, batch.tokens[lo:hi], (batch.offsets[b0:b1 + 1] - lo).astype(np.int32),
                      batch.density[b0:b1], batch.params, list(range(b0, b1)))
    o0, o1 = int(gpu["out_offsets"][b0]), int(gpu["out_offsets"][b1])
    g = dict(out=gpu["out"][o0:o1], out_offsets=(gpu["out_offsets"][b0:b1 + 1] - o0),
             keep=gpu["keep"][b0:b1], sel=gpu["sel"][lo:hi], pair=gpu["pair"][lo:hi], ratio=gpu["ratio"][b0:b1])
    return sub, g


def _compare_chunk(task):
    """Runs in a worker process (numpy and the oracle only; nothing here touches a GPU)."""
    sub, g, params, first = task
    try:
        from threadpoolctl import threadpool_limits
        limit = threadpool_limits(1)
    except ImportError:                                  # pragma: no cover
        limit = None
    try:
        rep = compare_batch(sub, g, params)
    except AssertionError as e:
        raise AssertionError(f"images {first}..{first + sub.batch - 1} (index inside the chunk first): {e}") from None
    finally:
        if limit is not None:
            limit.restore_original_limits()
    rep.notes = [f"chunk at image {first}: {n}" for n in rep.notes]
    return rep


def compare_batch_parallel(batch: synth.Batch, gpu: Dict, params: Optional[Dict] = None,
                           chunk: int = 16, workers: Optional[int] = None) -> Report:
    """compare_batch over every image of a fused result, the oracle spread over host
    processes.  The workers are started fresh (spawn), so they inherit nothing of this
    process's GPU state, and they import no GPU code."""
    import multiprocessing as mp
    from concurrent.futures import ProcessPoolExecutor
    workers = host_workers() if workers is None else workers
    tasks = []
    for b0 in range(0, batch.batch, chunk):
        b1 = min(batch.batch, b0 + chunk)
        sub, g = _slice_images(batch, gpu, b0, b1)
        tasks.append((sub, g, params, b0))
    total = Report()
    if workers <= 1 or len(tasks) <= 1:
        for t in tasks:
            _merge_reports(total, _compare_chunk(t))
        return total
    with ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn")) as pool:
        for rep in pool.map(_compare_chunk, tasks):
            _merge_reports(total, rep)
    return total
