"""GPU parity of rtprune_prune_splice: the fused call writing straight into the
prefill input.  Placement (sequence offsets, position ids, text rows) against the
oracle's splice; the merged visual rows inside the sequences against the oracle's
merge directly; and the whole against the packed output of rtprune_prune (same
kernels, so bit for bit)."""
import numpy as np
import pytest

from paper_2605_00392_amd import rtprune as rt, synth
from oracle import rtprune_oracle as orc
from tests import harness as hz

pytestmark = pytest.mark.gpu


def _text(rng, counts, d, dtype):
    off = np.zeros(len(counts) + 1, dtype=np.int32)
    off[1:] = np.cumsum(counts)
    rows = rng.standard_normal((int(off[-1]), d)).astype(np.float32)
    return (synth.f32_to_bf16_bits(rows) if dtype == "bf16" else rows), off


def _run(batch, prefix, poff, suffix, soff, mode, params=None):
    import torch
    dev = "cuda:0"
    p = rt.make_params(batch.params if params is None else params)
    db = rt.upload(batch, dev)
    ws = rt.alloc_workspace(db)
    B, total = db.B, db.total_tokens
    tdt = db.tokens.dtype

    def up(a):
        if a is None:
            return None
        t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev)
        return t.view(tdt) if a.dtype == np.uint16 else t
    pre, suf = up(prefix), up(suffix)
    po, so = up(poff), up(soff)
    prow = int(poff[-1]) if poff is not None else 0
    srow = int(soff[-1]) if soff is not None else 0
    cap = prow + srow + total + 3
    seq = torch.full((cap, db.D), 7.0, dtype=tdt, device=dev)
    seq_off = torch.full((B + 1,), -7, dtype=torch.int32, device=dev)
    pos = torch.full((cap,), -7, dtype=torch.int32, device=dev)
    keep = torch.full((max(B, 1),), -7, dtype=torch.int32, device=dev)
    sel = torch.full((max(total, 1),), -7, dtype=torch.int32, device=dev)
    pair = torch.full((max(total, 1),), -7, dtype=torch.int32, device=dev)
    ratio = torch.full((max(B, 1),), -7.0, dtype=torch.float32, device=dev)
    dens = torch.from_numpy(batch.density).to(dev)
    text = rt.make_text_spans(pre, po, prow, suf, so, srow)
    rt.check(rt.rtprune_prune_splice(db, dens, p, text, mode, seq, cap, seq_off, pos, keep, sel, pair, ratio, ws))
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) == 0
    return dict(seq=hz._np(seq), seq_off=seq_off.cpu().numpy(), pos=pos.cpu().numpy(),
                keep=keep.cpu().numpy(), sel=sel.cpu().numpy(), pair=pair.cpu().numpy(),
                ratio=ratio.cpu().numpy(), cap=cap)


@pytest.mark.parametrize("mode", [orc.POSITIONS_CONSECUTIVE, orc.POSITIONS_ORIGINAL])
@pytest.mark.parametrize("cfg,images", [(3, 5), (4, 4), (1, 1)])
def test_splice_matches_oracle_and_packed_output(cfg, images, mode, extra=None):
    batch = synth.gen_batch(cfg, images=range(images))
    if extra:
        batch.params.update(extra)
    rng = np.random.default_rng(100 + cfg)
    B, d = batch.batch, batch.tokens.shape[1]
    pc = rng.integers(0, 9, size=B)
    sc = rng.integers(0, 5, size=B)
    pc[0] = 0                                         # an image with no prefix
    prefix, poff = _text(rng, pc, d, batch.dtype)
    suffix, soff = _text(rng, sc, d, batch.dtype)
    g = _run(batch, prefix, poff, suffix, soff, mode)
    f = hz.run_prune(batch)                           # packed output of the same path
    np.testing.assert_array_equal(g["keep"][:B], f["keep"][:B])
    np.testing.assert_array_equal(g["sel"], f["sel"])
    at = 0
    for b in range(B):
        lo, hi = int(batch.offsets[b]), int(batch.offsets[b + 1])
        m = int(f["keep"][b])
        o0 = int(f["out_offsets"][b])
        kept = f["sel"][lo:lo + m]
        rows, pos = orc.splice_sequence(prefix[poff[b]:poff[b + 1]], f["out"][o0:o0 + m],
                                        suffix[soff[b]:soff[b + 1]], kept, hi - lo, mode)
        assert int(g["seq_off"][b]) == at
        np.testing.assert_array_equal(g["seq"][at:at + len(rows)], rows)
        np.testing.assert_array_equal(g["pos"][at:at + len(rows)], pos)
        at += len(rows)
    assert int(g["seq_off"][B]) == at
    # nothing beyond the last sequence is touched
    assert (g["pos"][at:] == -7).all()
    tail = g["seq"][at:]
    assert (tail == tail.flat[0]).all() if tail.size else True
    # and the visual rows inside the sequences, taken from `seq` itself (with the kept
    # counts, index lists, pairing and retention the splice call returned), are the rows
    # the oracle's merge gives, to the bars of every other parity test
    pre_n = np.diff(poff)
    vis, vis_off = [], np.zeros(B + 1, dtype=np.int32)
    for b in range(B):
        a = int(g["seq_off"][b]) + int(pre_n[b])
        vis.append(g["seq"][a:a + int(g["keep"][b])])
        vis_off[b + 1] = vis_off[b] + int(g["keep"][b])
    from_seq = dict(out=np.concatenate(vis, axis=0), out_offsets=vis_off, keep=g["keep"][:B], sel=g["sel"],
                    pair=g["pair"], ratio=g["ratio"][:B])
    rep = hz.compare_batch(batch, from_seq, staged=False)
    assert rep.images == B


def test_splice_through_the_merge_kernel_for_middling_pruned_sets():
    """63 pruned tokens per page, the matrix-core merge kernel for 17 to 64 switched on for a
    small batch: it writes into the sequence at each image's visual start like the others."""
    test_splice_matches_oracle_and_packed_output(9, 3, orc.POSITIONS_ORIGINAL, dict(mid_merge_min_images=1))


def test_splice_without_text_is_the_packed_output():
    batch = synth.gen_batch(2, images=range(3))
    g = _run(batch, None, None, None, None, orc.POSITIONS_CONSECUTIVE)
    f = hz.run_prune(batch)
    rows = int(f["out_offsets"][-1])
    np.testing.assert_array_equal(g["seq_off"], f["out_offsets"])
    np.testing.assert_array_equal(g["seq"][:rows], f["out"][:rows])
    for b in range(batch.batch):
        a, e = int(g["seq_off"][b]), int(g["seq_off"][b + 1])
        np.testing.assert_array_equal(g["pos"][a:e], np.arange(e - a))


def test_bad_text_offsets_set_the_status_word():
    import torch
    batch = synth.gen_batch(2, images=range(2))
    rng = np.random.default_rng(5)
    prefix, poff = _text(rng, [3, 2], batch.tokens.shape[1], batch.dtype)
    bad = poff.copy()
    bad[1] = 4
    bad[2] = 3                                       # decreasing
    dev = "cuda:0"
    db = rt.upload(batch, dev)
    ws = rt.alloc_workspace(db)
    pre = torch.from_numpy(prefix.view(np.int16)).to(dev).view(db.tokens.dtype)
    po = torch.from_numpy(bad).to(dev)
    cap = 5 + db.total_tokens
    seq = torch.full((cap, db.D), 7.0, dtype=db.tokens.dtype, device=dev)
    seq_off = torch.full((3,), -7, dtype=torch.int32, device=dev)
    text = rt.make_text_spans(pre, po, 5)
    rt.check(rt.rtprune_prune_splice(db, None, rt.make_params(batch.params), text, 0, seq, cap, seq_off, None,
                                     None, None, None, None, ws))
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).item()) & rt.RTP_DEV_BAD_OFFSETS
    assert (seq_off.cpu().numpy() == -7).all()
    assert (seq.float() == 7.0).all().item()
