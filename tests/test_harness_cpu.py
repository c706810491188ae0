"""Host-side checks of the parity harness itself: the whole-batch comparison that
fans the oracle out over worker processes accepts a result that is right and
rejects one with a planted mistake.  The stand-in "device result" here is built
from the oracle's own output (rounded to the token dtype); no GPU is involved."""
import numpy as np
import pytest

from oracle import rtprune_oracle as orc
from paper_2605_00392_amd import synth
from tests import harness as hz


def _stand_in_result(batch):
    p = orc.Params.from_dict(batch.params)
    res = orc.prune_batch(batch.tokens, batch.dtype, batch.offsets, batch.density, p)
    out_off = np.zeros(batch.batch + 1, dtype=np.int32)
    out_off[1:] = np.cumsum([r.m for r in res])
    sel = np.concatenate([np.concatenate([r.kept, r.prop]) for r in res]).astype(np.int32)
    pair = np.concatenate([np.concatenate([np.arange(r.m), r.pair]) for r in res]).astype(np.int32)
    rows = np.concatenate([orc.round_to_bf16(r.merged) for r in res], axis=0).astype(np.float32)
    return dict(out=synth.f32_to_bf16_bits(rows), out_offsets=out_off,
                keep=np.array([r.m for r in res], dtype=np.int32), sel=sel, pair=pair,
                ratio=np.array([r.retention for r in res], dtype=np.float32))


@pytest.fixture(scope="module")
def case():
    batch = synth.gen_batch(3, images=range(7))
    return batch, _stand_in_result(batch)


def test_parallel_compare_accepts_a_right_result_and_counts_every_image(case):
    batch, g = case
    rep = hz.compare_batch_parallel(batch, g, chunk=2, workers=3)
    serial = hz.compare_batch(batch, g)
    assert rep.images == serial.images == 7
    assert rep.pairs_checked == serial.pairs_checked == int((np.diff(batch.offsets) - g["keep"]).sum())
    assert rep.pairing_near_ties == 0 and rep.selection_near_ties == 0 and rep.ratio_boundary == 0
    assert rep.max_merge_row_rel == pytest.approx(serial.max_merge_row_rel)


def test_parallel_compare_rejects_a_planted_wrong_partner(case):
    batch, g = case
    bad = dict(g, pair=g["pair"].copy())
    # the last image with a pruned token: send its first pruned token to another kept row
    b = max(i for i in range(batch.batch) if g["keep"][i] < batch.offsets[i + 1] - batch.offsets[i])
    at = int(batch.offsets[b]) + int(g["keep"][b])
    bad["pair"][at] = (bad["pair"][at] + 1) % int(g["keep"][b])
    with pytest.raises(AssertionError, match="partner differs"):
        hz.compare_batch_parallel(batch, bad, chunk=2, workers=2)


def test_parallel_compare_rejects_unmerged_rows(case):
    batch, g = case
    bad = dict(g, out=g["out"].copy())
    b = 1
    lo, m = int(batch.offsets[b]), int(g["keep"][b])
    o0 = int(g["out_offsets"][b])
    bad["out"][o0:o0 + m] = batch.tokens[lo + g["sel"][lo:lo + m]]     # the kept rows, not merged
    if m < batch.offsets[b + 1] - lo:
        with pytest.raises(AssertionError):
            hz.compare_batch_parallel(batch, bad, chunk=3, workers=2)
