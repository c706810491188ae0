"""rtprune_prune_static, the variant of rtprune_prune that brings its own workspace (a fixed
array inside the library's device image) for callers that cannot allocate: its outputs must
equal rtprune_prune's bit for bit (same kernels), on calls in a row that reuse the array,
the later ones on smaller inputs, a batch beyond the array must be refused, and the call
recorded into a HIP graph must give the same on every replay."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2605_00392_amd import rtprune as rt  # noqa: E402
from paper_2605_00392_amd import synth  # noqa: E402
from tests import harness as hz  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    rt.load_library()


def _run_static(batch, device="cuda:0"):
    """rtprune_prune_static on a host batch, through the C ABI; outputs as numpy."""
    p = rt.make_params(batch.params)
    db = rt.upload(batch, device)
    B, total = db.B, db.total_tokens
    out = torch.zeros((max(total, 1), db.D), dtype=db.tokens.dtype, device=device)
    out_off = torch.full((B + 1,), -7, dtype=torch.int32, device=device)
    keep = torch.full((max(B, 1),), -7, dtype=torch.int32, device=device)
    sel = torch.full((max(total, 1),), -7, dtype=torch.int32, device=device)
    pair = torch.full((max(total, 1),), -7, dtype=torch.int32, device=device)
    ratio = torch.full((max(B, 1),), -7.0, dtype=torch.float32, device=device)
    dens = torch.from_numpy(np.ascontiguousarray(batch.density, dtype=np.float32)).to(device)
    torch.cuda.synchronize()
    rc = rt.rtprune_prune_static(db, dens, p, out, out_off, keep, sel, pair, ratio)
    torch.cuda.synchronize()
    return dict(rc=rc, out=hz._np(out), out_offsets=hz._np(out_off), keep=hz._np(keep)[:B],
                sel=hz._np(sel)[:total], pair=hz._np(pair)[:total], ratio=hz._np(ratio)[:B])


def _same(a, b, name):
    for k in ("out_offsets", "keep", "sel", "pair", "ratio", "out"):
        np.testing.assert_array_equal(a[k], b[k], err_msg=f"{name}: {k}")


def test_static_scratch_variant_equals_rtprune_prune_on_calls_in_a_row():
    # the calls below follow one another on one stream and share the library's one array:
    # first the largest, then smaller ones, which find the earlier calls' leftovers in it
    cases = [("c3, 48 pages, dynamic ratio", synth.gen_batch(3, images=range(48))),
             ("c2, 5 pages, fixed ratio", synth.gen_batch(2, images=range(5))),
             ("c4, 3 ragged tiled pages", synth.gen_batch(4, images=range(3))),
             ("c1, one fp32 image", synth.gen_batch(1))]
    want = []
    for name, batch in cases:
        ref = hz.run_prune(batch)
        assert ref["rc"] == 0 and ref["status"] == 0, name
        want.append(ref)
    for (name, batch), ref in zip(cases, want):
        print(f"static-scratch call: {name}", flush=True)
        got = _run_static(batch)
        assert got["rc"] == rt.RTP_OK, (name, rt.status_string(got["rc"]))
        assert (got["out_offsets"] >= 0).all(), name                 # written: no device-side error
        _same(got, ref, name)
    # and against the oracle, to the bars of every other parity test (first two cases)
    for (name, batch), _ in list(zip(cases, want))[:2]:
        rep = hz.compare_batch(batch, _run_static(batch), images=range(min(batch.batch, 6)))
        assert rep.images == min(batch.batch, 6)


def test_static_scratch_variant_refuses_a_batch_beyond_its_array():
    batch = synth.gen_batch(3, images=range(2))
    db = rt.upload(batch)
    # the same two images described as part of a batch far larger than the array holds
    db.B, db.total_tokens = 1024, 409600
    rc, need = rt.rtprune_workspace_bytes(db.B, db.total_tokens, db.max_tokens, db.D, db.dtype,
                                          rt.make_params(batch.params))
    assert rc == rt.RTP_OK and need > rt.RTPRUNE_STATIC_SCRATCH_BYTES
    out_off = torch.full((3,), -7, dtype=torch.int32, device="cuda:0")
    rc = rt.rtprune_prune_static(db, None, rt.make_params(batch.params, dynamic=0), 0x1000, out_off, None, None,
                                 None, None)
    torch.cuda.synchronize()
    assert rc == rt.RTP_EWORKSPACE
    assert (out_off.cpu().numpy() == -7).all()                        # nothing was enqueued


def test_static_scratch_variant_replays_from_a_captured_graph():
    # the callers this entry point is for: the whole call recorded into a HIP graph once,
    # then replayed, with the program's own eager work and waits between the replays;
    # every replay must give what the eager call gives
    batch = synth.gen_batch(3, images=range(24))
    other = synth.gen_batch(2, images=range(4))
    ref = hz.run_prune(batch)
    assert ref["rc"] == 0 and ref["status"] == 0
    device = "cuda:0"
    p = rt.make_params(batch.params)
    db = rt.upload(batch, device)
    B, total = db.B, db.total_tokens
    out = torch.zeros((total, db.D), dtype=db.tokens.dtype, device=device)
    out_off = torch.zeros((B + 1,), dtype=torch.int32, device=device)
    keep = torch.zeros((B,), dtype=torch.int32, device=device)
    sel = torch.zeros((total,), dtype=torch.int32, device=device)
    pair = torch.zeros((total,), dtype=torch.int32, device=device)
    ratio = torch.zeros((B,), dtype=torch.float32, device=device)
    dens = torch.from_numpy(np.ascontiguousarray(batch.density, dtype=np.float32)).to(device)
    outs = (out, out_off, keep, sel, pair, ratio)
    assert _run_static(batch)["rc"] == rt.RTP_OK          # first call on the device: set-up done
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        rc = rt.rtprune_prune_static(db, dens, p, *outs)  # on the capturing (current) stream
    assert rc == rt.RTP_OK
    for replay in range(3):
        print(f"graph replay {replay}", flush=True)
        for t in outs:                                    # fill kernels, not memset nodes;
            t.fill_(0 if t is out else -7)                # rows past the packed end stay as filled
        _same(_run_static(other), hz.run_prune(other), "eager call between replays")
        graph.replay()
        torch.cuda.synchronize()
        got = dict(out=hz._np(out), out_offsets=hz._np(out_off), keep=hz._np(keep),
                   sel=hz._np(sel), pair=hz._np(pair), ratio=hz._np(ratio))
        _same(got, ref, f"replay {replay}")
