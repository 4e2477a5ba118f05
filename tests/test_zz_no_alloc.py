"""The decode-aggregate entry point for callers that cannot allocate device memory
(cvlc_decode_aggregate_static) against cvlc_decode_aggregate, through the C ABI.

Collected last (file name), so that a failure here hides no other test; passes
alone in a fresh process and after the other tests.
"""
import numpy as np
import pytest
import torch

import cvlc_synth as syn
import paper_2402_03770_amd.cvlc as cv
from oracle import cvlc_oracle as orc

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _streams(d, n, seed):
    plan = orc.plan_alg1(d, int(0.9 * d), 7, -0.6)
    refs = [orc.encode(syn.update_vector(3, 100 * seed + c, d=d), plan, seed, c).words for c in range(n)]
    return refs, [torch.from_numpy(r.view(np.int32)).to(DEV) for r in refs]


def _abs_terms(refs, d, weights):
    tot = np.zeros(d)
    for r, w in zip(refs, weights):
        tot += np.abs(orc.decode_aggregate([r], d, weights=[1.0]).astype(np.float64)) * abs(float(np.float32(w)))
    return tot


def _both(dev, d, weights, start=None):
    """(static entry point's result and status word, workspace entry point's result and status word)."""
    out_s = torch.full((d,), float("nan"), dtype=torch.float32, device=DEV) if start is None else start.clone()
    out_w = out_s.clone()
    status = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    cv.decode_aggregate_static(dev, out_s, status, weights=weights, accumulate=start is not None)
    ws = cv.new_workspace(cv.decode_workspace_bytes(d, len(dev)), DEV)
    cv.decode_aggregate(dev, out_w, ws, weights=weights, accumulate=start is not None)
    st_w = cv.device_status(ws)
    torch.cuda.synchronize()
    return out_s.cpu().numpy(), int(status.item()), out_w.cpu().numpy(), st_w


def test_static_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    """Two calls in a row on the same device, the second with a smaller model and fewer clients (what the
    first left in the array must not matter), then a third in accumulate mode and a malformed stream."""
    for d, n, seed in ((300_007, 6, 1), (50_001, 2, 2)):
        refs, dev = _streams(d, n, seed)
        wts = [float(np.float32(v)) for v in np.linspace(0.25, 1.5, n)]
        got_s, st_s, got_w, st_w = _both(dev, d, wts)
        assert st_s == 0 and st_w == 0
        tol = 1e-5 * _abs_terms(refs, d, wts)
        ref = orc.decode_aggregate(refs, d, weights=wts).astype(np.float64)
        assert np.all(np.abs(got_s.astype(np.float64) - got_w.astype(np.float64)) <= tol)
        assert np.all(np.abs(got_s.astype(np.float64) - ref) <= tol)
    # one client: both entry points are bit exact
    got_s, st_s, got_w, st_w = _both(dev[:1], d, [1.0])
    assert st_s == 0 and np.array_equal(got_s.view(np.uint32), got_w.view(np.uint32))
    assert np.array_equal(got_s.view(np.uint32), orc.decode_aggregate(refs[:1], d, weights=[1.0]).view(np.uint32))
    # accumulate mode on top of what the output holds
    start = torch.from_numpy(np.random.default_rng(3).standard_normal(d).astype(np.float32)).to(DEV)
    got_s, st_s, got_w, st_w = _both(dev, d, wts, start=start)
    tol = 1e-5 * (_abs_terms(refs, d, wts) + np.abs(start.cpu().numpy().astype(np.float64)))
    assert st_s == 0 and np.all(np.abs(got_s.astype(np.float64) - got_w.astype(np.float64)) <= tol)
    # a malformed stream is reported through the status word the caller passed
    bad = refs[0].copy()
    bad[0] ^= 1
    got_s, st_s, got_w, st_w = _both([torch.from_numpy(bad.view(np.int32)).to(DEV), dev[1]], d, [1.0, 1.0])
    assert st_s == st_w and st_s & cv.DEV_STREAM


def test_static_entry_point_refuses_what_does_not_fit_and_allocates_nothing():
    d = 11_200_000
    assert cv.decode_workspace_bytes(d, 32) <= cv.DECODE_STATIC_BYTES < cv.decode_workspace_bytes(d, 64)
    out = torch.zeros(d, dtype=torch.float32, device=DEV)
    refs, dev = _streams(40_000, 1, 5)
    with pytest.raises(cv.CvlcError) as e:
        cv.decode_aggregate_static(dev * 64, out)           # 64 clients of this size need more than the array holds
    assert e.value.code == -4
    torch.cuda.synchronize()
    small = torch.zeros(40_000, dtype=torch.float32, device=DEV)
    free_before, _ = torch.cuda.mem_get_info()
    for _ in range(3):
        cv.decode_aggregate_static(dev, small)              # without a status word
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert free_after == free_before                        # the calls took no device memory
    assert np.array_equal(small.cpu().numpy().view(np.uint32),
                          orc.decode_aggregate(refs, 40_000, weights=None).view(np.uint32))
