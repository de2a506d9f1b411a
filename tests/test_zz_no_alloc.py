"""The entry point that allocates nothing (maaso_placement_sweep_noalloc) against
maaso_placement_sweep, through the C-ABI: same counts, ratios and best candidate, bit for bit, on
calls in a row that share the library's static scratch array - the second smaller than the first, so
that whatever the first left behind would show."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
from paper_2509_06362_amd import binding, workloads as W  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' on CPU-only machines)")
    binding.load_library()


def both(w, window=0):
    """(no-alloc outputs, ordinary outputs) as numpy arrays; each on a fresh context."""
    res = []
    for noalloc in (True, False):
        dw = binding.DeviceWorkload(w)
        try:
            out = dw.sweep(window=window, noalloc=noalloc)
            torch.cuda.synchronize()
            assert binding.maaso_ctx_device_status(dw.ctx) == 0
            res.append((out[0].cpu().numpy().view(np.uint32), out[1].cpu().numpy(),
                        int(out[2].cpu().numpy().view(np.uint32)[0])))
        finally:
            dw.close()
    return res


def test_two_calls_in_a_row_the_second_smaller():
    big = W.stressed(W.config1(n_cand=700, n_req=20000), seed=31)
    small = W.stressed(W.config4(n_cand=9, n_req=1500), seed=32)
    spread = 0
    for w in (big, small):
        print(f"no-alloc sweep {w.name} C={w.n_cand} I={w.i_pad} R={w.n_req}", flush=True)
        (cnt, ratio, best), (cnt0, ratio0, best0) = both(w)
        assert np.array_equal(cnt, cnt0)
        assert np.array_equal(ratio, ratio0)
        assert best == best0
        ref = oracle.placement_sweep(w)
        assert np.array_equal(cnt, ref["sat_count"]) and best == ref["best_cand"]
        spread = max(spread, len(np.unique(cnt)))
    assert spread > 1


def test_same_context_repeated_and_interleaved_with_the_ordinary_entry_point():
    w1 = W.stressed(W.config3(n_cand=600, n_req=9000), seed=33)
    w2 = W.stressed(W.config1(n_cand=40, n_req=700), seed=34)
    ref1, ref2 = oracle.placement_sweep(w1)["sat_count"], oracle.placement_sweep(w2)["sat_count"]
    d1, d2 = binding.DeviceWorkload(w1), binding.DeviceWorkload(w2)
    try:
        for noalloc1, noalloc2 in ((True, True), (False, True), (True, False), (True, True)):
            a = d1.sweep(noalloc=noalloc1)[0].clone()
            b = d2.sweep(noalloc=noalloc2)[0].clone()
            torch.cuda.synchronize()
            assert np.array_equal(a.cpu().numpy().view(np.uint32), ref1)
            assert np.array_equal(b.cpu().numpy().view(np.uint32), ref2)
        assert binding.maaso_ctx_device_status(d1.ctx) == 0
        assert binding.maaso_ctx_device_status(d2.ctx) == 0
    finally:
        d1.close()
        d2.close()


def test_capacity_aware_form_passes_through():
    w = W.stressed(W.config1(n_cand=40, n_req=3000), seed=35)
    w = W.replace(w, arrival_ticks=W.poisson_arrivals(W.rng_for(35, 3), 900.0, w.n_req))
    (cnt, ratio, best), (cnt0, ratio0, best0) = both(w, window=256)
    assert np.array_equal(cnt, cnt0) and np.array_equal(ratio, ratio0) and best == best0


def test_a_shape_beyond_the_scratch_is_refused():
    # 16 bytes per instance slot: 40,000 candidates of 32 slots need 20 MB of records
    w = W.config1(n_cand=40000, n_req=256)
    dw = binding.DeviceWorkload(w)
    try:
        with pytest.raises(binding.MaasoError) as e:
            dw.sweep(noalloc=True)
        assert e.value.status == -2
        assert "size" in str(e.value)
        cnt = dw.sweep(noalloc=False)[0]          # the ordinary entry point takes it
        torch.cuda.synchronize()
        assert int(cnt.cpu().numpy().view(np.uint32).max()) <= w.n_req
        # the largest shape of the five workloads that fits: config 1 in full
        assert 4 * 3 * 65536 + 16 * 4096 * 32 + (1 << 20) < binding.MAASO_NOALLOC_SCRATCH_BYTES
    finally:
        dw.close()
