"""spd_pairwise_static, the entry point that allocates nothing, against spd_pairwise (needs an
MI355X; run with -m gpu).  Collected last: it must pass alone in a fresh process and after every
other test."""
import numpy as np
import pytest

from gen import synth
from util import assert_distances_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def spd():
    import paper_2104_06357_amd as lib
    return lib


def _both(spd, h, A, B, metric, p=2.0):
    import torch
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    want = h.pairwise(dA, dB, metric, p)
    got = torch.full((A["n_rows"], B["n_rows"]), float("nan"), dtype=torch.float32, device="cuda")
    h.pairwise_static(dA, dB, metric, got, p)
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy()


def test_two_calls_in_a_row_the_second_smaller(spd):
    """Config 1 (10,000 x 10,000, three launches), then config 0 (256 x 256) through the same
    array, which still holds the first call's data: each must equal spd_pairwise."""
    h = spd.Handle()
    h.set_option("check_plan", 1)
    print("static entry: config 1, l1", flush=True)
    A, B = synth.workload(1)
    got, want = _both(spd, h, A, B, "l1")
    assert_distances_close(got, want, "static l1, config 1")
    assert np.array_equal(got, want)                    # same plan, same kernels: the same bits
    print("static entry: config 0, cosine and jensen_shannon", flush=True)
    A, B = synth.workload(0)
    for metric in ("cosine", "jensen_shannon"):
        got, want = _both(spd, h, A, B, metric)
        assert_distances_close(got, want, "static %s, config 0" % metric)
        assert np.array_equal(got, want)
    h.close()


def test_sliced_rows_keep_their_partial_sums_in_the_static_array(spd):
    """Rows of A cut into slices (their partial sums live in the scratch between two launches),
    a larger case first and a smaller one after it, and a second handle on the same array."""
    rng = np.random.default_rng(11)

    def wide(rows_a, rows_b):
        out = []
        for rows in (rows_a, rows_b):
            d = np.zeros((rows, 400))
            for r in range(rows):
                n = int(rng.choice([0, 3, 40, 150, 300, 400]))
                d[r, rng.choice(400, size=n, replace=False)] = rng.random(n) + 0.01
            out.append(synth.from_dense(np.asarray(d.astype(np.float32), dtype=np.float64)))
        return out

    for handle_no, (ra, rb) in enumerate(((90, 140), (20, 33))):
        h = spd.Handle()
        for name, value in (("split_len", 4), ("window", 64), ("force_kind", 3), ("lds_budget", 8192), ("check_plan", 1)):
            h.set_option(name, value)
        A, B = wide(ra, rb)
        plan = spd.testing.host_plan_summary(A["indptr"], B["indptr"], 400, "minkowski", split_len=4, window=64, force_kind=3,
                                     lds_budget=8192)
        assert plan["spilled_rows"] > 0
        for metric in ("minkowski", "chebyshev", "hellinger"):
            print("static entry: slices, handle", handle_no, metric, flush=True)
            got, want = _both(spd, h, A, B, metric, 3.0)
            assert_distances_close(got, want, "static %s with slices" % metric)
            assert np.array_equal(got, want)
        h.close()


def test_rejections(spd):
    import torch
    h = spd.Handle()
    A, B = synth.workload(0)
    out = torch.empty((256, 256), dtype=torch.float32, device="cuda")
    # no host copy of the row pointers: the call would have to wait for the stream
    dA, dB = spd.DeviceCsr.from_host(A, keep_host_indptr=False), spd.DeviceCsr.from_host(B)
    with pytest.raises(spd.SpdError) as e:
        h.pairwise_static(dA, dB, "l1", out)
    assert e.value.status_name == "SPD_ERR_NULL"
    # an index whose packed copy is larger than the array (4.6 M entries x 8 bytes)
    _, big = synth.workload(1, scale=12.0)
    assert int(big["indptr"][-1]) * 8 > 32 << 20
    small = synth.slice_rows(big, 0, 8)
    out = torch.empty((8, big["n_rows"]), dtype=torch.float32, device="cuda")
    with pytest.raises(spd.SpdError) as e:
        h.pairwise_static(spd.DeviceCsr.from_host(small), spd.DeviceCsr.from_host(big), "cosine", out)
    assert e.value.status_name == "SPD_ERR_WORKSPACE" and "allocates nothing" in str(e.value)
    # the handle still serves the ordinary entry point, and the static one, afterwards
    want = h.pairwise(spd.DeviceCsr.from_host(small), spd.DeviceCsr.from_host(big), "cosine")
    A, B = synth.workload(0)
    dA, dB = spd.DeviceCsr.from_host(A), spd.DeviceCsr.from_host(B)
    got = torch.empty((256, 256), dtype=torch.float32, device="cuda")
    h.pairwise_static(dA, dB, "l1", got)
    assert torch.equal(got, h.pairwise(dA, dB, "l1"))
    assert bool(torch.isfinite(want).all())
    h.close()
