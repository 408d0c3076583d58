"""The entry point that allocates nothing (btard_centered_clip_verify_noalloc, for callers
that cannot call hipMalloc or hand over a workspace): through the C ABI, against the
existing entry point with a caller's workspace, on two calls in a row, the second on a
smaller input (the library's scratch array then still holds the first call's state)."""
import pytest
import torch

import paper_2106_11257_amd as btard
from paper_2106_11257_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


def outputs(n, d, P, dev):
    out = {k: torch.full((n, P), float("nan"), dtype=torch.float64, device=dev)
           for k in ("norms", "weights", "proj")}
    out["colsum"] = torch.full((P,), float("nan"), dtype=torch.float64, device=dev)
    return (torch.full((d,), float("nan"), dtype=torch.float32, device=dev),
            torch.full((P,), -7, dtype=torch.int32, device=dev),
            torch.full((P,), float("nan"), dtype=torch.float64, device=dev), out)


def run_both(G, off, tau, eps, M, seed, flags, v0=None):
    n, d = G.shape
    P = len(off) - 1
    v, iters, sn, out = outputs(n, d, P, G.device)
    print(f"[noalloc] n={n} d={d} P={P} M={M} flags={flags} v0={'yes' if v0 is not None else 'mean'}",
          flush=True)
    btard.centered_clip_verify_noalloc(G, off, tau, eps, M, seed, v, iters, sn, out, v0=v0,
                                       flags=flags)
    want = btard.centered_clip_verify(G, off, tau, eps, M, seed, v0=v0, flags=flags)
    torch.cuda.synchronize()
    assert torch.equal(iters, want[1]) and (iters > 0).all()
    assert torch.equal(v, want[0])
    assert torch.equal(sn, want[2])
    for k in ("norms", "weights", "proj", "colsum"):
        assert torch.equal(out[k], want[3][k]), k


@pytest.mark.parametrize("flags", [0, 1])
def test_two_calls_in_a_row_the_second_smaller(dev, flags):
    big, off_big = workloads.generic_case(16, 300_007, 16, seed=41, device=dev, ld=300_016,
                                          spread=0.3, outliers=3)
    small, off_small = workloads.generic_case(7, 40_003, 5, seed=42, device=dev, spread=0.05,
                                              outliers=2)
    run_both(big, off_big, 1.0, 1e-6, 30, 0xA110C, flags)
    run_both(small, off_small, 0.6, 1e-7, 40, 0xA110D, flags)
    # and with a caller's start vector (per-iteration passes, the two separate last passes)
    v0 = small[1].clone()
    run_both(small, off_small, 0.6, 1e-7, 12, 0xA110E, flags, v0=v0)


def test_sizes_beyond_the_scratch_array_are_refused(dev):
    G, off = workloads.generic_case(17, 2000, 2, seed=43, device=dev)
    v, iters, sn, out = outputs(17, 2000, 2, dev)
    with pytest.raises(btard.BtardError) as e:
        btard.centered_clip_verify_noalloc(G, off, 1.0, 1e-6, 5, 1, v, iters, sn, out)
    assert e.value.status == -2                       # BTARD_ERR_WORKSPACE
    G16, off16 = workloads.generic_case(16, 2000, 2, seed=44, device=dev)
    v, iters, sn, out = outputs(16, 2000, 2, dev)
    with pytest.raises(btard.BtardError) as e:        # nothing in this call may wait for the device
        btard.centered_clip_verify_noalloc(G16, off16, 1.0, 1e-6, 5, 1, v, iters, sn, out,
                                           flags=btard.BTARD_FLAG_GRAM | btard.BTARD_FLAG_HOST_SYNC)
    assert e.value.status == -1
    torch.cuda.synchronize()
    assert int(iters[0]) == -7                        # untouched: refused before any launch
