"""The inversion entry point that allocates nothing (its working arrays are a device array inside the
library) against the ordinary kfac_invert, through the C ABI: two calls in a row, the second smaller."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2211_14133_amd import synth  # noqa: E402

pytestmark = pytest.mark.gpu


def test_invert_noalloc_matches_kfac_invert(oracle):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2211_14133_amd as k

    lib = k.load()
    assert lib.kfac_invert_noalloc_max_d() == 2048
    lam = 1e-3
    for call, d in enumerate((1300, 200)):  # ragged sizes spanning several panels; the second reuses the array
        print("noalloc invert d=%d" % d, flush=True)
        a = oracle.curvature(synth.activations(2, 8, call, 0, 2 * d + 8, d, gelu=(call == 0))).astype(np.float32)
        fd = torch.from_numpy(a).cuda()
        want_inv = torch.full((d, d), 3.0, device="cuda")
        want_info = k.kfac_invert(fd, lam, want_inv)
        got_inv = torch.full((d, d), 3.0, device="cuda")
        got_info = torch.full((1,), 77, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        k.kfac_invert_noalloc(fd, lam, got_inv, got_info)
        assert torch.cuda.memory_allocated() == before  # nothing taken from torch's allocator either
        torch.cuda.synchronize()
        assert int(want_info[0]) == 0 and int(got_info[0]) == 0
        assert torch.equal(got_inv, want_inv)  # the same kernels on the same data: bit for bit
        ref, _ = oracle.invert(a.astype(np.float64), lam)
        cond = np.linalg.cond(a.astype(np.float64) + lam * np.eye(d))
        assert oracle.rel_fro(got_inv.cpu().numpy(), ref) <= 2e-6 * cond + 1e-6
    # a failing matrix: info reports the pivot, the inverse is left alone
    m = torch.eye(300, device="cuda")
    m[170, 170] = -1.0
    inv = torch.full((300, 300), 3.0, device="cuda")
    info = torch.zeros(1, dtype=torch.int32, device="cuda")
    k.kfac_invert_noalloc(m, 0.0, inv, info)
    torch.cuda.synchronize()
    assert int(info[0]) == 171 and bool(torch.all(inv == 3.0))
    # beyond the built-in array: refused before anything is enqueued
    big = torch.eye(2049, device="cuda")
    with pytest.raises(k.KfacError):
        k.kfac_invert_noalloc(big, lam, torch.empty_like(big), info)
