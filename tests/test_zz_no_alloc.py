"""c2r_permute_noalloc (static device scratch, for callers that cannot allocate) against
c2r_permute on the same inputs: two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c2r():
    from paper_2504_01337_amd import c2r as m
    m.lib()
    return m


def _outputs(T, K, E_local, d, dtype):
    i32 = dict(dtype=torch.int32, device="cuda")
    return (torch.full((E_local,), -7, **i32), torch.full((E_local + 1,), -7, **i32),
            torch.full((T * K,), -1, **i32), torch.full((T * K,), -7, **i32),
            torch.zeros((T * K, d), dtype=dtype, device="cuda"))


def _case(c2r, seed, T, K, E, d, local):
    print(f"[no_alloc] T={T} K={K} E={E} d={d} local={local}", flush=True)
    rng = np.random.default_rng(seed)
    idx = rng.integers(0, E, size=(T, K)).astype(np.int32)
    idx[::11, 0] = -1                                   # empty slots
    x = torch.from_numpy(rng.standard_normal((T, d)).astype(np.float32)).to(torch.bfloat16).cuda()
    idx_d = torch.from_numpy(idx).cuda()
    if local:
        ls = np.full(E, -1, dtype=np.int32)
        keep = rng.permutation(E)[: E // 2]
        ls[np.sort(keep)] = np.arange(len(keep), dtype=np.int32)
        ls_d, E_local = torch.from_numpy(ls).cuda(), len(keep)
    else:
        ls_d, E_local = None, E
    ref = c2r.permute(x, idx_d, E, ls_d, E_local, out=_outputs(T, K, E_local, d, torch.bfloat16))
    got = c2r.permute_noalloc(x, idx_d, E, ls_d, E_local, out=_outputs(T, K, E_local, d, torch.bfloat16))
    torch.cuda.synchronize()
    for name, a, b in zip(("counts", "offsets", "perm", "inv_perm", "x_perm"), got, ref):
        assert torch.equal(a, b), name      # integer and byte work: bit exact
    assert int(got[1][-1]) > 0


def test_permute_noalloc_two_calls_second_smaller(c2r):
    # both sizes are above the one-launch switch point (49152 assignments), so both calls go
    # through the block histograms in the static array; the second reuses it with fewer blocks
    _case(c2r, 1, T=70000, K=4, E=60, d=64, local=False)
    _case(c2r, 2, T=20000, K=4, E=60, d=64, local=True)
    # and one below the switch point (no scratch is read)
    _case(c2r, 3, T=1000, K=2, E=8, d=64, local=False)


def test_permute_noalloc_rejects_sizes_beyond_its_array(c2r):
    import ctypes
    p = ctypes.c_void_p(0x1000)       # rejected on the host before anything is touched
    L = c2r.lib()
    assert L.c2r_permute_noalloc(p, 1, p, (1 << 22) // 4 + 1, 64, 8, 4, None, 8, p, p, p, p, p, None) == c2r.ERR_UNSUPPORTED
    assert L.c2r_permute_noalloc(p, 1, p, 16, 64, 8, 0, None, 8, p, p, p, p, p, None) == c2r.ERR_INVALID_ARG
