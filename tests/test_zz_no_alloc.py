"""The allocation-free entry point sc_block_qr_noalloc against sc_block_qr (same kernels, scratch in a fixed device
array inside the library): bitwise the same Q, R and Gram matrix on two calls in a row, the second on a smaller input
(the array keeps the first call's contents), no change in the device's free memory across the calls, and the size
limits as error codes."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_1802_04450_amd import binding
    binding.lib()
    return binding


def _block(n, ld, j, b, seed):
    rng = np.random.default_rng(seed)
    basis = rng.standard_normal((n, ld))
    basis[:, j + b - 1] = basis[:, j] if b > 2 else basis[:, j + b - 1]      # a dependent column when there is room
    return torch.from_numpy(basis).cuda()


def test_noalloc_block_qr_matches_block_qr_twice_in_a_row(B):
    shapes = [(70001, 48, 5, 32, 1), (1237, 21, 3, 8, 2)]       # large first, then smaller in every dimension
    # references from the allocating entry point, and everything the test needs on the device, before measuring
    cases = []
    for n, ld, j, b, seed in shapes:
        ref = _block(n, ld, j, b, seed)
        r0, g0 = B.sc_block_qr(ref, j, b)
        work = _block(n, ld, j, b, seed)
        r = torch.full((b, b), 7.0, dtype=torch.float64, device="cuda")
        g = torch.full((b, b), 7.0, dtype=torch.float64, device="cuda")
        cases.append((ref, r0, g0, work, r, g, j, b))
    # a first call creates whatever the runtime sets up lazily (the scratch array itself is part of the loaded code
    # object); from then on the free memory must not move
    warm = _block(100, 8, 0, 4, 9)
    rw = torch.empty((4, 4), dtype=torch.float64, device="cuda")
    assert B.sc_block_qr_noalloc(warm, 0, 4, rw, rw.clone()) == B.SC_OK
    B.sc_release_cache()
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for ref, r0, g0, work, r, g, j, b in cases:
        assert B.sc_block_qr_noalloc(work, j, b, r, g) == B.SC_OK
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0, (free0, free1)
    for ref, r0, g0, work, r, g, j, b in cases:
        assert torch.equal(work, ref)            # Q in place, and nothing outside the block touched
        assert torch.equal(r, r0) and torch.equal(g, g0)
        q = work[:, j:j + b].cpu().numpy()
        keep = np.abs(np.diag(r.cpu().numpy())) > 0
        assert keep.sum() >= b - 1
        assert np.max(np.abs(q[:, keep].T @ q[:, keep] - np.eye(int(keep.sum())))) < 1e-13


def test_noalloc_block_qr_rejects_what_its_scratch_cannot_hold(B):
    x = torch.zeros((64, 80), dtype=torch.float64, device="cuda")
    r = torch.zeros((64, 64), dtype=torch.float64, device="cuda")
    for b in (64, 3, 0, 33):
        with pytest.raises(B.ScError) as e:
            B.sc_block_qr_noalloc(x, 0, b, r, r)
        assert e.value.code == B.SC_EDOMAIN
    with pytest.raises(B.ScError) as e:
        B.sc_block_qr_noalloc(x, 70, 16, r, r)        # block does not fit the leading dimension
    assert e.value.code == B.SC_EDOMAIN
    assert torch.all(x == 0.0)
