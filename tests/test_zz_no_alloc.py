"""bbmm_tridiag_eig_batched_noalloc (the entry point for callers that cannot allocate device
memory) against bbmm_tridiag_eig_batched, through the C ABI: same kernel on a fixed work area
inside the library instead of a context buffer, so the results must be bit-identical -- on two
calls in a row, the second with a smaller input (the work area keeps the first call's contents),
and beyond the stated limit the call must refuse with a clear error."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def ctx():
    from paper_1809_11165_amd import binding
    c = binding.Context(0)
    yield c
    c.close()


def _batch(seed, batch, m):
    rng = np.random.default_rng(seed)
    diag = rng.uniform(0.5, 3.0, (batch, m))
    off = rng.uniform(-0.4, 0.4, (batch, max(m - 1, 0)))
    return diag, off


def test_noalloc_matches_the_allocating_entry_point_on_two_calls_in_a_row(ctx):
    import scipy.linalg as sla
    big = _batch(1, 64, 256)              # 16384 entries: the whole work area
    small = _batch(2, 3, 37)              # then a smaller batch over the first call's leftovers
    ref_big = ctx.bbmm_tridiag_eig_batched(*big)
    ref_small = ctx.bbmm_tridiag_eig_batched(*small)
    got_big = ctx.bbmm_tridiag_eig_batched_noalloc(*big)
    got_small = ctx.bbmm_tridiag_eig_batched_noalloc(*small)
    for got, ref in ((got_big, ref_big), (got_small, ref_small)):
        assert np.array_equal(got[0], ref[0])
        assert np.array_equal(got[1], ref[1])
    # and both are right: eigenvalues against LAPACK, unit first rows
    for (diag, off), (vals, first) in ((big, got_big), (small, got_small)):
        for b in (0, diag.shape[0] - 1):
            lam = sla.eigh_tridiagonal(diag[b], off[b], eigvals_only=True)
            assert np.allclose(np.sort(vals[b]), lam, rtol=1e-11, atol=1e-12)
            assert np.sum(first[b] ** 2) == pytest.approx(1.0, rel=1e-10)


def test_noalloc_single_rows_and_a_second_context(ctx):
    from paper_1809_11165_amd import binding
    diag, off = _batch(3, 5, 1)           # m = 1: no off-diagonal at all
    vals, first = ctx.bbmm_tridiag_eig_batched_noalloc(diag, off)
    assert np.array_equal(vals, diag) and np.all(first == 1.0)
    other = binding.Context(0)            # another context on the same GPU uses the same work area
    try:
        d2, o2 = _batch(4, 7, 50)
        a = other.bbmm_tridiag_eig_batched_noalloc(d2, o2)
        b = ctx.bbmm_tridiag_eig_batched(d2, o2)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    finally:
        other.close()


def test_noalloc_rejects_sizes_beyond_its_work_area(ctx):
    from paper_1809_11165_amd import binding
    diag, off = _batch(5, 65, 256)        # 16640 > 16384
    with pytest.raises(binding.BbmmError) as e:
        ctx.bbmm_tridiag_eig_batched_noalloc(diag, off)
    assert e.value.code == binding.EINVAL and "16384" in str(e.value)
    ctx.bbmm_tridiag_eig_batched(diag, off)            # the allocating entry point takes it
    # and the sweep-budget status comes back through the static work area too
    ctx.bbmm_tune("eig_sweeps", 1)
    try:
        with pytest.raises(binding.BbmmError) as e:
            ctx.bbmm_tridiag_eig_batched_noalloc(*_batch(6, 2, 40))
        assert e.value.code == binding.ENOCONV
    finally:
        ctx.bbmm_tune("eig_sweeps", 0)
