"""rad_sample_pack_static (the entry point that allocates nothing: its keep bitmap lies in a static device
array) against rad_sample_pack, entry for entry and bit for bit, on two calls in a row, the second with a
smaller input, so that what the first call left in the array is there when the second runs."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2007_10412_amd import binding as B
    c = B.rad_ctx_create()
    yield c
    B.rad_ctx_destroy(c)


def _both(ctx, rows, cols, scheme, p, dtype, seed):
    """Stores written by the two entry points from the same input and sampling parameters."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev
    print("sample_pack_static rows=%d cols=%d scheme=%d p=%g dtype=%d seed=%d" % (rows, cols, scheme, p, dtype, seed),
          flush=True)
    rng = np.random.default_rng(seed)
    x = dev(rng.standard_normal((rows, cols)).astype(np.float32), dtype)
    L = B.make_layer(rows, cols, 8, dtype=dtype, relu=False)
    sm = B.make_sampling(scheme, p, seed, 2, 1)
    out = []
    for static in (True, False):
        st = B.rad_store_create(ctx, L, scheme, p)
        try:
            if static:
                B.rad_sample_pack_static(ctx, sm, x, st)
            else:
                B.rad_sample_pack(ctx, sm, x, st)
            out.append(B.rad_store_export_csr(ctx, st, rows))
        finally:
            B.rad_store_destroy(st)
    return out


def _same(a, b):
    for u, v in zip(a, b):
        assert u.shape == v.shape
        assert np.array_equal(u.view(np.uint32) if u.dtype == np.float32 else u,
                              v.view(np.uint32) if v.dtype == np.float32 else v)


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("scheme,p", [(1, 0.1), (3, 0.1), (2, 0.1), (5, 0.1), (0, 1.0)])
def test_two_calls_in_a_row_match_rad_sample_pack(ctx, scheme, p, dtype):
    big = _both(ctx, 1024, 4096, scheme, p, dtype, seed=41)
    _same(*big)
    assert big[0][0][-1] > 0
    small = _both(ctx, 70, 1000, scheme, p, dtype, seed=42)      # ragged width, fewer rows: stale words lie beyond it
    _same(*small)
    assert small[0][0][-1] > 0


def test_largest_input_that_fits(ctx):
    """4096 x 4096 elements fill the 2 MiB array exactly."""
    from paper_2007_10412_amd import binding as B
    a, b = _both(ctx, 4096, 4096, B.RAD_FIXEDK_PER_EXAMPLE, 0.02, B.RAD_BF16, seed=43)
    _same(a, b)
    _same(*_both(ctx, 33, 96, B.RAD_BERNOULLI, 0.5, B.RAD_F32, seed=44))


def test_sizes_beyond_the_static_array_are_refused(ctx):
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev
    rows, cols = 4097, 4096
    L = B.make_layer(rows, cols, 8, dtype=B.RAD_BF16, relu=False)
    st = B.rad_store_create(ctx, L, B.RAD_BERNOULLI, 0.1)
    try:
        x = dev(np.zeros((rows, cols), dtype=np.float32), B.RAD_BF16)
        with pytest.raises(B.RadError) as e:
            B.rad_sample_pack_static(ctx, B.make_sampling(B.RAD_BERNOULLI, 0.1, 1), x, st)
        assert e.value.status == B.RAD_ERR_CAPACITY and "static scratch" in str(e.value)
    finally:
        B.rad_store_destroy(st)
    L = B.make_layer(64, 256, 8, dtype=B.RAD_BF16, relu=False)
    st = B.rad_store_create(ctx, L, B.RAD_PROJECT_SHARED, 0.1)
    try:
        x = dev(np.zeros((64, 256), dtype=np.float32), B.RAD_BF16)
        with pytest.raises(B.RadError) as e:
            B.rad_sample_pack_static(ctx, B.make_sampling(B.RAD_PROJECT_SHARED, 0.1, 1), x, st)
        assert e.value.status == B.RAD_ERR_UNSUPPORTED
    finally:
        B.rad_store_destroy(st)
