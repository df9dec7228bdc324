"""GPU parity of the sampler: keep sets, indices and stored values must equal
the oracle's bit for bit (they depend on the seed only, never on tiling)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import rad_oracle as R


@pytest.fixture(scope="module")
def ctx():
    from paper_2007_10412_amd import binding as B
    c = B.rad_ctx_create()
    yield c
    B.rad_ctx_destroy(c)


def _check_pack(ctx, rows, cols, scheme, p, seed, stream_id, step, dtype, rng):
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev
    from paper_2007_10412_amd.synth import bf16_round
    x = rng.standard_normal((rows, cols)).astype(np.float32)
    if dtype == B.RAD_BF16:
        x = bf16_round(x)
    print("case rows=%d cols=%d scheme=%d p=%g seed=%d dtype=%d" % (rows, cols, scheme, p, seed, dtype), flush=True)
    L = B.make_layer(rows, cols, 8, dtype=dtype, relu=False)
    st = B.rad_store_create(ctx, L, scheme, p)
    try:
        B.rad_sample_pack(ctx, B.make_sampling(scheme, p, seed, stream_id, step), dev(x, dtype), st)
        rp, col, val = B.rad_store_export_csr(ctx, st, rows)
        orp, ocol, oval, _ = R.sample_pack(x, scheme, p, seed, stream_id, step, dtype)
        assert np.array_equal(rp, orp)
        assert np.array_equal(col, ocol)
        assert np.array_equal(val.view(np.uint32), oval.view(np.uint32))     # one fp32 multiply, one rounding
        stats = B.rad_store_get_stats(ctx, st)
        es = 2 if dtype == B.RAD_BF16 else 4
        assert stats["nnz"] == orp[-1] and stats["value_bytes"] == orp[-1] * es
        assert stats["dense_bytes"] == rows * cols * es
    finally:
        B.rad_store_destroy(st)


@pytest.mark.parametrize("scheme", [1, 2, 3])
@pytest.mark.parametrize("rows,cols,p", [
    (150, 784, 0.1),        # config 1/2 first layer
    (150, 300, 0.1),        # k = 30
    (33, 37, 0.3),          # rows start inside a Philox quad (cols % 4 != 0), one ragged bucket
    (5, 1, 0.1),            # one column: k = 1
    (3, 1030, 0.5),         # five buckets with a ragged tail
    (64, 4096, 0.02),       # config 4 width
    (2, 16376, 0.1),        # widest fixed-k row
    (7, 300, 1.0),          # fraction one keeps everything
])
def test_pack_equals_oracle_f32(ctx, scheme, rows, cols, p):
    from paper_2007_10412_amd import binding as B
    rng = np.random.default_rng(rows * 1000 + cols)
    _check_pack(ctx, rows, cols, scheme, p, seed=77 + rows, stream_id=3, step=5, dtype=B.RAD_F32, rng=rng)


@pytest.mark.parametrize("scheme", [1, 2, 3])
def test_pack_equals_oracle_bf16(ctx, scheme):
    from paper_2007_10412_amd import binding as B
    rng = np.random.default_rng(5)
    _check_pack(ctx, 96, 4096, scheme, 0.1, seed=(1 << 40) + 9, stream_id=1, step=0, dtype=B.RAD_BF16, rng=rng)


def test_bernoulli_wide_row(ctx):
    from paper_2007_10412_amd import binding as B
    rng = np.random.default_rng(6)
    _check_pack(ctx, 3, 65535, B.RAD_BERNOULLI, 0.1, seed=4, stream_id=0, step=0, dtype=B.RAD_F32, rng=rng)


def test_exact_scheme_stores_everything(ctx):
    from paper_2007_10412_amd import binding as B
    rng = np.random.default_rng(7)
    _check_pack(ctx, 9, 50, B.RAD_EXACT, 1.0, seed=0, stream_id=0, step=0, dtype=B.RAD_F32, rng=rng)


@pytest.mark.parametrize("scheme", [2, 3])
def test_fixed_k_tie_rule(ctx, scheme):
    """Keys cut down to 6 bits collide constantly; ties at the cut must go to the lower column."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev
    rows, cols, p, seed, shift = 40, 1000, 0.1, 11, 26
    x = np.ones((rows, cols), dtype=np.float32)
    L = B.make_layer(rows, cols, 8, relu=False)
    st = B.rad_store_create(ctx, L, scheme, p)
    B.rad_debug_key_shift(ctx, shift)
    try:
        B.rad_sample_pack(ctx, B.make_sampling(scheme, p, seed, 2, 1), dev(x), st)
        rp, col, val = B.rad_store_export_csr(ctx, st, rows)
    finally:
        B.rad_debug_key_shift(ctx, 0)
        B.rad_store_destroy(st)
    k = R.fixed_k(p, cols)
    n_rows = 1 if scheme == 2 else rows
    keys = R.element_keys(seed, 2, 1, 0, n_rows * cols).reshape(n_rows, cols) >> np.uint32(shift)
    for b in range(rows):
        kr = keys[0 if scheme == 2 else b]
        want = np.sort(np.argsort(kr, kind="stable")[:k])
        assert np.array_equal(col[rp[b]:rp[b + 1]], want), b


def test_bad_arguments_are_status_codes(ctx):
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev
    L = B.make_layer(4, 16, 8)
    for bad_p in (0.0, -0.1, 1.5, float("nan")):
        with pytest.raises(B.RadError) as e:
            B.rad_store_create(ctx, L, B.RAD_BERNOULLI, bad_p)
        assert e.value.status == B.RAD_ERR_PARAM
    with pytest.raises(B.RadError) as e:
        B.rad_store_create(ctx, L, 9, 0.5)
    assert e.value.status == B.RAD_ERR_PARAM
    with pytest.raises(B.RadError) as e:
        B.rad_store_create(ctx, B.make_layer(0, 16, 8), B.RAD_BERNOULLI, 0.5)
    assert e.value.status == B.RAD_ERR_SHAPE
    with pytest.raises(B.RadError) as e:
        B.rad_store_create(ctx, B.make_layer(4, 70000, 8), B.RAD_BERNOULLI, 0.5)
    assert e.value.status == B.RAD_ERR_UNSUPPORTED
    st = B.rad_store_create(ctx, L, B.RAD_BERNOULLI, 0.5)
    try:
        with pytest.raises(B.RadError) as e:      # sampling must match the store
            B.rad_sample_pack(ctx, B.make_sampling(B.RAD_BERNOULLI, 0.25, 1), dev(np.zeros((4, 16), np.float32)), st)
        assert e.value.status == B.RAD_ERR_PARAM
        with pytest.raises(B.RadError) as e:
            B.rad_sample_pack(ctx, B.make_sampling(B.RAD_BERNOULLI, 0.5, 1), None, st)
        assert e.value.status == B.RAD_ERR_NULL
    finally:
        B.rad_store_destroy(st)
