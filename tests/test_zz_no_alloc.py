"""The allocation-free variant of the stand-alone sampler (staging in a static device array) against the allocating
one: same kernel, same inputs, so the tokens must be identical. Two calls in a row on the same device, the second
smaller than the first (it reuses the front of the array, whose back still holds the first call's rows), then a larger one again."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _case(n, V, seed):
    rng = np.random.default_rng(seed)
    rows = rng.normal(0.0, 1.3, (n, V)).astype(np.float32)
    params = [dict(temperature=0.0 if i % 5 == 4 else 0.8, top_k=[50, 1, 300, 1024][i % 4], top_p=[0.9, 1.0, 0.55][i % 3],
                   seed=int(rng.integers(1, 1 << 62))) for i in range(n)]
    return rows, params, rng.integers(0, 500, n)


def test_static_staging_gives_the_same_tokens_as_allocated_staging(lib):
    for n, V, seed in ((30, 128256, 1), (7, 5000, 2), (31, 128256, 3), (1, 37, 4)):
        rows, params, idx = _case(n, V, seed)
        want = lib.sample_rows(rows, params, idx)
        got = lib.sample_rows_static(rows, params, idx)
        assert np.array_equal(got, want), (n, V, got, want)
        assert np.all((got >= 0) & (got < V))


def test_static_staging_rejects_what_does_not_fit(lib):
    rows, params, idx = _case(33, 128256, 5)          # 33 x 128256 x 4 bytes exceed the 16 MiB array
    with pytest.raises(lib.BlinkError) as ei:
        lib.sample_rows_static(rows, params, idx)
    assert ei.value.code == lib.ERR_TOO_LARGE
    assert "static buffer" in str(ei.value)
