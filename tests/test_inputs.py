"""The seeded input generator: a pure function of (seed, tensor ordinal, index)."""
import numpy as np
import pytest

from paper_2203_08069_amd import inputs


def test_slices_agree_with_whole():
    whole = inputs.tensor(2, 0, (70000,), np.float32)
    for start, count in [(0, 10), (65530, 100), (69999, 1), (123, 0)]:
        assert np.array_equal(inputs.values(2, 0, start, count, np.float32), whole[start:start + count])


def test_threads_and_chunking_do_not_change_values():
    a = inputs.tensor(3, 1, (3, 5, 20011), np.float64, threads=1)
    b = inputs.tensor(3, 1, (3, 5, 20011), np.float64, threads=4)
    assert np.array_equal(a, b)
    pieces = [c.copy() for _, c in inputs.chunks(3, 1, a.size, np.float64, chunk_elems=7777)]
    assert np.array_equal(np.concatenate(pieces), a.ravel())


def test_streams_differ_by_seed_and_ordinal():
    base = inputs.values(0, 0, 0, 1000, np.float64)
    assert not np.array_equal(base, inputs.values(1, 0, 0, 1000, np.float64))
    assert not np.array_equal(base, inputs.values(0, 1, 0, 1000, np.float64))
    assert abs(np.corrcoef(base, inputs.values(0, 1, 0, 1000, np.float64))[0, 1]) < 0.15


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_uniform_range_and_moments(dtype):
    x = inputs.values(7, 0, 0, 1 << 18, dtype).astype(np.float64)
    assert x.min() >= -1.0 and x.max() <= 1.0
    assert abs(x.mean()) < 0.01
    assert abs(x.var() - 1.0 / 3.0) < 0.01


def test_float32_is_rounded_float64():
    a = inputs.values(5, 2, 100, 4096, np.float64)
    b = inputs.values(5, 2, 100, 4096, np.float32)
    assert np.array_equal(a.astype(np.float32), b)


@pytest.mark.parametrize("r", [1, 2, 3])
def test_small_integers(r):
    x = inputs.values(9, 0, 0, 1 << 16, np.float32, inputs.SMALLINT, r)
    assert np.array_equal(x, np.round(x))
    assert set(np.unique(x).tolist()) == set(float(v) for v in range(-r, r + 1))
    assert abs(x.mean()) < 0.05


def test_pinned_first_words():
    # SplitMix64 with state 0 yields 0xE220A8397B1DCDAF as its first output
    # (reference value of the published generator): checks the mixer constants.
    assert inputs._mix_scalar(0x9E3779B97F4A7C15) == 0xE220A8397B1DCDAF
    key = inputs.stream_key(0, 0)
    w = inputs.raw_bits(0, 0, 0, 3)
    for n in range(3):
        assert int(w[n]) == inputs._mix_scalar(key + (n + 1) * 0x9E3779B97F4A7C15)


def test_bad_arguments():
    with pytest.raises(ValueError):
        inputs.values(0, 0, 0, 4, np.int32)
    with pytest.raises(ValueError):
        inputs.values(0, 0, -1, 4, np.float32)
    with pytest.raises(ValueError):
        inputs.values(0, 0, 0, 4, np.float32, "gauss")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("kind", [inputs.UNIFORM, inputs.SMALLINT])
def test_torch_generator_reproduces_the_numpy_one(dtype, kind):
    """The torch-integer form of the generator (used to fill device tensors in place) must give
    the same bytes as the numpy one, across chunk boundaries and for large indices."""
    from paper_2203_08069_amd import device_inputs
    got = device_inputs.generate_on_device(4, 2, (3, 7, 1001), dtype, kind, device="cpu", chunk_elems=5000).numpy()
    assert np.array_equal(got, inputs.tensor(4, 2, (3, 7, 1001), dtype, kind))
    big = device_inputs.generate_on_device(9, 0, (1 << 16,), dtype, kind, r=2, device="cpu").numpy()
    assert np.array_equal(big, inputs.values(9, 0, 0, 1 << 16, dtype, kind, 2))
