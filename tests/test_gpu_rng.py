"""HIP path vs CPU oracle: Philox words bit-exact, Gaussians within 2 ulp (fp32).
The radius and the cos/sin factors are checked exhaustively over every
uniform the generator can produce."""
import numpy as np
import pytest

from oracle import perturbation as P
from oracle.philox import philox4x32
from tests.util import ulp_diff

pytestmark = pytest.mark.gpu


def test_philox_words_bit_exact_known_answers_and_random():
    from paper_2601_12917_amd.session import debug_philox
    ctr = np.array([[0, 0, 0, 0], [0xFFFFFFFF] * 4, [0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344]], dtype=np.uint32)
    assert debug_philox(ctr[:1], (0, 0))[0].tolist() == [0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8]
    assert debug_philox(ctr[1:2], (0xFFFFFFFF, 0xFFFFFFFF))[0].tolist() == [0x408F276D, 0x41C83B0E, 0xA20BC7C6, 0x6D5451FD]
    assert debug_philox(ctr[2:3], (0xA4093822, 0x299F31D0))[0].tolist() == [0xD16CFE09, 0x94FDCCEB, 0x5001E420, 0x24126EA1]
    rng = np.random.default_rng(0)
    c = rng.integers(0, 2 ** 32, size=(100003, 4), dtype=np.uint64).astype(np.uint32)
    key = (0xDEADBEEF, 0x12345678)
    assert np.array_equal(debug_philox(c, key), philox4x32(c, np.array(key, dtype=np.uint64)))
    assert debug_philox(c[:0], key).shape == (0, 4)


@pytest.mark.parametrize("bits", [32, 16])
def test_radius_exhaustive(bits):
    from paper_2601_12917_amd.session import debug_radius_table
    got = debug_radius_table(bits)
    n = np.arange(got.size, dtype=np.float64)
    u = (n + 0.5) * 2.0 ** (-23 if bits == 32 else -16)
    want = np.sqrt(-2.0 * np.log(u))
    err = np.abs(got.astype(np.float64) - want) / np.spacing(want.astype(np.float32)).astype(np.float64)
    assert err.max() <= 0.51, err.max()


@pytest.mark.parametrize("bits", [32, 16])
def test_cos_sin_exhaustive(bits):
    from paper_2601_12917_amd.session import debug_cossin_table
    c, s = debug_cossin_table(bits)
    v = np.arange(c.size, dtype=np.float64) * 2.0 ** (-24 if bits == 32 else -16)
    wc, ws = P.cos_sin_2pi(v)
    for got, want in ((c, wc), (s, ws)):
        zero = want == 0
        assert np.all(got[zero] == 0)
        assert ulp_diff(got[~zero], want[~zero].astype(np.float32)).max() <= 1.0
        # against the unrounded value: the rounded sum hi + lo is within 0.5 ulp + the hi/lo pair's own error
        rel = np.abs(got[~zero].astype(np.float64) / want[~zero] - 1.0)
        assert rel.max() <= 1.5 * 2.0 ** -24


@pytest.mark.parametrize("bits", [32, 16])
@pytest.mark.parametrize("first,n", [(0, 1 << 20), (5, 1000), (123457, 77), (7, 1), ((1 << 33) + 3, 4099)])
def test_gaussians_within_2_ulp(bits, first, n):
    from paper_2601_12917_amd.session import debug_gauss
    seed, step, tid, stream = (7 << 32) | 42, 9, 1234, 1
    got = debug_gauss(seed, step, tid, stream, bits, first, n)
    want = P.gauss_at(seed, step, tid, stream, np.arange(first, first + n, dtype=np.uint64), bits)
    assert np.all(np.isfinite(got))
    zero = want == 0
    assert np.all(got[zero] == 0)
    err = ulp_diff(got[~zero], want[~zero])
    assert err.max() <= 2.0, err.max()
    if n >= 1 << 20:
        assert np.mean(got == want) > 0.6          # mostly identical to the correctly rounded value


def test_gaussians_many_samples_within_2_ulp():
    from paper_2601_12917_amd.session import debug_gauss
    worst = 0.0
    for chunk in range(8):
        first = chunk * (1 << 40) + 4 * chunk
        got = debug_gauss(99, chunk, 5, 0, 32, first, 1 << 22)
        want = P.gauss_at(99, chunk, 5, 0, np.arange(first, first + (1 << 22), dtype=np.uint64), 32)
        nz = want != 0
        worst = max(worst, ulp_diff(got[nz], want[nz]).max())
    assert worst <= 2.0, worst
