"""The measurement helpers and the state-tile conversions move bytes only: bit-exact checks."""
import numpy as np
import pytest
import torch

from paper_2604_19877_amd import binding as sa
from gpu_util import Guarded

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_bytes", [16, 4096, 65536, 65536 + 48, 5 * 65536, 7 * 65536 + 16 * 1000 + 16])
def test_copy_bytes_is_exact_and_stays_in_bounds(n_bytes):
    rng = np.random.default_rng(n_bytes)
    src = rng.integers(0, 256, n_bytes, dtype=np.uint8)
    gs, gd = Guarded(src), Guarded(np.zeros(n_bytes, dtype=np.uint8))
    sa.sa_copy_bytes(gs.ptr(), gd.ptr(), n_bytes)
    torch.cuda.synchronize()
    assert np.array_equal(gd.read(), src) and np.array_equal(gs.read(), src)
    assert gs.bands_intact() and gd.bands_intact()


def test_copy_bytes_rejects_bad_arguments():
    t = torch.zeros(64, dtype=torch.uint8, device="cuda")
    for args in ((None, t, 16), (t, t.data_ptr() + 8, 16), (t, t, 24)):
        with pytest.raises(sa.SaError) as e:
            sa.sa_copy_bytes(*args)
        assert e.value.status == sa.SA_EINVAL
    sa.sa_copy_bytes(t, t, 0)


@pytest.mark.parametrize("dk", [64, 128])
def test_state_pack_and_unpack_round_trip(dk):
    n_tiles = 5
    rng = np.random.default_rng(dk)
    tiles = rng.standard_normal((n_tiles, dk, dk)).astype(np.float32)
    a, b, c = Guarded(tiles), Guarded(np.zeros_like(tiles)), Guarded(np.zeros_like(tiles))
    assert sa.sa_state_tile_bytes(dk, dk) == dk * dk * 4
    sa.sa_state_pack(a.ptr(), b.ptr(), n_tiles, dk, dk)
    sa.sa_state_unpack(b.ptr(), c.ptr(), n_tiles, dk, dk)
    torch.cuda.synchronize()
    assert np.array_equal(c.read(), tiles) and a.bands_intact() and b.bands_intact() and c.bands_intact()


@pytest.mark.parametrize("kind", [0, 1, 2])
def test_stream_tiles_touches_its_tiles_only(kind):
    n_tiles = 6
    rng = np.random.default_rng(kind)
    tiles = rng.standard_normal((n_tiles, 128, 128)).astype(np.float32)
    g = Guarded(tiles)
    sa.sa_stream_tiles(kind, g.ptr(), n_tiles)
    torch.cuda.synchronize()
    got = g.read()
    assert g.bands_intact()
    if kind == 0:
        assert np.array_equal(got, tiles)
    elif kind == 1:
        assert (got == got.flat[0]).all()
    else:
        np.testing.assert_allclose(got, tiles * np.float32(0.999), rtol=1e-6)
