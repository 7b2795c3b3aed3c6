"""Pack / unpack of halo rows against oracle/partition_oracle.py: bit-exact in both payload precisions."""
import numpy as np
import pytest

from oracle import partition_oracle as P
from paper_2507_03840_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2507_03840_amd import binding
    binding.load_library()
    return binding


@pytest.mark.parametrize("lmax,E,n,n_idx", [(0, 8, 10, 7), (2, 16, 100, 333), (4, 32, 500, 257), (4, 64, 50, 50), (3, 128, 20, 5)])
@pytest.mark.parametrize("half", [False, True])
def test_pack_unpack_bit_exact(B, lmax, E, n, n_idx, half):
    import torch
    rng = np.random.default_rng([21, lmax, E])
    x = synth.node_features(rng, n, lmax, E)
    idx = rng.integers(0, n, n_idx).astype(np.int32)
    m = B.Egnn(lmax, E, 6, 4.0, 1.0)
    buf = m.egnn_pack_rows(B.to_device(x), B.to_device(idx), half=half)
    ref = P.pack_rows(x, idx, np.float16 if half else np.float32)
    got = buf.cpu().numpy()
    assert got.dtype == ref.dtype and np.array_equal(got.view(np.uint16 if half else np.uint32), ref.view(np.uint16 if half else np.uint32))
    n_owned = 13
    full = synth.node_features(rng, n_owned + n_idx, lmax, E)
    out = m.egnn_unpack_rows(buf, B.to_device(full), n_owned).cpu().numpy()
    assert np.array_equal(out, P.unpack_rows(full, n_owned, ref))


def test_pack_rows_empty_and_out_of_range_indices(B):
    import torch
    m = B.Egnn(1, 8, 6, 4.0, 1.0)
    x = B.to_device(synth.node_features(np.random.default_rng(0), 6, 1, 8))
    assert m.egnn_pack_rows(x, torch.zeros(0, dtype=torch.int32, device="cuda")).shape[0] == 0
    got = m.egnn_pack_rows(x, torch.tensor([-5, 99], dtype=torch.int32, device="cuda")).cpu().numpy()   # clamped
    assert np.array_equal(got[0], x.cpu().numpy()[0]) and np.array_equal(got[1], x.cpu().numpy()[5])
