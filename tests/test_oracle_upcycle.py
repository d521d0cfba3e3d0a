"""Pins for the oracle's upcycling initialiser and the pack / unpack of trained experts."""
import numpy as np
from scipy import stats

from oracle import spes_oracle as O


def test_philox_matches_library_generator():
    """numpy's Philox is the same 4x64-10 function; it advances its counter before producing a block."""
    for counter, key in [((0, 0, 0, 0), (0, 0)), ((5, 7, 0, 0), (1234, 0)), ((2**64 - 2, 3, 9, 1), (2**63 + 11, 77))]:
        raw = [int(v) for v in np.random.Philox(counter=np.array(counter, dtype=np.uint64), key=np.array(key, dtype=np.uint64)).random_raw(4)]
        nxt = ((counter[0] + 1) % 2**64, counter[1] + ((counter[0] + 1) >> 64), counter[2], counter[3])
        assert raw == list(O.philox4x64(nxt, key))


def test_draws_are_uniform_bytes_and_standard_normals():
    sel, z = [], []
    for g in range(20000):
        s, n = O.upcycle_draws(g, seed=99, stream_id=3)
        sel += s; z += n
    sel, z = np.array(sel), np.array(z)
    assert sel.min() >= 0 and sel.max() <= 255
    frac = (sel < 128).mean()
    assert abs(frac - 0.5) < 4 * 0.5 / np.sqrt(sel.size)
    assert stats.kstest(z, "norm").pvalue > 1e-3
    assert abs(z.mean()) < 4 / np.sqrt(z.size) and abs(z.std() - 1.0) < 0.02
    # selection and value are independent draws: the selected half is as normal as the rest
    assert stats.kstest(z[sel < 128], "norm").pvalue > 1e-3
    # Box-Muller pairs: r^2 = z0^2 + z1^2 is exponential with mean 2
    r2 = z[0::2] ** 2 + z[1::2] ** 2
    assert stats.kstest(r2, "expon", args=(0, 2)).pvalue > 1e-3


def test_upcycle_init_structure():
    rng = np.random.default_rng(0)
    dense = rng.normal(size=256) * 0.02
    out = O.upcycle_init(dense, 6, 0.5, 0.02, seed=7)
    changed = out != dense[None, :]
    assert abs(changed.mean() - 0.5) < 0.06                      # half of the parameters receive noise
    np.testing.assert_array_equal(out[~changed], np.broadcast_to(dense, out.shape)[~changed])
    noise = (out - dense[None, :])[changed]
    assert abs(noise.std() - 0.02) < 0.003 and abs(noise.mean()) < 0.003
    assert not np.array_equal(out[0], out[1])                    # experts get different draws
    np.testing.assert_array_equal(out, O.upcycle_init(dense, 6, 0.5, 0.02, seed=7))
    assert not np.array_equal(out, O.upcycle_init(dense, 6, 0.5, 0.02, seed=8))
    assert not np.array_equal(out, O.upcycle_init(dense, 6, 0.5, 0.02, seed=7, stream_id=1))
    np.testing.assert_array_equal(O.upcycle_init(dense, 3, 0.0, 0.02, seed=7), np.broadcast_to(dense, (3, 256)))
    allp = O.upcycle_init(dense, 3, 1.0, 0.02, seed=7)
    assert (allp != dense[None, :]).all()
    # the noise of the selected entries does not depend on the fraction
    sel = out[:3] != dense[None, :]
    np.testing.assert_array_equal(allp[sel], out[:3][sel])


def test_pack_unpack_round_trip():
    rng = np.random.default_rng(1)
    store = rng.normal(size=(7, 12))
    tr = [1, 4, 6]
    packed = O.pack_experts(store, tr)
    np.testing.assert_array_equal(packed, store[[1, 4, 6]])
    new = rng.normal(size=packed.shape)
    out = O.unpack_experts(store, tr, new)
    np.testing.assert_array_equal(out[tr], new)
    rest = [e for e in range(7) if e not in tr]
    np.testing.assert_array_equal(out[rest], store[rest])
    np.testing.assert_array_equal(O.unpack_experts(store, tr, packed), store)
