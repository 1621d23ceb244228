"""The input generators: explicit harmonics agree with the oracle's general definition,
graphs have the requested shape, everything is reproducible from the seed."""
import numpy as np

from oracle import so3
from paper_2501_13986_amd import synth


def test_sh_edge_attr_matches_oracle_definition():
    v = synth.unit_vectors(3, 200)
    assert np.abs(np.linalg.norm(v, axis=1) - 1).max() < 1e-14
    for lmax in range(4):
        assert np.abs(synth.sh_edge_attr(v, lmax) - so3.real_sh_all(lmax, v)).max() < 1e-12


def test_periodic_graph_shape_and_symmetry():
    recv, send, unit = synth.periodic_graph(7, 2000, 32.0)
    E = recv.shape[0]
    assert abs(E / 2000 - 32.0) < 1.5
    assert np.all(recv != send)
    assert np.abs(np.linalg.norm(unit, axis=1) - 1).max() < 1e-12
    fwd = set(zip(recv.tolist(), send.tolist()))
    assert len(fwd) == E                                     # no duplicate edges
    assert all((s, r) in fwd for r, s in list(fwd)[:500])    # both directions present
    r2, s2, u2 = synth.periodic_graph(7, 2000, 32.0)
    assert np.array_equal(recv, r2) and np.array_equal(send, s2) and np.array_equal(unit, u2)


def test_normal_reproducible():
    a, b = synth.normal(4, (5, 3)), synth.normal(4, (5, 3))
    assert np.array_equal(a, b) and a.dtype == np.float64
