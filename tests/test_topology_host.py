"""Host side of the comparison-topology rounds: ceca_topology_round against the oracle's definitions
and the argument checks of ceca_mix_rounds (nothing here touches a device)."""
import ctypes

import numpy as np
import pytest

from oracle import topologies as OT


@pytest.fixture(scope="module")
def api():
    import paper_2306_00256_amd as P
    P.lib()
    return P


def _as_tuple(m):
    return tuple(m.shift[: m.m]), tuple(m.w[: m.m]), m.w_self


@pytest.mark.parametrize("n", [1, 2, 3, 5, 6, 8, 31, 100, 130, 258, 1026, 4096, 65536])
def test_rounds_match_the_definitions(api, n):
    from paper_2306_00256_amd import binding as Bn
    tau = OT.num_rounds(n)
    cases = [(Bn.TOPO_RING, 0, OT.ring(n)), (Bn.TOPO_STATIC_EXP, 5, OT.static_exponential(n))]
    cases += [(Bn.TOPO_ONE_PEER_EXP, k, OT.one_peer_exponential(n, k)) for k in range(2 * tau + 1)]
    for kind, k, want in cases:
        shifts, w, w_self = _as_tuple(api.ceca_topology_round(kind, n, k))
        assert shifts == want.shifts, (kind, n, k)
        assert w == tuple(np.float32(x) for x in want.weights)
        # the rounded weights sum to one exactly (in real arithmetic) and w_self is the exact weight rounded
        assert float(np.float64(w_self) + sum(np.float64(x) for x in w)) == 1.0
        assert abs(w_self - want.w_self) <= 2e-7


def test_host_errors(api):
    from paper_2306_00256_amd import binding as Bn
    L = api.lib()
    for kind, n, k in [(7, 4, 0), (Bn.TOPO_RING, 0, 0), (Bn.TOPO_RING, 4, -1), (Bn.TOPO_STATIC_EXP, 1 << 20, 0)]:
        with pytest.raises(api.CecaError) as e:
            api.ceca_topology_round(kind, n, k)
        assert e.value.code == Bn.CECA_EINVAL
    buf = (ctypes.c_float * 256)()
    p = ctypes.addressof(buf)
    ok = api.ceca_topology_round(Bn.TOPO_RING, 4, 0)
    spec = (Bn.Mix * 1)(ok)
    call = lambda *a: L.ceca_mix_rounds(*a)
    assert call(None, p, 4, 8, 8, spec, 1, 0, 1, None) == Bn.CECA_EINVAL
    assert call(p, p, 4, 8, 8, None, 1, 0, 1, None) == Bn.CECA_EINVAL
    assert call(p, p, 5000, 8, 8, spec, 1, 0, 1, None) == Bn.CECA_EINVAL          # more than 4096 agents
    assert call(p, p, 4, 8, 4, spec, 1, 0, 1, None) == Bn.CECA_EINVAL             # ld < d
    assert call(p, p, 4, 8, 8, spec, 0, 0, 1, None) == Bn.CECA_EINVAL             # empty period
    assert call(p, p, 4, 8, 8, spec, 17, 0, 1, None) == Bn.CECA_EINVAL
    assert call(p, p, 4, 8, 8, spec, 1, 0, 0, None) == Bn.CECA_EINVAL             # no rounds
    assert call(p, p + 32, 4, 8, 8, spec, 1, 0, 1, None) == Bn.CECA_EINVAL        # partial overlap
    bad = Bn.Mix(); bad.m = 1; bad.shift[0] = 4; bad.w[0] = 0.5; bad.w_self = 0.5
    assert call(p, p, 4, 8, 8, (Bn.Mix * 1)(bad), 1, 0, 1, None) == Bn.CECA_EINVAL   # shift outside [0, n)
    bad.m = 17
    assert call(p, p, 4, 8, 8, (Bn.Mix * 1)(bad), 1, 0, 1, None) == Bn.CECA_EINVAL
    many = api.ceca_topology_round(Bn.TOPO_STATIC_EXP, 4096, 0)                    # 12 peers per round
    assert call(p, p, 4096, 8, 8, (Bn.Mix * 6)(*([many] * 6)), 6, 0, 1, None) == Bn.CECA_EINVAL   # 72 peers over the period
