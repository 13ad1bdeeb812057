"""The library's host-side layer-range profiler (rc_layer_profile) against the oracle's; no GPU needed."""
import numpy as np
import pytest

from oracle import relay_oracle as R
from paper_2603_13289_amd import binding as rc


def _cases():
    rng = np.random.default_rng(11)
    out = []
    for L, n in ((12, 40), (32, 500), (64, 77), (5, 3), (2, 1)):
        depth = np.arange(L) / max(L - 1, 1)
        s = 1.0 - 0.2 * np.exp(-((depth - 0.45) / 0.18) ** 2) - 0.03 * depth      # U shape, partial recovery
        base = rng.random(n)
        share = 1.0 - np.exp(-0.4 * np.arange(L))
        pattern = np.stack([share[l] * base + (1 - share[l]) * rng.random(n) for l in range(L)], axis=1)
        d = (1.0 - s)[None, :] * (0.5 + pattern)
        out.append(d.astype(np.float32))
    ties = np.round(out[1], 2)            # many equal deviations
    out.append(ties.astype(np.float32))
    return out


@pytest.mark.parametrize("idx", range(6))
@pytest.mark.parametrize("params", [(0.99, 5, 2.0, 2), (0.97, 3, 1.0, 3), (0.5, 8, 4.0, 1)])
def test_layer_profile_matches_oracle(idx, params):
    d = _cases()[idx]                              # [n][L] float32
    tau, tail, lam, cons = params
    want = R.profile_layers(d.astype(np.float64), tau_st=float(np.float32(tau)), tail=tail, lam=float(np.float32(lam)),
                            consecutive=cons)
    (l_start, l_det, l_end), s, rho = rc.rc_layer_profile(d.T, tau, tail, lam, cons)
    assert np.allclose(s, want.s, atol=1e-12) and np.allclose(rho, want.rho, atol=1e-12)
    assert (l_start, l_det, l_end) == (want.l_start, want.l_det, want.l_end)
    assert 0 <= l_start and l_start <= l_end < d.shape[1] and l_det <= l_end


def test_layer_profile_hand_worked_detection_layer():
    """The library's profiler on rankings written out by hand: rho, the first positive-to-negative change of the
    second difference at l* = 5 and l_det = l* + 1 = 6 are typed-in numbers (tests/hand_profiles.py)."""
    from tests import hand_profiles as H
    (l_start, l_det, l_end), s, rho = rc.rc_layer_profile(H.deviations().T.astype(np.float32))
    assert (l_start, l_det, l_end) == H.TRIPLE == (2, 6, 8)
    assert np.allclose(rho, H.RHO, atol=1e-12) and np.allclose(s, H.S, atol=1e-6)
    flat = rc.rc_layer_profile(H.deviations(ranks=[H.RANKS[0]] + [H.RANKS[5]] * 11).T.astype(np.float32))[0]
    assert flat == (2, 3, 8)


def test_layer_profile_argument_errors():
    d = np.zeros((3, 4), np.float32)
    for bad in (dict(tail=0), dict(consecutive=0), dict(lam=-1.0)):
        with pytest.raises(rc.RcError) as e:
            rc.rc_layer_profile(d, **bad)
        assert e.value.status == rc.RC_E_INVALID_ARG
    with pytest.raises(rc.RcError) as e:
        rc.rc_layer_profile(np.zeros((1, 4), np.float32))
    assert e.value.status == rc.RC_E_INVALID_ARG
    with pytest.raises(rc.RcError) as e:
        rc.rc_layer_profile(np.zeros((200, 4), np.float32))
    assert e.value.status == rc.RC_E_CAPACITY
