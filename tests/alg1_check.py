"""Comparison of an Algorithm-1 output with the oracle (shared by the GPU tests; not a test itself).

A coordinate passes if the output is the oracle's within 1e-5 of the conditioning scale; or, where
the oracle's decision margin is below the rounding noise of an fp32 evaluation of the multi-Krum
averages (4e-6 of the scale), the runner-up's; or, for the few coordinates where more than two
averages are nearly equidistant from the median, any choice the oracle's plain per-coordinate check
accepts (oracle.alg1_accepts).  Returns how many coordinates passed only through the second or third
door: the count the tests bound."""
import numpy as np

import oracle as O


def compare(got, G, ext, sets, beta, what=""):
    got = np.asarray(got)
    ref, scale, margin, alt = O.coordwise_alg1(G, ext, sets, beta, want_extra=True)
    tol = 1e-5 * np.maximum(np.abs(ref), scale) + 1e-37
    ok = np.abs(got - ref) <= tol
    ok_alt = (margin <= 4e-6 * scale) & (np.abs(got - alt) <= 1e-5 * np.maximum(np.abs(alt), scale) + 1e-37)
    rest = np.flatnonzero(~(ok | ok_alt))
    assert rest.size <= 64, f"{what}: {rest.size} coordinates differ beyond a runner-up choice"
    for c in rest:
        assert O.alg1_accepts(G[:, c], ext, sets, beta, got[c]), (
            f"{what}: coordinate {int(c)}: got {got[c]!r}, oracle {ref[c]!r}, runner-up {alt[c]!r}, margin {margin[c]!r}")
    worst = float(np.max(np.where(ok, np.abs(got - ref) / tol, 0.0))) if got.size else 0.0
    return int(np.sum(~ok)), worst
