"""Validity of an extracted list on given distances (shared by the GPU tests; not a test itself)."""
import numpy as np

import oracle as O


def replay(D, f, sel, sets, tau):
    """Validity of an extracted list (and, if given, of the averaged sets) on the distances D.
    Returns the smallest relative gap the oracle itself saw at a decision (winner / runner-up, and
    with sets the q-th / (q+1)-th score)."""
    n = D.shape[0]
    active = np.ones(n, np.uint8)
    clear = np.inf
    for t, w in enumerate(sel):
        assert active[w], f"round {t}: gradient {w} extracted twice"
        S = O.krum_scores(D, f, active)
        k = int(active.sum())
        q = max(k - f - 2, 0)
        order = sorted(np.flatnonzero(active), key=lambda i: (S[i], i))
        best = S[order[0]]
        assert S[w] <= best + tau * max(best, 1e-300), f"round {t}: winner {w} has score {S[w]}, best {best}"
        # (scores that tie exactly - no neighbours left, or two gradients that are each other's only
        # neighbour - tie on both sides and go to the smaller index on both)
        if len(order) > 1 and S[order[1]] != best:
            clear = min(clear, (S[order[1]] - best) / max(S[order[1]], 1e-300))
        if sets is not None:
            members = np.flatnonzero(sets[t])
            assert len(members) == min(q, k) and all(active[i] for i in members)
            if 0 < q < k:
                worst_in = max(S[i] for i in members)
                others = [S[i] for i in order if i not in set(members.tolist())]
                assert worst_in <= min(others) + tau * max(worst_in, 1e-300), f"round {t}: averaged set"
                if S[order[q]] != S[order[q - 1]]:
                    clear = min(clear, (S[order[q]] - S[order[q - 1]]) / max(S[order[q]], 1e-300))
        active[w] = 0
    return clear
