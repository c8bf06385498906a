"""The inequality behind abandoning a transport problem early (CPU only).

The device solver (successive shortest paths with potentials, sources served in turn) drops a pair of the pruned
search once  cost of the flow so far + supply left of the current source x max(its search distances so far, its
cheapest edge) + sum over sources not yet served of weight x cheapest edge  exceeds the cut-off.  That expression is
the value of a feasible point of the dual programme, so it can never exceed the optimum.  Here a serial model of that
search, written for this test alone, evaluates the expression after every search on random problems (with exact
matches, ties and uniform weights) and holds it against its own optimum and against the LP oracle."""
import numpy as np

import oracle

FAR, EPS = 1e300, 1e-13


def solve_with_bounds(a, b, c):
    h1, h2 = c.shape
    sup, dem = a / a.sum(), b / b.sum()
    x1 = sup.copy()
    phiS, phiT, f, total = np.zeros(h1), np.zeros(h2), np.zeros((h2, h1)), 0.0
    cheapest = c.min(axis=1)
    tail = float(x1 @ cheapest)
    seen = [tail]
    for s in range(h1):
        tail = max(tail - x1[s] * cheapest[s], 0.0)
        paid = 0.0
        while sup[s] > EPS:
            dT = np.maximum(c[s] + phiS[s] - phiT, 0)
            used, vis = np.zeros(h2, bool), np.zeros(h1, bool)
            way, par, dS = np.full(h2, s), np.full(h1, -1), np.zeros(h1)
            vis[s] = True
            Dt = None
            for _ in range(h2):
                cand = np.where(~used, dT, FAR)
                u = int(np.argmin(cand))
                bv = cand[u]
                if bv >= FAR:
                    break
                used[u] = True
                if dem[u] > 0:
                    Dt = bv
                    delta, p = min(sup[s], dem[u]), way[u]
                    while par[p] >= 0:
                        delta = min(delta, f[par[p], p])
                        p = way[par[p]]
                    total += delta * (bv - phiS[s] + phiT[u])
                    uu, p, emptied = u, way[u], False
                    while True:
                        f[uu, p] += delta
                        up = par[p]
                        if up < 0:
                            break
                        left = f[up, p] - delta
                        f[up, p] = left if left > EPS else 0.0
                        emptied |= left <= EPS
                        uu, p = up, way[up]
                    sup[s] = sup[s] - delta if sup[s] - delta > EPS else 0.0
                    dem[u] = dem[u] - delta if dem[u] - delta > EPS else 0.0
                    if sup[s] == 0 or emptied or dem[u] > 0:
                        break
                for p in range(h1):
                    if f[u, p] > 0 and not vis[p]:
                        vis[p], dS[p], par[p] = True, bv, u
                        nd = bv + np.maximum(c[p] + phiS[p] - phiT, 0)
                        better = ~used & (nd < dT)
                        dT[better], way[better] = nd[better], p
            if Dt is None:
                sup[s] = 0
                break
            mS, mT = vis & (dS < Dt), used & (dT < Dt)
            phiS[mS] += dS[mS] - Dt
            phiT[mT] += dT[mT] - Dt
            paid += Dt
            seen.append(total + sup[s] * max(paid, cheapest[s]) + tail)
    return total, seen


def test_the_bound_never_exceeds_the_optimum_and_ends_on_it():
    rng = np.random.default_rng(5)
    for trial in range(150):
        h1, h2, m = int(rng.integers(1, 14)), int(rng.integers(1, 14)), int(rng.integers(1, 5))
        X, Y = rng.standard_normal((h1, m)), rng.standard_normal((h2, m))
        if trial % 3 == 0:
            same = min(h1, h2, 3)
            Y[:same] = X[:same]                         # words the two histograms share
        if trial % 5 == 0:
            X, Y = np.round(X), np.round(Y)             # many equal distances
        c = np.sqrt(((X[:, None, :] - Y[None, :, :]) ** 2).sum(2))
        a, b = rng.random(h1) + 0.01, rng.random(h2) + 0.01
        if trial % 7 == 0:
            a, b = np.ones(h1), np.ones(h2)
        total, seen = solve_with_bounds(a, b, c)
        assert abs(total - oracle.emd(a, b, c)) <= 1e-7 * max(total, 1e-3)          # the model solves the programme
        assert max(seen) <= total + 1e-12 * max(total, 1e-3)                         # never above the optimum
        assert abs(seen[-1] - total) <= 1e-12 * max(total, 1e-3)                     # and tight at the end
        row_min_bound = float((a / a.sum()) @ c.min(axis=1))
        assert abs(seen[0] - row_min_bound) < 1e-12                                  # starts at the one-sided RWMD
