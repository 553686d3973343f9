"""Search for the sparsification recipe (R-Sparse, Sec. 3.5, Algorithm "Search Algorithm for
Sparsification Recipe") -- TEST INFRASTRUCTURE, plain Python, the algorithm's steps in the paper's
order and notation.

rho = (rho_1 .. rho_L), rho_i = share of layer i's budget given to the sparse part.  A population
G of P recipes is improved for T generations: every individual i gets a mutant
m^i = rho^{x1} + p_m (rho^{x2} - rho^{x3}) (x1, x2, x3 drawn from {1..P}), crossed over coordinate-wise
with its parent, rho_hat^i = m^i where alpha > p_c and rho^i where alpha <= p_c (alpha uniform in (0,1)
per coordinate); the next generation is the P lowest-loss members of G u G_hat, S the best of them.
Group-wise strategy (Sec. 3.5): the coordinates are optimised one group at a time, all others held
at the values of the most recent best individual S.

Readings where the paper is silent: x1, x2, x3 are independent draws (they may coincide); recipes are
clamped to [lo, hi] after mutation (rho is a ratio); Top_K keeps K = P and breaks ties by age (older
first) then index; every group starts from a fresh random population in its own coordinates, with S
itself as individual 0 so that the best loss never gets worse; the random numbers are
u_k = (splitmix64(seed, k) >> 11) * 2^-53, consumed in the order written below.
"""
from __future__ import annotations

MASK = (1 << 64) - 1


def _splitmix64(seed: int, k: int) -> int:
    z = (seed + (k + 1) * 0x9E3779B97F4A7C15) & MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
    return z ^ (z >> 31)


class _Uniform:
    def __init__(self, seed: int):
        self.seed, self.k = seed & MASK, 0

    def __call__(self) -> float:
        u = (_splitmix64(self.seed, self.k) >> 11) * (1.0 / 9007199254740992.0)
        self.k += 1
        return u


def search_recipe(loss, n_layers, population=32, generations=5, p_m=0.5, p_c=0.5, group_size=28,
                  seed=0, lo=0.0, hi=1.0, rho_start=None):
    """Returns (S, loss(S), history) with history = best loss after the initial population and after
    every generation of every group, in order."""
    L, P, T = int(n_layers), int(population), int(generations)
    u = _Uniform(seed)
    S = [float(v) for v in rho_start] if rho_start is not None else [lo + (hi - lo) * u() for _ in range(L)]
    S_loss = float(loss(list(S)))
    history = [S_loss]
    for g0 in range(0, L, group_size):
        coords = list(range(g0, min(L, g0 + group_size)))
        # population: individual 0 is S, the others are random in this group's coordinates
        G = [list(S)]
        for _ in range(1, P):
            ind = list(S)
            for c in coords:
                ind[c] = lo + (hi - lo) * u()
            G.append(ind)
        G_loss = [S_loss] + [float(loss(list(ind))) for ind in G[1:]]
        for _t in range(T):
            G_hat, G_hat_loss = [], []
            for i in range(P):
                x1, x2, x3 = int(u() * P), int(u() * P), int(u() * P)
                child = list(G[i])
                for c in coords:
                    alpha = u()
                    m = G[x1][c] + p_m * (G[x2][c] - G[x3][c])
                    m = min(max(m, lo), hi)
                    child[c] = m if alpha > p_c else G[i][c]
                G_hat.append(child)
                G_hat_loss.append(float(loss(list(child))))
            # Top_K over G u G_hat: P lowest losses; ties: members of G before G_hat, then by index
            pool = [(G_loss[i], 0, i, G[i]) for i in range(P)] + [(G_hat_loss[i], 1, i, G_hat[i]) for i in range(P)]
            pool.sort(key=lambda e: (e[0], e[1], e[2]))
            G = [list(e[3]) for e in pool[:P]]
            G_loss = [e[0] for e in pool[:P]]
            history.append(G_loss[0])
        S, S_loss = list(G[0]), G_loss[0]
    return S, S_loss, history
