"""Definition-level evaluation of the paper's cost model in pure Python (itertools), used only to
pin the oracle on tiny instances. Written directly from Eqs. 1-4; shares nothing with oracle/."""
import itertools
import math


def weights_entry(lat, bw, d, e, c, div):
    """2 (alpha + (c/div) / beta) with alpha, beta the two-direction averages (Sec. 2, Eqs. 2-3)."""
    alpha = (lat[d][e] + lat[e][d]) / 2.0
    beta = (bw[d][e] + bw[e][d]) / 2.0
    return 2.0 * (alpha + (c / div) / beta)


def datap_cost(W_dp, groups):
    """Eq. 2 and the max over stages below it. Sums in the listed order of each group."""
    worst = -math.inf
    for C in groups:
        for d in C:
            s = 0.0
            for e in C:
                if e != d:
                    s = s + W_dp[d][e]
            worst = max(worst, s)
    return worst


def matching_cost(W_pp, Ca, Cb):
    """Eq. 3: min over perfect matchings of the max matched weight."""
    best = math.inf
    for pi in itertools.permutations(range(len(Cb))):
        best = min(best, max(W_pp[Ca[i]][Cb[pi[i]]] for i in range(len(Ca))))
    return best


def open_tsp(G):
    """Eq. 4: cheapest Hamiltonian path, free end points; each path summed left to right."""
    n = len(G)
    if n <= 1:
        return 0.0
    best = math.inf
    for order in itertools.permutations(range(n)):
        s = 0.0
        for k in range(n - 1):
            s = s + G[order[k]][order[k + 1]]
        best = min(best, s)
    return best


def comm_cost(W_dp, W_pp, groups):
    """Eq. 1."""
    n = len(groups)
    G = [[0.0] * n for _ in range(n)]
    for a in range(n):
        for b in range(a + 1, n):
            G[a][b] = G[b][a] = matching_cost(W_pp, groups[a], groups[b])
    return datap_cost(W_dp, groups) + open_tsp(G)


def groups_of(perm, D_dp):
    return [list(perm[j:j + D_dp]) for j in range(0, len(perm), D_dp)]


def all_partitions(devs, size):
    """Every unordered partition of `devs` into blocks of `size` (blocks listed with their
    smallest element ascending)."""
    devs = list(devs)
    if not devs:
        yield []
        return
    first, rest = devs[0], devs[1:]
    for others in itertools.combinations(rest, size - 1):
        block = [first] + list(others)
        remaining = [d for d in rest if d not in others]
        for tail in all_partitions(remaining, size):
            yield [block] + tail
