"""Definition-level restatement, in pure Python integers and lists, of the search half of the method
(Sec. 3.4: hybrid genetic algorithm and local search) under this build's stated reading of it.
Used only to pin the oracle; shares nothing with oracle/ and is written from the prose of the
reading, not from the oracle's code:

  * random words: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), key = (seed low 32 bits, seed
    high 32 bits), counter = (t // 4, candidate k, generation g, stream), the t-th draw is word
    t % 4 of that block; streams: 0 initial population, 1 parent selection, 2 crossover, 3 mutation;
    an integer in [0, n) is (word * n) >> 32;
  * initial candidate k: the identity shuffled by Fisher-Yates downwards (i = N-1 .. 1, exchange
    position i with position randint(i + 1)), the first exchange using draw 0, the next draw 1, ...;
  * offspring k of generation g: parents = selection draws 0 and 1 (each randint(P)); the child is a
    copy of parent 1; crossover step s = 0 .. m_x-1 uses draws 2s (a device d = randint(N)) and
    2s + 1 (a slot = randint(D_dp)): if the stage of d in the child differs from the stage of d in
    parent 2, d changes places with whichever device sits at that slot of parent 2's stage in the
    child; both draws are taken whether used or not; mutation step s uses draws 2s and 2s + 1 as two
    positions (each randint(N)) whose contents are exchanged;
  * local search round r (four-candidate and Kernighan-Lin neighbourhoods): the stage pair is the
    (r mod D_pp (D_pp - 1) / 2)-th in lexicographic order; the proposed swap is applied iff it makes
    the true cost strictly smaller;
  * replacement: the P smallest of parents + offspring under (cost, origin index), parents numbered
    before offspring, in ascending order.

Every function takes a `fault` argument naming a deliberate mistake (None = the reading itself);
the tests use the faulty variants to show that the comparison with the oracle would catch them.
"""
import itertools

MASK32 = 0xFFFFFFFF
STREAM_INIT, STREAM_SELECT, STREAM_CROSSOVER, STREAM_MUTATION = 0, 1, 2, 3


def philox4x32_10(counter, key):
    """Ten rounds of the Philox-4x32 bijection. Each round: (hi0, lo0) = 0xD2511F53 * c0,
    (hi1, lo1) = 0xCD9E8D57 * c2, new counter = (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0); the key
    is bumped by (0x9E3779B9, 0xBB67AE85) after every round but the last (a bump after the last
    one changes nothing)."""
    c = [int(x) & MASK32 for x in counter]
    k = [int(x) & MASK32 for x in key]
    for rnd in range(10):
        prod0 = 0xD2511F53 * c[0]
        prod1 = 0xCD9E8D57 * c[2]
        c = [(prod1 >> 32) ^ c[1] ^ k[0], prod1 & MASK32, (prod0 >> 32) ^ c[3] ^ k[1], prod0 & MASK32]
        k = [(k[0] + 0x9E3779B9) & MASK32, (k[1] + 0xBB67AE85) & MASK32]
    return c


def draw_word(seed, stream, g, k, t, fault=None):
    counter = [t // 4, k, g, stream]
    if fault == "counter_words_swapped":
        counter = [t // 4, g, k, stream]
    if fault == "stream_and_generation_swapped":
        counter = [t // 4, k, stream, g]
    key = [seed & MASK32, (seed >> 32) & MASK32]
    if fault == "key_words_swapped":
        key = key[::-1]
    return philox4x32_10(counter, key)[t % 4]


def randint(word, n):
    return (word * n) >> 32


def init_candidate(seed, k, N, fault=None):
    perm = list(range(N))
    t = 0
    for i in range(N - 1, 0, -1):
        tt = i if fault == "shuffle_draw_index_is_i" else t
        j = randint(draw_word(seed, STREAM_INIT, 0, k, tt, fault), i + 1)
        if fault == "shuffle_range_excludes_i":
            j = randint(draw_word(seed, STREAM_INIT, 0, k, tt, fault), i)
        perm[i], perm[j] = perm[j], perm[i]
        t += 1
    return perm


def stage_of(perm, D_dp, device):
    return perm.index(device) // D_dp


def make_offspring(seed, g, k, population, D_dp, m_x, m_m, fault=None):
    """Returns (child, (parent 1 index, parent 2 index))."""
    P, N = len(population), len(population[0])
    p1 = randint(draw_word(seed, STREAM_SELECT, g, k, 0, fault), P)
    p2 = randint(draw_word(seed, STREAM_SELECT, g, k, 1, fault), P)
    if fault == "parents_exchanged":
        p1, p2 = p2, p1
    child = list(population[p1])
    other = list(population[p2])
    for s in range(m_x):
        d = randint(draw_word(seed, STREAM_CROSSOVER, g, k, 2 * s, fault), N)
        slot = randint(draw_word(seed, STREAM_CROSSOVER, g, k, 2 * s + 1, fault), D_dp)
        here = stage_of(child, D_dp, d)
        there = stage_of(other, D_dp, d)
        if fault == "parent2_stage_read_from_child":
            there = stage_of(child, D_dp, other[child.index(d)])
        if fault == "parent2_stage_by_position":
            there = other[d] // D_dp        # reads parent 2 as if it were indexed by device
        if here == there:
            continue
        qa, qb = child.index(d), there * D_dp + slot
        child[qa], child[qb] = child[qb], child[qa]
    for s in range(m_m):
        a = randint(draw_word(seed, STREAM_MUTATION, g, k, 2 * s, fault), N)
        b = randint(draw_word(seed, STREAM_MUTATION, g, k, 2 * s + 1, fault), N)
        child[a], child[b] = child[b], child[a]
    return child, (p1, p2)


def stage_pair_of_round(r, D_pp):
    pairs = list(itertools.combinations(range(D_pp), 2))
    return pairs[r % len(pairs)]


def gain4_proposal(W_pp, perm, D_dp, D_pp, r):
    """The paper's four-candidate neighbourhood (Sec. 3.4, "Improving Local Search Strategy") for
    round r: positions (a, b) of the swap of largest Gain. The fastest link of a stage is the first
    smallest W_pp over slot pairs i < i'; candidates in the order (d1,d1'), (d1,d2'), (d2,d1'),
    (d2,d2'); Gain(x<->y) = mean_{C_j'} w[x][.] - w[x][partner of x] + mean_{C_j} w[y][.] -
    w[y][partner of y], each mean a slot-order sum from 0.0 divided by D_dp, the four terms combined
    left to right; the first largest wins."""
    j, jp = stage_pair_of_round(r, D_pp)
    Cj, Cjp = perm[j * D_dp:(j + 1) * D_dp], perm[jp * D_dp:(jp + 1) * D_dp]

    def fastest(C):
        best = None
        for i in range(D_dp):
            for i2 in range(i + 1, D_dp):
                w = W_pp[C[i]][C[i2]]
                if best is None or w < best[0]:
                    best = (w, i, i2)
        return best[1], best[2]

    s, sp = fastest(Cj), fastest(Cjp)
    cands = []
    for xi in (0, 1):
        for yi in (0, 1):
            x, mx = Cj[s[xi]], Cj[s[1 - xi]]
            y, my = Cjp[sp[yi]], Cjp[sp[1 - yi]]
            sx = 0.0
            for e in Cjp:
                sx = sx + W_pp[x][e]
            sy = 0.0
            for e in Cj:
                sy = sy + W_pp[y][e]
            gain = ((sx / D_dp - W_pp[x][mx]) + sy / D_dp) - W_pp[y][my]
            cands.append((gain, j * D_dp + s[xi], jp * D_dp + sp[yi]))
    best = cands[0]
    for c in cands[1:]:
        if c[0] > best[0]:
            best = c
    return best[1], best[2]


def four_candidates(W_pp, perm, D_dp, D_pp, r):
    """The four swaps round r's stage pair offers (Sec. 3.4, "Improving Local Search Strategy": the end points
    d1, d2 of the fastest link inside C_j and d1', d2' of the fastest inside C_j'), as position pairs in the
    order (d1,d1'), (d1,d2'), (d2,d1'), (d2,d2'). Fastest = first smallest W_pp over slot pairs i < i'."""
    j, jp = stage_pair_of_round(r, D_pp)
    ends = []
    for st in (j, jp):
        C = perm[st * D_dp:(st + 1) * D_dp]
        best = None
        for i, i2 in itertools.combinations(range(D_dp), 2):
            if best is None or W_pp[C[i]][C[i2]] < best[0]:
                best = (W_pp[C[i]][C[i2]], st * D_dp + i, st * D_dp + i2)
        ends.append(best[1:])
    return [(a, b) for a in ends[0] for b in ends[1]]


def local_search_best4(cost_fn, W_pp, perm, D_dp, D_pp, rounds):
    """The second reading of the paper's neighbourhood: per round the four candidates are all priced by the true
    cost, the cheapest (the first on ties) is applied iff it is strictly cheaper than the current allocation.
    Returns (perm, cost, applied)."""
    perm = list(perm)
    cur = cost_fn(perm)
    applied = []
    for r in range(rounds):
        best = None
        for a, b in four_candidates(W_pp, perm, D_dp, D_pp, r):
            trial = list(perm)
            trial[a], trial[b] = trial[b], trial[a]
            c = cost_fn(trial)
            if best is None or c < best[0]:
                best = (c, trial, (a, b))
        if best[0] < cur:
            cur, perm = best[0], best[1]
            applied.append(best[2])
        else:
            applied.append(None)
    return perm, cur, applied


def kl_proposal(W_pp, perm, D_dp, D_pp, r):
    """The Kernighan-Lin neighbourhood the paper compares with (Sec. 3.4, "Existing Local Search
    Strategy") for round r: among all swaps of a device x of C_j with a device y of C_j', the first
    (slot of x, then slot of y) of largest gain_KL = sum_{C_j'} w[x][.] - sum_{C_j minus x} w[x][.]
    + sum_{C_j} w[y][.] - sum_{C_j' minus y} w[y][.] - 2 w[x][y], sums in slot order from 0.0, the
    five terms combined left to right."""
    j, jp = stage_pair_of_round(r, D_pp)
    Cj, Cjp = perm[j * D_dp:(j + 1) * D_dp], perm[jp * D_dp:(jp + 1) * D_dp]
    best = None
    for sx, x in enumerate(Cj):
        for sy, y in enumerate(Cjp):
            ext_x = int_x = ext_y = int_y = 0.0
            for e in Cjp:
                ext_x = ext_x + W_pp[x][e]
            for e in Cj:
                if e != x:
                    int_x = int_x + W_pp[x][e]
            for e in Cj:
                ext_y = ext_y + W_pp[y][e]
            for e in Cjp:
                if e != y:
                    int_y = int_y + W_pp[y][e]
            gain = (((ext_x - int_x) + ext_y) - int_y) - 2.0 * W_pp[x][y]
            if best is None or gain > best[0]:
                best = (gain, j * D_dp + sx, jp * D_dp + sy)
    return best[1], best[2]


def local_search(cost_fn, W_pp, perm, D_dp, D_pp, rounds, proposal):
    """`rounds` rounds on one candidate with the given proposal rule; returns (perm, cost, applied)
    where applied[r] is the (a, b) swapped in round r or None. cost_fn(perm) is the true cost."""
    perm = list(perm)
    cur = cost_fn(perm)
    applied = []
    for r in range(rounds):
        a, b = proposal(W_pp, perm, D_dp, D_pp, r)
        trial = list(perm)
        trial[a], trial[b] = trial[b], trial[a]
        c = cost_fn(trial)
        if c < cur:
            perm, cur = trial, c
            applied.append((a, b))
        else:
            applied.append(None)
    return perm, cur, applied


def local_search_gain4(cost_fn, W_pp, perm, D_dp, D_pp, rounds):
    return local_search(cost_fn, W_pp, perm, D_dp, D_pp, rounds, gain4_proposal)[:2]


def replace(parents, parent_cost, offspring, offspring_cost):
    """Survivors (rows, costs): the len(parents) best under (cost, origin), parents first."""
    pool = [(c, i, row) for i, (row, c) in enumerate(zip(parents, parent_cost))]
    pool += [(c, len(parents) + i, row) for i, (row, c) in enumerate(zip(offspring, offspring_cost))]
    pool.sort(key=lambda e: (e[0], e[1]))
    keep = pool[:len(parents)]
    return [list(e[2]) for e in keep], [e[0] for e in keep]


def evolve(cost_fn, W_pp, seed, generations, P, lam, N, D_dp, D_pp, m_x, m_m, ls_moves, fault=None):
    """The generation-wise evolutionary loop with the four-candidate local search.
    Returns (population, cost, best_trace)."""
    pop = [init_candidate(seed, k, N, fault) for k in range(P)]
    cost = [cost_fn(row) for row in pop]
    trace = []
    for g in range(generations):
        off, off_cost = [], []
        for k in range(lam):
            child, _ = make_offspring(seed, g, k, pop, D_dp, m_x, m_m, fault)
            child, c = local_search_gain4(cost_fn, W_pp, child, D_dp, D_pp, ls_moves)
            off.append(child)
            off_cost.append(c)
        pop, cost = replace(pop, cost, off, off_cost)
        trace.append(cost[0])
    return pop, cost, trace
