"""Plain-Python definition of the scale-up model (TEST INFRASTRUCTURE ONLY, like the rest of
oracle/): the speed-up of a replication strategy P (Section 4.1, Eq. 1-4), the greedy scale-up
(Algorithm 1) expressed as a fold over the offers (node, layer) that the continuity ordering
produces, and the integer batch shares that minimise Eq. 1's slowest instance.  Written from the
paper's definitions; shares no code with the library."""
import functools
import math


def compute_load(p, bs, capacity, d, l):
    """Eq. 1: W(P) = sum over layers of the slowest instance's d^2 * bs_ij * l / C_ij."""
    total = 0.0
    for i in range(len(p)):
        total += max(d * d * bs[i][j] * l / capacity[i][j] for j in range(p[i]))
    return total


def comm_load(p, bs, bandwidth, d, l, delta):
    """Eq. 2: T(P) = delta * sum over layers and replicas j >= 1 of d * bs_ij * l / B_ij."""
    total = 0.0
    for i in range(len(p)):
        for j in range(1, p[i]):
            total += d * bs[i][j] * l / bandwidth[i][j]
    return delta * total


def speedup(p, bs, capacity, bandwidth, d, l, delta):
    """Eq. 3: S(P) = W(P0) / (W(P) + T(P)); P0 runs each layer's whole batch on its original."""
    n = len(p)
    p0 = [1] * n
    bs0 = [[sum(bs[i][:p[i]])] for i in range(n)]
    cap0 = [[capacity[i][0]] for i in range(n)]
    return compute_load(p0, bs0, cap0, d, l) / (compute_load(p, bs, capacity, d, l) + comm_load(p, bs, bandwidth, d, l, delta))


def speedup_homo(p, gamma):
    """Eq. 4: 1 / (gamma + (1 - gamma) / n * sum_i 1 / p_i)."""
    n = len(p)
    return 1.0 / (gamma + (1.0 - gamma) / n * sum(1.0 / v for v in p))


def longest_run_through(held, layer):
    """Length of the block of consecutive layer indices that contains `layer` once it is held."""
    s = set(held) | {layer}
    lo = layer
    while lo - 1 in s:
        lo -= 1
    hi = layer
    while hi + 1 in s:
        hi += 1
    return hi - lo + 1


def sort_candidates_by_continuity(held, n, max_replicas):
    """Layers node g could still take, best first: the one that gives the node its longest run of
    consecutive layers, the lower index on ties; at most max_replicas of them."""
    held = set(held)
    out = []
    while len(out) < max_replicas:
        free = [i for i in range(n) if i not in held]
        if not free:
            break
        best = max(free, key=lambda i: (longest_run_through(held, i), -i))
        held.add(best)
        out.append(best)
    return out


def scale_up_offers(n, node_available, replica_size, placed):
    """What Algorithm 1 considers, in its order: for every node with room for at least one replica
    (nodes in the given order), the layers it does not hold yet in continuity order, as many as
    fit.  A node's offers depend on that node's own holdings only."""
    offers = []
    for g, avail in enumerate(node_available):
        held = [i for i in range(n) if placed[g][i]]
        offers += [(g, layer) for layer in sort_candidates_by_continuity(held, n, avail // replica_size)]
    return offers


def plan_scale_up(p, gamma, node_available, replica_size, placed=None):
    """Algorithm 1 as a left fold over the offers: an offer is taken when one more instance of
    that layer raises the speed-up of Eq. 4 above the best seen so far.  Returns (P*, placed,
    speed-up)."""
    n = len(p)
    start_placed = [list(row) for row in placed] if placed is not None else [[0] * n for _ in node_available]

    def take(state, offer):
        p_now, placed_now, best = state
        g, layer = offer
        p_new = [v + (1 if i == layer else 0) for i, v in enumerate(p_now)]
        sp = speedup_homo(p_new, gamma)
        if sp <= best:
            return state
        placed_new = [[1 if (gi == g and i == layer) else v for i, v in enumerate(row)] for gi, row in enumerate(placed_now)]
        return p_new, placed_new, sp

    offers = scale_up_offers(n, node_available, replica_size, start_placed)
    return functools.reduce(take, offers, (list(p), start_placed, speedup_homo(list(p), gamma)))


# ---- batch shares from capacities (Eq. 1) ----------------------------------------------------
def slowest_instance(shares, capacity):
    """The factor of Eq. 1 that the shares decide: max_j bs_j / C_j (d^2 l is common to all j)."""
    return max(b / c for b, c in zip(shares, capacity))


def shares_from_capacity(n, capacity):
    """Integer shares bs_j >= 0, sum n, that minimise max_j bs_j / C_j.  Start from the
    capacity-weighted form of the paper's contiguous split - boundaries floor(n * C_{<j} / C_total),
    which is floor(j n / k) for equal capacities (15 -> 7 + 8) - then, while handing one unit from
    a slowest instance (lowest index) to the instance that would be fastest with one more (lowest
    index) lowers that slowest instance below its current time, do so."""
    k = len(capacity)
    total = sum(capacity)
    bounds = [math.floor(n * sum(capacity[:j]) / total) for j in range(k)] + [n]
    shares = [bounds[j + 1] - bounds[j] for j in range(k)]
    while True:
        worst = max(range(k), key=lambda j: (shares[j] / capacity[j], -j))
        taker = min(range(k), key=lambda j: ((shares[j] + 1) / capacity[j], j))
        if shares[worst] == 0 or (shares[taker] + 1) / capacity[taker] >= shares[worst] / capacity[worst]:
            return shares
        shares[worst] -= 1
        shares[taker] += 1
