"""Plain-Python definition of the scale-up model (TEST INFRASTRUCTURE ONLY, like the rest of
oracle/): the speed-up of a replication strategy P (Section 4.1, Eq. 1-4) and the greedy
scale-up with its continuity ordering (Algorithm 1).  Written from the paper's definitions, one
step per statement; shares no code with the library."""


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


def plan_scale_up(p, gamma, node_available, replica_size, placed=None):
    """Algorithm 1.  Returns (P*, placed, speed-up)."""
    n = len(p)
    p = list(p)
    placed = [list(row) for row in placed] if placed is not None else [[0] * n for _ in node_available]
    best = speedup_homo(p, gamma)
    for g, avail in enumerate(node_available):
        max_replicas = avail // replica_size
        if max_replicas < 1:
            continue
        held = [i for i in range(n) if placed[g][i]]
        for layer in sort_candidates_by_continuity(held, n, max_replicas):
            trial = list(p)
            trial[layer] += 1
            sp = speedup_homo(trial, gamma)
            if sp > best:
                best, p = sp, trial
                placed[g][layer] = 1
    return p, placed, best
