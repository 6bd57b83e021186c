"""Oracle for STAR-H, the heuristic synchronization-mode choice (test infrastructure).

Written from the paper's definitions, with exact rational arithmetic where the
inputs allow it (pass Fractions or floats):
  straggler      d_i = (T_i - min T)/min T > threshold                     (Section 2)
  static x-order T_x = (1 + phi/(x M/N)) t_x                                (Section 4.3.1, Eq. 1)
  dynamic        T_d = 1 / sum_i 1/((1 + phi/(n_ci M/N)) t_ci)              (Eq. 2)
  all-reduce     T_a = (1 + phi/((N-x+q) M/N)) (t_ring + t_w)               (Eq. 3)
Readings (the paper does not fix them; the library states the same ones):
t_x = the x-th smallest iteration time (when x gradient reports have arrived);
groups of a static mode = consecutive runs of x workers in ascending iteration
time; clusters by complete-linkage agglomerative
clustering, merging the pair of clusters whose union has the smallest range
while range / (fastest member of the union) <= cluster_threshold; ties between
modes go to the higher order, the dynamic mode must be strictly faster; no
straggler -> SSGD.
"""
from fractions import Fraction


def stragglers(T, threshold):
    tmin = min(T)
    return [(t - tmin) / tmin > threshold for t in T]


def sorted_workers(T):
    return sorted(range(len(T)), key=lambda k: (T[k], k))


def time_static(T, phi, M, x):
    N = len(T)
    t_x = sorted(T)[x - 1]
    return (1 + phi / (x * M / N)) * t_x


def clusters(T, cluster_threshold):
    """Agglomerative, complete linkage, over all pairs of clusters (brute force)."""
    cl = [[k] for k in sorted_workers(T)]
    while len(cl) > 1:
        best = None
        for a in range(len(cl)):
            for b in range(a + 1, len(cl)):
                u = cl[a] + cl[b]
                rng = max(T[k] for k in u) - min(T[k] for k in u)        # complete linkage in one dimension
                key = (rng, min(T[k] for k in u), a, b)
                if best is None or key < best[0]:
                    best = (key, a, b, u)
        (rng, lo, _, _), a, b, u = best
        if rng / lo > cluster_threshold:
            break
        cl = [c for i, c in enumerate(cl) if i not in (a, b)] + [u]
    cl = [sorted(c, key=lambda k: (T[k], k)) for c in cl]
    cl.sort(key=lambda c: (max(T[k] for k in c), c))
    return cl


def time_dynamic(T, phi, M, cl):
    N = len(T)
    rate = 0
    for c in cl:
        rate += 1 / ((1 + phi / (len(c) * M / N)) * max(T[k] for k in c))
    return 1 / rate


def select_ps(T, phi, M, straggler_threshold=Fraction(1, 5), cluster_threshold=Fraction(1, 5)):
    N = len(T)
    Tx = {x: time_static(T, phi, M, x) for x in range(1, N + 1)}
    cl = clusters(T, cluster_threshold)
    Td = time_dynamic(T, phi, M, cl)
    strag = stragglers(T, straggler_threshold)
    best_x = max(range(1, N + 1), key=lambda x: (-Tx[x], x))          # least time, ties to the higher order
    dynamic = Td < Tx[best_x]
    if not any(strag):
        best_x, dynamic = N, False
    order = sorted_workers(T)
    if dynamic:
        mode, x, groups, best = "dynamic", 0, cl, Td
    else:
        mode = "ssgd" if best_x == N else ("asgd" if best_x == 1 else "static")
        x, best = best_x, Tx[best_x]
        groups = [order[lo:lo + best_x] for lo in range(0, N, best_x)]
    return {"mode": mode, "x": x, "time": best, "Tx": [Tx[x] for x in range(1, N + 1)], "Td": Td, "groups": groups,
            "clusters": cl, "stragglers": strag}


def select_ar(T, child_T, phi, M, waits, straggler_threshold=Fraction(1, 5)):
    N = len(T)
    order = sorted_workers(T)
    X = sum(stragglers(T, straggler_threshold))
    best = ((1 + phi / (N * M / N)) * max(T), 0, 0)                    # plain ring
    table = {(0, None): best[0]}
    for x in range(1, min(X, N - 1) + 1):
        removed = order[N - x:]
        t_ring = max(T[k] for k in order[:N - x])
        for tw in waits:
            q = sum(1 for k in removed if child_T[k] <= tw)
            Ta = (1 + phi / ((N - x + q) * M / N)) * (t_ring + tw)
            table[(x, tw)] = Ta
            if Ta < best[0]:
                best = (Ta, x, tw)
    return {"time": best[0], "x": best[1], "wait": best[2], "table": table}
