"""Head-wise plan selection for one layer -- TEST INFRASTRUCTURE, not the product.

Sec. 3.4.2, Eq. 2 of DiTFastAttnV2.  Every head h takes at most one method m of the candidate set
(X[h, m] in {0, 1}, sum_m X[h, m] <= 1); a head without a method runs full attention.  Subject to
    sum_h sum_m X[h, m] * I[h, m] <= delta            (the layer's influence budget)
    X[h, m] = 1  only if  I[h, m] <= (c / n) * delta   (no head takes more than c/n of the budget; n = heads)
the total latency  sum_h ( L_full + sum_m X[h, m] * (L[m] - L_full) )  is minimised.  (The printed
objective lists the method latencies only; a head that keeps full attention has to cost L_full for the
minimum to mean anything, which is the reading taken here.)

The oracle is the definition: every one of the (M + 1)^H assignments is tried.  Pure Python, small H only.
Nothing in the product path may import this module.
"""
import itertools


def solve(influence, latency, latency_full, delta, c):
    """influence: H x M nested sequence; latency: M values.  Returns (best total latency, list of every
    assignment reaching it); an assignment is a tuple of H entries, -1 = full attention, else the method index."""
    H = len(influence)
    M = len(latency)
    assert H <= 8, "brute force: small instances only"
    cap = c / H * delta
    best, best_set = None, []
    for assign in itertools.product(range(-1, M), repeat=H):
        total_i, total_l, ok = 0.0, 0.0, True
        for h, m in enumerate(assign):
            if m < 0:
                total_l += latency_full
                continue
            if influence[h][m] > cap:
                ok = False
                break
            total_i += influence[h][m]
            total_l += latency[m]
        if not ok or total_i > delta:
            continue
        if best is None or total_l < best - 1e-12 * max(1.0, abs(best)):
            best, best_set = total_l, [assign]
        elif abs(total_l - best) <= 1e-12 * max(1.0, abs(best)):
            best_set.append(assign)
    return best, best_set
