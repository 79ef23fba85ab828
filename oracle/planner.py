"""Communication model and overlap planning, written out from the paper's own arithmetic.

TEST INFRASTRUCTURE ONLY (see oracle/ref.py).

Sec. 2.4.1 (analysis of communication overhead): with a ring all-reduce between C clusters the
link between two clusters carries 2 (C - 1) / C of what every worker holds.  Sec. 2.3 (one-step
delay): the exchange of outer step t-1 runs beside the H local steps of outer step t, so it is
hidden when it takes no longer than H local steps.
"""


def comm_seconds(payload_bytes, clusters, bits_per_second):
    between = 2 * (clusters - 1) * payload_bytes / clusters
    return between * 8 / bits_per_second


def factor_payload_bytes(m, n, r, qbits, group):
    """Both quantised factors of one m x n matrix at rank r: codes plus one fp32 scale per group."""
    total = 0
    for side in (m, n):
        count = side * r
        total += (count // 2 if qbits == 4 else count) + 4 * (count // group)
    return total


def stage_payload_bytes(shapes, r, qbits, group, extra_bytes=0, iters=1):
    """What one worker sends per outer step: both factors of every matrix once per power
    iteration of the round, plus the tensors sent without low-rank."""
    return extra_bytes + iters * sum(factor_payload_bytes(m, n, min(r, m, n), qbits, group)
                                     for m, n in shapes)


def plan_overlap(shapes, qbits, group, extra_bytes, rmin, rmax, clusters, bits_per_second,
                 step_seconds, H, iters=1):
    """Largest rank whose exchange hides behind H local steps; if none does, rmin and the
    smallest H that hides it.  Exhaustive over the ranks."""
    def seconds(r):
        return comm_seconds(stage_payload_bytes(shapes, r, qbits, group, extra_bytes, iters),
                            clusters, bits_per_second)
    fits = [r for r in range(rmin, rmax + 1) if seconds(r) <= H * step_seconds]
    if fits:
        r = max(fits)
        return r, H, seconds(r)
    t = seconds(rmin)
    h = 1
    while h * step_seconds < t:
        h += 1
    return rmin, h, t
