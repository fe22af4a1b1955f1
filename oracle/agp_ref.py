"""Reference of the strategy selection of Section 4.3 (Algorithm 3): TEST INFRASTRUCTURE ONLY.

k = t_iter(1)/N.  For every GPU count i = 2..P and every strategy c with a measured
coefficient b = beta_c(i): keep i*b/(i-1) when it does not exceed k.  Return the (c, i) of the
smallest kept term, or (None, 1) when nothing was kept."""


def agp_select(t_iter1, n_nodes, beta, max_gpus):
    """beta: dict {(strategy, gpus): seconds per node}; table order = dict order."""
    k = t_iter1 / n_nodes
    kept = []
    for i in range(2, max_gpus + 1):
        for (c, gpus), b in beta.items():
            if gpus != i:
                continue
            term = i * b / (i - 1)
            if term <= k:
                kept.append((term, c, i))
    if not kept:
        return None, 1
    term, c, i = min(kept, key=lambda t: t[0])
    return c, i
