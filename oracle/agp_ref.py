"""Reference of the strategy selection of Section 4.3 (Algorithm 3): TEST INFRASTRUCTURE ONLY.

With k = t_iter(1)/N, a measured coefficient b = beta_c(i) (strategy c on i GPUs, 2 <= i <= P) is
admissible when i*b/(i-1) <= k (the p = 1 case of the scaling inequality of Section 4.3); the
selection is the admissible entry with the smallest term.  The paper's argmin leaves ties open;
the reading taken here (and by the library): fewer GPUs first, then the entry listed first."""


def agp_select(t_iter1, n_nodes, beta, max_gpus):
    """beta: dict {(strategy, gpus): seconds per node}; "listed first" = dict order.
    Returns (strategy, gpus), or (None, 1) when no entry is admissible."""
    k = t_iter1 / n_nodes
    admissible = [(i * b / (i - 1), i, position, c)
                  for position, ((c, i), b) in enumerate(beta.items())
                  if 2 <= i <= max_gpus and i * b / (i - 1) <= k]
    if not admissible:
        return None, 1
    _, i, _, c = min(admissible)   # by (term, gpus, position); position is unique, c is never compared
    return c, i
