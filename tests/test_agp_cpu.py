"""Strategy selection (Algorithm 3) — host-only entry point of the library against the reference
and against cases worked by hand from the inequality s*beta_c(s)/(s-1) <= t_iter(1)/N."""
import itertools

import numpy as np
import pytest

from oracle import agp_ref


def test_hand_worked_cases():
    import paper_2604_16715_amd as gta
    # t_iter(1) = 1 s, N = 1e6 nodes -> k = 1e-6.  Terms: AG@2 = 2*4e-7/1 = 8e-7 (kept),
    # AG@4 = 4*6e-7/3 = 8e-7 (kept, tie -> first in table order wins), A2A@2 = 2*6e-7 = 1.2e-6 (dropped),
    # A2A@4 = 4*3e-7/3 = 4e-7 (kept, smallest) -> GP-A2A on 4 GPUs; estimate = 1/4 + 3e-7*1e6 = 0.55 s.
    table = [(0, 2, 4e-7), (0, 4, 6e-7), (1, 2, 6e-7), (1, 4, 3e-7)]
    c, s, est = gta.gta_agp_select(1.0, 1_000_000, table, 8)
    assert (c, s) == (1, 4) and est == pytest.approx(0.55, rel=1e-12)
    # limiting the machine to 2 GPUs leaves only AG@2
    c, s, est = gta.gta_agp_select(1.0, 1_000_000, table, 2)
    assert (c, s) == (0, 2) and est == pytest.approx(0.5 + 0.4, rel=1e-12)
    # a graph whose single-GPU iteration is too short to pay for any communication stays on one GPU
    c, s, est = gta.gta_agp_select(0.1, 1_000_000, table, 8)
    assert (c, s) == (-1, 1) and est == 0.1
    # the boundary value itself is admissible (the paper's test is <=)
    c, s, _ = gta.gta_agp_select(8e-7 * 1_000_000, 1_000_000, [(0, 2, 4e-7)], 8)
    assert (c, s) == (0, 2)
    with pytest.raises(gta.GtaError):
        gta.gta_agp_select(0.0, 10, table, 8)


def test_matches_reference_on_random_tables():
    import paper_2604_16715_amd as gta
    rng = np.random.Generator(np.random.Philox(3))
    for trial in range(200):
        P = int(rng.integers(2, 9))
        n = int(rng.integers(1000, 10_000_000))
        t1 = float(rng.uniform(0.01, 5.0))
        beta = {}
        for i, c in itertools.product(range(2, P + 1), (0, 1, 2)):
            if rng.random() < 0.8:
                beta[(c, i)] = float(rng.uniform(0.0, 3.0) * t1 / n)
        c_ref, s_ref = agp_ref.agp_select(t1, n, beta, P)
        # the reference scans gpus ascending, then strategies in table order: present the table that way
        table = [(c, i, b) for i in range(2, P + 1) for (c, g), b in beta.items() if g == i]
        c, s, _ = gta.gta_agp_select(t1, n, table, P)
        assert (c if c >= 0 else None, s) == (c_ref, s_ref), trial
