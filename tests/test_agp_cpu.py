"""Strategy selection (Algorithm 3).  Cases worked by hand from the inequality
s*beta_c(s)/(s-1) <= t_iter(1)/N pin the reference (oracle/agp_ref.py) first; the library's host-only
entry point is then held to the same cases and to the reference on random tables, including tables
built to contain ties and boundary values."""
import itertools

import numpy as np
import pytest

from oracle import agp_ref

# (t_iter(1), N, table [(strategy, gpus, beta)], P) -> (strategy, gpus, estimated t_iter or None)
HAND = {
    # k = 1e-6.  AG@2 = 2*4e-7/1 = 8e-7 (kept), AG@4 = 4*6e-7/3 = 8e-7 (kept), A2A@2 = 2*6e-7 = 1.2e-6
    # (dropped), A2A@4 = 4*3e-7/3 = 4e-7 (kept, smallest) -> GP-A2A on 4; estimate 1/4 + 3e-7*1e6 = 0.55 s
    "smallest_term_wins": ((1.0, 1_000_000, [(0, 2, 4e-7), (0, 4, 6e-7), (1, 2, 6e-7), (1, 4, 3e-7)], 8), (1, 4, 0.55)),
    # the same table on a 2-GPU machine: only AG@2 is admissible (A2A@2 exceeds k); 1/2 + 4e-7*1e6 = 0.9 s
    "machine_limit": ((1.0, 1_000_000, [(0, 2, 4e-7), (0, 4, 6e-7), (1, 2, 6e-7), (1, 4, 3e-7)], 2), (0, 2, 0.9)),
    # k = 1e-7: every term exceeds it -> stay on one GPU
    "nothing_admissible": ((0.1, 1_000_000, [(0, 2, 4e-7), (0, 4, 6e-7), (1, 2, 6e-7), (1, 4, 3e-7)], 8), (None, 1, 0.1)),
    # boundary: beta = 2^-22 on 2 GPUs -> term 2^-21 exactly; N = 2^20, t = 0.5 -> k = 2^-21 exactly: kept
    "boundary_is_admissible": ((0.5, 1 << 20, [(0, 2, 2.0 ** -22)], 8), (0, 2, None)),
    # one ulp below the boundary: dropped
    "just_below_boundary": ((0.5 * (1 - 2.0 ** -52), 1 << 20, [(0, 2, 2.0 ** -22)], 8), (None, 1, None)),
    # tie at the minimum across GPU counts: 4 GPUs: 4*1.5*2^-22/3 = 2^-21; 2 GPUs: 2*2^-22 = 2^-21 -> fewer GPUs,
    # whichever is listed first
    "tie_prefers_fewer_gpus": ((1.0, 1 << 20, [(0, 4, 1.5 * 2.0 ** -22), (1, 2, 2.0 ** -22)], 8), (1, 2, None)),
    "tie_prefers_fewer_gpus_listed_last": ((1.0, 1 << 20, [(1, 2, 2.0 ** -22), (0, 4, 1.5 * 2.0 ** -22)], 8), (1, 2, None)),
    # tie at the minimum at the same GPU count: the entry listed first
    "tie_same_gpus_first_listed": ((1.0, 1 << 20, [(1, 2, 2.0 ** -22), (0, 2, 2.0 ** -22), (2, 2, 2.0 ** -21)], 8), (1, 2, None)),
    # the term, not the raw coefficient, is minimised: AG@2 has the smaller beta (3e-7 -> term 6e-7), A2A@8 the
    # smaller term (8*3.2e-7/7 = 3.657e-7) -> GP-A2A on 8; estimate 1/8 + 3.2e-7*1e6 = 0.445 s
    "term_not_raw_coefficient": ((1.0, 1_000_000, [(0, 2, 3e-7), (1, 8, 3.2e-7)], 8), (1, 8, 0.445)),
    # entries beyond the machine, or for one GPU, are ignored even when they have the smallest term
    "entries_outside_2_to_P_ignored": ((1.0, 1000, [(0, 16, 1e-9), (1, 1, 0.0), (0, 8, 5e-4)], 8), (0, 8, None)),
}


def as_beta(table):
    return {(c, i): b for c, i, b in table}


@pytest.mark.parametrize("name", sorted(HAND))
def test_reference_on_hand_worked_cases(name):
    (t1, n, table, P), (c, s, _) = HAND[name]
    assert agp_ref.agp_select(t1, n, as_beta(table), P) == (c, s)


@pytest.mark.parametrize("name", sorted(HAND))
def test_library_on_hand_worked_cases(name):
    import paper_2604_16715_amd as gta
    (t1, n, table, P), (c, s, est) = HAND[name]
    got_c, got_s, got_est = gta.gta_agp_select(t1, n, table, P)
    assert (got_c if got_c >= 0 else None, got_s) == (c, s)
    if est is not None:
        assert got_est == pytest.approx(est, rel=1e-12)


def test_library_rejects_bad_arguments():
    import paper_2604_16715_amd as gta
    with pytest.raises(gta.GtaError):
        gta.gta_agp_select(0.0, 10, [(0, 2, 1e-7)], 8)
    with pytest.raises(gta.GtaError):
        gta.gta_agp_select(1.0, 10, [(0, 2, -1e-7)], 8)


def test_library_matches_reference_on_random_tables():
    """Continuous tables (ties have probability zero) and tables drawn from a few dyadic values, where
    ties at the minimum and terms equal to k are common; table order is shuffled."""
    import paper_2604_16715_amd as gta
    rng = np.random.Generator(np.random.Philox(3))
    ties = boundaries = 0
    for trial in range(600):
        P = int(rng.integers(2, 9))
        dyadic = trial % 2 == 1
        n = 1 << int(rng.integers(10, 22)) if dyadic else int(rng.integers(1000, 10_000_000))
        t1 = float(2.0 ** int(rng.integers(-3, 2))) if dyadic else float(rng.uniform(0.01, 5.0))
        k = t1 / n
        table = []
        for i, c in itertools.product(range(2, P + 1), (0, 1, 2)):
            if rng.random() < 0.8:
                if dyadic:   # beta such that i*beta/(i-1) is k times a small dyadic factor (exactly, for i-1 a power of two)
                    b = k * float(rng.choice([0.25, 0.5, 1.0, 2.0])) * (i - 1) / i
                else:
                    b = float(rng.uniform(0.0, 3.0) * k)
                table.append((c, i, b))
        order = rng.permutation(len(table))
        table = [table[j] for j in order]
        terms = sorted(i * b / (i - 1) for _, i, b in table if i * b / (i - 1) <= k)
        ties += len(terms) > 1 and terms[0] == terms[1]
        boundaries += any(t == k for t in terms)
        c_ref, s_ref = agp_ref.agp_select(t1, n, as_beta(table), P)
        c, s, _ = gta.gta_agp_select(t1, n, table, P)
        assert (c if c >= 0 else None, s) == (c_ref, s_ref), (trial, table)
    assert ties > 50 and boundaries > 50   # the dyadic tables did exercise both


@pytest.mark.parametrize("old,new", [
    ("i * b / (i - 1) <= k]", "i * b / (i - 1) < k]"),            # boundary excluded
    ("if 2 <= i <= max_gpus and", "if 2 <= i and"),                # machine size ignored
    ("(i * b / (i - 1), i, position, c)", "(i * b / (i - 1), -i, position, c)"),   # ties to MORE GPUs
    ("(i * b / (i - 1), i, position, c)", "(i * b / (i - 1), i, -position, c)"),   # ties to the entry listed last
    ("(i * b / (i - 1), i, position, c)", "(b, i, position, c)"),                  # raw coefficient instead of the term
    ("k = t_iter1 / n_nodes", "k = t_iter1"),                                      # k not per node
])
def test_planted_mistakes_in_the_reference_are_caught_by_the_hand_worked_cases(old, new):
    """The hand-worked cases alone (no library involved) notice each of these one-token mistakes."""
    import inspect
    text = inspect.getsource(agp_ref)
    assert text.count(old) == 1
    scope: dict = {}
    exec(compile(text.replace(old, new), "agp_ref_mutant", "exec"), scope)
    wrong = 0
    for (t1, n, table, P), (c, s, _) in HAND.values():
        got = scope["agp_select"](t1, n, as_beta(table), P)
        if -got[1] == s:            # the mutant that negates the GPU count returns it negated
            got = (got[0], -got[1])
        wrong += got != (c, s)
    assert wrong > 0
