"""Host logic: the baby-step / giant-step planner (Sec. 3.2, rotation counts of App. A.2.2)."""
from paper_2604_09975_amd import plan
from paper_2604_09975_amd import workload as W


def test_counts_follow_the_formula():
    assert plan.key_switches(3, 9, 256, 32) == (93, 63)
    assert plan.key_switches(12, 3, 256, 8) == (84, 93)
    assert plan.key_switches(1, 1, 64, 64) == (63, 0)


def test_benchmark_plans_are_the_planner_s_choice():
    for spec in (W.BERT_QKV,) + W.GPT2_LAYERS:
        G, B_out = -(-spec.d_in // spec.C), -(-spec.d_out // spec.C)
        assert plan.choose_n1(G, B_out, spec.C) == spec.N1, spec.name


def test_equal_costs_minimise_the_plain_count():
    # with equal unit costs the choice minimises G*(N1-1) + B_out*(N2-1)
    for G, B_out, C in [(3, 9, 256), (12, 3, 256), (1, 1, 64), (5, 5, 120)]:
        n1 = plan.choose_n1(G, B_out, C, 1.0, 1.0)
        best = min(sum(plan.key_switches(G, B_out, C, d)) for d in plan.divisors(C))
        assert sum(plan.key_switches(G, B_out, C, n1)) == best
