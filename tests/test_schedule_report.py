"""The paper's qualitative claims about schedule quality (Sec. 5, non-overlapped communication vs brute force),
checked on seeded synthetic profiles through the library's scheduler and Eq. (7) evaluator."""
from paper_2502_11058_amd import schedule_report as R


def test_alg2_close_to_optimum_and_better_than_equal_partition():
    for L, enp, alg2, opt, same in R.layers_sweep(trials=60, seed=1):
        assert opt <= alg2 <= enp                 # exact optimum <= heuristic <= equal-number partition (on average)
        assert alg2 - opt <= 0.02                 # "slightly longer in a few cases": within 2 % of a backward period
        assert same >= 0.4                        # and identical on a large share of instances


def test_period_time_falls_with_bandwidth_and_partial_sync_beats_full_sync():
    rows = R.bandwidth_sweep("gpt2_small")
    for col in (1, 2, 3, 4):
        assert all(rows[i][col] >= rows[i + 1][col] for i in range(len(rows) - 1))
    for g, full, enp, alg2, opt in rows:
        assert opt <= alg2 <= enp <= full


def test_solution_set_stays_within_its_bound_and_far_below_brute_force():
    # Sec. 3.3: the pruned search visits exponentially fewer candidates than all cuts
    for L, H, cuts, bound, size, t_alg2, t_opt in R.complexity_sweep(trials=5):
        assert 1 <= size <= bound
        assert cuts >= size
    big = [r for r in R.complexity_sweep(trials=3) if r[0] >= 64]
    assert all(r[2] > 1e6 * r[4] for r in big)
