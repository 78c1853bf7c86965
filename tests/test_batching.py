"""Request batching (the paper's appendix A.2): properties the description fixes, brute force on
small inputs, and the degenerate cases."""
import itertools
import random

import pytest

from paper_2411_11217_amd.batching import MicroBatch, Request, batch_requests


def reqs(lens):
    return [Request(i, n) for i, n in enumerate(lens)]


def test_every_request_is_placed_once_or_aborted():
    rng = random.Random(1)
    for _ in range(50):
        lens = [rng.randint(1, 600) for _ in range(rng.randint(0, 60))]
        n_ub, ubs, gen = rng.randint(1, 6), rng.randint(1, 12), rng.randint(0, 64)
        cache = rng.randint(200, 6000)
        mbs, aborted = batch_requests(reqs(lens), n_ub, ubs, gen, cache)
        ids = [r.rid for mb in mbs for r in mb.requests] + [r.rid for r in aborted]
        assert sorted(ids) == list(range(len(lens)))
        assert len(mbs) <= n_ub
        for mb in mbs:
            assert 1 <= len(mb.requests) <= ubs
            assert mb.prompt_tokens + len(mb.requests) * gen <= cache     # the KV cache of the micro-batch fits
            assert mb.decode_tokens == len(mb.requests)


def test_longest_first_into_the_lightest_gives_the_textbook_greedy_partition():
    # no limits in play: the classic longest-processing-time partition
    mbs, aborted = batch_requests(reqs([7, 5, 4, 3, 3, 2]), n_ub=2, ubs=100, gen_len=0, cache_size=10**9)
    assert not aborted
    assert sorted(sorted(r.input_len for r in mb.requests) for mb in mbs) == [[2, 3, 7], [3, 4, 5]]
    assert sorted(mb.prompt_tokens for mb in mbs) == [12, 12]


def test_balance_is_within_the_longest_request():
    rng = random.Random(7)
    for _ in range(30):
        lens = [rng.randint(16, 512) for _ in range(64)]
        mbs, aborted = batch_requests(reqs(lens), n_ub=4, ubs=64, gen_len=0, cache_size=10**9)
        assert not aborted and len(mbs) == 4
        loads = [mb.prompt_tokens for mb in mbs]
        assert max(loads) - min(loads) <= max(lens)                # greedy bound for open bins


def test_against_brute_force_optimum_on_tiny_inputs():
    # the greedy makespan is within 4/3 - 1/(3m) of the optimum (Graham's bound for longest-first)
    rng = random.Random(3)
    for _ in range(40):
        lens = [rng.randint(1, 30) for _ in range(7)]
        m = 3
        best = min(max(sum(l for l, b in zip(lens, assign) if b == k) for k in range(m))
                   for assign in itertools.product(range(m), repeat=len(lens)))
        mbs, _ = batch_requests(reqs(lens), n_ub=m, ubs=100, gen_len=0, cache_size=10**9)
        greedy = max(mb.prompt_tokens for mb in mbs)
        assert best <= greedy <= (4 / 3 - 1 / (3 * m)) * best + 1e-9


def test_cache_limit_aborts_and_full_micro_batches_close():
    # prompt tokens + gen_len per request must fit the cache: 100 + 50 > 140 aborts the long request,
    # 30 + 50 fits, then 30 + 20 + 2 * 50 = 150 > 140 aborts the last one
    mbs, aborted = batch_requests(reqs([100, 30, 20]), n_ub=1, ubs=8, gen_len=50, cache_size=140)
    assert [r.input_len for r in aborted] == [100, 20]
    assert [[r.input_len for r in mb.requests] for mb in mbs] == [[30]]
    # with room for the long one it is placed first and the others no longer fit
    mbs, aborted = batch_requests(reqs([100, 30, 20]), n_ub=1, ubs=8, gen_len=50, cache_size=160)
    assert [r.input_len for r in aborted] == [30, 20] and [[r.input_len for r in mb.requests] for mb in mbs] == [[100]]
    # ubs closes micro-batches; when all are closed the rest is aborted
    mbs, aborted = batch_requests(reqs([9, 8, 7, 6, 5, 4]), n_ub=2, ubs=2, gen_len=0, cache_size=10**9)
    assert sorted(sorted(r.input_len for r in mb.requests) for mb in mbs) == [[6, 9], [7, 8]]
    assert sorted(r.input_len for r in aborted) == [4, 5]


def test_degenerate_inputs():
    assert batch_requests([], 3, 4, 8, 100) == ([], [])
    mbs, aborted = batch_requests(reqs([5]), 3, 4, 8, 100)
    assert len(mbs) == 1 and not aborted and isinstance(mbs[0], MicroBatch)
    with pytest.raises(ValueError):
        batch_requests(reqs([1]), 0, 1, 1, 1)
    # equal lengths keep arrival order inside the sort: deterministic output
    a = batch_requests(reqs([4] * 10), 2, 5, 0, 10**9)
    b = batch_requests(reqs([4] * 10), 2, 5, 0, 10**9)
    assert [[r.rid for r in mb.requests] for mb in a[0]] == [[r.rid for r in mb.requests] for mb in b[0]]


def test_prompt_length_stand_in_has_the_papers_mean_and_maximum_and_packs_evenly():
    # the paper's table of workload configurations gives 77 / 418 (MTBench), 242 / 256, 1693 / 1984
    import numpy as np
    from moe_workloads import prompt_lengths
    for s_avg, s_max in ((77, 418), (242, 256), (1693, 1984)):
        lens = prompt_lengths(1024, seed=5, s_avg=s_avg, s_max=s_max)
        assert lens.shape == (1024,) and lens.min() >= 4 and lens.max() == s_max
        assert abs(lens.mean() - s_avg) < 0.01 * s_avg
        assert np.array_equal(lens, prompt_lengths(1024, seed=5, s_avg=s_avg, s_max=s_max))      # seeded
        assert not np.array_equal(lens, prompt_lengths(1024, seed=6, s_avg=s_avg, s_max=s_max))
        mbs, aborted = batch_requests([Request(i, int(v)) for i, v in enumerate(lens)], 8, 128, gen_len=64, cache_size=1 << 40)
        tokens = [mb.prompt_tokens for mb in mbs]
        assert not aborted and sum(tokens) == lens.sum() and max(tokens) - min(tokens) <= s_max
