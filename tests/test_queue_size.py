"""Queue-depth rule (paper Eq. 22-23): oracle pinned by the paper's worked example, library checked
against the oracle.  Host arithmetic only - runs without a GPU."""
import math
import os
import random

import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
MB, GB = 10 ** 6, 10 ** 9


def worked_examples():
    rows = []
    for line in open(os.path.join(HERE, "golden", "queue_size_worked_example.txt")):
        if line.strip() and not line.startswith("#"):
            name, prep, comp, peak, total, q = line.split()
            rows.append((name, float(prep), float(comp), float(peak), float(total), int(q)))
    return rows


def test_oracle_reproduces_the_papers_worked_example():
    rows = worked_examples()
    assert rows
    for name, prep, comp, peak_mb, total_gb, printed in rows:
        for margin in (5, 10):                                    # the paper's 5-10 % safety margin
            for per_batch in (50 * MB, 561 * MB, 2 * GB):
                q, cap = oracle.queue_size(prep, comp, int(total_gb * GB), int(peak_mb * MB), margin, per_batch)
                assert q == printed, (name, margin, per_batch, q)
                assert cap > printed


def test_oracle_closed_forms():
    # never below 2 when memory allows; capped by memory; ceil, not round
    assert oracle.queue_size(1.0, 10.0, 100 * GB, 1 * GB, 10, 1 * GB) == (2, 98)
    assert oracle.queue_size(30.0, 10.0, 100 * GB, 1 * GB, 10, 1 * GB)[0] == 3
    assert oracle.queue_size(30.0001, 10.0, 100 * GB, 1 * GB, 10, 1 * GB)[0] == 4
    assert oracle.queue_size(1000.0, 1.0, 10 * GB, 1 * GB, 10, 1 * GB) == (8, 8)      # floor(8.9) = 8
    assert oracle.queue_size(1000.0, 1.0, 2 * GB, 1 * GB, 0, 1 * GB) == (1, 1)
    assert oracle.queue_size(1000.0, 1.0, 2 * GB, 1 * GB, 5, 1 * GB) == (0, 0)


def test_library_matches_oracle():
    from paper_2601_04707_amd import mqg
    for name, prep, comp, peak_mb, total_gb, printed in worked_examples():
        assert mqg.mqg_queue_size(prep, comp, int(total_gb * GB), int(peak_mb * MB), 10, 561 * MB)[0] == printed
    rnd = random.Random(0)
    for _ in range(3000):
        prep = rnd.uniform(0.01, 500.0)
        comp = rnd.uniform(0.01, 50.0)
        total = rnd.randrange(1, 300) * GB + rnd.randrange(0, GB)
        peak = rnd.randrange(0, total // 2)
        margin = rnd.randrange(0, 11)
        per = rnd.randrange(1, 4 * GB)
        assert mqg.mqg_queue_size(prep, comp, total, peak, margin, per) == oracle.queue_size(prep, comp, total, peak, margin, per)
    # exact multiples: ceil must not overshoot
    for k in range(1, 40):
        assert mqg.mqg_queue_size(k * 2.5, 2.5, 288 * GB, GB, 10, GB)[0] == max(2, k)


def test_library_refuses_bad_arguments():
    from paper_2601_04707_amd import mqg
    for args in [(0.0, 1.0, GB, 0, 5, MB), (1.0, 0.0, GB, 0, 5, MB), (1.0, 1.0, 0, 0, 5, MB), (1.0, 1.0, GB, 0, 5, 0),
                 (1.0, 1.0, GB, 0, 101, MB), (1.0, 1.0, GB, 2 * GB, 5, MB), (float("nan"), 1.0, GB, 0, 5, MB)]:
        with pytest.raises(mqg.MqgError) as e:
            mqg.mqg_queue_size(*args)
        assert e.value.code == mqg.MQG_ERR_INVALID_ARG
