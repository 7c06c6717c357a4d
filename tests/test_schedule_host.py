"""The library's host-side learning-rate helper (no GPU work) against the oracle's schedule (section 4.1)."""
import numpy as np
import pytest

from oracle import tsm_oracle as O
from paper_1910_00932_amd import binding as B


def test_lr_schedule_matches_oracle_over_a_run():
    for tb, wb in ((8, 8), (64, 8), (12288, 8), (512, 64)):
        for e in np.linspace(0.0, 101.0, 405):
            got, ref = B.tsm_lr_schedule(e, tb, wb), O.lr_schedule(e, tb, wb)
            assert abs(got - ref) <= 1e-15 + 1e-12 * abs(ref), (tb, wb, e, got, ref)
    assert abs(B.tsm_lr_schedule(3.0, 64, 8, 10.0, 50.0) - O.lr_schedule(3.0, 64, 8, 10.0, 50.0)) < 1e-15
    assert abs(B.tsm_lr_schedule(30.0, 64, 8, 10.0, 50.0) - O.lr_schedule(30.0, 64, 8, 10.0, 50.0)) < 1e-15


def test_lr_schedule_rejects_bad_arguments():
    for args in ((-1.0, 64, 8, 5.0, 100.0), (1.0, 0, 8, 5.0, 100.0), (1.0, 64, 0, 5.0, 100.0), (1.0, 64, 8, 5.0, 5.0)):
        with pytest.raises(B.TsmError):
            B.tsm_lr_schedule(*args)
