"""The pins are only worth something if a wrong oracle fails them: every mistake planted by oracle/mutation_check.py
(in a temporary copy of the oracle, on the CPU) must make some CPU test fail, and the mutants it marks as equivalent
must not.  Each mutant is one run of the CPU suite in a child process; they run a few at a time."""
from oracle import mutation_check


def test_every_planted_mistake_fails_a_pin():
    res = mutation_check.run(jobs=4)
    assert len(res) >= 30
    broken = [(n, msg) for n, caught, msg, _ in res if caught is None]
    assert not broken, broken
    missed = [n for n, caught, _, equiv in res if not caught and not equiv]
    assert not missed, missed
    wrongly_marked = [n for n, caught, _, equiv in res if caught and equiv]
    assert not wrongly_marked, wrongly_marked
