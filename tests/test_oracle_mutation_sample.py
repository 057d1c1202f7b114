"""Do the pins catch a mistake?  A bounded sample of the mutation check (every 45th mutant of
tests/oracle_mutation_check.py: one small mistake planted in a copy of the oracle's C source,
the copy built and the pins run against it).  A sampled mutant may survive only if its mutated
line is on the committed list of mutants that change nothing a caller can see
(tests/golden/oracle_mutation_survivors.txt, written by a full run of that script)."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, HERE)

import oracle_mutation_check as mc  # noqa: E402


def test_sampled_mutants_are_killed_or_known_to_be_harmless():
    allowed = {line.strip() for line in open(mc.SURVIVORS) if line.strip() and not line.startswith("#")}
    todo = mc.all_mutants()
    assert len(todo) > 800
    sample = todo[7::45]
    assert 15 <= len(sample) <= 30
    res = mc.run_mutants(sample, workers=4, threads_each=2)
    killed = [r for r in res if r[2] == "killed"]
    unexpected = [(ln + 1, new.strip()) for ln, new, verdict in res
                  if verdict == "survived" and new.strip() not in allowed]
    assert not unexpected, f"mutants that pass every pin and are not known to be harmless: {unexpected}"
    assert len(killed) >= len(sample) // 2      # the sample is not made of equivalent mutants
