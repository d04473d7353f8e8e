"""Reader for the small text fixtures under tests/golden/."""
import os


def read_replacement_traces(golden_dir):
    cases = []
    with open(os.path.join(golden_dir, "replacement_traces.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, acc, exp = [p.strip() for p in line.split(":")]
            policy, cap = head.split()
            accesses = [int(x) for x in acc.split()]
            expected = [tuple(int(v) for v in e.split(",")) for e in exp.split()]
            cases.append((policy, int(cap), accesses, expected))
    return cases
