"""Reader for the small text fixtures under tests/golden/."""
import os

_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_records(name):
    """`group key v1 v2 ...` lines -> {group: {key: [float, ...]}}; '#' starts a comment."""
    out = {}
    with open(os.path.join(_DIR, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            parts = line.split()
            out.setdefault(parts[0], {})[parts[1]] = [float(x) for x in parts[2:]]
    return out
