"""Writes tests/golden/schedule_pins.json from the oracle alone (run from the repo root:
`python tests/golden/make_schedule_golden.py`).  The stored lists freeze the canonical reading of
Algorithm 1 / Algorithm 2 / Fig. 4 so that an accidental change of the oracle shows up as a diff;
their validity is established separately by the brute-force tests."""
import hashlib
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import schedule as sch  # noqa: E402


def digest(rings):
    return hashlib.sha256(",".join(str(x) for ring in rings for x in ring).encode()).hexdigest()


def main():
    pins = {"rings": {}, "sha256": {}, "arrival": {}, "out_mapping": {}, "in_mapping": {}}
    for n in (4, 8, 16):
        rings = sch.hamilton_rings(n)
        pins["rings"][str(n)] = rings
        pins["out_mapping"][str(n)] = sch.out_mapping(rings)
        pins["in_mapping"][str(n)] = sch.in_mapping(rings)
    for n in (4, 8, 12, 16, 20, 24, 32, 64):
        pins["sha256"][str(n)] = digest(sch.hamilton_rings(n))
    for n, rank in ((4, 0), (8, 3), (8, 0), (16, 5), (8, 7)):
        pins["arrival"]["%d/%d" % (n, rank)] = sch.arrival_table(sch.hamilton_rings(n), rank)
    path = os.path.join(ROOT, "tests", "golden", "schedule_pins.json")
    with open(path, "w") as f:
        json.dump(pins, f, separators=(",", ":"))
        f.write("\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
