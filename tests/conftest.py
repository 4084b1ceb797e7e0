import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box only)")


def read_golden(name):
    """Rows of a '|'-separated golden file (comment and blank lines dropped, fields stripped)."""
    rows = []
    with open(os.path.join(GOLDEN, name), encoding="utf-8") as f:
        for line in f:
            line = line.rstrip("\n")
            if not line.strip() or line.startswith("#"):
                continue
            rows.append([field.strip() for field in line.split("|")])
    return rows


def parse_rows(spec):
    return [tuple(int(x) for x in row.split(":")) for row in spec.split(",") if row]


def parse_ids(spec):
    return [int(x) for x in spec.split(",") if x.strip()]
