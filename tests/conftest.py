import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _parse_mesh(text):
    mesh = {}
    for tok in text.split():
        name, size = tok.split(":")
        mesh[name] = int(size)
    return mesh


def load_chains():
    """Blocks of tests/golden/paper_chains.txt -> dicts(cite, mesh, start, steps=[(op, args, type_text)])."""
    blocks, cur = [], None
    with open(os.path.join(GOLDEN, "paper_chains.txt")) as fh:
        for raw in fh:
            line = raw.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("cite:"):
                cur = {"cite": line[5:].strip(), "mesh": None, "start": None, "steps": [], "_op": None}
                blocks.append(cur)
            elif line.startswith("mesh:"):
                cur["mesh"] = _parse_mesh(line[5:])
            elif line.startswith("["):
                if cur["start"] is None:
                    cur["start"] = line
                else:
                    op = cur["_op"]
                    cur["steps"].append((op[0], op[1:], line))
                    cur["_op"] = None
            else:
                cur["_op"] = line.split()
    for b in blocks:
        b.pop("_op")
    return blocks


def load_values():
    out = {}
    with open(os.path.join(GOLDEN, "paper_values.txt")) as fh:
        for raw in fh:
            line = raw.strip()
            if not line or line.startswith("#"):
                continue
            key, val, _cite = [p.strip() for p in line.split("|")]
            out[key] = val
    return out


@pytest.fixture(scope="session")
def paper_chains():
    return load_chains()


@pytest.fixture(scope="session")
def paper_values():
    return load_values()


def parse_mesh(text):
    return _parse_mesh(text)
