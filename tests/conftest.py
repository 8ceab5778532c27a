import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: test needs a real MI355X (run with -m gpu)")


HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="session")
def aten_philox(tmp_path_factory):
    """Independent Philox4x32-10: ATen's header-only engine compiled into a tiny CLI."""
    import torch

    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    exe = str(tmp_path_factory.mktemp("pin") / "pin_philox_aten")
    subprocess.run(["g++", "-std=c++17", "-O1", "-I" + inc,
                    os.path.join(HERE, "pin_philox_aten.cpp"), "-o", exe], check=True)

    def run(triples):
        text = "".join(f"{s} {q} {o}\n" for s, q, o in triples)
        out = subprocess.run([exe], input=text, capture_output=True, text=True, check=True)
        rows = [list(map(int, line.split())) for line in out.stdout.strip().splitlines()]
        assert len(rows) == len(triples)
        return rows

    return run
