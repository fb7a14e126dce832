"""The C ABI from a plain C program: no PyTorch, hipMalloc memory, the library's own allocation fallback.

(The file name sorts before the other GPU tests on purpose: the program is started as a child process while
this process has not touched the GPU yet.)"""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "c_abi", "abi_example")


def expected_lines():
    with open(os.path.join(ROOT, "tests", "golden", "abi_example_expected.txt")) as fh:
        return [l.strip() for l in fh if l.strip() and not l.startswith("#")]


def test_expected_text_matches_the_oracle():
    """The hand-derived text is what the oracle gives for the same matrix (CPU only)."""
    import numpy as np
    from oracle import unisparse_oracle as O
    r = np.array([2, 4, 0, 2, 1, 2], np.int32); c = np.array([3, 3, 0, 1, 1, 2], np.int32)
    v = np.array([5, 6, 1, 3, 2, 4], np.float32); x = np.array([1, 10, 100, 1000], np.float32)
    csr = O.convert(5, 4, r, c, v, O.CSR()); dia = O.convert(5, 4, r, c, v, O.DIA())
    fmt = lambda name, a: name + " " + " ".join(f"{t:g}" for t in a)
    got = [fmt("csr.ptr", csr.levels[1].ptr), fmt("csr.idx", csr.levels[1].idx), fmt("csr.val", csr.val),
           fmt("y", O.spmv(csr, x)), fmt("dia.offsets", dia.levels[0].idx), fmt("dia.val", dia.val),
           fmt("y_dia", O.spmv(dia, x)), "bad US_ERR_INDEX_RANGE"]
    assert got == expected_lines()


@pytest.mark.gpu
def test_plain_c_program_drives_the_library():
    assert os.path.exists(EXE), "tests/c_abi/abi_example is built by __graft_entry__.build()"
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    assert [l.strip() for l in r.stdout.splitlines() if l.strip()] == expected_lines()
