"""The (value, index) reduction rule of the head and commit kernels, compiled for the host and run on the CPU:
ties go to the lowest index, NaN never wins, and a row of NaN logits yields a token inside the vocabulary
(token 0), so the next step's embedding read cannot leave the table."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "host", "argmax_rule.hip")


@pytest.fixture(scope="module")
def rule(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("host") / "argmax_rule")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    res = subprocess.run([hipcc, "--cuda-host-only", "-O1", "-std=c++17", "-o", exe, SRC], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr

    def run(cases):
        text = "\n".join(f"{vocab} {len(v)} " + " ".join(str(x) for x in v) for vocab, v in cases) + "\n"
        out = subprocess.run([exe], input=text, capture_output=True, text=True, check=True).stdout.split("\n")
        return [tuple(int(t) for t in line.split()) for line in out if line.strip()]
    return run


def test_ties_nan_and_out_of_range_rows(rule):
    cases = [
        (8, [0.5, 2.0, 2.0, -1.0, 2.0, 0.0, 1.0, 1.5]),          # three equal maxima: the lowest index
        (8, ["nan", 1.0, "nan", 3.0, "nan", 3.0, 0.0, "nan"]),    # NaN never wins; tie among the finite ones
        (8, ["nan"] * 8),                                          # nothing wins: token 0, inside the vocabulary
        (8, ["-inf"] * 8),                                         # -inf equals the start value: lowest index wins
        (5, ["inf", 1.0, "inf", "nan", 2.0]),
        (3, [1.0, 5.0, 2.0, 9.0, 3.0]),                            # a candidate beyond the vocabulary cannot leave the rule
        (100, [float(i % 17) for i in range(100)]),
    ]
    want = [1, 3, 0, 0, 0, 0, 16]
    got = rule(cases)
    assert len(got) == len(want)
    for (a, b), w in zip(got, want):
        assert a == b == w, (a, b, w)
