"""The C ABI from the C side: ppsd_cli (plain C++, links libppsd.so through include/ppsd.h only) decodes workload C1
in every schedule and must commit one token stream (the method is lossless, Sec. 5.1), also through
ppsd_decode_static_scratch and with direct launches."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLI = os.path.join(ROOT, "paper_2509_19368_amd", "ppsd_cli")


def _run(*args):
    if not os.path.exists(CLI):
        pytest.fail(f"{CLI} is missing: build it with `python -m paper_2509_19368_amd.build`")
    res = subprocess.run([CLI, *args], capture_output=True, text=True, timeout=240)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-2000:]
    return res.stdout


def test_every_schedule_commits_one_stream_from_c():
    out = _run("C1", "--check")
    assert "check ok" in out and "MISMATCH" not in out
    for name in ("vanilla", "serial", "overlap", "pipeline"):
        assert name in out


def test_static_scratch_and_direct_launches_from_c():
    a = _run("C1", "--check", "--static-scratch")
    b = _run("C1", "--check", "--no-graph")
    assert "check ok" in a and "check ok" in b


def test_three_stage_partition_and_bad_arguments_from_c():
    out = _run("C1", "--mode", "pipeline", "--later-stage", "2", "--decode", "40")
    assert "pipeline" in out and "streams 3" in out
    res = subprocess.run([CLI, "C1", "--mode", "pipeline", "--later-stage", "99"], capture_output=True, text=True, timeout=60)
    assert res.returncode == 4 and "pipeline_stage_layers" in res.stderr
