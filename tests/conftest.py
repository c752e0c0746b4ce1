import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny_shape():
    """A small GQA decoder that the no-cache brute force finishes in seconds."""
    import synth_inputs as S
    return S.Workload("tiny", n_layers=3, exit_layer=1, d_model=32, n_heads=4, n_kv_heads=2,
                      head_dim=8, d_ffn=48, vocab=64, dtype="fp32", damp=0.3, seed=7,
                      prompt_len=5, decode_len=12)
