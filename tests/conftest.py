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
    """A small Qwen3-shaped model: 2 layers, GQA group 2, head_dim 16, fp32 blob."""
    import synth
    return synth.ModelShape("tiny-f32", hidden=64, n_layers=2, n_q_heads=4, n_kv_heads=2,
                            head_dim=16, ffn=96, vocab=50, dtype=synth.F32)
