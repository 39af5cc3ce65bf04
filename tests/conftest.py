import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny_model_cpu():
    """Tiny config: canonical CPU tensors + oracle model (bf16 weights, seed 0x2505)."""
    from paper_2505_22758_amd import synth
    from oracle import oracle
    S = synth.TINY
    seed = 0x2505
    layers = [synth.make_layer(S, seed, l, synth.WDTYPE_BF16, "cpu") for l in range(S.n_layers)]
    head = synth.make_head(S, seed, synth.WDTYPE_BF16, "cpu")
    return S, seed, layers, head, oracle.OracleModel(S, layers, head)
