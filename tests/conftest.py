import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny():
    """Config-0 workload with its three CPU-checker models and inputs."""
    from rsd_inputs import workload, model_weights_np, prompt_tokens, prompt_lengths, uniforms
    from oracle import rsd_oracle as O

    w = workload("cfg0")
    models = [O.OracleModel(s, model_weights_np(w.seed, i, s)) for i, s in enumerate(w.shapes)]
    return dict(w=w, models=models, tokens=prompt_tokens(w), lens=prompt_lengths(w),
                u_draft=uniforms(w, "U_DRAFT", w.max_ctx), u_target=uniforms(w, "U_TARGET", w.max_ctx),
                u_gate=uniforms(w, "U_GATE", w.max_steps))
