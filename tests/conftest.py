import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


@pytest.fixture(scope="session")
def tiny_shape():
    from seeded_inputs import StageShape
    return StageShape("fd_tiny", n_layers=2, d_model=16, n_heads=2, head_dim=8, d_ffn=24, seq=6,
                      micro_batch=2, n_microbatches=2, dtype="f32", seed=7)
