import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: CPU test that takes more than ~20 s")


@pytest.fixture(scope="session")
def codebooks():
    """Small K-Means codebooks from the oracle (fp16-representable), keyed by sub_dim."""
    from oracle import nsn_oracle as O
    from paper_2505_18231_amd import synth
    out = {}
    for sub in (4, 8):
        cb, _, _ = O.build_codebook(synth.codebook_samples(77, 1 << 14, sub), 256, 6)
        out[sub] = cb
    return out


@pytest.fixture(scope="session")
def gpu_api():
    import torch
    from paper_2505_18231_amd import api
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    api.lib()  # fails loudly if libnsn.so is not built
    return api


@pytest.fixture
def select_variant(gpu_api):
    """select_variant("decode", "lut") / ("encode", "valu") picks the alternative kernel for this test;
    the library's variants are back to what they were when the test ends."""
    api, saved = gpu_api, {}

    def pick(op_name, impl):
        op = {"encode": api.NSN_OP_ENCODE, "decode": api.NSN_OP_DECODE}[op_name]
        variant = api.NSN_VARIANT_ALT if impl in ("lut", "valu") else api.NSN_VARIANT_DEFAULT
        prev = api.nsn_select_variant(op, variant)
        saved.setdefault(op, prev)
    yield pick
    for op, prev in saved.items():
        api.nsn_select_variant(op, prev)
