import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def has_gpu():
    import torch
    return torch.cuda.is_available()


def pytest_terminal_summary(terminalreporter):
    """GPU runs: the largest logit error each shape reached against the oracle (relative to the row's largest logit
    on the bf16 path, absolute on the fp32 path), next to the bounds the tests enforce."""
    try:
        import gpu_common
    except Exception:
        return
    if not gpu_common.ACHIEVED:
        return
    terminalreporter.write_line("achieved logit error per shape (fp32 path: absolute; bf16 path: relative to the row's "
                                "largest logit) and the bound enforced:")
    for name, err in sorted(gpu_common.ACHIEVED.items()):
        m = gpu_common.MEASURED.get(name)
        cap = gpu_common.FP32_ABS_BOUND if name in ("tiny", "fp32_gqa") else gpu_common.BF16_REL_BOUND
        terminalreporter.write_line("  %-24s %.3e   bound %s" % (name, err, ("%.1e" % min(cap, 10 * m)) if m else "default"))
