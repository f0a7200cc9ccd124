import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped (not failed) where no GPU is visible."""
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(autouse=True)
def _library_switches_at_their_defaults(request):
    """The library's three process-wide test and tuning switches (forced GEMM variant, forced attention kernel, bound of
    the log-softmax waits) are put back after every GPU test, whatever the test did with them, so that no test changes
    what a later one runs or measures."""
    yield
    if "gpu" not in request.keywords:
        return
    from paper_2511_17826_amd import binding as tb
    tb.tbik_set_gemm_variant(tb.VARIANT_AUTO)
    tb.tbik_set_attention_variant(0)
    tb.tbik_set_row_wait_limit(1 << 14)


def read_tree_pins():
    """Parse tests/golden/tree_pins.txt -> list of (name, [float32 leaves], T_bits, seq_bits)."""
    import numpy as np
    out = []
    with open(os.path.join(ROOT, "tests", "golden", "tree_pins.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, leaves, t_hex, s_hex = [c.strip() for c in line.split(";")]
            vals = []
            for tok in leaves.split():
                if tok == "0":
                    vals.append(np.float32(0.0))
                else:
                    e = int(tok[1:]) * (1 if tok[0] == "p" else -1)
                    vals.append(np.float32(2.0 ** e))
            out.append((name, vals, int(t_hex, 16), int(s_hex, 16)))
    return out
