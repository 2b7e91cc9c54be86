import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


TUNING_KEYS = ("SEGKV_TARGET_GROUPS", "SEGKV_MIN_PCHUNK", "SEGKV_PATH", "SEGKV_MFMA_WAVES",
               "SEGKV_HEADS_PER_WAVE", "SEGKV_PAIR_HEADS", "SEGKV_PREFILL", "SEGKV_XCD_HEAD_ORDER")


@pytest.fixture
def planner_env():
    """Force the launch planner through the library's test-only overrides: they are read
    from the environment once, so every change is followed by segkv_reload_tuning()."""
    import paper_2401_05391_amd as segkv
    lib = segkv.load_library()
    saved = {k: os.environ.get(k) for k in TUNING_KEYS}

    def set_env(**kw):
        for k, v in kw.items():
            assert k in TUNING_KEYS, k
            os.environ[k] = str(v)
        lib.segkv_reload_tuning()
    yield set_env
    for k, v in saved.items():
        if v is None:
            os.environ.pop(k, None)
        else:
            os.environ[k] = v
    lib.segkv_reload_tuning()
