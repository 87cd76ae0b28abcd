import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


_capture_manager = None


def progress(msg):
    """A progress line of a long test that reaches the terminal even while pytest captures output (a run that
    prints nothing for minutes is taken for a hung one), and a log file in the run's output folder if that
    folder exists.  Called by the work itself (a layer checked, a stage uploaded), never from a timer."""
    line = f"[progress] {msg}"
    if _capture_manager is not None:
        with _capture_manager.global_and_fixture_disabled():
            print(line, file=sys.stderr, flush=True)
    else:
        print(line, file=sys.stderr, flush=True)
    out_dir = os.path.join(ROOT, "gpurun_out")
    if os.path.isdir(out_dir):
        try:
            with open(os.path.join(out_dir, "test_progress.log"), "a") as f:
                f.write(line + "\n")
        except OSError:
            pass


def pytest_configure(config):
    global _capture_manager
    _capture_manager = config.pluginmanager.getplugin("capturemanager")
    config.addinivalue_line("markers", "gpu: needs a MI355X; runs the HIP path through the C ABI")
    config.addinivalue_line("markers", "slow: full-size model workloads (minutes)")


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)
