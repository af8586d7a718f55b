import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

_config = None
_last = [0.0]


def pytest_configure(config):
    global _config
    _config = config
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def progress(msg, every=20.0):
    """A line on the real terminal (past pytest's capture), at most one per `every` seconds: long checks
    (the full-size steps compare gigabytes of tensors on the CPU) show that they are alive."""
    now = time.time()
    if now - _last[0] < every:
        return
    _last[0] = now
    line = "[%s] %s" % (time.strftime("%H:%M:%S"), msg)
    capman = _config.pluginmanager.getplugin("capturemanager") if _config is not None else None
    if capman is not None:
        with capman.global_and_fixture_disabled():
            print(line, flush=True)
    else:
        print(line, flush=True)
