"""Progress lines of long tests.  A full-size parity test spends minutes inside the fp64 oracle; with pytest's output
capture on, nothing it prints is seen until it ends, and a run that is silent for minutes looks hung to whoever
watches it.  `progress` writes one line to the real stdout, capture or not; tests call it at the steps of their own
work (weights drawn, oracle done, GPU done)."""

import time

_capture_manager = None
_t0 = time.time()


def set_capture_manager(manager):
    global _capture_manager
    _capture_manager = manager


def progress(msg):
    if _capture_manager is None:
        print(msg, flush=True)
        return
    with _capture_manager.global_and_fixture_disabled():
        print(f"\n[progress +{time.time() - _t0:.0f}s] {msg}", end="", flush=True)
