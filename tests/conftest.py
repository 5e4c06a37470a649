import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    _sanitizer_run()


def _sanitizer_run():
    """CPU sanitizer job.  With PCG_SANITIZE=1 the CPU suite runs against builds of the oracle and
    of libpcg's host side that carry AddressSanitizer and UndefinedBehaviorSanitizer (made here if
    missing or stale).  An instrumented library can only be loaded into a Python that has the
    sanitizer runtime preloaded, so the whole run is started as

        LD_PRELOAD=$(python -c "from paper_2511_13732_amd import build; print(build.asan_runtime())")${LD_PRELOAD:+:$LD_PRELOAD} \\
        ASAN_OPTIONS=detect_leaks=0 PCG_SANITIZE=1 python -m pytest tests -q -m "not gpu"

    (leak detection off: the interpreter itself does not free everything at exit).  Any finding
    aborts the process with the sanitizer's report."""
    from paper_2511_13732_amd import build as hip_build
    if not hip_build.sanitize_requested():
        return
    runtime = hip_build.asan_runtime()
    if os.path.basename(runtime) not in os.environ.get("LD_PRELOAD", ""):
        raise pytest.UsageError(
            f"PCG_SANITIZE=1 needs the sanitizer runtime preloaded: run with LD_PRELOAD={runtime} "
            "ASAN_OPTIONS=detect_leaks=0 (prepend to any LD_PRELOAD that is already set)")
    if (not os.path.exists(hip_build.LIB_SAN)
            or any(os.path.getmtime(os.path.join(hip_build.CSRC, f)) > os.path.getmtime(hip_build.LIB_SAN)
                   for f in hip_build.SOURCES + hip_build.HEADERS)):
        hip_build.build(sanitize=True)
    import oracle
    oracle.build()


def pytest_collection_modifyitems(config, items):
    import torch
    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
