import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionfinish(session, exitstatus):
    """After a GPU session: the two margins (worst error / bound) of every oracle comparison, worst first,
    to gpurun_out/parity_margins.txt (the scratch folder of GPU runs; nothing reads it back)."""
    mod = sys.modules.get("test_gpu_parity")
    margins = getattr(mod, "MARGINS", None)
    if not margins:
        return
    try:
        out_dir = os.path.join(ROOT, "gpurun_out")
        os.makedirs(out_dir, exist_ok=True)
        with open(os.path.join(out_dir, "parity_margins.txt"), "w") as f:
            f.write("# primary = max|err| / (tol * max|ref|), guard = max over elements of |err| / guard bound\n")
            for what, dtype, primary, guard in sorted(margins, key=lambda m: -max(m[2], m[3])):
                f.write(f"{primary:6.3f} {guard:6.3f} {dtype:5s} {what}\n")
    except OSError:
        pass
