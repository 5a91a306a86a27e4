import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests need the card; everything else runs anywhere.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_sessionfinish(session, exitstatus):
    """bf16 parity comparisons of this run as a table, parity_bf16.md in the directory that the
    environment variable MC_TEST_REPORT_DIR names (nothing is written without it): per comparison
    the device's and the noise floor's distance from the exact oracle, the bound that applied and
    the statistics with power."""
    try:
        import gpu_common
    except Exception:
        return
    recs = gpu_common.PARITY_RECORDS
    if not recs:
        return
    out_dir = os.environ.get("MC_TEST_REPORT_DIR")
    if not out_dir:
        return
    try:
        os.makedirs(out_dir, exist_ok=True)
        with open(os.path.join(out_dir, "parity_bf16.md"), "w") as f:
            f.write("| comparison | rows x cols | max-abs | floor max-abs | rel L2 | floor rel L2 | bound used | "
                    "RMS / floor RMS | worst row | bias / RMS | frac > 2e-2 | floor frac > 2e-2 | floor frac > 1.6e-2 |\n")
            f.write("|---|---|---|---|---|---|---|---|---|---|---|---|---|\n")
            for r in recs:
                f.write(f"| {r['what']} | {r['rows']} x {r['cols']} | {r['err']:.2e} | {r['floor_err']:.2e} | {r['rel']:.2e} | "
                        f"{r['floor_rel']:.2e} | {r['which']} | {r['rms_ratio']:.2f} | {r['rms_ratio_row']:.2f} | "
                        f"{r['bias']:.3f} | {r['frac']:.1e} | {r['floor_frac']:.1e} | {r['floor_frac_scaled']:.1e} |\n")
    except OSError:
        pass
