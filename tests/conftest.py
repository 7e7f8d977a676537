import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: full-size case, minutes of host time")


def pytest_collection_modifyitems(config, items):
    # GPU tests are selected explicitly with -m gpu; without a device they are skipped, not failed.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


@pytest.fixture(autouse=True)
def _parity_report(request):
    """After every GPU test: one line saying what its comparisons with the oracle really covered."""
    try:
        from tests import gpu_util
    except Exception:
        yield
        return
    gpu_util.REPORT.clear()
    yield
    if not gpu_util.REPORT:
        return
    import json
    kinds = {}
    for k, rec in gpu_util.REPORT:
        kinds.setdefault(k, []).append(rec)
    parts = []
    if "logits" in kinds:
        L = kinds["logits"]
        parts.append(f"logit checks {len(L)}: max abs err {max(r['err'] for r in L):.3g}, max err/range "
                     f"{max(r['err'] / max(r['range'], 1e-30) for r in L):.3g}")
    if "ids" in kinds:
        I = kinds["ids"]
        parts.append(f"argmax rows held exact {sum(r['compared'] for r in I)}/{sum(r['rows'] for r in I)}, "
                     f"in the band between 1e-2 and the id margin {sum(r['band'] for r in I)} "
                     f"(of them different {sum(r['band_mismatch'] for r in I)})")
    if "step" in kinds:
        S = kinds["step"]
        parts.append(f"steps {len(S)}: revealed set held against the oracle's in {sum(r['set_compared'] for r in S)} "
                     f"(equal in {sum(r['set_equal'] for r in S)}); candidate rows held exact {sum(r['id_rows'] for r in S)}/"
                     f"{sum(r['rows'] for r in S)}, band {sum(r['band'] for r in S)} (different {sum(r['band_mismatch'] for r in S)}); "
                     f"max conf rel err {max(r['cerr'] for r in S):.3g}")
    if "carry" in kinds:
        K = kinds["carry"]
        parts.append(f"carry checks {len(K)} (id held exact in {sum(r['compared'] for r in K)})")
    if "count" in kinds:
        parts += [f"{r['what']} {r['n']}" for r in kinds["count"]]
    line = f"[parity] {request.node.name}: " + "; ".join(parts)
    print(line, flush=True)
    try:
        os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(ROOT, "gpurun_out", "parity_report.jsonl"), "a") as f:
            f.write(json.dumps({"test": request.node.name, "records": gpu_util.REPORT}) + "\n")
    except OSError:
        pass
