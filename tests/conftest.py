import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _plant_oracle_mistake(spec: str) -> None:
    """JSON ``[module, old, new]``: re-executes ``oracle/<module>.py`` with one piece of its source replaced.  Only
    ``test_oracle_mutations.py`` sets this (in child processes), to show that the pins catch the mistake."""
    import importlib
    import json
    module, old, new = json.loads(spec)
    m = importlib.import_module("oracle." + module)
    with open(m.__file__) as f:
        src = f.read()
    if old not in src:
        raise RuntimeError(f"planted mistake does not apply: {old!r} not in oracle/{module}.py")
    exec(compile(src.replace(old, new, 1), m.__file__, "exec"), m.__dict__)


if os.environ.get("SPIN_ORACLE_MUTATION"):
    _plant_oracle_mistake(os.environ["SPIN_ORACLE_MUTATION"])


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the GPU box)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are only meaningful where a device is visible.
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
