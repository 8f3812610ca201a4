"""Progress lines and measured-gap records of the GPU tests.

pytest captures what a test prints, so a test that works silently for minutes
looks hung from outside.  ``say`` therefore writes every line three ways: to
stderr (shown with a failure), to the terminal with capturing suspended, and
to ``gpu_test_progress.log`` in the results folder ``OUT_DIR`` under the repository root.
``record`` keeps measured quantities (strip-set gaps, score errors) in
``parity_gaps.json`` in the same folder so that they can be quoted afterwards.
"""
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT_DIR = os.path.join(ROOT, "gpurun_out")
_config = None
_t0 = time.time()


def set_config(config) -> None:
    global _config
    _config = config


def _to_file(name: str, text: str, mode: str = "a") -> None:
    try:
        os.makedirs(OUT_DIR, exist_ok=True)
        with open(os.path.join(OUT_DIR, name), mode) as f:
            f.write(text)
    except OSError:
        pass


def say(msg: str) -> None:
    line = f"[gpu-case +{time.time() - _t0:6.1f}s] {msg}"
    print(line, file=sys.stderr, flush=True)
    _to_file("gpu_test_progress.log", line + "\n")
    cap = _config.pluginmanager.getplugin("capturemanager") if _config is not None else None
    if cap is not None:
        with cap.global_and_fixture_disabled():
            print(line, flush=True)


def record(key: str, value) -> None:
    """Store ``value`` (JSON-serialisable) under ``key`` in ``OUT_DIR``/parity_gaps.json."""
    path = os.path.join(OUT_DIR, "parity_gaps.json")
    data = {}
    try:
        with open(path) as f:
            data = json.load(f)
    except (OSError, ValueError):
        pass
    data[key] = value
    _to_file("parity_gaps.json", json.dumps(data, indent=1, sort_keys=True) + "\n", mode="w")
