"""Reader for workloads/calib.json (per-tensor scales written by oracle/calibrate.py).
Plain data access: the scales are inputs to the layers on both the CPU-oracle and GPU side."""
import json
import os

_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "calib.json")
_cache = None


def load():
    global _cache
    if _cache is None:
        with open(_PATH) as f:
            _cache = json.load(f)
    return _cache
