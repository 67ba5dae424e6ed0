"""Reader for the hand-worked cases in tests/golden/gac_len8_cases.txt."""
import os
from typing import Dict, List

_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "gac_len8_cases.txt")
_VECTORS = ("d", "g", "sums", "gprime")


def load_cases() -> List[Dict]:
    cases: List[Dict] = []
    cur: Dict = {}
    with open(_PATH) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = [s.strip() for s in line.split(":", 1)]
            if key == "case":
                cur = {"case": val}
                cases.append(cur)
            elif key in _VECTORS:
                cur[key] = [float(x) for x in val.split()]
            elif key == "regime":
                cur[key] = val
            else:
                cur[key] = float(val)
    return cases
