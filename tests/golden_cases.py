"""Reader for tests/golden/worked_examples.txt (hand-derived fixtures)."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "worked_examples.txt")

_VEC_KEYS = ("x", "min", "max", "scale", "zero_point", "given_scale", "given_zero_point",
             "codes", "xhat", "mask")


def load_cases(path=GOLDEN):
    cases, cur = [], None
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, rest = line.partition(" ")
            if key == "case":
                cur = {"name": rest.strip()}
                cases.append(cur)
            elif key == "bits":
                cur["bits"] = int(rest)
            elif key == "dtype":
                cur["dtype"] = rest.strip()
            elif key == "shape":
                cur["shape"] = tuple(int(t) for t in rest.split())
            elif key in _VEC_KEYS:
                cur[key] = np.array([float(t) for t in rest.split()], dtype=np.float64)
            else:
                raise ValueError("unknown key %r in %s" % (key, path))
    return cases


def to_storage(values, dtype):
    """float values -> the array the oracle / library takes (float32, or uint16 bf16 bits)."""
    f = np.asarray(values, np.float32)
    if dtype == "f32":
        return f
    bits = f.view(np.uint32)
    assert not np.any(bits & 0xFFFF), "fixture value is not bfloat16-representable"
    return (bits >> 16).astype(np.uint16)


def from_storage(arr):
    if arr.dtype == np.uint16:
        return (arr.astype(np.uint32) << 16).view(np.float32)
    return arr
