"""Reader for the tiny text fixtures under tests/golden/."""
import os

HERE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load(name):
    out = {}
    with open(os.path.join(HERE, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, vals = line.split(":", 1)
            nums = [float(v) for v in vals.split()]
            out[key.strip()] = nums[0] if len(nums) == 1 else nums
    return out
