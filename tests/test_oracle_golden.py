"""Change detector: the oracle still produces the digests stored by tests/golden/make_golden.py."""
import json
import os
import importlib.util

import numpy as np

from paper_2603_09237_amd import configs

HERE = os.path.dirname(os.path.abspath(__file__))


def test_cfg1_digest_unchanged():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    got = mod.digest(configs.CONFIGS[1])
    with open(os.path.join(HERE, "golden", "cfg1_update_step.json")) as f:
        ref = json.load(f)
    for k, v in ref.items():
        assert np.allclose(got[k], v, rtol=1e-9, atol=1e-12), k
