"""Writes tests/golden/cfg1_update_step.json from the CPU oracle alone.

Run from the repo root: `python tests/golden/make_golden.py`.  It imports only the oracle and
the seeded input generator; nothing here touches the HIP path.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import morlax_oracle as orc            # noqa: E402
from paper_2603_09237_amd import configs, inputs   # noqa: E402


def digest(cfg):
    d = inputs.make_all(cfg)
    res = orc.update_step(cfg, d["w"], d["hparams_actor_old"], d["hparams_critic_old"],
                          d["hparams_actor"], d["hparams_critic"], d["obs"], d["rewards"],
                          d["dones"], d["eps"], cfg.gamma, cfg.lam, cfg.clip_eps,
                          cfg.minibatches, cfg.epochs, keep=True)
    g = res["grads"][0]
    return {
        "stats": [float(x) for x in g["stats"]],
        "dhp_actor_l2": float(np.linalg.norm(g["dhp_actor"])),
        "dhp_critic_l2": float(np.linalg.norm(g["dhp_critic"])),
        "dhp_actor_first4": [float(x) for x in g["dhp_actor"][:4]],
        "adv_s_sum": float(res["adv_s"].sum()),
        "vtarg_l2": float(np.linalg.norm(res["vtarg"])),
        "logp_old_sum": float(res["logp_old"].sum()),
    }


if __name__ == "__main__":
    out = digest(configs.CONFIGS[1])
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg1_update_step.json"), "w") as f:
        json.dump(out, f, indent=1)
    print(json.dumps(out, indent=1))
