#!/usr/bin/env python3
"""One-GPU benchmark of the MORLAX update step (paper Sec. III-C) on synthetic trajectories.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--no-cpu-baseline]

A step is one pass of the whole hot path: two hypernet forwards, the rollout forward of the actor
(sampling actions and their log-density) and critic families over all T x N cells, the vector GAE scan,
then for every epoch and minibatch hypernet forward, grouped forward, clipped-PPO / value loss, grouped
backward and hypernet backward for both nets.  No optimiser step (the gradients are the product).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published dense peaks used for the roofline fractions
PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
# grouped-GEMM launch kinds -> kernel that serves them (bf16 at full size: the persistent direct-to-LDS
# kernel; small or fp32 problems: k_gemm_dma / k_grouped_gemm)
KERNEL_OF_KIND = {
    "fwd_first": "k_grouped_gemm<x rows, W0(p), EpiFwd> forward, first layer",
    "fwd_hidden": "k_gemm_pers<SRC_KCONTIG, SRC_KCONTIG, EpiFwd> forward, W x W layers (rollout + update)",
    "dx_hidden": "k_gemm_pers<SRC_KCONTIG, SRC_KSTRIDED, EpiDx> dX, W x W layers",
    "dw_hidden": "k_gemm_pers<SRC_KSTRIDED, SRC_KSTRIDED, EpiDw> dW, W x W layers",
    "dw_first": "k_grouped_gemm<SRC_KSTRIDED, SRC_X_KSTRIDED, EpiDw> dW, first layer",
}

# HBM bytes per launch of a GEMM launch kind, from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this script scaled by
# a copy of known size (profiles/grouped_gemm_cfg5_hbm_traffic.txt); workloads without such a run report null
MEASURED_TRAFFIC_BYTES = {("cfg5-largest-K6-P128-N16384-T64-4x512-silu-bf16-4mbx2ep", "fwd_hidden"): 1073.3e6}


def cpu_baseline(cfg_full):
    """The oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np
    from oracle import morlax_oracle as orc
    from paper_2603_09237_amd import inputs
    from paper_2603_09237_amd.configs import scaled
    try:
        from threadpoolctl import threadpool_info
        threads = max([int(i.get("num_threads", 1)) for i in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    # sample: the first P_s preferences with their n_g environments each, all T, all minibatches/epochs
    flops_full = cfg_full.P * cfg_full.n_g * cfg_full.T * cfg_full.width ** 2 * cfg_full.n_hidden * 2.0 * 2 * \
        (1 + 3 * cfg_full.epochs)
    p_s = int(max(2, min(cfg_full.P, round(cfg_full.P * 1.5e12 / max(flops_full, 1.0)))))
    cfg = scaled(cfg_full, P=p_s, N=p_s * cfg_full.n_g, name=cfg_full.name + f"-sample-P{p_s}")
    d = inputs.make_all(cfg)
    t0 = time.perf_counter()
    orc.update_step(cfg, d["w"], d["hparams_actor_old"], d["hparams_critic_old"], d["hparams_actor"],
                    d["hparams_critic"], d["obs"], d["rewards"], d["dones"], d["eps"], cfg.gamma, cfg.lam,
                    cfg.clip_eps, cfg.minibatches, cfg.epochs, emulate_bf16=(cfg.wdtype == 1))
    dt = time.perf_counter() - t0
    return {"value": cfg.T * cfg.N / dt, "unit": "env-steps/s", "cores": threads, "kind": "oracle",
            "sample": f"one update step on P={p_s} of {cfg_full.P} preferences (N={cfg.N} of {cfg_full.N} "
                      f"environments, all T={cfg.T} steps, {cfg.minibatches} minibatches x {cfg.epochs} epochs); "
                      f"cost per env-step does not depend on P; {dt:.1f} s of numpy float64"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--streams", type=int, default=1, choices=(1, 2),
                    help="1 (default): every launch on one stream, so that the per-kernel durations behind `roofline` are "
                         "those of kernels running alone; 2: actor and critic chains on their own HIP streams (faster "
                         "step, but concurrent kernels stretch each other's durations)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device copy (a kernel of known traffic, to scale hardware byte counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (collectives and sharding are not part of it); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_09237_amd import inputs
    from paper_2603_09237_amd.configs import CONFIGS
    from paper_2603_09237_amd.step import UpdateStep

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    cfg = CONFIGS[a.config]
    st = UpdateStep(cfg, two_streams=(a.streams == 2))
    st.load_inputs(inputs.make_all(cfg))
    torch.cuda.synchronize()
    for _ in range(a.warmup):
        st.run()
    torch.cuda.synchronize()
    if a.calib_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    st.ctx.profile_begin()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        st.run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = st.ctx.profile_end()

    env_steps = cfg.T * cfg.N
    dtype = "bf16" if cfg.wdtype == 1 else "f32"
    kind = max(prof, key=lambda k: prof[k][0])
    ms, launches, flops = prof[kind]
    gemm_ms = sum(v[0] for v in prof.values())
    peak = PEAK_TFLOPS[dtype]
    achieved = flops / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
    out = {
        "metric": "env_steps_per_sec_per_update_step",
        "value": env_steps * a.steps / dt,
        "unit": "env-steps/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": dt / a.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "K": cfg.K, "P": cfg.P, "N": cfg.N, "T": cfg.T, "obs_dim": cfg.obs_dim,
                   "act_dim": cfg.act_dim, "mlp": f"{cfg.n_hidden}x{cfg.width}", "rank": cfg.rank,
                   "minibatches": cfg.minibatches, "epochs": cfg.epochs, "env_steps_per_step": env_steps,
                   "optimizer_step": "not included"},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": MEASURED_TRAFFIC_BYTES.get((cfg.name, kind)),
                     "kernel": KERNEL_OF_KIND[kind], "launches_per_step": launches / a.steps,
                     "avg_launch_ms": ms / max(launches, 1), "flop_per_launch": flops / max(launches, 1),
                     "all_gemm_ms_per_step": gemm_ms / a.steps,
                     "all_gemm_tflops": sum(v[2] for v in prof.values()) / (gemm_ms * 1e-3) / 1e12 if gemm_ms else 0.0,
                     "per_kind_ms_per_step": {k: v[0] / a.steps for k, v in prof.items()}},
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
