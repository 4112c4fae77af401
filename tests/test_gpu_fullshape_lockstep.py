"""Lock-step parity at the FULL row count and vocabulary width of the benchmark workloads: the HIP path and the CPU
oracle free-run several steps from the same seed on the same logits (drawn on the device in the recipe of the workload
and downloaded for the oracle), in the launch shape bench.py times, and are compared after every step: tokens,
ESS, resampling flags, ancestors, weights, sums, histories and live KV bytes, with only oracle-flagged excuses
(see test_gpu_trajectory).  The KV cache keeps its full row length but one head of one layer, so that the oracle's
copies fit comfortably in host memory.

cfg4 runs four steps of an exponent ramp (generic-exponent instantiation) and four at the held exponent 4 (the
integer instantiation on 4-wave workgroups, one per row, that the default bench line times) on all 2048 rows.
"""
import numpy as np
import pytest
import torch

from paper_2602_10273_amd import synth
from test_gpu_trajectory import run_lockstep

pytestmark = pytest.mark.gpu


def _device_logits(w, seed):
    def fn(t):
        x = synth.logits_torch(w, t, seed)
        if w.dtype == "bf16":
            return x.view(torch.int16).cpu().numpy().view(np.uint16), x
        return x.cpu().numpy(), x
    return fn


@pytest.mark.parametrize("name,fused", [("cfg2", False), ("cfg3", True), ("cfg5", False), ("cfg5", True)])
def test_full_shape_lockstep_8_steps(name, fused):
    w = synth.scaled(synth.WORKLOADS[name], layers=1, H=1)
    st = run_lockstep(w, seed=5, steps=8, grow_kv=False, logits_fn=_device_logits(w, 5), fused=fused)
    print(name, st)
    assert st["resamples"] > 0
    assert st["token_ties"] + st["ess_band"] + st["pos_band"] <= 2


@pytest.mark.parametrize("fused", [False, True])
def test_full_shape_lockstep_cfg4_ramp_then_held_exponent(fused):
    # kappa raised so that resampling fires within eight steps (the workload's own 0.5 needs tens of steps for that)
    w = synth.scaled(synth.WORKLOADS["cfg4"], layers=1, H=1, ramp=4, kappa=0.98)
    st = run_lockstep(w, seed=6, steps=8, grow_kv=False, logits_fn=_device_logits(w, 6), fused=fused)
    print("cfg4", st)
    assert st["steps"] == 8 and st["resamples"] > 0
    assert st["token_ties"] + st["ess_band"] + st["pos_band"] <= 2
