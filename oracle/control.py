"""CPU oracle of the scheduler's control loop -- TEST INFRASTRUCTURE ONLY.

Paper Sec. 3.3, last part: a light loop that runs every few hundred milliseconds moves the share r
reserved for the prefill queue and that queue's flush time-out tau_pre.  The paper fixes directions:
KV-link utilisation below its target -> raise r or shorten tau_pre (prefill must go faster); decode
stalls rising -> lower r (decode gets more of the batch); the loop also tries to bring the prefill P95
wait down.  It gives no amounts, no order and no rule for relaxing tau_pre again; the reading taken
(amounts as parameters, r before tau_pre, prefill before decode, relax when nothing else applies) is
the four rules below, in this order.  Plain floats (Python's float is fp64; r is kept as the nearest
fp32 after each period, as the library stores it).

Pins (tests/test_oracle_pins.py): the paper's directional statements as properties, the bounds,
a fixed point on target, and a closed loop against a toy plant.  The amounts are parameters of the
reading, so beyond those properties this function is "parity unpinned".
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np


@dataclass
class Config:
    r_min: float
    r_max: float
    r_step: float
    tau_factor: float
    tau_min_s: float
    tau_max_s: float
    u_kv_target: float
    u_kv_band: float
    stall_target: float
    wait_p95_budget_s: float


def _f32(x: float) -> float:
    return float(np.float32(x))


def period(cfg: Config, r: float, tau: float, u_kv: float, decode_stall: float, decode_stall_prev: float,
           wait_p95_s: float):
    """One period.  Unknown signals are NaN.  Returns (r, tau, rules) with rules = the set of rule numbers applied."""
    r = min(max(_f32(r), _f32(cfg.r_min)), _f32(cfg.r_max))
    tau = min(max(tau, cfg.tau_min_s), cfg.tau_max_s)
    rules = set()
    starved = not math.isnan(u_kv) and _f32(u_kv) < _f32(_f32(cfg.u_kv_target) - _f32(cfg.u_kv_band))
    if starved:                                                   # 1: the KV link is under-used
        if r < _f32(cfg.r_max):
            r = min(_f32(cfg.r_max), _f32(r + _f32(cfg.r_step)))
        else:
            tau = max(cfg.tau_min_s, tau / _f32(cfg.tau_factor))
        rules.add(1)
    waited = not math.isnan(wait_p95_s)
    if waited and wait_p95_s > cfg.wait_p95_budget_s:            # 2: prefill requests wait too long
        tau = max(cfg.tau_min_s, tau / _f32(cfg.tau_factor))
        rules.add(2)
    if (not starved and not math.isnan(decode_stall) and not math.isnan(decode_stall_prev)
            and _f32(decode_stall) > _f32(cfg.stall_target) and _f32(decode_stall) > _f32(decode_stall_prev)):
        r = max(_f32(cfg.r_min), _f32(r - _f32(cfg.r_step)))     # 3: decode stalls are rising
        rules.add(3)
    if not rules and (not waited or wait_p95_s <= 0.5 * cfg.wait_p95_budget_s):
        tau = min(cfg.tau_max_s, tau * _f32(cfg.tau_factor))     # 4: nothing presses: relax
        rules.add(4)
    return r, tau, rules
