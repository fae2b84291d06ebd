"""Oracle for the network-sensing controller -- TEST INFRASTRUCTURE.

Algorithm 1 (network sensing and ratio adjustment) with Eq. (1) EBB =
data_size / RTT, Eq. (2) BDP = BtlBw * RTprop and Eq. (3) the ratio update,
followed by the gate of Algorithm 2 Step 1 (the quantization step) that
decides the value width for the step.

Python floats are IEEE doubles, so every +, *, /, max, min below is the same
operation a C double would perform.

Readings where the paper is silent (each also listed in the design notes):
  * beta1 (start-up increment) is not printed; 0.1 = 10 * beta2 is used.
  * the RTT criterion that ends start-up (Sec. 4.1 gives no number): the last transmission time exceeds
    rtt_excess * RTprop, rtt_excess = 2 (the only figure the paper gives for an
    RTT-reactive trigger, in its discussion of MLT); start-up also ends after
    startup_max steps or when the ratio reaches its cap.  On the call that ends
    start-up, Eq. (3) is applied at once.
  * data_size in Eq. (3) is the size transmitted in the interval just measured.
  * BtlBw / RTprop windows: win == 0 is the literal all-time max / min; win > 0
    keeps the last `win` intervals.
  * tr_q = 0.1, tr_d = 0; an unknown L2 norm (< 0) passes the density test.
  * quant_mode 0 (build contract): 8-bit codes below tr_q, 4-bit below tr_q4;
    quant_mode 1 (paper's own): 16-bit floats below tr_q; quant_mode 2: never.
    Whenever values are quantized the ratio handed to top-k is doubled
    (Algorithm 2 Step 1), capped at `cap`; the controller's own ratio is not.

parity unpinned: beyond the closed forms of Eq. (3) and hand values of
Eq. (1)/(2) the start-up exit, windows and gate thresholds above are readings,
not facts the paper fixes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

STARTUP, NETSENSE = 0, 1


@dataclass
class CtlParams:
    alpha: float = 0.5        # Eq. (3); value printed in Sec. 4.1
    beta1: float = 0.1        # Algorithm 1 Step 1 (value not printed)
    beta2: float = 0.01       # Eq. (3); value printed in Sec. 4.1
    floor: float = 0.005      # Eq. (3) lower bound
    cap: float = 1.0          # Eq. (3) upper bound
    init: float = 0.01        # Algorithm 1 Step 1 initial ratio
    bdp_frac: float = 0.9     # Eq. (3) trigger fraction of BDP
    rtt_excess: float = 2.0
    tr_q: float = 0.1
    tr_q4: float = 0.01
    tr_d: float = 0.0
    startup_max: int = 10
    win_bw: int = 10
    win_rt: int = 100
    quant_mode: int = 0


@dataclass
class CtlState:
    p: CtlParams
    ratio: float
    phase: int = STARTUP
    startup_steps: int = 0
    ebb: List[float] = field(default_factory=list)
    rtt: List[float] = field(default_factory=list)
    btlbw: float = 0.0
    rtprop: float = 0.0
    bdp: float = 0.0


def ctl_init(p: CtlParams | None = None) -> CtlState:
    p = p or CtlParams()
    return CtlState(p=p, ratio=p.init)


def choose_ratio(s: CtlState, last_payload_bytes: float, last_tx_seconds: float,
                 dense_bytes: float = 0.0, last_l2norm: float = -1.0) -> Tuple[float, int]:
    """One controller decision before a transmission.  -> (ratio for top-k, bits)."""
    p = s.p
    measured = last_payload_bytes > 0.0 and last_tx_seconds > 0.0
    if measured:
        # Eq. (1)
        s.ebb.append(last_payload_bytes / last_tx_seconds)
        s.rtt.append(last_tx_seconds)
        ebb = s.ebb[-p.win_bw:] if p.win_bw > 0 else s.ebb
        rtt = s.rtt[-p.win_rt:] if p.win_rt > 0 else s.rtt
        s.btlbw = max(ebb)
        s.rtprop = min(rtt)
        # Eq. (2)
        s.bdp = s.btlbw * s.rtprop
        if s.phase == STARTUP:
            excessive = last_tx_seconds > p.rtt_excess * s.rtprop
            if excessive or s.startup_steps >= p.startup_max or s.ratio >= p.cap:
                s.phase = NETSENSE
            else:
                s.ratio = min(p.cap, s.ratio + p.beta1)
                s.startup_steps += 1
        if s.phase == NETSENSE:
            # Eq. (3)
            if last_payload_bytes > p.bdp_frac * s.bdp:
                s.ratio = max(p.floor, s.ratio * p.alpha)
            else:
                s.ratio = min(p.cap, s.ratio + p.beta2)
    ratio_out, bits = s.ratio, 32
    if p.quant_mode != 2 and s.ratio < p.tr_q and (last_l2norm < 0.0 or last_l2norm > p.tr_d):
        bits = 16 if p.quant_mode == 1 else (4 if s.ratio < p.tr_q4 else 8)
        ratio_out = min(p.cap, 2.0 * s.ratio)
    return ratio_out, bits
