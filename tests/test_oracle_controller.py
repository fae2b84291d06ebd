"""Pins for the controller oracle: Eq. (1)-(3) and Algorithm 1 with the printed constants."""
import os

import pytest

from oracle import CtlParams, choose_ratio, ctl_init
from oracle.controller import NETSENSE, STARTUP

GOLD = os.path.join(os.path.dirname(__file__), "golden", "eq3_closed_forms.txt")


def _netsense_only(init, **kw):
    # startup_max = 0: the first measurement ends start-up; windows 0 = all-time max / min
    return ctl_init(CtlParams(init=init, startup_max=0, win_bw=0, win_rt=0, quant_mode=2, **kw))


def test_eq3_closed_forms_golden():
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        head, _, tail = line.partition(":")
        kind, r0, steps = head.split()
        r0, steps = float(r0), int(steps)
        if kind == "congested":
            # a constant (bytes, time) sample makes BDP == bytes, so bytes > 0.9 * BDP each step
            s = _netsense_only(r0)
            got = [choose_ratio(s, 1e6, 0.5)[0] for _ in range(steps)]
            assert got == [float(x) for x in tail.split()]
        else:
            # one large sample fixes BtlBw; later small samples at the same time stay below 0.9*BDP
            s = _netsense_only(r0)
            s.phase = NETSENSE
            s.ebb.append(1e9), s.rtt.append(1.0)
            n = 0
            while s.ratio < 1.0:
                choose_ratio(s, 1e3, 1.0)
                n += 1
                assert n <= 1000
            assert n == steps and s.ratio == 1.0


def test_eq1_eq2_by_hand():
    s = _netsense_only(0.5)
    choose_ratio(s, 8e6, 0.25)          # EBB = 32e6 B/s
    assert s.btlbw == 32e6 and s.rtprop == 0.25 and s.bdp == 8e6
    choose_ratio(s, 3e6, 0.125)         # EBB = 24e6; max stays 32e6; min RTT 0.125
    assert s.btlbw == 32e6 and s.rtprop == 0.125 and s.bdp == 4e6
    # 3e6 <= 0.9 * 4e6 -> additive increase after the first (congested) halving
    assert s.ratio == 0.25 + 0.01


def test_first_call_returns_initial_ratio():
    s = ctl_init()
    assert choose_ratio(s, 0.0, 0.0) == (0.02, 8)      # 0.01 < tr_q: 8-bit codes, ratio doubled
    assert s.ratio == 0.01 and s.phase == STARTUP
    s = ctl_init(CtlParams(quant_mode=2))
    assert choose_ratio(s, 0.0, 0.0) == (0.01, 32)


def test_startup_ramp_and_exit_on_excessive_rtt():
    s = ctl_init(CtlParams(quant_mode=2))
    choose_ratio(s, 0, 0)
    # uncongested: time barely grows -> +beta1 per step
    r = [choose_ratio(s, 1e5 * (i + 1), 0.010 + 1e-4 * i)[0] for i in range(3)]
    assert r == pytest.approx([0.11, 0.21, 0.31], abs=1e-12) and s.phase == STARTUP
    # the next transmission takes > 2 x RTprop: start-up ends and Eq. (3) halves at once
    r4 = choose_ratio(s, 4e5, 0.050)[0]
    assert s.phase == NETSENSE and r4 == pytest.approx(0.155, abs=1e-12)


def test_startup_limited_number_of_steps():
    s = ctl_init(CtlParams(startup_max=4, quant_mode=2, beta1=0.05))
    for i in range(4):
        choose_ratio(s, 1e5, 0.01)
    assert s.phase == STARTUP and s.startup_steps == 4
    choose_ratio(s, 1e5, 0.01)
    assert s.phase == NETSENSE


def test_sliding_window_forgets_old_bandwidth():
    s = ctl_init(CtlParams(init=0.5, startup_max=0, win_bw=3, win_rt=3, quant_mode=2))
    choose_ratio(s, 1e9, 1.0)
    for _ in range(3):
        choose_ratio(s, 1e6, 1.0)
    assert s.btlbw == 1e6                      # the 1e9 sample left the window
    s = _netsense_only(0.5)
    choose_ratio(s, 1e9, 1.0)
    for _ in range(30):
        choose_ratio(s, 1e6, 1.0)
    assert s.btlbw == 1e9                      # all-time maximum


def test_failure_reaction_and_recovery():
    """A collapsed link (huge transmission time) drives the ratio to the floor by halving;
    once the payload fits the BDP again it recovers by +0.01 per step."""
    s = ctl_init(CtlParams(init=0.64, startup_max=0, quant_mode=2))
    seen = [choose_ratio(s, 5e8, 100.0)[0] for _ in range(9)]
    assert seen[:7] == [0.32, 0.16, 0.08, 0.04, 0.02, 0.01, 0.005] and seen[-1] == 0.005
    s.ebb[:] = [1e12]
    before = s.ratio
    after = choose_ratio(s, 1e3, 100.0)[0]
    assert after == before + 0.01


def test_quantization_gate():
    p = CtlParams(init=0.05, quant_mode=0)
    assert choose_ratio(ctl_init(p), 0, 0) == (0.1, 8)
    p = CtlParams(init=0.008, quant_mode=0)
    assert choose_ratio(ctl_init(p), 0, 0) == (0.016, 4)
    p = CtlParams(init=0.05, quant_mode=1)
    assert choose_ratio(ctl_init(p), 0, 0) == (0.1, 16)       # the paper's 32 -> 16 bit cast
    p = CtlParams(init=0.2, quant_mode=0)
    assert choose_ratio(ctl_init(p), 0, 0) == (0.2, 32)       # ratio >= tr_q: no quantization
    p = CtlParams(init=0.05, quant_mode=0, tr_d=1.0)
    assert choose_ratio(ctl_init(p), 0, 0, 0.0, 0.5) == (0.05, 32)   # L2 <= tr_d: sparse signal
    assert choose_ratio(ctl_init(p), 0, 0, 0.0, 2.0) == (0.1, 8)
    assert choose_ratio(ctl_init(p), 0, 0, 0.0, -1.0) == (0.1, 8)    # unknown norm passes
    p = CtlParams(init=0.7, quant_mode=0, tr_q=0.9)
    assert choose_ratio(ctl_init(p), 0, 0) == (1.0, 8)        # doubled ratio is capped


def test_eq3_boundary_is_strict():
    """Eq. (3) halves only when data_size > 0.9 * BDP; a payload of exactly 0.9 * BDP still takes
    the additive branch."""
    s = _netsense_only(0.5)
    s.phase = NETSENSE
    s.ebb.append(1e7), s.rtt.append(1.0)       # BtlBw = 1e7 B/s, RTprop = 1 s: BDP = 1e7 bytes
    edge = 0.9 * 1e7
    assert choose_ratio(s, edge, 1.0)[0] == 0.5 + 0.01 and s.bdp == 1e7
    above = edge * (1.0 + 2.0 ** -52)
    assert above > edge
    assert choose_ratio(s, above, 1.0)[0] == (0.5 + 0.01) * 0.5
