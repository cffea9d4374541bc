"""Rough cycle model of one CU running a generated decode kernel.  Test infrastructure only.

Four waves (one per SIMD) replay the instruction trace that the functional emulator recorded for
wave 0.  Costs: every wave issues in order, 4 cycles per instruction (16 for the quarter-rate
transcendentals, n+1 for s_nop n); each SIMD has its own MFMA pipe that is busy 32 cycles per
v_mfma_f32_32x32x16_bf16; LDS is one shared server that spends 4 cycles per wave-wide read
(1024 B of ds_read_b128 at the measured 256 B/clk, 512 B of ds_read_b64_tr_b16 at the measured
128 B/clk) and returns data 64 cycles later; s_waitcnt lgkmcnt blocks on those returns; s_barrier
joins the four waves.  Global memory latency, bank conflicts, instruction fetch and clock
throttling are not modelled: the result is a lower bound on the time of a pass, used to compare
schedules, not a prediction of the measured rate."""
from __future__ import annotations

import collections

import gfx950_emu as emu

LDS_LATENCY = 64
MFMA_BUSY = 32


def record_trace(run, wave_id=0):
    """Runs `run()` (something that drives emu.Workgroup) and returns the program counters wave
    `wave_id` of the first workgroup executed."""
    trace = []
    orig = emu.Wave.step
    first_wg = []

    def step(self):
        if not first_wg:
            first_wg.append(self.wg)
        if self.id == wave_id and self.wg is first_wg[0]:
            trace.append(self.pc)
        orig(self)

    emu.Wave.step = step
    try:
        run()
    finally:
        emu.Wave.step = orig
    return trace


def simulate(ins, trace, nwaves=4):
    """Returns (list of (pc, time) for wave 0, stall counters, total cycles)."""
    t = [0.0] * nwaves
    mfma_free = [0.0] * nwaves
    lds_free = 0.0
    pend = [collections.deque() for _ in range(nwaves)]
    pos = [0] * nwaves
    marks = []
    stall = collections.Counter()
    n = len(trace)
    while min(pos) < n:
        cand = [w for w in range(nwaves) if pos[w] < n and ins[trace[pos[w]]][0] != "s_barrier"]
        if not cand:
            tb = max(t)
            for w in range(nwaves):
                stall["barrier"] += tb - t[w]
                t[w] = tb + 8
                pos[w] += 1
            continue
        w = min(cand, key=lambda x: t[x])
        pc = trace[pos[w]]
        m, ops, mods = ins[pc]
        if w == 0:
            marks.append((pc, t[w]))
        if m.startswith("v_mfma"):
            start = max(t[w], mfma_free[w])
            stall["mfma_pipe"] += start - t[w]
            mfma_free[w] = start + MFMA_BUSY
            t[w] = start + 4
        elif m.startswith("ds_read"):
            begin = max(t[w], lds_free)
            lds_free = begin + 4
            pend[w].append(lds_free + LDS_LATENCY)
            t[w] += 4
        elif m == "s_waitcnt":
            lg = None
            for o in ops + list(mods):
                if o.startswith("lgkmcnt"):
                    lg = int(o[8:-1])
            if lg is not None:
                while len(pend[w]) > lg:
                    done = pend[w].popleft()
                    if done > t[w]:
                        stall["lds_wait"] += done - t[w]
                        t[w] = done
            t[w] += 1
        elif m == "s_nop":
            t[w] += int(ops[0]) + 1
        elif m in emu.TRANS:
            t[w] += 16
        else:
            t[w] += 4
        pos[w] += 1
    return marks, stall, max(t)


def cycles_per_pass(ins, labels, trace, loop_label, passes_per_loop=2):
    marks, stall, total = simulate(ins, trace)
    at = [tm for pc, tm in marks if pc == labels[loop_label]]
    if len(at) < 3:
        raise ValueError("trace too short")
    steady = [b - a for a, b in zip(at[1:-1], at[2:])]
    return sum(steady) / len(steady) / passes_per_loop, stall
