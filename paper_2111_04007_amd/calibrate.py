"""Calibration of one stage's compute-time parameters over the micro-batch size m.

The paper's morphing needs, per cut-point, the forward and backward compute times
F(m) and B(m) measured on a few micro-batches of random inputs (Job Morphing,
"Scale-invariant Calibration", parameter table), and then takes the lowest m at
which F(m)/m stops improving ("Parametrized Simulation").  `sweep` measures them on
the GPU through the stage library for a middle stage (F, and recompute+backward)
and for a last stage (forward that keeps internals, backward without recompute);
`pick_micro_batch` is the selection rule.
"""
from __future__ import annotations

from typing import Dict, List, Sequence


def pick_micro_batch(ms: Sequence[int], time_per_example: Sequence[float], rel_gain: float = 0.03) -> int:
    """Lowest m at which time/example stops improving: the first m (ascending) such
    that no larger measured m is better by more than `rel_gain` (relative).  The
    paper gives the rule in words only; the threshold is this build's reading."""
    if len(ms) != len(time_per_example) or not ms:
        raise ValueError("ms and time_per_example must be non-empty and of equal length")
    order = sorted(range(len(ms)), key=lambda i: ms[i])
    for pos, i in enumerate(order):
        t = time_per_example[i]
        if all(time_per_example[j] >= t * (1.0 - rel_gain) for j in order[pos + 1:]):
            return ms[i]
    return ms[order[-1]]


def sweep(cfg, m_values: Sequence[int], n_mb: int = 4, reps: int = 3, device="cuda:0") -> List[Dict]:
    """For each micro-batch size m: mean milliseconds of one forward F(m), one
    recompute+backward call RB(m), one keeping forward FK(m) and one backward on
    stored activations B(m), each over n_mb micro-batches x reps repetitions, timed
    with events on the stream the library launches on."""
    import torch
    from . import binding as B, synth

    out = []
    dev = torch.device(device)
    stream = torch.cuda.current_stream(dev)
    for m in m_values:
        c = cfg.replace(micro_batch=int(m), n_micro_batches=n_mb, wgrad_group=1)
        params, xs, dys = synth.device_random_stage(c, dev)
        st = B.Stage(c, dev, params_flat=params)
        ys = torch.empty_like(xs)
        dxs = torch.empty_like(xs)

        def timed(fn):
            fn()  # warm-up
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            torch.cuda.synchronize(dev)
            return e0.elapsed_time(e1) / (reps * n_mb)

        def fwd():
            for i in range(n_mb):
                st.forward(i, xs[i], ys[i], stream)

        def rb():
            for i in range(n_mb):
                st.backward_recompute(i, dys[i], dxs[i], stream)

        st.grad_accum_reset(stream)
        t_f = timed(fwd)
        # backward_recompute consumes a slot: re-arm the slots (untimed) before each batch
        ev = []
        for r in range(reps + 1):
            fwd()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            rb()
            e1.record(stream)
            ev.append((e0, e1))
        torch.cuda.synchronize(dev)
        t_rb = sum(a.elapsed_time(b) for a, b in ev[1:]) / (reps * n_mb)
        # last-stage pair: time the keeping forwards and the stored backwards separately
        last = []
        for r in range(reps + 1):
            for i in range(n_mb):
                e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
                e[0].record(stream)
                st.forward_keep(i, xs[i], ys[i], stream)
                e[1].record(stream)
                st.backward_stored(i, dys[i], dxs[i], stream)
                e[2].record(stream)
                if r:  # repetition 0 is the warm-up
                    last.append(e)
        torch.cuda.synchronize(dev)
        fk = sum(e[0].elapsed_time(e[1]) for e in last) / len(last)
        bs = sum(e[1].elapsed_time(e[2]) for e in last) / len(last)
        st.close()
        del st, params, xs, dys, ys, dxs
        torch.cuda.empty_cache()
        out.append({"m": int(m), "F_ms": t_f, "RB_ms": t_rb, "Fkeep_ms": fk, "B_ms": bs,
                    "F_per_example_ms": t_f / m, "RB_per_example_ms": t_rb / m,
                    "Fkeep_per_example_ms": fk / m, "B_per_example_ms": bs / m})
    return out
