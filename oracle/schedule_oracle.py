"""CPU oracle for the nested pipeline schedule (pure integer logic).

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and smoke/bench baseline
legs), never by the product path, and sharing no code with it.

The scheduling rule follows the paper's BuildSchedule algorithm (Sec. 3.1,
"Compute operator" / "Memory efficiency", and the BuildSchedule figure): the
LLM schedule is kept verbatim; W encoder-forward units are warmed up; after
every LLM column, each op of the column is inspected: when the LLM output of
its unit is complete the unit's generator forward and backward run
back-to-back, and when the encoder-input gradient of its unit is complete the
unit's encoder backward runs, immediately followed by the next pending
encoder forward.

The paper leaves ``columns``, ``llm_output_ready`` and ``encoder_grad_ready``
as names.  Reading used here for ONE pipeline stage that is both the entry
and the exit stage of the LLM:
  * a unit is ``unit_size`` consecutive microbatches (the paper's pp_size);
  * the LLM schedule is local 1F1B at unit granularity with ``depth`` units in
    flight (depth 3 is the smallest order satisfying the paper's order
    property F_i, F_{i+1}, F_{i+2} < G_i < F_{i+3});  one column = the ops of
    one unit in one direction;
  * the LLM output of unit u is ready at the forward of u's last microbatch;
  * the encoder gradient of unit u is ready at the backward of u's last
    microbatch.

Ops are tuples ``(kind, index)`` with kind in
  "E" enc_fwd(unit)  "e" enc_bwd(unit)  "g" gen_fwd+gen_bwd(unit) is emitted
  as two ops "G" (gen_fwd) and "H" (gen_bwd);  "F"/"B" LLM fwd/bwd(microbatch).
Pins: tests/test_oracle_schedule.py (hand expansion fixtures, invariants).
"""
from __future__ import annotations

from typing import List, Tuple

Op = Tuple[str, int]


def partition_microbatches(M: int, unit_size: int) -> List[List[int]]:
    return [list(range(s, min(s + unit_size, M))) for s in range(0, M, unit_size)]


def llm_schedule_1f1b(M: int, unit_size: int = 1, depth: int = 3) -> List[List[Op]]:
    """Columns of one stage's 1F1B order at unit granularity."""
    units = partition_microbatches(M, unit_size)
    U = len(units)
    fwd = lambda u: [("F", m) for m in units[u]]
    bwd = lambda u: [("B", m) for m in units[u]]
    cols = [fwd(u) for u in range(min(depth, U))]
    nxt = min(depth, U)
    for u in range(U):
        cols.append(bwd(u))
        if nxt < U:
            cols.append(fwd(nxt)); nxt += 1
    return cols


def build_schedule(llm_columns: List[List[Op]], M: int, unit_size: int, W: int,
                   has_generator: bool = True) -> List[Op]:
    units = partition_microbatches(M, unit_size)
    unit_of = {m: u for u, mbs in enumerate(units) for m in mbs}
    schedule: List[Op] = []
    next_unit = 0
    while next_unit < min(W, len(units)):
        schedule.append(("E", next_unit)); next_unit += 1
    for column in llm_columns:
        schedule += column
        for kind, m in column:
            u = unit_of[m]
            last = units[u][-1]
            if has_generator and kind == "F" and m == last:
                schedule += [("G", u), ("H", u)]
            if kind == "B" and m == last:
                schedule.append(("e", u))
                if next_unit < len(units):
                    schedule.append(("E", next_unit)); next_unit += 1
    return schedule


def compute_efficient_schedule(llm_columns: List[List[Op]], M: int, unit_size: int,
                               has_generator: bool = True) -> List[Op]:
    """The baseline order the paper contrasts with (Sec. 2.2 "Compute-efficient
    systems"): every encoder forward first, then the LLM schedule (generator
    units where their inputs appear), every encoder backward at the end."""
    units = partition_microbatches(M, unit_size)
    unit_of = {m: u for u, mbs in enumerate(units) for m in mbs}
    schedule: List[Op] = [("E", u) for u in range(len(units))]
    for column in llm_columns:
        schedule += column
        for kind, m in column:
            u = unit_of[m]
            if has_generator and kind == "F" and m == units[u][-1]:
                schedule += [("G", u), ("H", u)]
    schedule += [("e", u) for u in range(len(units))]
    return schedule


def sequential_schedule(M: int, unit_size: int, has_generator: bool = True) -> List[Op]:
    """One unit at a time, nothing overlapped (reference order for gradients)."""
    out: List[Op] = []
    for u, mbs in enumerate(partition_microbatches(M, unit_size)):
        out.append(("E", u))
        out += [("F", m) for m in mbs]
        if has_generator:
            out += [("G", u), ("H", u)]
        out += [("B", m) for m in mbs]
        out.append(("e", u))
    return out


def live_counts(schedule: List[Op], M: int, unit_size: int):
    """Replay: peak number of encoder units, generator units and LLM
    microbatches whose activations are alive at the same time."""
    enc = gen = llm = 0
    peak = {"enc": 0, "gen": 0, "llm": 0}
    for kind, _ in schedule:
        if kind == "E": enc += 1
        elif kind == "e": enc -= 1
        elif kind == "G": gen += 1
        elif kind == "H": gen -= 1
        elif kind == "F": llm += 1
        elif kind == "B": llm -= 1
        peak["enc"] = max(peak["enc"], enc)
        peak["gen"] = max(peak["gen"], gen)
        peak["llm"] = max(peak["llm"], llm)
    assert enc == gen == llm == 0
    return peak


def format_schedule(schedule: List[Op]) -> str:
    return " ".join(f"{k}{i}" for k, i in schedule)
