"""CPU oracle for the multi-stage nested schedule and its replay (host logic only).

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and bench baseline legs),
never by the product path, and sharing no code with it.

What it follows.  Sec. 3.1 of the paper: the LLM runs a user-given pipeline
schedule over P ranks ("e.g. interleaved 1F1B"), encoder and generator work is
grouped in units of P microbatches that every rank processes locally (one
microbatch of the unit per rank), and BuildSchedule (the figure of that name)
nests the units into the unchanged LLM schedule: W encoder units are warmed
up; after every LLM column the generator forward+backward of a unit is placed
once its LLM output is complete, and the encoder backward of a unit (followed
by the next pending encoder forward) once its input gradient is complete.
Sec. 2.2 "Performance analysis" gives the closed forms the replay is pinned
to: 1F1B bubble rate (P-1)/(M+P-1); peak modality activations (M/P)*A_m for
the compute-efficient order, P*A_m on the first stage for the memory-efficient
order, W units for the nested order.

Readings (the paper leaves ``columns``, ``llm_output_ready`` and
``encoder_grad_ready`` as names and prints no rank programs):
  * LLM schedules: V = 1 is the classic 1F1B order (rank r warms up P-r-1
    forwards); V >= 2 is the interleaved order of the virtual-pipeline
    literature (rank r warms up 2(P-r-1) + (V-1)P forwards; the k-th forward
    slot of a rank runs chunk (k div P) mod V of microbatch
    (k div PV)*P + k mod P, backward slots walk the chunks in reverse).
    M must be a multiple of P.  Model chunk c of rank r is pipeline position
    c*P + r.
  * column j of the LLM schedule = the j-th LLM op of every rank.
  * a rank works on ONE microbatch of every unit (microbatch u*P + r on rank
    r).  For rank r the LLM output of unit u is ready at the forward of that
    microbatch through the last chunk on the last rank.  (Waiting for the
    unit's last microbatch instead would deadlock: under 1F1B the last rank
    runs the backward of a microbatch right after its forward, and that
    backward needs the generator's gradient.)  The encoder gradient of unit u
    is ready, for every rank, at the backward of the unit's LAST microbatch
    through chunk 0 on rank 0 (one gradient scatter per unit).
  * every rank program carries the same unit ops in the same order; encoder
    ops sit at the same column on all ranks, generator ops at the column of
    the rank's own microbatch.
  * cross-rank edges of the replay: a forward needs the same (microbatch,
    chunk) forward of the previous pipeline position, the first position needs
    the encoder output of that microbatch (computed by rank m mod P); a
    backward needs the backward of the next position, the last position needs
    the generator backward of that microbatch's rank (or, without generator,
    only its own forward); generator forward of rank r needs the last-position
    forward of microbatch u*P + r; encoder backward of rank r needs the
    first-position backward of microbatch u*P + r.
  * memory-efficient order: the encoder of microbatch m runs inside the
    first-position forward/backward on rank 0, the generator inside the
    last-position forward on rank P-1 (one 1F1B pipeline, Sec. 2.2).

Ops are tuples (kind, index, chunk): kind "F"/"B" LLM forward/backward of a
microbatch through a chunk; "E"/"e" encoder forward/backward of a unit;
"G"/"H" generator forward/backward of a unit (chunk = 0 for unit ops).

Pins: tests/test_oracle_pipeline.py.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

Op = Tuple[str, int, int]

NESTED, COMPUTE_EFFICIENT, MEMORY_EFFICIENT = "nested", "compute_efficient", "memory_efficient"


def llm_rank_schedule(P: int, V: int, M: int, rank: int) -> List[Op]:
    """LLM ops of one rank, in execution order."""
    if M % P != 0:
        raise ValueError("M must be a multiple of P")
    total = M * V
    if V == 1:
        warm = min(P - rank - 1, total)
    else:
        warm = min(2 * (P - rank - 1) + (V - 1) * P, total)

    def fwd(k):
        return ("F", (k // (P * V)) * P + k % P, (k // P) % V)

    def bwd(k):
        return ("B", (k // (P * V)) * P + k % P, V - 1 - (k // P) % V)

    ops: List[Op] = [fwd(k) for k in range(warm)]
    nf, nb = warm, 0
    while nf < total:                      # steady state: one forward, one backward
        ops.append(fwd(nf)); nf += 1
        ops.append(bwd(nb)); nb += 1
    while nb < total:                      # cool-down
        ops.append(bwd(nb)); nb += 1
    return ops


def build_rank_schedule(order: str, P: int, V: int, M: int, W: int, has_generator: bool,
                        rank: int) -> List[Op]:
    """Program of one rank: its LLM ops with the unit ops nested per `order`."""
    llm = [llm_rank_schedule(P, V, M, r) for r in range(P)]
    U = M // P
    if order == MEMORY_EFFICIENT:
        return list(llm[rank])
    prog: List[Op] = []
    nxt = 0
    warm = U if order == COMPUTE_EFFICIENT else min(W, U)
    while nxt < warm:
        prog.append(("E", nxt, 0)); nxt += 1
    for j in range(len(llm[0])):
        prog.append(llm[rank][j])
        for r in range(P):
            kind, m, c = llm[r][j]
            u = m // P
            last_of_unit = m % P == P - 1
            if has_generator and kind == "F" and r == P - 1 and c == V - 1 and m % P == rank:
                prog += [("G", u, 0), ("H", u, 0)]
            if kind == "B" and r == 0 and c == 0 and last_of_unit and order == NESTED:
                prog.append(("e", u, 0))
                if nxt < U:
                    prog.append(("E", nxt, 0)); nxt += 1
    if order == COMPUTE_EFFICIENT:
        prog += [("e", u, 0) for u in range(U)]
    return prog


def replay(order: str, P: int, V: int, M: int, W: int, has_generator: bool,
           llm_fwd: Sequence[float], llm_bwd: Sequence[float],
           enc_fwd: Sequence[float], enc_bwd: Sequence[float],
           gen_fwd: Sequence[float], gen_bwd: Sequence[float],
           p2p: float = 0.0, act_llm: float = 0.0,
           act_enc: Optional[Sequence[float]] = None,
           act_gen: Optional[Sequence[float]] = None) -> Dict[str, object]:
    """Event replay of the P rank programs.

    llm_fwd/llm_bwd: [P*V] seconds per (rank, chunk), index rank*V + chunk.
    enc_*/gen_*: [M] seconds per microbatch.  act_llm: bytes one (microbatch,
    chunk) keeps between its forward and backward; act_enc/act_gen: [M] bytes
    per microbatch kept between the unit's forward and backward.
    Returns makespan, busy seconds and activation high-water marks per rank.
    """
    act_enc = list(act_enc) if act_enc is not None else [0.0] * M
    act_gen = list(act_gen) if act_gen is not None else [0.0] * M
    progs = [build_rank_schedule(order, P, V, M, W, has_generator, r) for r in range(P)]
    fused = order == MEMORY_EFFICIENT
    done: Dict[Tuple[int, Op], float] = {}          # (rank, op) -> finish time
    pos = [0] * P
    clock = [0.0] * P
    busy = [0.0] * P

    def edge(src_rank: int, op: Op, dst_rank: int) -> Optional[float]:
        t = done.get((src_rank, op))
        if t is None:
            return None
        return t + (p2p if src_rank != dst_rank else 0.0)

    def ready_and_cost(r: int, op: Op):
        kind, i, c = op
        deps: List[Optional[float]] = []
        if kind == "F":
            cost = llm_fwd[r * V + c]
            if r > 0:
                deps.append(edge(r - 1, op, r))
            elif c > 0:
                deps.append(edge(P - 1, ("F", i, c - 1), r))
            elif fused:
                cost += enc_fwd[i]
            else:
                deps.append(edge(i % P, ("E", i // P, 0), r))
            if fused and has_generator and r == P - 1 and c == V - 1:
                cost += gen_fwd[i] + gen_bwd[i]
        elif kind == "B":
            cost = llm_bwd[r * V + c]
            if r < P - 1:
                deps.append(edge(r + 1, op, r))
            elif c < V - 1:
                deps.append(edge(0, ("B", i, c + 1), r))
            elif has_generator and not fused:
                deps.append(edge(i % P, ("H", i // P, 0), r))
            if fused and r == 0 and c == 0:
                cost += enc_bwd[i]
        elif kind == "E":
            cost = enc_fwd[i * P + r]
        elif kind == "e":
            cost = enc_bwd[i * P + r]
            deps.append(edge(0, ("B", i * P + r, 0), r))
        elif kind == "G":
            cost = gen_fwd[i * P + r]
            deps.append(edge(P - 1, ("F", i * P + r, V - 1), r))
        elif kind == "H":
            cost = gen_bwd[i * P + r]
        else:
            raise ValueError(kind)
        if any(d is None for d in deps):
            return None, cost
        return max([0.0] + [d for d in deps if d is not None]), cost

    remaining = sum(len(p) for p in progs)
    while remaining:
        progressed = False
        for r in range(P):
            while pos[r] < len(progs[r]):
                op = progs[r][pos[r]]
                t_ready, cost = ready_and_cost(r, op)
                if t_ready is None:
                    break
                start = max(clock[r], t_ready)
                clock[r] = start + cost
                busy[r] += cost
                done[(r, op)] = clock[r]
                pos[r] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise RuntimeError("rank programs deadlock")
    makespan = max(clock)

    # activation high-water marks follow from each rank's program alone
    peak, peak_enc, peak_gen, peak_llm = [], [], [], []
    for r in range(P):
        live_l = live_e = live_g = 0.0
        pk = pe = pg = pl = 0.0
        for kind, i, c in progs[r]:
            if kind == "F":
                live_l += act_llm
                if fused and r == 0 and c == 0:
                    live_e += act_enc[i]
                if fused and has_generator and r == P - 1 and c == V - 1:
                    pg = max(pg, act_gen[i])
                    pk = max(pk, live_l + live_e + live_g + act_gen[i])
            elif kind == "E":
                live_e += act_enc[i * P + r]
            elif kind == "G":
                live_g += act_gen[i * P + r]
            pk = max(pk, live_l + live_e + live_g)
            pe, pg, pl = max(pe, live_e), max(pg, live_g), max(pl, live_l)
            if kind == "B":
                live_l -= act_llm
                if fused and r == 0 and c == 0:
                    live_e -= act_enc[i]
            elif kind == "e":
                live_e -= act_enc[i * P + r]
            elif kind == "H":
                live_g -= act_gen[i * P + r]
        peak.append(pk); peak_enc.append(pe); peak_gen.append(pg); peak_llm.append(pl)
    return {"makespan": makespan, "busy": busy, "peak": peak, "peak_enc": peak_enc,
            "peak_gen": peak_gen, "peak_llm": peak_llm,
            "bubble": 1.0 - sum(busy) / (P * makespan) if makespan > 0 else 0.0}


# ---------------------------------------------------------------------------
# communication operators and the deadlock check (Sec. 3.1 "Communication
# operator", Sec. 3.2; the executor-interface figure names insert_comm_ops and
# deadlock_check without defining them)
#
# Reading.  Every cross-rank data dependency of a compute op becomes a RECV
# placed right before it and every tensor another rank consumes a SEND placed
# right after it.  A message is identified by (what, microbatch, edge):
#   ACT   forward activation into pipeline position `edge`      (edge-1 -> edge)
#   GRAD  gradient w.r.t. the input of pipeline position `edge` (edge -> edge-1)
#   FEAT  encoder features of a microbatch to the entry rank 0  (owner m mod P -> 0)
#   FGRAD input-embedding gradient back to the encoder owner    (0 -> m mod P)
#   OUT   LLM output of a microbatch to its generator owner     (P-1 -> m mod P)
#   OGRAD generator-input gradient back to the exit rank        (m mod P -> P-1)
# Edges whose two ends sit on one rank need no message.  Sends are posted
# asynchronously and never block; a RECV blocks until its SEND was posted
# (the executor waits on receive handles before consuming, Sec. 3.2).
# ---------------------------------------------------------------------------

def comm_rank_schedule(order: str, P: int, V: int, M: int, W: int, has_generator: bool,
                       rank: int) -> List[tuple]:
    """Rank program with communication operators.  Compute ops stay (kind, index, chunk);
    comm ops are ("SEND" | "RECV", peer, what, microbatch, edge)."""
    r = rank
    last = P * V - 1
    fused = order == MEMORY_EFFICIENT
    out: List[tuple] = []
    for op in build_rank_schedule(order, P, V, M, W, has_generator, r):
        kind, i, c = op
        pre: List[tuple] = []
        post: List[tuple] = []
        if kind in "FB":
            pos = c * P + r
            if kind == "F":
                if pos > 0 and (pos - 1) % P != r:
                    pre.append(("RECV", (pos - 1) % P, "ACT", i, pos))
                if pos == 0 and not fused and i % P != r:
                    pre.append(("RECV", i % P, "FEAT", i, 0))
                if pos < last and (pos + 1) % P != r:
                    post.append(("SEND", (pos + 1) % P, "ACT", i, pos + 1))
                if pos == last and has_generator and not fused and i % P != r:
                    post.append(("SEND", i % P, "OUT", i, last))
            else:
                if pos < last and (pos + 1) % P != r:
                    pre.append(("RECV", (pos + 1) % P, "GRAD", i, pos + 1))
                if pos == last and has_generator and not fused and i % P != r:
                    pre.append(("RECV", i % P, "OGRAD", i, last))
                if pos > 0 and (pos - 1) % P != r:
                    post.append(("SEND", (pos - 1) % P, "GRAD", i, pos))
                if pos == 0 and not fused and i % P != r:
                    post.append(("SEND", i % P, "FGRAD", i, 0))
        else:
            m = i * P + r
            if kind == "E" and r != 0:
                post.append(("SEND", 0, "FEAT", m, 0))
            if kind == "e" and r != 0:
                pre.append(("RECV", 0, "FGRAD", m, 0))
            if kind == "G" and r != P - 1:
                pre.append(("RECV", P - 1, "OUT", m, last))
            if kind == "H" and r != P - 1:
                post.append(("SEND", P - 1, "OGRAD", m, last))
        out += pre + [op] + post
    return out


def check_comm(order: str, P: int, V: int, M: int, W: int, has_generator: bool) -> Dict[str, object]:
    """Runs the P rank programs with eager sends and blocking receives.

    A compute op also waits for the tensors its own rank produces for it; an op placed
    before its local producer therefore shows up as a deadlock.
    Returns {"deadlock": bool, "messages": total sends, "unmatched": sends without a
    receive plus receives without a send, "fifo": whether, for every ordered pair of
    ranks, messages are received in the order they were sent (what a transport that
    matches by order alone needs), "max_inflight": largest number of posted but not
    yet received messages on one ordered pair}."""
    progs = [comm_rank_schedule(order, P, V, M, W, has_generator, r) for r in range(P)]
    sends = {}
    recvs = {}
    for r, prog in enumerate(progs):
        for op in prog:
            if op[0] == "SEND":
                sends[(r, op[1]) + op[2:]] = sends.get((r, op[1]) + op[2:], 0) + 1
            elif op[0] == "RECV":
                recvs[(op[1], r) + op[2:]] = recvs.get((op[1], r) + op[2:], 0) + 1
    unmatched = sum(abs(sends.get(k, 0) - recvs.get(k, 0)) for k in set(sends) | set(recvs))
    unmatched += sum(v - 1 for v in sends.values() if v > 1)

    last = P * V - 1
    fused = order == MEMORY_EFFICIENT

    def local_inputs(r: int, op: tuple) -> List[tuple]:
        """Tensors a compute op consumes that its own rank produces (no message exists for
        them, so the producer must simply have run already)."""
        kind, i, c = op
        need: List[tuple] = []
        if kind == "F":
            p_ = c * P + r
            if p_ > 0 and (p_ - 1) % P == r:
                need.append(("F", i, c - 1))
            if p_ == 0 and not fused and i % P == r:
                need.append(("E", i // P, 0))
        elif kind == "B":
            p_ = c * P + r
            need.append(("F", i, c))
            if p_ < last and (p_ + 1) % P == r:
                need.append(("B", i, c + 1))
            if p_ == last and has_generator and not fused and i % P == r:
                need.append(("H", i // P, 0))
        elif kind == "e":
            need.append(("E", i, 0))
            if r == 0:
                need.append(("B", i * P, 0))
        elif kind == "G" and r == P - 1:
            need.append(("F", i * P + r, V - 1))
        elif kind == "H":
            need.append(("G", i, 0))
        return need

    posted = set()
    ran = [set() for _ in range(P)]
    pos = [0] * P
    inflight: Dict[Tuple[int, int], int] = {}
    max_inflight = 0
    sent_order: Dict[Tuple[int, int], list] = {}
    recv_order: Dict[Tuple[int, int], list] = {}
    remaining = sum(len(p) for p in progs)
    deadlock = False
    while remaining:
        progressed = False
        for r in range(P):
            while pos[r] < len(progs[r]):
                op = progs[r][pos[r]]
                if op[0] == "SEND":
                    key = (r, op[1]) + op[2:]
                    posted.add(key)
                    pair = (r, op[1])
                    inflight[pair] = inflight.get(pair, 0) + 1
                    max_inflight = max(max_inflight, inflight[pair])
                    sent_order.setdefault(pair, []).append(op[2:])
                elif op[0] == "RECV":
                    key = (op[1], r) + op[2:]
                    if key not in posted:
                        break
                    pair = (op[1], r)
                    inflight[pair] -= 1
                    recv_order.setdefault(pair, []).append(op[2:])
                else:
                    if any(n not in ran[r] for n in local_inputs(r, op)):
                        break                      # consumes a tensor its own rank has not produced yet
                    ran[r].add(op)
                pos[r] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            deadlock = True
            break
    fifo = (not deadlock) and all(sent_order.get(k, []) == recv_order.get(k, []) for k in set(sent_order) | set(recv_order))
    return {"deadlock": deadlock, "messages": sum(sends.values()), "unmatched": unmatched, "fifo": fifo,
            "max_inflight": max_inflight}
