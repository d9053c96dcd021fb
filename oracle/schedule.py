"""CPU oracle for the schedule side: building blocks, repetition, pass orders, lifetime accounting.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file; the C++ schedule
generator in the library is a separate implementation and the two share no code.

Follows the paper's construction (Section 2): lay out the passes of ONE microbatch on a
device x time grid (the building block), repeat the block every T cells for the next microbatch
(legal only if no two passes land in one cell), and keep each device's pass order when bubbles are
squeezed out.  T is the number of unit passes a device runs per microbatch: 6 here (2 F, 2 B, 2 W).

V-shape blocks (Section 3, Section 3.1, Appendix A notation, Appendix F tables): the model is cut
into 2d chunks; device i holds chunk i ("chunk 0" of the device) and chunk 2d-1-i ("chunk 1").
Adjacent F passes of the first half are delta0 cells apart, of the second half delta1 cells apart;
B passes of the second half (which run device 0 -> d-1) use delta0 and B passes of the first half
use delta1.  Three same-device offsets complete the block: F turn-around on the last device, F->B
turn-around on the first device, B turn-around on the last device.  W passes then take, in the
order of their B passes, the first cell after their own B that is still free modulo T.

Readings where the paper is unclear (all listed in the design notes of the repository):
 * Appendix F's tables label the two B columns the other way round from Section 3.1's text; the
   text is followed (the literal table reading collides for every d).
 * The same-device offsets of V-ZB are found by brute force in the paper and never printed;
   (1, 1, 1) is used.  best_vzb_offsets() below repeats the brute force and is pinned to that.
 * The optional reordering step of Section 2 is not part of build(); reordered() applies it, with
   the readings stated there (warm-up moves may not raise a device's peak; the cool-down phase of
   a device starts after its last F).
 * A 1F1B stage is two consecutive chunks with B and W fused per chunk, upper chunk first.

Parity pins (tests/test_oracle_schedule.py): Section 3.2's exact peak formulas for every d, Table
1's peaks for 1F1B and V-ZB, Equation 1 as an upper bound, independence of n, balance across
devices, Table 1's bubble column, the bubble rate formula of Appendix D.3 for 1F1B, Appendix E.1's
condition for V-Half to have no repeating bubble, and for the reordering: unchanged peaks, the
least possible makespan for V-ZB.

PARITY UNPINNED by the paper (it prints nothing these could be checked against; what pins them is
this repository's own reading, stated in the tests):
 * the per-device ORDER of V-ZB (its same-device offsets are not printed; its peak is pinned);
 * reordered_passes: the paper prints no reordered order; two small grids worked by hand from
   Appendix C's two steps pin this reading of them;
 * adaptive_search: the winner's optimality is checked by a second brute force, but which of
   several equally fast blocks wins (the first in loop order) is this repository's rule;
 * the tensor-byte track of peak_bytes: pinned by hand to this repository's tensor table (the
   paper pins units only);
 * one_f_one_b_v_block (1F1B-V, Appendix H): the paper states the placement, the fused backward
   and the 2/3 asymptote (all pinned) but no offsets: the order is this repository's earliest fit.
"""
from __future__ import annotations

from dataclasses import dataclass
from itertools import product

T = 6
KINDS = ("1f1b", "vzb", "vhalf", "vmin")
# Further building blocks (Section 3.4, Appendix H), kept apart from KINDS: the paper describes them
# in a sentence each and its drawings are not available, so their pass orders are this
# repository's construction (see one_f_one_b_v_block).
MORE_KINDS = ("1f1bv",)
FUSED_KINDS = ("1f1b", "1f1bv")     # B and W of a chunk run as one pass


@dataclass(frozen=True)
class Pass:
    time: int      # cell index of the pass in the repeated (unsqueezed) grid
    device: int
    op: str        # "F", "B" or "W"
    chunk: int     # 0 or 1: which of the device's two chunks
    mb: int        # microbatch

    @property
    def key(self):
        return (self.op, self.chunk, self.mb)


def model_chunk(kind: str, d: int, device: int, chunk: int) -> int:
    """Position of a device's chunk in the model (0 .. 2d-1)."""
    if kind == "1f1b":
        return 2 * device + chunk
    return device if chunk == 0 else 2 * d - 1 - device


def vshape_params(kind: str, d: int):
    """(delta0, delta1, F turn on last device, F->B turn on first device, B turn on last device)."""
    if kind == "vmin":      # Table 1 row V-Min; Appendix F first table
        return 1, 1, 1, (3 if d % 3 == 0 else 1), 1
    if kind == "vhalf":     # Table 1 row V-Half; Appendix F second table
        return 2, 1, 2, (4 if d % 2 == 0 else 1), 1
    if kind == "vzb":       # Table 1 row V-ZB; same-device offsets not printed
        return 4, 2, 1, 1, 1
    raise ValueError(kind)


def vshape_block(d: int, delta0: int, delta1: int, a: int, b: int, c: int):
    """Cell index of each pass of one microbatch: dict (op, chunk) -> list over devices.
    Returns None if repeating the block every T cells would put two F/B passes in one cell."""
    tF0 = [i * delta0 for i in range(d)]
    tF1 = [0] * d
    tF1[d - 1] = tF0[d - 1] + a
    for i in range(d - 2, -1, -1):
        tF1[i] = tF1[i + 1] + delta1
    tB1 = [0] * d
    tB1[0] = tF1[0] + b
    for i in range(1, d):
        tB1[i] = tB1[i - 1] + delta0
    tB0 = [0] * d
    tB0[d - 1] = tB1[d - 1] + c
    for i in range(d - 2, -1, -1):
        tB0[i] = tB0[i + 1] + delta1
    tW1, tW0 = [0] * d, [0] * d
    for i in range(d):
        used = {tF0[i] % T, tF1[i] % T, tB1[i] % T, tB0[i] % T}
        if len(used) != 4:
            return None
        for tB, tW in ((tB1, tW1), (tB0, tW0)):     # chunk 1's B comes first on every device
            t = tB[i] + 1
            while t % T in used:
                t += 1
            used.add(t % T)
            tW[i] = t
    return {("F", 0): tF0, ("F", 1): tF1, ("B", 1): tB1, ("B", 0): tB0, ("W", 1): tW1, ("W", 0): tW0}


def one_f_one_b_block(d: int):
    """1F1B at chunk granularity: a stage's F covers two cells (lower chunk first), its fused
    backward four cells (B, W of the upper chunk, then B, W of the lower chunk).  Adjacent stages'
    forwards are 2 cells apart and backwards 4 cells apart (Table 1)."""
    tF = [2 * i for i in range(d)]
    tBW = [2 * d + 4 * (d - 1 - i) for i in range(d)]
    return {("F", 0): tF, ("F", 1): [t + 1 for t in tF],
            ("B", 1): tBW, ("W", 1): [t + 1 for t in tBW],
            ("B", 0): [t + 2 for t in tBW], ("W", 0): [t + 3 for t in tBW]}


def _fits(free, lengths):
    """Can passes of these lengths (cells in a row, modulo T) still be packed into the free residues?"""
    if not lengths:
        return True
    L = lengths[0]
    for r in sorted(free):
        cells = {(r + k) % T for k in range(L)}
        if len(cells) == L and cells <= free and _fits(free - cells, lengths[1:]):
            return True
    return False


def one_f_one_b_v_block(d: int, f_turn: int | None = None):
    """1F1B-V (Appendix H): the V-shape placement applied to 1F1B's block, WITHOUT splitting B and W:
    a chunk's backward is one fused pass of two cells (B, then W at once), and a device holds chunk i
    and chunk 2d-1-i.  The paper gives no offsets (its drawing is not available); this is an
    earliest-fit block.  Passes are placed in dependency order - F of the first half down the devices,
    F of the second half back up, the fused backward of the second half down, of the first half up -
    each at the first cell at or after the END of the pass it depends on (a fused pass hands its
    gradient on when the whole pass has ended, as in 1F1B) such that its own cells are free modulo T
    on its device and the device's passes still to come can be fitted into what stays free (the six
    residues of a device are exactly filled: 1 + 1 + 2 + 2 cells, so the block repeats without
    collision by construction).  One free parameter, the extra delay `f_turn` (0 .. T-1 cells) of the
    forward's turn on the last device, is chosen like V-ZB's same-device offsets (Section 3.1's brute
    force): least peak of live units, then least unit-time makespan, at n = 3d microbatches, first
    such value.  The peak tends to 2/3 of 1F1B's (pinned in the tests against the paper's statement),
    balanced over the devices."""
    if f_turn is None:
        best = None
        for a in range(T):
            blk = one_f_one_b_v_block(d, a)
            passes = repeat(blk, d, 3 * d)
            score = (max(peak_units_of(passes, "1f1bv", d)), makespan_of(passes, "1f1bv", d))
            if best is None or score < best[0]:
                best = (score, blk)
        return best[1]
    free = [set(range(T)) for _ in range(d)]

    def place(i, ready, length, later):
        t = ready
        while True:
            cells = {(t + k) % T for k in range(length)}
            if cells <= free[i] and _fits(free[i] - cells, later):
                free[i] -= cells
                return t
            t += 1

    tF0, tF1, tB1, tB0 = [0] * d, [0] * d, [0] * d, [0] * d
    for i in range(d):
        tF0[i] = place(i, 0 if i == 0 else tF0[i - 1] + 1, 1, [1, 2, 2])
    for i in range(d - 1, -1, -1):
        tF1[i] = place(i, (tF0[d - 1] + f_turn if i == d - 1 else tF1[i + 1]) + 1, 1, [2, 2])
    for i in range(d):
        tB1[i] = place(i, tF1[0] + 1 if i == 0 else tB1[i - 1] + 2, 2, [2])
    for i in range(d - 1, -1, -1):
        tB0[i] = place(i, (tB1[d - 1] if i == d - 1 else tB0[i + 1]) + 2, 2, [])
    return {("F", 0): tF0, ("F", 1): tF1, ("B", 1): tB1, ("W", 1): [t + 1 for t in tB1],
            ("B", 0): tB0, ("W", 0): [t + 1 for t in tB0]}


def block(kind: str, d: int):
    if d < 1:
        raise ValueError("d must be positive")
    if kind == "1f1b":
        return one_f_one_b_block(d)
    if kind == "1f1bv":
        return one_f_one_b_v_block(d)
    blk = vshape_block(d, *vshape_params(kind, d))
    if blk is None:
        raise ValueError(f"{kind} block collides for d={d}")
    return blk


def repeat(blk, d: int, n: int):
    """All passes of n microbatches: microbatch j's block is shifted by j*T.  Checks that no cell
    of any device is used twice."""
    passes = []
    seen = set()
    for (op, chunk), times in blk.items():
        for i in range(d):
            for j in range(n):
                t = times[i] + j * T
                if (i, t) in seen:
                    raise ValueError("collision")
                seen.add((i, t))
                passes.append(Pass(t, i, op, chunk, j))
    return passes


def device_orders(passes, d: int):
    """Per-device pass order: by cell index (squeezing keeps it)."""
    return [sorted((p for p in passes if p.device == i), key=lambda p: p.time) for i in range(d)]


def global_order(passes):
    """One-stream replay order: by cell index, ties between devices by device index.  Every
    dependency of a pass sits in a strictly earlier cell, so this is a topological order."""
    return sorted(passes, key=lambda p: (p.time, p.device))


def build(kind: str, d: int, n: int):
    return repeat(block(kind, d), d, n)


# --------------------------------------------------------------------------- lifetime accounting

def _order_peak(order, kind: str) -> int:
    live = peak = 0
    for p in order:
        if kind == "1f1b":
            if p.op == "F" and p.chunk == 0:
                live += 2
            elif p.op == "W" and p.chunk == 0:
                peak = max(peak, live)
                live -= 2
        else:
            if p.op == "F":
                live += 1
            elif p.op == "W":
                peak = max(peak, live)
                live -= 1
        peak = max(peak, live)
    return peak


def peak_units_of(passes, kind: str, d: int):
    """Peak number of live activation units per device for any pass list (Section 2.2: a unit is
    allocated when its F starts and retained until both its B and W are done).  For 1F1B the unit
    of allocation is the stage: both chunks' units are taken when the stage's F starts and returned
    when its fused backward ends."""
    return [_order_peak(order, kind) for order in device_orders(passes, d)]


def peak_units(kind: str, d: int, n: int):
    return peak_units_of(build(kind, d, n), kind, d)


def peak_bytes(kind: str, d: int, n: int, unit_bytes: int, stats_bytes: int):
    """Per device: (peak pool bytes, peak tensor bytes).

    Pool bytes count whole units of unit_bytes from F start to W end.  Tensor bytes follow the
    tensor table at pass boundaries: a unit weighs unit_bytes until its B has ended and
    unit_bytes - stats_bytes (the fp32 statistics are dead) from then until its W ends."""
    out = []
    units = peak_units(kind, d, n)
    for i, order in enumerate(device_orders(build(kind, d, n), d)):
        live = peak = 0
        for p in order:
            if kind == "1f1b":
                if p.op == "F" and p.chunk == 0:
                    live += 2 * unit_bytes
                elif p.op == "B":
                    peak = max(peak, live)
                    live -= stats_bytes
                elif p.op == "W" and p.chunk == 0:
                    live -= 2 * (unit_bytes - stats_bytes)
            else:
                if p.op == "F":
                    live += unit_bytes
                elif p.op == "B":
                    peak = max(peak, live)
                    live -= stats_bytes
                elif p.op == "W":
                    live -= unit_bytes - stats_bytes
            peak = max(peak, live)
        assert live == 0
        out.append((units[i] * unit_bytes, peak))
    return out


def lifespans(blk, d: int):
    """Per device, per chunk: cells from the start of F to the end of W."""
    return [[blk[("W", c)][i] + 1 - blk[("F", c)][i] for c in (0, 1)] for i in range(d)]


def equation1_bound(kind: str, d: int):
    """Equation 1: per device, sum over its chunks of ceil(lifespan / T) units.  For 1F1B the two
    chunks of a stage live from the stage's F start to the end of its fused backward."""
    blk = block(kind, d)
    out = []
    for i in range(d):
        if kind == "1f1b":
            l = blk[("W", 0)][i] + 1 - blk[("F", 0)][i]
            out.append(2 * -(-l // T))
        else:
            out.append(sum(-(-l // T) for l in lifespans(blk, d)[i]))
    return out


# --------------------------------------------------------------------------- squeezing (unit times)

def _dependencies(p: Pass, kind: str, d: int):
    """Keys (op, model chunk, microbatch) of the passes p waits for.  F of a model chunk needs F of
    the previous chunk (same microbatch); B needs B of the next chunk (the last chunk's B needs its
    own F); W needs its own B.  In 1F1B a stage's backward is one fused pass, so the stage before
    it waits for the end of that pass."""
    mc = model_chunk(kind, d, p.device, p.chunk)
    last = 2 * d - 1
    if p.op == "F":
        return [("F", mc - 1, p.mb)] if mc > 0 else []
    if p.op == "B":
        if mc == last:
            return [("F", mc, p.mb)]
        if kind == "1f1b" and p.chunk == 1:
            # B and W are one fused pass: the next stage hands its gradient over only when that
            # whole pass (which ends with its lower chunk's W) is done
            return [("W", mc + 1, p.mb)]
        if kind == "1f1bv":
            return [("W", mc + 1, p.mb)]      # the next chunk's fused pass ends with its W
        return [("B", mc + 1, p.mb)]
    return [("B", mc, p.mb)]


def _asap(orders, kind: str, d: int, dur):
    """Run every device's order as early as dependencies allow: a device runs one pass at a time in
    its fixed order.  Returns ({key: start}, {key: end}, finish time)."""
    start, end = {}, {}
    nxt = [0] * d
    free_at = [0.0] * d
    remaining = sum(len(o) for o in orders)
    while remaining:
        progressed = False
        for i in range(d):
            while nxt[i] < len(orders[i]):
                p = orders[i][nxt[i]]
                deps = _dependencies(p, kind, d)
                if any(dep not in end for dep in deps):
                    break
                k = (p.op, model_chunk(kind, d, p.device, p.chunk), p.mb)
                start[k] = max([free_at[i]] + [end[dep] for dep in deps])
                end[k] = free_at[i] = start[k] + dur[p.op]
                nxt[i] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise RuntimeError("deadlock: orders contradict dependencies")
    return start, end, max(free_at)


def _asap_finish(passes, kind: str, d: int, dur):
    return _asap(device_orders(passes, d), kind, d, dur)[2]


def makespan_of(passes, kind: str, d: int, tf: float = 1.0, tb: float = 1.0, tw: float = 1.0):
    """Finish time of any pass list when every device runs its order as early as it can."""
    return _asap_finish(passes, kind, d, {"F": tf, "B": tb, "W": tw})


def squeezed_makespan(kind: str, d: int, n: int, tf: float = 1.0, tb: float = 1.0, tw: float = 1.0):
    """Finish time of the squeezed schedule with the given pass durations."""
    return _asap_finish(build(kind, d, n), kind, d, {"F": tf, "B": tb, "W": tw})


def bubbles(kind: str, d: int, n: int):
    """Unit-time idle cells per device after squeezing: makespan minus the 6n cells of work."""
    return squeezed_makespan(kind, d, n) - T * n


def best_vzb_offsets(d: int, n: int | None = None):
    """The brute force of Section 3.1 for V-ZB's same-device offsets: among collision-free
    (a, b, c) below the repeating interval, those with the least (max peak units, squeezed
    makespan at unit pass times); returned sorted."""
    n = n or 4 * d
    scored = []
    for a, b, c in product(range(1, T), repeat=3):
        blk = vshape_block(d, 4, 2, a, b, c)
        if blk is None:
            continue
        passes = repeat(blk, d, n)
        peak = 0
        for order in device_orders(passes, d):
            live = 0
            for p in order:
                live += p.op == "F"
                peak = max(peak, live)
                live -= p.op == "W"
        span = _asap_finish(passes, "vzb", d, {"F": 1, "B": 1, "W": 1})
        scored.append(((peak, span), (a, b, c)))
    best = min(s for s, _ in scored)
    return sorted(t for s, t in scored if s == best)


# --------------------------------------------------------------------------- reordering (Appendix C)

def reordered(kind: str, d: int, n: int):
    """Reordering applied to the schedule that build(kind, d, n) gives; see reordered_passes."""
    return reordered_passes(build(kind, d, n), kind, d)


def reordered_passes(passes, kind: str, d: int):
    """The optional third step of Section 2, after the two greedy heuristics of Appendix C, on the
    squeezed grid with unit pass times.  Returns the passes with `time` set to their cell in the
    final squeezed grid (so device_orders / global_order apply unchanged).

    Warm-up: cells are visited left to right (devices in index order within a column); a vacant
    cell of a device that lies before that device's first B is filled with the first later pass of
    the same device whose dependencies have all ended by that cell, every other pass staying where
    it is.  Reading: a move is refused if it would lift the device's peak of live units above its
    peak before reordering (the paper states that reordering leaves the peak unchanged, Section 2).
    Cool-down: on every device the W passes after its last F are taken out, the rest is squeezed,
    and the vacant cells after the last F are then filled left to right, each with the first
    removed W (in their former order) whose B has ended; what is left goes to the end.
    A 1F1B stage (and a 1F1B-V chunk) runs B and W fused, so nothing of it can move: such a schedule
    is returned squeezed only."""
    unit = {"F": 1, "B": 1, "W": 1}
    key = lambda p: (p.op, model_chunk(kind, d, p.device, p.chunk), p.mb)
    orders = device_orders(passes, d)
    start, end, _ = _asap(orders, kind, d, unit)
    if kind not in FUSED_KINDS:
        base_peak = [_order_peak(o, kind) for o in orders]
        cells = [{int(start[key(p)]): p for p in orders[i]} for i in range(d)]
        first_b = [min(c for c, p in cells[i].items() if p.op == "B") for i in range(d)]
        for t in range(max(first_b)):
            for i in range(d):
                if t >= first_b[i] or t in cells[i]:
                    continue
                for c in sorted(c for c in cells[i] if c > t):
                    p = cells[i][c]
                    if any(end[dep] > t for dep in _dependencies(p, kind, d)):
                        continue
                    trial = dict(cells[i])
                    del trial[c]
                    trial[t] = p
                    if _order_peak([trial[x] for x in sorted(trial)], kind) > base_peak[i]:
                        continue
                    cells[i] = trial
                    start[key(p)], end[key(p)] = t, t + 1
                    break
        orders = [[cells[i][c] for c in sorted(cells[i])] for i in range(d)]
        kept, removed = [], []
        for order in orders:
            last_f = max(j for j, p in enumerate(order) if p.op == "F")
            kept.append([p for j, p in enumerate(order) if not (p.op == "W" and j > last_f)])
            removed.append([p for j, p in enumerate(order) if p.op == "W" and j > last_f])
        start, end, _ = _asap(kept, kind, d, unit)
        orders = []
        for i in range(d):
            cells_i = {int(start[key(p)]): p for p in kept[i]}
            pending = list(removed[i])
            t = max(c for c, p in cells_i.items() if p.op == "F") + 1
            while pending:
                if t not in cells_i:
                    ready = [w for w in pending if end[("B", model_chunk(kind, d, w.device, w.chunk), w.mb)] <= t]
                    if ready:
                        cells_i[t] = ready[0]
                        pending.remove(ready[0])
                t += 1
            orders.append([cells_i[c] for c in sorted(cells_i)])
        start, end, _ = _asap(orders, kind, d, unit)
    return [Pass(int(start[key(p)]), p.device, p.op, p.chunk, p.mb) for order in orders for p in order]


# --------------------------------------------------------------------------- adaptive search (Appendix A)

def vshape_block_split(d: int, K: int, d0_lo: int, d1_lo: int, d0_hi: int, d1_hi: int, a: int, b: int, c: int):
    """V-shape block whose offsets differ between the first K devices and the rest (Appendix A's
    two-part constraint, devices numbered 1..d there):
        delta F_i^0 = delta B_i^1 = d0_lo for 1 <= i < K,   d0_hi for K <= i < d,
        delta F_i^1 = delta B_i^0 = d1_lo for 1 < i <= K,   d1_hi for K < i <= d,
    with the three same-device offsets a, b, c of vshape_block (they fix which residue modulo T each
    pass of the first device takes: the "permutation of the first device").  K = d is the uniform
    block.  Returns None on a collision."""
    down = [d0_lo if i + 1 < K else d0_hi for i in range(d - 1)]      # device i -> i+1 (0-based i)
    up = [d1_lo if i + 1 <= K else d1_hi for i in range(1, d)]        # device i -> i-1, stored at i-1
    tF0 = [0] * d
    for i in range(d - 1):
        tF0[i + 1] = tF0[i] + down[i]
    tF1 = [0] * d
    tF1[d - 1] = tF0[d - 1] + a
    for i in range(d - 1, 0, -1):
        tF1[i - 1] = tF1[i] + up[i - 1]
    tB1 = [0] * d
    tB1[0] = tF1[0] + b
    for i in range(d - 1):
        tB1[i + 1] = tB1[i] + down[i]
    tB0 = [0] * d
    tB0[d - 1] = tB1[d - 1] + c
    for i in range(d - 1, 0, -1):
        tB0[i - 1] = tB0[i] + up[i - 1]
    tW1, tW0 = [0] * d, [0] * d
    for i in range(d):
        used = {tF0[i] % T, tF1[i] % T, tB1[i] % T, tB0[i] % T}
        if len(used) != 4:
            return None
        for tB, tW in ((tB1, tW1), (tB0, tW0)):
            t = tB[i] + 1
            while t % T in used:
                t += 1
            used.add(t % T)
            tW[i] = t
    return {("F", 0): tF0, ("F", 1): tF1, ("B", 1): tB1, ("B", 0): tB0, ("W", 1): tW1, ("W", 0): tW0}


def search_candidates(d: int, max_delta: int):
    """Parameter tuples (K, d0_lo, d1_lo, d0_hi, d1_hi, a, b, c) in the order the search visits
    them.  K = 1 would use the `hi` offsets everywhere and K = d the `lo` ones, so the uniform
    blocks are visited once, as K = d with hi = lo."""
    deltas = range(1, max_delta + 1)
    for K in range(2 if d > 1 else 1, d + 1):
        for d0_lo, d1_lo in product(deltas, deltas):
            for d0_hi, d1_hi in (product(deltas, deltas) if K < d else [(d0_lo, d1_lo)]):
                for a, b, c in product(range(1, T + 1), repeat=3):
                    yield K, d0_lo, d1_lo, d0_hi, d1_hi, a, b, c


def adaptive_search(d: int, n: int, limit_units: int, tf: float = 1.0, tb: float = 1.0, tw: float = 1.0,
                    max_delta: int = T, reorder: bool = True):
    """Appendix A as an exhaustive loop: every two-part block within the offset range is repeated
    (collisions dropped), dropped if some device's peak of live units over the n microbatches
    exceeds the limit, squeezed and (optionally) reordered, and timed with the given pass times;
    the first block with the least finish time wins.  Returns (finish time, parameters, passes)
    or None when no block fits the limit."""
    best = None
    for params in search_candidates(d, max_delta):
        blk = vshape_block_split(d, *params)
        if blk is None:
            continue
        passes = repeat(blk, d, n)
        if max(peak_units_of(passes, "vshape", d)) > limit_units:
            continue
        if reorder:
            passes = reordered_passes(passes, "vshape", d)
        span = makespan_of(passes, "vshape", d, tf, tb, tw)
        if best is None or span < best[0]:
            best = (span, params, passes)
    return best

