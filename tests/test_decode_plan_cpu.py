"""CPU models of the grouped-query decode path (decode_plan_kernel + decode_gqa_kernel): no attention
arithmetic, only what decides whether an access is in bounds and whether a read sees its writer.

1. Index model: the planning rule (pieces of S rows, S doubled until the list fits) and the row walk of the
   attention kernel, checked against the segment capacities for long-context-like length mixes.
2. Workgroup-local protocol: the per-item use of the LDS cells s_next / s_part / s_last with ONE barrier per
   item (two more for a piece of a split segment).  All interleavings of the wavefronts of one workgroup are
   enumerated (explicit-state search) for 4 and for 8 wavefronts per workgroup; every read must return the
   value written for the same item.  Two planted mistakes (single-buffered cells) must be caught.
3. Cross-workgroup protocol: two workgroups claim items from the counter and hand the partial results of a
   split segment to the last arriver.  All interleavings of their global events are enumerated, with stores
   landing asynchronously; the arrival count may only be raised once the workgroup's own partial has landed
   (the wait in front of the arrival).  Without that wait the model finds the stale read.
"""
import itertools

import numpy as np


# ------------------------------------------------------------------------------------------- 1. indices
def plan_and_walk(base_lens, T, S0, NT, N=8192, steps=(1, 2, 100, 511, 512)):
    """Mirror of the index arithmetic: returns (S, pieces, highest row touched)."""
    n, BR = len(base_lens), NT * 16
    pieces_cap = n * (2 + N // 512)
    caps = base_lens + T
    worst = 0
    for t in steps:
        len_old = base_lens + t - 1
        app = len_old < caps
        ln = len_old + app
        S = S0
        while True:
            nps = np.maximum(1, (ln + S - 1) // S)
            total = int(nps.sum())
            if total <= pieces_cap or S >= 1 << 24:
                break
            S *= 2
        assert total <= pieces_cap
        assert S % BR == 0, "a block must not straddle two pieces"
        at = np.concatenate([[0], np.cumsum(nps)])
        for i in range(n):
            covered = 0
            for k in range(int(nps[i])):
                assert at[i] + k < pieces_cap
                row_lo = k * S
                row_hi = min(int(ln[i]), row_lo + S)
                nblk = (row_hi - row_lo + BR - 1) // BR if row_hi > row_lo else 0
                for blk in range(nblk):
                    r0 = row_lo + blk * BR
                    full = r0 + BR <= len_old[i]
                    hi_row = r0 + BR - 1 if full else min(int(ln[i]), r0 + BR) - 1
                    assert hi_row < caps[i], (i, k, blk, hi_row, caps[i])
                    assert r0 + BR <= row_lo + S
                    worst = max(worst, hi_row)
                covered += max(0, row_hi - row_lo)
            assert covered == ln[i], "the pieces of a segment cover its rows exactly once"
            if app[i]:
                assert (len_old[i] // S) < nps[i], "the appended row lies inside one piece"
    return S, total, worst


def test_plan_indices_stay_inside_the_segments():
    rng = np.random.default_rng(0)
    # lengths of the long-context workload: tens of rows in half of the layers, thousands in others
    per_layer = np.array([1641, 39, 1093, 32, 2072, 33, 33, 1811, 2103, 1962, 1104, 2255, 2128, 33, 543, 137, 35,
                          2598, 38, 42, 126, 34, 600, 36, 33, 41, 2446, 2153, 905, 39, 33, 37])
    base = np.concatenate([np.maximum(1, per_layer + rng.integers(-20, 20, 32)) for _ in range(4)])
    for S0 in (128, 256, 512, 1024, 2048, 4096):
        for NT in (1, 2, 4):
            S, total, worst = plan_and_walk(base, 512, S0, NT)
            assert S >= S0 and total >= len(base) and worst < (base + 512).max()
    # degenerate mixes: all minimal, all maximal, a single long segment among empty-ish ones
    for base in (np.ones(128, np.int64), np.full(128, 8192, np.int64),
                 np.concatenate([[8192], np.ones(127, np.int64)])):
        plan_and_walk(base, 512, 1024, 2)


# ------------------------------------------------------------------------------------------- 2. LDS protocol
def wavefront_program(tid, W, items, double_next=True, double_part=True):
    """Events of one wavefront (its first lane stands for it) over the item sequence.  items[i] = True for a
    piece of a split segment.  Cells are double-buffered by the parity of the item counter."""
    ops = []
    for it, split in enumerate(items):
        pn = it & 1 if double_next else 0
        pp = it & 1 if double_part else 0
        if tid == 0:
            ops.append(("w", ("s_next", pn), it))            # claim of the following item
        ops.append(("w", ("s_part", pp, tid), it))           # this wavefront's row of the merge buffer
        ops.append(("bar",))
        ops.append(("r", ("s_next", pn), it))
        ops.append(("r_rows", pp, it))                       # the merge reads every wavefront's row
        if split:
            ops.append(("bar",))
            if tid == 0:
                ops.append(("w", ("s_last", it & 1), it))
            ops.append(("bar",))
            ops.append(("r", ("s_last", it & 1), it))
    return ops


def explore_workgroup(W, items, **kw):
    """All interleavings of W wavefronts; returns the first violated read or None.  Wavefronts other than 0
    run the same program, so states that differ by a permutation of them are identified."""
    progs = [wavefront_program(t, W, items, **kw) for t in range(W)]

    start = tuple([0] * W)
    seen, stack = {start}, [(start, {})]
    # memory is carried explicitly: the last value written to each cell in this interleaving
    while stack:
        pcs, mem = stack.pop()
        at_bar = [pcs[t] < len(progs[t]) and progs[t][pcs[t]][0] == "bar" for t in range(W)]
        done = [pcs[t] >= len(progs[t]) for t in range(W)]
        succ = []
        if all(a or d for a, d in zip(at_bar, done)) and any(at_bar):
            assert all(at_bar), "a wavefront left the loop while others wait at a barrier"
            succ.append((tuple(p + 1 for p in pcs), mem))
        else:
            for t in range(W):
                if done[t] or at_bar[t]:
                    continue
                op = progs[t][pcs[t]]
                m2 = mem
                if op[0] == "w":
                    m2 = dict(mem)
                    m2[op[1]] = op[2]
                elif op[0] == "r":
                    if mem.get(op[1]) != op[2]:
                        return (t, op, mem.get(op[1]))
                elif op[0] == "r_rows":
                    for w in range(W):
                        if mem.get(("s_part", op[1], w)) != op[2]:
                            return (t, op, w, mem.get(("s_part", op[1], w)))
                nxt = list(pcs)
                nxt[t] += 1
                succ.append((tuple(nxt), m2))
        for pcs2, m2 in succ:
            # the row a wavefront last wrote is a function of its program counter, so the sorted counters of
            # wavefronts 1..W-1 identify the s_part rows up to that permutation; the other cells belong to wavefront 0
            key = (pcs2[0], tuple(sorted(pcs2[1:])), tuple(sorted((k, v) for k, v in m2.items() if k[0] != "s_part")))
            if key not in seen:
                seen.add(key)
                stack.append((pcs2, m2))
    return None


def test_lds_cells_are_read_by_the_item_that_wrote_them():
    for W in (4, 8):
        for items in itertools.product([False, True], repeat=3 if W == 8 else 4):
            assert explore_workgroup(W, list(items)) is None, (W, items)


def test_lds_model_catches_single_buffered_cells():
    # with one barrier per item, a cell that is not double-buffered is overwritten by the next item's writer
    # while a slower wavefront has not read it yet
    assert explore_workgroup(4, [False, False, False], double_next=False) is not None
    assert explore_workgroup(4, [False, False, False], double_part=False) is not None


# ------------------------------------------------------------------------------------------- 3. hand-off
def explore_handoff(items, n_wg=2, wait_before_arrival=True):
    """items: list of (segment, nsplit).  Workgroup i starts with item i and claims item counter + n_wg.
    Global events of a workgroup per item: claim, [store partial (lands later), wait, arrive, maybe combine],
    or the direct output.  Returns a description of the first violation or None."""
    total = len(items)

    def step(state):
        """yields successor states; a state is (wg tuple, counter, arrive dict, landed set, issued set, out dict)"""
        wgs, counter, arrive, landed, issued, out, done_items = state
        # asynchronous landing of issued stores
        for piece in issued - landed:
            yield (wgs, counter, arrive, landed | {piece}, issued, out, done_items), None
        for i, (item, pc, nxt) in enumerate(wgs):
            if item is None or item >= total:
                continue
            seg, nsplit = items[item]
            w = list(wgs)
            if pc == 0:                                        # claim the following item first
                w[i] = (item, 1, counter + n_wg)
                yield (tuple(w), counter + 1, arrive, landed, issued, out, done_items), None
            elif pc == 1:
                if item in done_items:
                    yield None, f"item {item} processed twice"
                    return
                if nsplit == 1:
                    if seg in out:
                        yield None, f"segment {seg} written twice"
                        return
                    o2 = dict(out); o2[seg] = "direct"
                    w[i] = (nxt, 0, None)
                    yield (tuple(w), counter, arrive, landed, issued, o2, done_items | {item}), None
                else:
                    w[i] = (item, 2, nxt)                      # partial stores issued
                    yield (tuple(w), counter, arrive, landed, issued | {item}, out, done_items | {item}), None
            elif pc == 2:                                      # wait for the own partial, then count in
                if wait_before_arrival and item not in landed:
                    continue                                   # blocked until the store has landed
                a2 = dict(arrive); old = a2.get(seg, 0); a2[seg] = old + 1
                w[i] = (item, 3 if old == nsplit - 1 else 4, nxt)
                yield (tuple(w), counter, a2, landed, issued, out, done_items), None
            elif pc == 3:                                      # last arriver: every piece must be readable
                pieces = [j for j, (s, _) in enumerate(items) if s == seg]
                missing = [j for j in pieces if j not in landed]
                if missing:
                    yield None, f"last arriver of segment {seg} reads pieces {missing} before they landed"
                    return
                if seg in out:
                    yield None, f"segment {seg} written twice"
                    return
                o2 = dict(out); o2[seg] = "combined"
                w[i] = (nxt, 0, None)
                yield (tuple(w), counter, arrive, landed, issued, o2, done_items), None
            elif pc == 4:
                w[i] = (nxt, 0, None)
                yield (tuple(w), counter, arrive, landed, issued, out, done_items), None

    def freeze(s):
        wgs, counter, arrive, landed, issued, out, done_items = s
        return (wgs, counter, tuple(sorted(arrive.items())), tuple(sorted(landed)), tuple(sorted(issued)),
                tuple(sorted(out.items())), tuple(sorted(done_items)))

    start = (tuple((i if i < total else None, 0, None) for i in range(n_wg)), 0, {}, frozenset(), frozenset(), {},
             frozenset())
    seen, stack, finals = {freeze(start)}, [start], 0
    while stack:
        s = stack.pop()
        succ = list(step(s))
        if not succ:
            wgs, _, _, _, _, out, done_items = s
            if any(item is not None and item < total for item, _, _ in wgs):
                return "deadlock"
            if len(done_items) != total or set(out) != {seg for seg, _ in items}:
                return f"finished with items {sorted(done_items)} and outputs {out}"
            finals += 1
        for s2, err in succ:
            if err:
                return err
            k = freeze(s2)
            if k not in seen:
                seen.add(k)
                stack.append(s2)
    assert finals > 0
    return None


def test_split_segment_handoff_all_interleavings():
    # segment 0 in two pieces, segment 1 whole, segment 2 in two pieces, in list order and interleaved
    for items in ([(0, 2), (0, 2)], [(0, 2), (0, 2), (1, 1)], [(0, 2), (1, 1), (0, 2)],
                  [(0, 2), (2, 2), (1, 1), (0, 2), (2, 2)], [(0, 3), (0, 3), (1, 1), (0, 3)]):
        for n_wg in (1, 2, 3):
            assert explore_handoff(items, n_wg=n_wg) is None, (items, n_wg)


def test_handoff_model_catches_a_missing_wait():
    err = explore_handoff([(0, 2), (0, 2)], n_wg=2, wait_before_arrival=False)
    assert err is not None and "before they landed" in err
