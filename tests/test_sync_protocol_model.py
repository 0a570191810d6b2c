"""A model of how the 8-wavefront kernel hands K/V tiles from the wavefronts that load them to the wavefronts that read
them (the copy/GEMM overlap of Section 6 of the paper, done here with arrival counters in LDS instead of barriers),
explored over EVERY interleaving of a few wavefronts on the CPU.

The protocol, as the kernel runs it (ring of four buffers per operand, tile t of K and of V in buffer t mod 4):

  prologue   every wavefront loads its share of K tiles 0..3 and V tiles 0..2, waits for them, barrier;
             reads K tile 0; barrier.
  iteration j  reads V tile j and K tile j+1.
  boundary j   waits for its own outstanding loads; counts its arrival j (counter j mod 4); waits until the counter
             of iteration j-1 shows that all wavefronts made arrival j-1; then issues its share of K tile j+4 into
             the buffer of K tile j, and of V tile j+3 into the buffer of V tile j-1.

A load may land at any moment between its issue and the issuing wavefront's next wait for its loads: the model
overwrites the buffer's share at once (the worst case for a wavefront still reading the old tile) and calls it
complete only at that wait (the worst case for a wavefront about to read the new one).  The search visits every
reachable state of the scheduler's choices and checks three things: no read of a share that is not the expected
tile or not complete, no state from which no wavefront can move before all are done, and that every wavefront
finishes.  A read is checked when it begins and again when it ends, so an overwrite during the iteration shows too.
Two planted mistakes (one shared arrival counter; no wait for the others' arrivals) must be caught.
"""
import pytest

RING = 4


class Hazard(Exception):
    pass


def explore(waves, n_tiles, one_counter=False, no_wait=False):
    """Exhaustive search.  A wavefront's program is a list of steps; a state is (pcs, counters, buffers).
    Buffers: for K and V, per slot, per wavefront share: (tile held, complete?)."""
    # program of one wavefront, per iteration j: its reads begin, its reads end, then the boundary in three steps:
    # "arrive" (wait for the own loads, count the arrival), "wait" (for the others' arrival j-1), "load" (refill)
    prog = []
    for j in range(n_tiles):
        prog += [("read", j), ("read", j)]   # the iteration's reads begin ... and end
        if j + 1 < n_tiles:
            prog += [("arrive", j), ("wait", j), ("load", j)]
    n_steps = len(prog)

    def initial():
        k = tuple(tuple((t, True) for _ in range(waves)) for t in range(RING))           # K tiles 0..3
        v = tuple(tuple((t if t < RING - 1 else -1, True) for _ in range(waves)) for t in range(RING))  # V 0..2
        counters = (0,) * (1 if one_counter else RING)
        return (tuple([0] * waves), counters, k, v)

    def check_read(buf, tile, what):
        if tile >= n_tiles:
            return
        for share in buf[tile % RING]:
            if share != (tile, True):
                raise Hazard(f"{what} tile {tile}: a share holds {share}")

    def step(state, w):
        """The state after wavefront w takes its next step, or None if it cannot move."""
        pcs, counters, k, v = state
        kind, j = prog[pcs[w]]
        if kind == "read":
            check_read(v, j, "V")
            check_read(k, j + 1, "K")
        elif kind == "arrive":
            # the wait for the wavefront's own loads: its shares in flight are complete now
            k = tuple(tuple((t, True) if i == w else (t, c) for i, (t, c) in enumerate(slot)) for slot in k)
            v = tuple(tuple((t, True) if i == w else (t, c) for i, (t, c) in enumerate(slot)) for slot in v)
            idx = 0 if one_counter else j % RING
            counters = tuple(c + 1 if i == idx else c for i, c in enumerate(counters))
        elif kind == "wait":
            if j > 0 and not no_wait:
                if one_counter:
                    if counters[0] < waves * j:
                        return None
                elif counters[(j - 1) % RING] < waves * ((j - 1) // RING + 1):
                    return None
        elif kind == "load":
            kt, vt = j + RING, j - 1 + RING
            if kt < n_tiles:
                k = tuple(tuple((kt, False) if (s == kt % RING and i == w) else sh for i, sh in enumerate(slot))
                          for s, slot in enumerate(k))
            if vt < n_tiles:
                v = tuple(tuple((vt, False) if (s == vt % RING and i == w) else sh for i, sh in enumerate(slot))
                          for s, slot in enumerate(v))
        pcs = tuple(p + 1 if i == w else p for i, p in enumerate(pcs))
        return (pcs, counters, k, v)

    seen, stack, finished, lead = set(), [initial()], 0, 0
    while stack:
        state = stack.pop()
        if state in seen:
            continue
        seen.add(state)
        pcs = state[0]
        its = [prog[p][1] if p < n_steps else n_tiles - 1 for p in pcs]
        lead = max(lead, max(its) - min(its))
        if all(p == n_steps for p in pcs):
            finished += 1
            continue
        moved = False
        for w in range(waves):
            if pcs[w] == n_steps:
                continue
            nxt = step(state, w)
            if nxt is not None:
                moved = True
                stack.append(nxt)
        if not moved:
            raise Hazard(f"deadlock at {pcs}")
    assert finished >= 1
    return len(seen), lead


@pytest.mark.parametrize("waves,n_tiles", [(2, 12), (3, 9), (4, 6)])
def test_every_interleaving_is_safe(waves, n_tiles):
    states, lead = explore(waves, n_tiles)
    print(f"{waves} wavefronts, {n_tiles} tiles: {states} states, largest lead {lead} iterations")
    assert states > 100
    # the slack is real and bounded: to leave boundary j a wavefront needs everyone's arrival j-1, so while it reads
    # iteration j+1 the slowest may still stand in boundary j-1 (its reads of iteration j-1 over), and no further back
    assert lead == 2


def test_one_shared_counter_is_caught():
    # a wavefront arrives before it waits, so it can be two arrivals ahead of the slowest: a single running count
    # then passes while one wavefront has not arrived (the first version of the kernel made this mistake)
    with pytest.raises(Hazard):
        explore(3, 9, one_counter=True)


def test_no_wait_for_the_others_is_caught():
    with pytest.raises(Hazard):
        explore(2, 10, no_wait=True)
