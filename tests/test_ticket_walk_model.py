"""A plain Python model of the ordered persistent schedule's walk over the chunk table (no GPU).

The kernels hand out table entries like this: the table is cut into blocks of `span` entries; workgroup b of G owns
blocks b and b + G and then takes block 2G + ticket, where ticket is an atomic increment of one counter, requested one
block ahead.  Full chunks (the first nfull entries) go through a two-stage pipeline that always holds the current and
the next entry; the short chunks behind them are handled one at a time.  The model runs G workgroups as coroutines
that may be interleaved in any order at every atomic, and checks what must hold for every interleaving:

  * every entry in [0, nchunks) is handled exactly once, full ones by the pipeline, short ones by the tail loop;
  * what the pipeline computes is the entry whose loads it issued into that register set;
  * every workgroup leaves, whatever its tickets were (also when its last ticket lies past the table or was never
    looked at), and the number of tickets drawn is what the reset at the end of the launch has to clear.
"""
import random

import pytest


class Queue:
    def __init__(self):
        self.next = 0
        self.done = 0
        self.tickets_drawn = 0


def workgroup(b, G, span, nfull, nchunks, q, handled, log):
    """One persistent workgroup.  Yields at every point where another workgroup's atomic may come first."""
    st = dict(blk=b, second=b + G, second_pending=True, j=0, ticket=None)

    def next_entry():
        if st["j"] == span:                       # enter the next block
            st["j"] = 0
            if st["second_pending"]:
                st["blk"] = st["second"]
                st["second_pending"] = False
            else:
                assert st["ticket"] is not None   # a ticket is only looked at after it was requested
                st["blk"] = 2 * G + st["ticket"]
            yield                                 # other workgroups may draw tickets first
            st["ticket"] = q.next                 # the atomic increment, for the block after the next one
            q.next += 1
            q.tickets_drawn += 1
        e = st["blk"] * span + st["j"]
        st["j"] += 1
        return e

    e = yield from next_entry()
    n = yield from next_entry()
    assert e < n
    if e < nfull:
        reg_a = e                                 # loads of entry e issued into register set a
        while True:
            reg_b = n if n < nfull else e         # past the full chunks: the own chunk again, values unused
            assert reg_a == e
            handled[e].append(("pipeline", b))    # compute + store a
            n2 = yield from next_entry()
            if n >= nfull:
                e, n = n, n2
                break
            reg_a = n2 if n2 < nfull else n
            assert reg_b == n
            handled[n].append(("pipeline", b))    # compute + store b
            e = n2
            n = yield from next_entry()
            if e >= nfull:
                break
    while e < nchunks:
        handled[e].append(("tail", b))
        e = n
        n = yield from next_entry()
    log["left"] += 1
    q.done += 1
    if q.done == G:                               # the workgroup that completes the count zeroes the queue
        log["tickets_at_reset"] = q.next
        q.done = 0
        q.next = 0


def run_launch(G, span, nfull, nchunks, order, seed=0):
    q = Queue()
    handled = [[] for _ in range(nchunks)]
    log = {"left": 0}
    alive = [workgroup(b, G, span, nfull, nchunks, q, handled, log) for b in range(G)]
    rng = random.Random(seed)
    k = 0
    while alive:
        if order == "random":
            i = rng.randrange(len(alive))
        elif order == "round_robin":
            i = k % len(alive)
        elif order == "first_to_completion":      # one workgroup runs alone until it leaves
            i = 0
        else:                                     # the last workgroup always goes first
            i = len(alive) - 1
        k += 1
        try:
            next(alive[i])
        except StopIteration:
            alive.pop(i)
    assert log["left"] == G
    assert q.next == 0 and q.done == 0
    assert log["tickets_at_reset"] == q.tickets_drawn          # every ticket was drawn before the reset in this model
    for entry, hs in enumerate(handled):
        assert len(hs) == 1, "entry %d handled %d times (G=%d span=%d nfull=%d nchunks=%d)" % (entry, len(hs), G, span, nfull, nchunks)
        assert hs[0][0] == ("pipeline" if entry < nfull else "tail")
    return q.tickets_drawn


def grid_for(G, nchunks):
    """The launch never has more workgroups than pairs of chunks (what the host does)."""
    return max(1, min(G, (nchunks + 1) // 2))


@pytest.mark.parametrize("span", [1, 2, 4])
@pytest.mark.parametrize("G", [1, 2, 3, 4, 5, 6, 7, 8, 9, 64, 256])
def test_every_entry_exactly_once_small_tables(G, span):
    for nchunks in list(range(1, 40)) + [63, 64, 65, 127, 200, 257, 300]:
        fulls = sorted({0, 1, nchunks // 2, max(0, nchunks - 1), nchunks} & set(range(nchunks + 1)))
        for nfull in fulls:
            g = grid_for(G, nchunks)
            for order in ("round_robin", "first_to_completion", "last_first"):
                run_launch(g, span, nfull, nchunks, order)
            run_launch(g, span, nfull, nchunks, "random", seed=nchunks * 7 + nfull)


@pytest.mark.parametrize("span", [1, 2, 4])
def test_all_splits_of_small_tables_under_random_interleavings(span):
    for nchunks in range(1, 26):
        for nfull in range(0, nchunks + 1):
            for G in (1, 2, 3, 5, 8):
                for seed in range(3):
                    run_launch(grid_for(G, nchunks), span, nfull, nchunks, "random", seed=seed)


def test_more_workgroups_than_the_host_would_launch_still_terminate():
    # workgroups whose very first block lies past the table draw at most their look-ahead tickets and leave
    for G, nchunks in ((8, 3), (64, 10), (9, 1)):
        for span in (1, 2, 4):
            for order in ("round_robin", "random", "last_first"):
                run_launch(G, span, nchunks // 2, nchunks, order, seed=1)


def test_a_leaving_workgroup_holds_a_ticket_it_never_looked_at():
    # G = 1, six full chunks: the walk is 0, 1, then tickets 0.. -> blocks 2, 3, 4, 5, 6, 7: the entries 6 and 7 are past
    # the table, and one more ticket is outstanding when the workgroup leaves; the reset has to come after it
    drawn = run_launch(1, 1, 6, 6, "round_robin")
    assert drawn >= 6
