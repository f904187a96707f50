"""Brute-force pLogP event simulator -- TEST INFRASTRUCTURE ONLY.

Replays the send/receive schedule of each collective strategy under the
pLogP rules the paper's models are built from (Section 2: gap g(z) of a
message of size z, latency L) and returns the completion time in exact
rational arithmetic.  It knows nothing of the closed forms of Tables 1 and
2: it only knows who sends what to whom and in which order, so it checks
the oracle's transcription of those tables from the outside.

Rules:
  * A node runs its program (a list of sends and receives) in order.
  * A send of z bytes that starts at time t keeps the sender busy until
    t + g(z); the message is at the receiver at t + g(z) + L.
  * A receive completes when the message is there (waiting costs nothing
    else); the node's clock moves to that time.
  * The gap holds at the receiving end as well (it is the least interval
    between consecutive transmissions or receptions of a node): a reception
    of z bytes completes no earlier than g(z) after the node's previous
    reception did.  In the schedules of Tables 1 and 2 every node has one
    parent, whose sends already lie a gap apart, so the rule only shows where
    several nodes send to one (Gather, Barrier).
  * A node forwards only what it has fully received.
The completion time of a collective is the largest clock over all nodes.
"""
from __future__ import annotations

from fractions import Fraction
from typing import Callable, Dict, List, Tuple

Action = Tuple  # ("send", dst, size, tag) | ("recv", src, tag)


def run(programs: Dict[int, List[Action]], g: Callable[[int], Fraction], L: Fraction) -> Fraction:
    """Execute the per-node programs; return the time the last node finishes."""
    clock = {n: Fraction(0) for n in programs}
    pc = {n: 0 for n in programs}
    last_reception = {n: None for n in programs}     # when the node's previous reception completed
    arrival: Dict[Tuple[int, int, object], Tuple[Fraction, int]] = {}
    progressed = True
    while progressed:
        progressed = False
        for n, prog in programs.items():
            while pc[n] < len(prog):
                act = prog[pc[n]]
                if act[0] == "send":
                    _, dst, size, tag = act
                    end = clock[n] + g(size)
                    clock[n] = end
                    key = (n, dst, tag)
                    assert key not in arrival, "duplicate message"
                    arrival[key] = (end + L, size)
                else:
                    _, src, tag = act
                    key = (src, n, tag)
                    if key not in arrival:
                        break                    # not sent yet: come back later
                    there, size = arrival[key]
                    if last_reception[n] is not None:
                        there = max(there, last_reception[n] + g(size))
                    last_reception[n] = there
                    clock[n] = max(clock[n], there)
                pc[n] += 1
                progressed = True
    for n, prog in programs.items():
        assert pc[n] == len(prog), "deadlock in schedule of node %d" % n
    return max(clock.values())


# ---------------------------------------------------------------- schedules

def _payload(progs, src, dst, size, tag, rendezvous):
    """src hands `size` bytes to dst; with rendezvous, a 1-byte request and a
    1-byte reply go first."""
    if rendezvous:
        progs[src].append(("send", dst, 1, ("req", tag)))
        progs[dst].append(("recv", src, ("req", tag)))
        progs[dst].append(("send", src, 1, ("ack", tag)))
        progs[src].append(("recv", dst, ("ack", tag)))
    progs[src].append(("send", dst, size, tag))
    progs[dst].append(("recv", src, tag))


def bcast_flat(P, m, rendezvous=False, seg=None):
    """Root sends the message (or its k segments, one child after the other)
    to each of the P-1 other nodes in turn."""
    progs = {n: [] for n in range(P)}
    for child in range(1, P):
        if seg is None:
            _payload(progs, 0, child, m, "msg", rendezvous)
        else:
            k = -(-m // seg)
            for c in range(k):
                _payload(progs, 0, child, seg, ("seg", c), False)
    return progs


def bcast_chain(P, m, rendezvous=False, seg=None):
    """Node i passes the message on to node i+1; with segments, segment by
    segment (pipeline)."""
    progs = {n: [] for n in range(P)}
    if seg is None:
        for n in range(P - 1):
            _payload(progs, n, n + 1, m, "msg", rendezvous)
        return progs
    k = -(-m // seg)
    # each node alternates: receive segment c, forward segment c
    for c in range(k):
        for n in range(P - 1):
            progs[n].append(("send", n + 1, seg, ("seg", c)))
            progs[n + 1].append(("recv", n, ("seg", c)))
    return progs


def _binomial_children(P):
    """Binomial tree on P nodes rooted at 0: node n's children are n + 2^j for
    every 2^j larger than n's lowest set bit range, largest subtree first."""
    children = {n: [] for n in range(P)}
    top = 1
    while top < P:
        top <<= 1
    for n in range(P):
        j = top >> 1
        while j >= 1:
            if n % (2 * j) == 0 and n + j < P:
                children[n].append((n + j, j))      # (child, size of its subtree slot)
            j >>= 1
    return children


def bcast_binomial(P, m, rendezvous=False, seg=None):
    progs = {n: [] for n in range(P)}
    children = _binomial_children(P)
    order = sorted(range(P), key=lambda n: bin(n).count("1"))   # parents before children
    for n in order:
        for child, _ in children[n]:
            if seg is None:
                _payload(progs, n, child, m, "msg", rendezvous)
            else:
                k = -(-m // seg)
                for c in range(k):
                    _payload(progs, n, child, seg, ("seg", c), False)
    return progs


def bcast_binary(P, m):
    """Heap-ordered binary tree: node n sends to 2n+1 then to 2n+2."""
    progs = {n: [] for n in range(P)}
    for n in range(P):
        for child in (2 * n + 1, 2 * n + 2):
            if child < P:
                _payload(progs, n, child, m, "msg", False)
    return progs


def scatter_flat(P, m):
    progs = {n: [] for n in range(P)}
    for child in range(1, P):
        _payload(progs, 0, child, m, "part", False)
    return progs


def scatter_chain(P, m):
    """Node i keeps its share and passes the shares of all later nodes on."""
    progs = {n: [] for n in range(P)}
    for n in range(P - 1):
        _payload(progs, n, n + 1, (P - 1 - n) * m, "rest", False)
    return progs


def scatter_binomial(P, m):
    """Binomial tree; a child receives its own share together with the shares
    of its whole subtree (P a power of two: a subtree slot of size j holds j
    nodes)."""
    progs = {n: [] for n in range(P)}
    children = _binomial_children(P)
    order = sorted(range(P), key=lambda n: bin(n).count("1"))
    for n in order:
        for child, slot in children[n]:
            count = min(slot, P - child)
            _payload(progs, n, child, count * m, "part", False)
    return progs


def gather_flat(P, m):
    """Every node sends its share straight to the root, all at once; the root takes
    them in one after the other."""
    progs = {n: [] for n in range(P)}
    for child in range(1, P):
        _payload(progs, child, 0, m, "part", False)
    return progs


def gather_chain(P, m):
    """The last node sends its share to its neighbour, which adds its own and passes
    both on, and so on down to the root."""
    progs = {n: [] for n in range(P)}
    for n in range(P - 1, 0, -1):
        _payload(progs, n, n - 1, (P - n) * m, "rest", False)
    return progs


def gather_binomial(P, m):
    """The binomial tree of the Scatter, every message reversed: a node first takes
    in the shares of its subtrees, the smallest first, then sends everything it
    holds to its parent."""
    progs = {n: [] for n in range(P)}
    children = _binomial_children(P)
    order = sorted(range(P), key=lambda n: -bin(n).count("1"))   # children before parents
    parent = {c: n for n in range(P) for c, _ in children[n]}
    slot_of = {c: slot for n in range(P) for c, slot in children[n]}
    for n in order:
        for child, slot in sorted(children[n], key=lambda cs: cs[1]):
            progs[n].append(("recv", child, "part"))
        if n != 0:
            count = min(slot_of[n], P - n)
            progs[n].append(("send", parent[n], count * m, "part"))
    return progs


def barrier_flat(P):
    """Every node reports to the root with one byte; the root then releases each
    of them with one byte."""
    progs = {n: [] for n in range(P)}
    for child in range(1, P):
        _payload(progs, child, 0, 1, "in", False)
    for child in range(1, P):
        _payload(progs, 0, child, 1, "out", False)
    return progs


def barrier_binomial(P):
    """Binomial fan-in of one-byte messages (subtrees report smallest first), then
    the binomial broadcast of one byte."""
    progs = gather_binomial(P, 0)
    for n in progs:                                   # the reports carry one byte, whatever the subtree
        progs[n] = [("send", a[1], 1, "in") if a[0] == "send" else ("recv", a[1], "in") for a in progs[n]]
    out = bcast_binomial(P, 1)
    for n in progs:
        progs[n] += [("send", a[1], 1, "out") if a[0] == "send" else ("recv", a[1], "out") for a in out[n]]
    return progs


def completion_time(strategy: int, P: int, m: int, s: int, g, L) -> Fraction:
    """Replay strategy id (0..12 in the order of Tables 1 and 2, then Gather
    13..15 and Barrier 16, 17)."""
    L = Fraction(L)
    table = {
        0: lambda: bcast_flat(P, m),
        1: lambda: bcast_flat(P, m, rendezvous=True),
        2: lambda: bcast_flat(P, m, seg=s),
        3: lambda: bcast_chain(P, m),
        4: lambda: bcast_chain(P, m, rendezvous=True),
        5: lambda: bcast_chain(P, m, seg=s),
        6: lambda: bcast_binary(P, m),
        7: lambda: bcast_binomial(P, m),
        8: lambda: bcast_binomial(P, m, rendezvous=True),
        9: lambda: bcast_binomial(P, m, seg=s),
        10: lambda: scatter_flat(P, m),
        11: lambda: scatter_chain(P, m),
        12: lambda: scatter_binomial(P, m),
        13: lambda: gather_flat(P, m),
        14: lambda: gather_chain(P, m),
        15: lambda: gather_binomial(P, m),
        16: lambda: barrier_flat(P),
        17: lambda: barrier_binomial(P),
    }
    return run(table[strategy](), g, L)
