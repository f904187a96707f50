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
    arrival: Dict[Tuple[int, int, object], Fraction] = {}
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
                    arrival[key] = end + L
                else:
                    _, src, tag = act
                    key = (src, n, tag)
                    if key not in arrival:
                        break                    # not sent yet: come back later
                    clock[n] = max(clock[n], arrival[key])
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


def completion_time(strategy: int, P: int, m: int, s: int, g, L) -> Fraction:
    """Replay strategy id (0..12, the order of Tables 1 and 2)."""
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
    }
    return run(table[strategy](), g, L)
