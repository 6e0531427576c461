"""Model check of the slot hand-over protocol of the paper's Communicator
(Section "Communicator"): a buffer written by a producer and read by a consumer,
reused over several iterations, synchronised only by flag words.

Model: each agent issues its program in order; its flag and data writes go into
a FIFO of its own and reach memory at an arbitrary later moment (in order) - a
late write.  Waits and reads look at memory only: the unit that polls a flag is
not the unit that posted the agent's own earlier write, so nothing is forwarded.
All interleavings of agent steps and write deliveries are explored.

Claim of the paper: with binary flags a late write can satisfy a future wait and
the consumer reads stale data; with monotonically increasing counters
(producer: wait semEmpty == i, write, semFull = i + 1; consumer: wait
semFull == i + 1, read, semEmpty = i + 1) it cannot."""
from collections import deque

ITER = 3


def programs(kind):
    prod, cons = [], []
    for i in range(ITER):
        if kind == "counter":
            prod += [("wait", "empty", i), ("write", "data", i), ("write", "full", i + 1)]
            cons += [("wait", "full", i + 1), ("read", i), ("write", "empty", i + 1)]
        else:   # binary flags: the waiter resets the flag it waited for
            prod += [("wait", "empty", 1), ("write", "empty", 0), ("write", "data", i), ("write", "full", 1)]
            cons += [("wait", "full", 1), ("write", "full", 0), ("read", i), ("write", "empty", 1)]
    return prod, cons


def explore(kind):
    """Returns (stale_read_possible, deadlock_possible)."""
    prod, cons = programs(kind)
    mem0 = (("data", -1), ("empty", 0 if kind == "counter" else 1), ("full", 0))
    start = (0, 0, mem0, (), ())           # pcs, visible memory, pending writes of P and of C
    seen, todo = {start}, deque([start])
    stale = deadlock = False
    while todo:
        pp, pc, mem, qp, qc = todo.popleft()
        m = dict(mem)
        nxt = []

        def view(q):                       # waits and reads see memory only, never a pending write
            return m
        for who, pc_, prog, q in (("P", pp, prod, qp), ("C", pc, cons, qc)):
            if pc_ < len(prog):
                op = prog[pc_]
                v = view(q)
                if op[0] == "wait":
                    if v[op[1]] == op[2]:
                        nxt.append((who, pc_ + 1, q, None))
                elif op[0] == "write":
                    nxt.append((who, pc_ + 1, q + ((op[1], op[2]),), None))
                else:                      # read: must see the data of its own iteration
                    if v["data"] != op[1]:
                        stale = True
                    nxt.append((who, pc_ + 1, q, None))
        for who, q in (("P", qp), ("C", qc)):
            if q:
                nxt.append((who, None, q[1:], q[0]))
        if not nxt and (pp < len(prod) or pc < len(cons)):
            deadlock = True
        for who, newpc, newq, deliver in nxt:
            m2 = dict(m)
            if deliver:
                m2[deliver[0]] = deliver[1]
            st = (newpc if who == "P" and newpc is not None else pp,
                  newpc if who == "C" and newpc is not None else pc,
                  tuple(sorted(m2.items())),
                  newq if who == "P" else qp, newq if who == "C" else qc)
            if st not in seen:
                seen.add(st)
                todo.append(st)
    return stale, deadlock


def test_binary_flags_admit_a_stale_read_when_a_write_is_late():
    stale, _ = explore("binary")
    assert stale


def test_monotonic_counters_never_read_stale_data_and_never_deadlock():
    stale, deadlock = explore("counter")
    assert not stale and not deadlock
