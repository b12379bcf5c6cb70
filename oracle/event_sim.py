"""Event-driven execution of the fault-tolerant reduce: every process runs its own
program, blocks in its receives, and time passes only through sends and waits.

TEST INFRASTRUCTURE ONLY (see the package docstring).  This is a discrete-event
simulation with one coroutine per process, an event queue ordered by time and
per-process mailboxes.  It exists to pin the timed mode of ``ftred_oracle.c``
(which stamps times onto its round loop) with code that shares nothing with it
but the tree and group structure, and to show that values, statuses and message
counts of the event-driven execution are those of the round model.

The model (the paper gives no timing model; what it does say: section "Related
work", last paragraph: the active phase is a property of a process, processes
run their phases one after the other without regard to the progress of others;
section "Up-Correction", last paragraph, and the proof of the liveness property
in section "Reduce / Properties": a receive from a failed sender ends by a
time-out after which the failure monitor confirms the failure, and is retried
while the monitor says the sender lives):

* every process starts at time 0 and runs: for t = 1 .. f (while t <= group
  size - 1) send its input to its exchange target of round t, then receive from
  its exchange source of round t; then receive from each child in child order,
  then send to its parent.  The root receives from its children in order until
  a message without the failed bit is there, and delivers.
* a send takes ``t_msg`` of the sender's time; the message is in the receiver's
  mailbox when the send ends.  A receive ends at once when the message is
  already there, at its arrival otherwise.  A receiver that has waited
  ``t_timeout`` (>= 1) asks the monitor; if the sender has failed before that
  moment it gives up, else it waits another ``t_timeout``, and so on.  A
  message that arrives at the very moment of a time-out is received.
* failures keep the labels of the round model: a process with ``fail_round`` r
  stops when it reaches the first step whose round is >= r (0: it never
  starts); the exchange of round t is the step of round t, the receives from
  the children and the send to the parent are the step of round f + 1 + height
  (the root: f + D).  The moment it stops is the time the monitor knows.
"""
from __future__ import annotations

import heapq

NEVER = None


def _virt(p, root):
    # root relabelling (section "Reduce"): the root and process 0 swap places
    if root == 0:
        return p
    return 0 if p == root else (root if p == 0 else p)


def run_reduce(struct, x, combine, fail, t_msg, t_timeout, root=0, f=None):
    """struct: the arrays of ``oracle.structure`` (physical ranks); x[p]: the input of process p (any value
    ``combine`` takes); fail: {physical rank: fail_round}.  Returns a dict: status ('ok', 'root_failed',
    'no_clean'), result, t_done, t_proc[p] (time at which p finished its part, None if it failed first),
    msgs_uc, msgs_tree."""
    P = len(struct["parent"])
    parent = [int(v) for v in struct["parent"]]
    group = [int(v) for v in struct["group"]]
    gpos = [int(v) for v in struct["gpos"]]
    gsize = [int(v) for v in struct["gsize"]]
    send_round = [int(v) for v in struct["send_round"]]
    subtree = [int(v) for v in struct["subtree"]]
    D = int(struct["D"])
    kids = [[] for _ in range(P)]
    for p in range(P):
        if parent[p] >= 0:
            kids[parent[p]].append(p)
    for p in range(P):
        kids[p].sort(key=lambda q: _virt(q, root))
    members = {}
    for p in range(P):
        if group[p] >= 0:
            members.setdefault(group[p], {})[gpos[p]] = p
    last_round = f + D

    now = [0] * P                      # each process's own clock
    stopped_at = {}                    # physical rank -> time it failed
    mailbox = [dict() for _ in range(P)]          # (kind, src) -> (arrival, payload)
    waiting = [None] * P               # (kind, src) a process is blocked on
    events = []                        # (time, order, seq, what, ...)
    seq = [0]
    out = dict(status=None, result=None, t_done=NEVER, t_proc=[NEVER] * P, msgs_uc=0, msgs_tree=0)

    def alive_for(p, step_round):
        r = fail.get(p)
        return r is None or (r != 0 and step_round < r)

    def program(p):
        # yields ('send', dst, kind, payload) and ('recv', kind, src) -> payload or None
        val = x[p]
        if group[p] >= 0:
            gs = gsize[p]
            mem = members[group[p]]
            for t in range(1, f + 1):
                if t > gs - 1:
                    break
                if not alive_for(p, t):
                    if p == root:
                        out["status"] = "root_failed"
                    return
                yield ("send", mem[(gpos[p] + t) % gs], "uc", x[p])
                got = yield ("recv", "uc%d" % t, mem[(gpos[p] - t) % gs])
                if got is not None:
                    val = combine(val, got)
        if p != root:
            if not alive_for(p, send_round[p]):
                return
            flag = False
            for c in kids[p]:
                got = yield ("recv", "tree", c)
                if got is None:
                    flag = True
                else:
                    val = combine(val, got[0])
                    flag = flag or got[1]
            yield ("send", parent[p], "tree", (val, flag))
            yield ("done",)
        else:
            if not alive_for(p, last_round):
                out["status"] = "root_failed"
                return
            for c in kids[p]:
                got = yield ("recv", "tree", c)
                if got is None or got[1]:
                    continue
                # is the root's value in the message already?  Yes iff the child's subtree holds a member of the
                # root's up-correction group (section "Reduce / Algorithm")
                included = group[p] >= 0 and any(q != p and subtree[q] == subtree[c] for q in members[group[p]].values())
                out["result"] = got[0] if included else combine(val, got[0])
                out["status"] = "ok"
                out["t_done"] = now[p]
                yield ("done",)
                return
            out["status"] = "no_clean"
            out["t_done"] = now[p]
            yield ("done",)

    progs = [program(p) for p in range(P)]
    uc_round_of = [0] * P              # exchange messages carry their round in the mailbox key

    def push(time, order, *what):
        seq[0] += 1
        heapq.heappush(events, (time, order, seq[0]) + what)

    def step(p, answer=None):
        """Run process p from its clock until it blocks, ends or fails."""
        try:
            act = progs[p].send(answer)
            while True:
                if act[0] == "send":
                    _, dst, kind, payload = act
                    now[p] += t_msg
                    if kind == "uc":
                        uc_round_of[p] += 1
                        key = ("uc%d" % uc_round_of[p], p)
                        out["msgs_uc"] += 1
                    else:
                        key = (kind, p)
                        out["msgs_tree"] += 1
                    push(now[p], 0, "arrive", dst, key, payload)
                    act = progs[p].send(None)
                elif act[0] == "recv":
                    key = (act[1], act[2])
                    if key in mailbox[p]:
                        act = progs[p].send(mailbox[p].pop(key))
                        continue
                    waiting[p] = key
                    push(now[p] + t_timeout, 1, "timeout", p, key)
                    return
                else:                               # done
                    out["t_proc"][p] = now[p]
                    progs[p].close()
                    return
        except StopIteration:
            # the program ended early: the process failed at this moment (or the root gave up)
            if p not in stopped_at and out["t_proc"][p] is NEVER:
                stopped_at[p] = now[p]

    for p in range(P):
        step(p)
    while events:
        ev = heapq.heappop(events)
        time, what = ev[0], ev[3]
        if what == "arrive":
            _, _, _, _, dst, key, payload = ev
            if dst in stopped_at or out["t_proc"][dst] is not NEVER:
                continue                            # no reaction from a failed process; nobody waits any more
            if waiting[dst] == key:
                waiting[dst] = None
                now[dst] = max(now[dst], time)
                step(dst, payload)
            else:
                mailbox[dst][key] = payload
        else:
            _, _, _, _, p, key = ev
            if waiting[p] != key:
                continue
            src = key[1]
            if src in stopped_at and stopped_at[src] < time:
                waiting[p] = None
                now[p] = time
                step(p, None)
            else:
                push(time + t_timeout, 1, "timeout", p, key)
    return out
