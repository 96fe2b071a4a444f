"""Oracle for the pipeline-execution model (EdgeShard Sec. 4.2 "Pipeline Execution
Optimization", Fig. 5).  Test infrastructure only: slow, plain, integer time.

Two independent formulations, neither shared with the library:
  * simulate_ticks: a clock that advances one tick at a time; every stage, when idle, takes
    the waiting task that arrived first (ties: lower iteration, then lower micro-batch).
    All times must be non-negative integers.  Covers both strategies.
  * bubbles_recurrence: for the Bubbles strategy the order on every stage is fixed
    (iteration-major, micro-batch-minor), so finish times follow the textbook pipeline
    recurrence F[i][m][s] = max(arrival from s-1, F[i][m-1][s], barrier_i) + duration.
"""


def simulate_ticks(t_prefill, t_decode, c_prefill, c_decode, c_return, n_micro, n_decode, no_bubbles):
    S, MB, IT = len(t_prefill), n_micro, 1 + n_decode
    waiting = [[] for _ in range(S)]          # (arrival tick, iteration, micro-batch)
    for m in range(MB):
        waiting[0].append((0, 0, m))
    running = [None] * S                      # (finish tick, iteration, micro-batch)
    busy = [0] * S
    arrivals = []                             # (tick, stage, iteration, micro-batch) still in flight
    home = {}                                 # (iteration, micro-batch) -> tick back at the source
    done, total, now, makespan = 0, S * MB * IT, 0, 0
    while done < total or arrivals:
        for a in [a for a in arrivals if a[0] == now]:
            arrivals.remove(a)
            waiting[a[1]].append((a[0], a[2], a[3]))
        # zero-length tasks can cascade within one tick: repeat until nothing changes
        changed = True
        while changed:
            changed = False
            for s in range(S):
                if running[s] is not None and running[s][0] == now:
                    _, it, m = running[s]
                    running[s] = None
                    done += 1
                    changed = True
                    if s + 1 < S:
                        c = c_prefill[s] if it == 0 else c_decode[s]
                        if c == 0:
                            waiting[s + 1].append((now, it, m))
                        else:
                            arrivals.append((now + c, s + 1, it, m))
                    else:
                        home[(it, m)] = now + c_return
                        makespan = max(makespan, now + c_return)
                        if it + 1 < IT:
                            if no_bubbles:
                                nxt = [(now + c_return, it + 1, m)]
                            elif all((it, mm) in home for mm in range(MB)):
                                gate = max(home[(it, mm)] for mm in range(MB))
                                nxt = [(gate, it + 1, mm) for mm in range(MB)]
                            else:
                                nxt = []
                            for (tk, i2, m2) in nxt:
                                if tk == now:
                                    waiting[0].append((tk, i2, m2))
                                else:
                                    arrivals.append((tk, 0, i2, m2))
            for s in range(S):
                if running[s] is None and waiting[s]:
                    task = min(waiting[s])
                    waiting[s].remove(task)
                    dur = t_prefill[s] if task[1] == 0 else t_decode[s]
                    running[s] = (now + dur, task[1], task[2])
                    busy[s] += dur
                    changed = True
        now += 1
        if now > 10 ** 7:
            raise RuntimeError("simulation does not end")
    return makespan, busy


def bubbles_recurrence(t_prefill, t_decode, c_prefill, c_decode, c_return, n_micro, n_decode):
    S, MB, IT = len(t_prefill), n_micro, 1 + n_decode
    gate = 0.0
    free = [0.0] * S
    makespan = 0.0
    for it in range(IT):
        t = t_prefill if it == 0 else t_decode
        c = c_prefill if it == 0 else c_decode
        back = []
        for m in range(MB):
            arrive = gate
            for s in range(S):
                start = max(arrive, free[s])
                free[s] = start + t[s]
                arrive = free[s] + (c[s] if s + 1 < S else c_return)
            back.append(arrive)
        gate = max(back)
        makespan = max(makespan, gate)
    return makespan
