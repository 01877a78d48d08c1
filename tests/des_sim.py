"""A small discrete-event simulator of two in-order device queues with events.

Test helper, independent of both the product's predictor and the oracle's
recurrence: it knows nothing about layers or slots, only queue semantics.

  ("copy", dur, tag)      occupies the queue for dur
  ("exec", dur, tag)      occupies the queue for dur
  ("record", ev)          event ev takes the time at which the queue reaches this op
  ("wait", ev)            queue stalls until the LAST record of ev issued before this wait
                          (in host issue order) has completed; no-op if never recorded

Ops are given as one host-ordered list of (queue_name, op); each queue runs its
own ops in order.  Returns per-op (start, end) times in host order.
"""


def simulate(host_ops):
    # resolve each wait to the index of the record it refers to (host order semantics)
    last_record = {}
    resolved = []
    for idx, (q, op) in enumerate(host_ops):
        if op[0] == "record":
            last_record[op[1]] = idx
            resolved.append(None)
        elif op[0] == "wait":
            resolved.append(last_record.get(op[1], None))
        else:
            resolved.append(None)
    queues = {}
    for idx, (q, op) in enumerate(host_ops):
        queues.setdefault(q, []).append(idx)
    t_queue = {q: 0.0 for q in queues}
    head = {q: 0 for q in queues}
    done = {}    # idx -> (start, end)
    progressed = True
    while progressed:
        progressed = False
        for q, lst in queues.items():
            while head[q] < len(lst):
                idx = lst[head[q]]
                op = host_ops[idx][1]
                t = t_queue[q]
                if op[0] == "wait":
                    dep = resolved[idx]
                    if dep is not None:
                        if dep not in done:
                            break
                        t = max(t, done[dep][1])
                    done[idx] = (t_queue[q], t)
                elif op[0] == "record":
                    done[idx] = (t, t)
                else:
                    done[idx] = (t, t + op[1])
                    t = t + op[1]
                t_queue[q] = t
                head[q] += 1
                progressed = True
    if any(head[q] < len(lst) for q, lst in queues.items()):
        raise RuntimeError("deadlock in simulated queues")
    return [done[i] for i in range(len(host_ops))]
