"""Oracle for the micrograph-merging bookkeeping (paper section 5.3), plain Python.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Written from the section's text: pick the
time step with the fewest root vertices, deal each model's roots of that step evenly to the
model's other steps, and in the examination period keep merging one more step per epoch while
the epoch time drops, undoing the first merge that does not help.
"""


def min_step(counts):
    totals = [sum(row[t] for row in counts) for t in range(len(counts[0]))]
    return totals.index(min(totals))


def apply(counts, ts):
    out = []
    for row in counts:
        others = [t for t in range(len(row)) if t != ts]
        share, extra = divmod(row[ts], len(others))
        new = []
        for k, t in enumerate(others):
            new.append(row[t] + share + (1 if k < extra else 0))
        out.append(new)
    return out


def examination(n_servers, epoch_times):
    """epoch_times(n_steps, epoch) -> run time.  Returns the list of step counts used per epoch."""
    used = []
    steps, prev, settled = n_servers, None, n_servers == 1
    epoch = 0
    while len(used) < 12:
        used.append(steps)
        t = epoch_times(steps, epoch)
        epoch += 1
        if settled:
            continue
        if prev is None:
            prev, steps = t, steps - 1
        elif t < prev:
            prev = t
            if steps > 1:
                steps -= 1
            else:
                settled = True
        else:
            steps, settled = steps + 1, True
    return used
