"""Level schedule of records over ring slots (oracle side).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

The paper's workers exchange whole parameter vectors over a network (Section
4.1); here a Send is a reference to a ring slot (Section 6.1's rotating queues,
index iter mod #queues), so records that touch no common slot in a conflicting
way may run side by side.  A record reads the slots of its sources and writes
its out slot.  Running the waves in order, members of a wave in any order,
must equal running the records in sequence order.
"""


def assign_waves(records, N, D):
    """Earliest wave per record: one after the last earlier writer of anything
    it reads, after every earlier reader of the slot it writes, and after the
    last earlier writer of that slot."""
    last_write = [[-1] * D for _ in range(N)]
    last_read = [[-1] * D for _ in range(N)]
    waves = []
    for r in records:
        w = 0
        for j, sl in zip(r.src_worker, r.src_slot):
            w = max(w, last_write[j][sl] + 1)
        o = r.out_slot
        w = max(w, last_read[r.worker][o] + 1, last_write[r.worker][o] + 1)
        for j, sl in zip(r.src_worker, r.src_slot):
            last_read[j][sl] = max(last_read[j][sl], w)
        last_write[r.worker][o] = w
        last_read[r.worker][o] = -1
        waves.append(w)
    return waves


def check_waves(records, waves, N, D):
    """True iff every conflicting pair (read-after-write, write-after-read,
    write-after-write on one slot) keeps its sequence order across waves, and
    no worker appears twice in a wave.  Written by pairs, not by the recurrence
    above, so it also judges wave numbers that some other code produced."""
    touched = {}
    for e, r in enumerate(records):
        for j, sl in zip(r.src_worker, r.src_slot):
            touched.setdefault((j, sl), []).append((e, "r"))
        touched.setdefault((r.worker, r.out_slot), []).append((e, "w"))
    for acc in touched.values():
        for x in range(len(acc)):
            e, me = acc[x]
            for y in range(x + 1, len(acc)):
                f, mf = acc[y]
                if e == f or (me == "r" and mf == "r"):
                    continue
                if not waves[e] < waves[f]:
                    return False
    seen = set()
    for e, r in enumerate(records):
        if (waves[e], r.worker) in seen:
            return False
        seen.add((waves[e], r.worker))
    return True
