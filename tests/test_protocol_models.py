"""Host-side models of the two hand-shakes inside the decode kernel, explored over every interleaving (CPU only).

The kernel's workgroups talk through a few counters in device memory.  These tests do not run the kernel: they restate
each protocol as a small state machine per workgroup (one atomic step = one access to shared state), let a scheduler pick
any runnable workgroup at every step, and walk the whole state space.  The hardware facts they assume are the ones the
kernel relies on: workgroups are dispatched in the order of their numbers, at most `capacity` are resident, a resident
workgroup runs until it ends, and a dispatched workgroup's next step is eventually taken.

1. A decode step in one call under splits by length (Sec. 2.2: the cache grows at its end; the split count of a sequence
   depends on its length).  The protocol that counted only the workgroups that had work is shown to let a late workgroup
   read the raised length; the protocol in the library (every workgroup counts itself once it has read the tables, the
   sequence's last workgroup in dispatch order raises the length when the count is complete) never does, never deadlocks,
   raises the length exactly once and leaves its counter at zero.
2. The merge of the splits: a workgroup counts itself on the arrival counter only after its partial is in memory; the one
   that counts last reads all partials.  Counting before the stores have landed (what a workgroup-scope fence alone gives)
   is shown to let the merging workgroup read a stale partial.
"""

import pytest


def explore(initial, steps_of, runnable, done):
    """Every state reachable from `initial`; `steps_of(state)` yields the successor states, one per runnable workgroup.
    Returns (all final states, whether some reachable state has no successor without being done = a deadlock)."""
    seen, stack, finals, deadlock = {initial}, [initial], set(), False
    while stack:
        st = stack.pop()
        nxt = list(steps_of(st))
        if not nxt:
            if done(st):
                finals.add(st)
            else:
                deadlock = True
            continue
        for n in nxt:
            if n not in seen:
                seen.add(n)
                stack.append(n)
    return finals, deadlock


# ---------------------------------------------------------------------------------------------------------------------
# 1. raising len16 while workgroups of the sequence may still have to read it
# ---------------------------------------------------------------------------------------------------------------------
def splits_used(tokens, splits, longest):
    return max(1, min(splits, -(-tokens * splits // longest)))        # ceil(tokens * splits / longest)


def append_model(n_heads, splits, capacity, tokens, longest, counts_everybody):
    """One sequence, n_heads KV heads, `splits` workgroups per head; workgroup number = split * n_heads + head (the head
    varies fastest, as in the kernel's grid).  State: (pc per workgroup, S each one computed, len16, per-head arrivals,
    sequence counter, number of times len16 was raised).  pc: 0 = not dispatched, 1 = dispatched (next: read the tables),
    2 = has work (next: arrive), 3 = waiting to raise the length, 9 = ended."""
    n = n_heads * splits
    last_wg = n - 1
    init = (tuple([0] * n), tuple([0] * n), tokens, tuple([0] * n_heads), 0, 0)

    def steps(st):
        pc, seen_s, len16, arrive, seq_ctr, raised = st
        resident = sum(1 for p in pc if p not in (0, 9))
        for w in range(n):
            head, split = w % n_heads, w // n_heads
            p = pc[w]
            if p == 0:                                               # dispatch: in order, if there is room
                if resident < capacity and all(q != 0 for q in pc[:w]):
                    yield (pc[:w] + (1,) + pc[w + 1:], seen_s, len16, arrive, seq_ctr, raised)
            elif p == 1:                                             # reads len16 (the tables), works out its split count
                s = splits_used(len16, splits, longest)
                ns = seen_s[:w] + (s,) + seen_s[w + 1:]
                if counts_everybody:                                 # the library: every workgroup counts itself here
                    nseq = seq_ctr + 1
                    if split >= s:
                        npc = 3 if w == last_wg else 9
                    else:
                        npc = 2
                    yield (pc[:w] + (npc,) + pc[w + 1:], ns, len16, arrive, nseq, raised)
                else:                                                # the earlier protocol: the ones without work just leave
                    yield (pc[:w] + (9 if split >= s else 2,) + pc[w + 1:], ns, len16, arrive, seq_ctr, raised)
            elif p == 2:                                             # its work is done: arrival on the head's counter
                s = seen_s[w]
                old = arrive[head]
                is_last = old == s - 1
                narr = arrive[:head] + ((0 if is_last else old + 1),) + arrive[head + 1:]
                if counts_everybody:
                    npc = 3 if w == last_wg else 9
                    yield (pc[:w] + (npc,) + pc[w + 1:], seen_s, len16, narr, seq_ctr, raised)
                else:                                                # the heads' last workgroups count; the last of them raises the length
                    if is_last:
                        if seq_ctr == n_heads - 1:
                            yield (pc[:w] + (9,) + pc[w + 1:], seen_s, len16 + 1, narr, 0, raised + 1)
                        else:
                            yield (pc[:w] + (9,) + pc[w + 1:], seen_s, len16, narr, seq_ctr + 1, raised)
                    else:
                        yield (pc[:w] + (9,) + pc[w + 1:], seen_s, len16, narr, seq_ctr, raised)
            elif p == 3:                                             # the sequence's last workgroup: waits for the full count
                if seq_ctr == n:
                    yield (pc[:w] + (9,) + pc[w + 1:], seen_s, len16 + 1, arrive, 0, raised + 1)

    done = lambda st: all(p == 9 for p in st[0])
    return explore(init, steps, None, done)


@pytest.mark.parametrize("n_heads,splits,capacity", [(1, 3, 2), (2, 3, 3), (2, 4, 4), (1, 4, 1)])
def test_counting_every_workgroup_keeps_the_split_count_of_a_launch_fixed(n_heads, splits, capacity):
    longest = 12
    for tokens in (4, 8, 9, 12):             # 4 -> 5 and 8 -> 9 cross a multiple of longest / splits for 3 or 4 splits
        finals, deadlock = append_model(n_heads, splits, capacity, tokens, longest, counts_everybody=True)
        assert not deadlock and finals
        s0 = splits_used(tokens, splits, longest)
        for pc, seen_s, len16, arrive, seq_ctr, raised in finals:
            assert set(seen_s) == {s0}                               # everybody computed the count from the old length
            assert len16 == tokens + 1 and raised == 1
            assert seq_ctr == 0 and set(arrive) == {0}               # the counters are ready for the next launch


def test_counting_only_the_workgroups_with_work_lets_a_late_one_read_the_raised_length():
    # 3 splits, longest 12: a sequence of 8 tokens uses 2 splits, of 9 tokens 3.  With room for two workgroups the third
    # is dispatched after the first two have ended, i.e. after the length has been raised.
    finals, deadlock = append_model(1, 3, 2, 8, 12, counts_everybody=False)
    bad = [f for f in finals if len(set(f[1])) > 1 or set(f[3]) != {0}]
    assert bad, "the earlier protocol should have an interleaving in which a workgroup disagrees about the split count"
    # ... and in that interleaving the head's arrival counter is left off by one for the next launch
    assert any(set(f[3]) != {0} for f in bad)
    # with room for every workgroup the same protocol can still go wrong or right, depending on the order
    finals_all, _ = append_model(1, 3, 3, 8, 12, counts_everybody=False)
    assert any(len(set(f[1])) == 1 for f in finals_all)


# ---------------------------------------------------------------------------------------------------------------------
# 2. the merge of the splits: partial in memory before the arrival is counted
# ---------------------------------------------------------------------------------------------------------------------
def merge_model(splits, waits_for_acknowledgement):
    """One (sequence, KV head).  A workgroup issues the store of its partial; the store lands in memory at some later
    step of its own (the memory system's, not the workgroup's); the workgroup counts itself either after the store has
    landed (the library: it waits for the acknowledgement) or right after issuing it; the one that counts last reads all
    partials.  memory[s] is 'old' (the previous launch's partial) until split s's store lands.
    State: (pc per workgroup, landed flags, counter, what the merging workgroup read).  pc: 0 store issued next,
    1 arrival next, 9 ended."""
    init = (tuple([0] * splits), tuple([False] * splits), 0, None)

    def steps(st):
        pc, landed, ctr, read = st
        for w in range(splits):
            if pc[w] == 0:                                           # issues its stores
                yield (pc[:w] + (1,) + pc[w + 1:], landed, ctr, read)
            elif pc[w] == 1:
                if waits_for_acknowledgement and not landed[w]:
                    continue                                         # (sits in its wait; the landing below is what lets it go on)
                is_last = ctr == splits - 1
                yield (pc[:w] + (9,) + pc[w + 1:], landed, 0 if is_last else ctr + 1, tuple(landed) if is_last else read)
        for w in range(splits):                                      # a store that has been issued lands
            if pc[w] != 0 and not landed[w]:
                yield (pc, landed[:w] + (True,) + landed[w + 1:], ctr, read)

    done = lambda st: all(p == 9 for p in st[0]) and all(st[1])
    return explore(init, steps, None, done)


@pytest.mark.parametrize("splits", [1, 2, 3, 4])
def test_merging_workgroup_reads_only_partials_that_have_landed(splits):
    finals, deadlock = merge_model(splits, waits_for_acknowledgement=True)
    assert not deadlock and finals
    for pc, landed, ctr, read in finals:
        assert read is not None and all(read), "a partial was read before it had landed"
        assert ctr == 0


def test_counting_before_the_stores_have_landed_can_merge_a_stale_partial():
    finals, deadlock = merge_model(2, waits_for_acknowledgement=False)
    assert not deadlock
    assert any(not all(f[3]) for f in finals)
