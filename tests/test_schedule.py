"""The window schedule (Sec. 1, Fig. 1, Sec. 3.3) as the library issues it,
checked on the host: the Fig. 1 worked setting, and by simulating the two
streams with random durations -- every layer is computed once per pass in
order, from a slot that holds exactly that layer for the whole compute, with
at most n_slots layers on the device."""
import os
import random

import pytest

from paper_2410_08791_amd import binding as sp

COPY, FWD, BWD = 0, 1, 2
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fig1_schedule.txt")


def test_fig1_setting_matches_the_paper():
    want = [tuple(l.split()) for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    ops = sp.trace_schedule(8, 4, 2)
    got = [("L" if k == COPY else "X", str(layer)) for k, layer, *_ in ops]
    assert got == want
    # never more than k = 4 layers on the device: slots are 0..3
    assert {s for _, _, s, _, _ in ops} == {0, 1, 2, 3}


def simulate(ops, n_layers, n_slots, seed):
    """Run the op list on a copy stream and a compute stream with random durations."""
    rnd = random.Random(seed)
    t_copy = t_comp = 0.0
    last_copy_end = {}      # layer -> end time of its most recent copy (in issue order)
    last_comp_end = {}      # layer -> end time of its most recent compute
    slot_events = {s: [] for s in range(n_slots)}   # (begin, end, kind, layer)
    computes = []
    for kind, layer, slot, wait, ps in ops:
        assert 0 <= slot < n_slots and 0 <= layer < n_layers
        if kind == COPY:
            start = t_copy
            if wait >= 0:
                start = max(start, last_comp_end.get(wait, 0.0))
            end = start + rnd.uniform(0.1, 3.0)
            t_copy = end
            last_copy_end[layer] = end
            slot_events[slot].append((start, end, "copy", layer))
        else:
            start = max(t_comp, last_copy_end.get(layer, 0.0))
            end = start + rnd.uniform(0.1, 3.0)
            t_comp = end
            last_comp_end[layer] = end
            slot_events[slot].append((start, end, "comp", layer))
            computes.append((ps, kind, layer))
    # per slot: events in issue order must not overlap in time, and every compute
    # must follow a copy of the same layer with no other copy in between
    for s, evs in slot_events.items():
        content = None
        t = 0.0
        for b, e, kind, layer in evs:
            assert b >= t - 1e-12, f"slot {s}: {kind} of layer {layer} starts before the previous op ended"
            t = e
            if kind == "copy":
                content = layer
            else:
                assert content == layer, f"slot {s} holds {content}, computing {layer}"
    return computes


@pytest.mark.parametrize("training", [False, True])
def test_schedule_invariants_over_a_grid(training):
    for L in range(1, 10):
        for N in range(1, L + 1):
            for p in range(1, max(N, 2)):
                for wrap in ([False, True] if not training else [False]):
                    passes = 4
                    ops = sp.trace_schedule(L, N, p, training=training, wrap=wrap, passes=passes)
                    computes = simulate(ops, L, N, seed=L * 1000 + N * 100 + p * 10 + wrap)
                    # every layer once per pass, in order (reverse order on backward passes)
                    for ps in range(passes):
                        seq = [l for q, k, l in computes if q == ps]
                        bwd = training and ps % 2 == 1
                        assert seq == (list(range(L - 1, -1, -1)) if bwd else list(range(L))), (L, N, p, ps)
                        kinds = {k for q, k, l in computes if q == ps}
                        assert kinds == ({BWD} if bwd else {FWD})
                    copies = [(ps, l) for k, l, s, w, ps in ops if k == COPY]
                    if N == L:      # fully resident: L copies in all, none after the first pass
                        assert len(copies) == L and all(ps == 0 for ps, _ in copies)
                    elif training:  # the turn re-uses the N layers still resident
                        per_pass = [sum(1 for ps, _ in copies if ps == q) for q in range(passes)]
                        assert per_pass[0] == L and all(c == L - N for c in per_pass[1:]), per_pass
                    elif wrap:      # steady state: L copies per call, none at the start of a call
                        per_pass = [sum(1 for ps, _ in copies if ps == q) for q in range(passes)]
                        assert per_pass[0] == L + N and all(c == L for c in per_pass[1:]), per_pass
                        for q in range(1, passes):
                            first = next(i for i, o in enumerate(ops) if o[4] == q)
                            assert ops[first][0] == FWD
                    else:           # each layer copied at most once per pass; only layers
                        for q in range(passes):   # left over from the previous pass are skipped
                            got = sorted(l for ps, l in copies if ps == q)
                            assert len(set(got)) == len(got) and L - N <= len(got) <= L
                        assert sorted(l for ps, l in copies if ps == 0) == list(range(L))


@pytest.mark.parametrize("training", [False, True])
def test_pinned_layers_are_copied_once_and_the_rest_stream(training):
    """Layers 0..R-1 sit in slots 0..R-1 from their first use on and are never copied
    again; the other layers use only the slots R..N-1; compute order and slot contents
    stay right (same replay as above)."""
    for L in range(2, 10):
        for N in range(2, L):
            for R in range(1, N):
                for p in range(1, max(N - R, 2)):
                    for wrap in ([False, True] if not training else [False]):
                        passes = 4
                        ops = sp.trace_schedule(L, N, p, training=training, wrap=wrap, passes=passes, pinned=R)
                        computes = simulate(ops, L, N, seed=L * 1000 + N * 100 + R * 10 + p)
                        for ps in range(passes):
                            seq = [l for q, k, l in computes if q == ps]
                            bwd = training and ps % 2 == 1
                            assert seq == (list(range(L - 1, -1, -1)) if bwd else list(range(L)))
                        copies = [(ps, l, s) for k, l, s, w, ps in ops if k == COPY]
                        for l in range(R):
                            assert [(ps, s) for ps, ll, s in copies if ll == l] == [(0, l)]
                        assert all(s >= R for ps, l, s in copies if l >= R)
                        assert all((s >= R) == (l >= R) for k, l, s, w, ps in ops if k != COPY)
                        per_pass = [sum(1 for ps, l, s in copies if ps == q and l >= R) for q in range(passes)]
                        ring = N - R
                        if training:    # the turn re-uses what the ring still holds
                            assert per_pass[0] == L - R and all(c == L - R - ring for c in per_pass[1:])
                        elif wrap:      # steady state: every streamed layer once per call
                            assert per_pass[0] == L - R + ring and all(c == L - R for c in per_pass[1:])


def test_backward_stops_above_frozen_layers():
    """Training with F frozen layers and no input gradient: the backward pass covers layers
    L-1..F only, never copies a layer below F, and the next forward starts at layer 0 again."""
    for L in range(2, 9):
        for N in range(1, L + 1):
            for F in range(0, L + 1):
                for R in ([0] if N < 2 or N == L else [0, 1]):
                    ops = sp.trace_schedule(L, N, 1, training=True, passes=4, pinned=R, frozen=F)
                    computes = simulate(ops, L, N, seed=L * 100 + N * 10 + F)
                    for ps in range(4):
                        seq = [l for q, k, l in computes if q == ps]
                        assert seq == (list(range(L - 1, F - 1, -1)) if ps % 2 else list(range(L))), (L, N, F, ps)
                    assert all(l >= F for k, l, s, w, ps in ops if k == COPY and ps % 2 == 1)


def test_pinned_zero_is_the_plain_schedule():
    for L, N, p in [(8, 4, 2), (12, 5, 3), (7, 7, 1)]:
        assert sp.trace_schedule(L, N, p, passes=3, wrap=True) == sp.trace_schedule(L, N, p, passes=3, wrap=True, pinned=0)


def test_refill_happens_in_groups_of_p():
    ops = sp.trace_schedule(12, 5, 3)
    kinds = "".join("L" if k == COPY else "X" for k, *_ in ops)
    assert kinds == "LLLLL" + "XXX" + "LLL" + "XXX" + "LLL" + "XXX" + "L" + "XXX"
    # a refill waits for exactly the layer it replaces
    for k, layer, slot, wait, _ in ops:
        if k == COPY and layer >= 5:
            assert wait == layer - 5


def test_trace_argument_errors():
    for args in [(0, 1, 1), (4, 0, 1), (4, 5, 1), (4, 2, 0)]:
        with pytest.raises(sp.SuperpipeError):
            sp.trace_schedule(*args)
    for pinned in (-1, 2, 3):
        with pytest.raises(sp.SuperpipeError):
            sp.trace_schedule(4, 2, 1, pinned=pinned)


@pytest.mark.parametrize("training", [False, True])
def test_rewritten_layers_cross_the_link_again_and_only_they(training):
    """sp_weights_updated in the schedule: every pass after an update computes a rewritten layer
    from a copy issued after the update; layers that were not rewritten keep their residency."""
    per_call = 2 if training else 1
    for L, N, p, pinned, upd in [(6, 6, 1, 0, [1, 4]), (6, 3, 1, 1, [0, 5]), (8, 4, 2, 2, [1, 2, 7]),
                                 (5, 2, 1, 0, [0, 1, 2, 3, 4]), (4, 4, 1, 0, [])]:
        calls = 3
        plain = sp.trace_schedule(L, N, p, training=training, passes=calls * per_call, pinned=pinned)
        ops = sp.trace_schedule(L, N, p, training=training, passes=calls * per_call, pinned=pinned, updated=upd)
        for seed in range(3):
            comp = simulate(ops, L, N, seed)
            assert len(comp) == calls * per_call * L
        # a rewritten layer: in each call after the first, its first compute is preceded by a copy
        # of it issued in the same call
        for call in range(1, calls):
            first_pass = call * per_call
            seen_copy = set()
            checked = set()
            for kind, layer, slot, wait, ps in ops:
                if ps < first_pass or ps >= first_pass + per_call:
                    continue
                if kind == COPY:
                    seen_copy.add(layer)
                elif layer in upd and layer not in checked:
                    assert layer in seen_copy, (L, N, upd, call, layer)
                    checked.add(layer)
            assert checked == set(upd)
        n_copies = lambda o: sum(1 for k, *_ in o if k == COPY)
        if N == L:
            # resident: the plain schedule copies each layer once, updates add one copy per call
            assert n_copies(plain) == L and n_copies(ops) == L + (calls - 1) * len(upd)
        else:
            assert n_copies(plain) <= n_copies(ops) <= n_copies(plain) + (calls - 1) * len(upd)


def test_trace_with_updates_argument_errors():
    import ctypes as C
    bad = (C.c_int * 1)(9)
    assert sp.sp_trace_schedule_updated(4, 2, 0, 1, 0, 0, 2, bad, 1, None, 0) == sp.SP_ERR_INVALID_ARG
    assert sp.sp_trace_schedule_updated(4, 2, 0, 1, 0, 0, 2, None, 1, None, 0) == sp.SP_ERR_INVALID_ARG
    assert sp.sp_trace_schedule_updated(4, 2, 0, 1, 0, 0, 2, None, 0, None, 0) > 0
