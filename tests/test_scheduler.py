"""Embedding tracker, Algorithm 1 and Algorithm 2: the oracle against what the paper fixes, then the C++ library
against the oracle (bit-exact integers).  Host only: no test here needs a GPU."""
import numpy as np
import pytest

from oracle import TrackedRequest, encoder_batches, schedule_round
from paper_2509_24381_amd.binding import RsError, Scheduler

T, M = False, True


# ------------------------------------------------------------------ oracle pins
def test_tracker_walkthrough_of_section_3_1_case0():
    """Figure 'embedding tracker', Case0: [Text1, MM1, Text2, MM2].  Text1 is prefilled while MM1 is encoded; MM1's
    arrival triggers the prefill of MM1 and Text2; MM2's arrival that of MM2."""
    r = TrackedRequest(1, [(T, 7), (M, 20), (T, 5), (M, 11)])
    assert r.schedulable_tokens() == 7
    s, q = schedule_round([r], 1000)
    assert [(x[1], x[2]) for x in s] == [(0, 7)] and q == [r]
    assert r.schedulable_tokens() == 0                      # waiting for the encoder
    r.mark_ready(1)
    assert r.schedulable_tokens() == 25                     # MM1 + Text2
    s, q = schedule_round(q, 1000)
    assert [(x[1], x[2]) for x in s] == [(7, 25)]
    r.mark_ready(3)
    s, q = schedule_round(q, 1000)
    assert [(x[1], x[2]) for x in s] == [(32, 11)] and q == []


def test_tracker_case1_consecutive_items_need_no_text_between():
    """Case1: two consecutive multimodal items: MM1 can be prefilled while MM2 is still being encoded."""
    r = TrackedRequest(2, [(M, 9), (M, 4), (T, 3)])
    assert r.schedulable_tokens() == 0
    r.mark_ready(0)
    assert r.schedulable_tokens() == 9
    r.mark_ready(1)
    assert r.schedulable_tokens() == 16


@pytest.mark.parametrize("seed", range(4))
def test_paper_walkthroughs_from_the_fixture(seed):
    """tests/golden/tracker_walkthroughs.json restates the paper's two walkthroughs of the tracker (section 3.1) as event
    sequences without token counts; with any counts, the oracle and the library must prefill exactly the named segments,
    whole and in order, at every step."""
    import json
    import os
    rng = np.random.default_rng(seed)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tracker_walkthroughs.json")
    for case in json.load(open(path))["cases"]:
        names = case["segments"]
        segs = [(n.startswith("MM"), int(rng.integers(1, 50))) for n in names]
        begin = np.concatenate([[0], np.cumsum([n for _, n in segs])])
        r = TrackedRequest(7, segs)
        lib = Scheduler(10 ** 6)
        lib.add_request(7, segs)
        q = [r]
        for step in case["steps"]:
            for n in step["ready"]:
                r.mark_ready(names.index(n))
                lib.mark_ready(7, names.index(n))
            want = [names.index(n) for n in step["prefilled"]]
            first = int(begin[want[0]]) if want else r.prefilled
            count = int(sum(segs[k][1] for k in want))
            assert r.schedulable_tokens() == count == lib.schedulable_tokens(7), (case["name"], step)
            s, q = schedule_round(q, 10 ** 6)
            assert [(x[1], x[2]) for x in s] == [(first, count)], (case["name"], step)
            entries = lib.next_round()
            assert [(e[1], e[2]) for e in entries] == [(first, count)], (case["name"], step)
        assert q == [] and lib.queue_length() == 0, case["name"]


def test_out_of_order_encoder_results_do_not_unlock_later_tokens():
    r = TrackedRequest(3, [(T, 2), (M, 5), (M, 6)])
    r.mark_ready(2)
    assert r.schedulable_tokens() == 2          # MM at segment 1 still blocks
    r.mark_ready(1)
    assert r.schedulable_tokens() == 13


def test_algorithm1_worked_example():
    """Items of 300, 800, 200, 1024 and 50 tokens with C = 1024: 300+800 closes the first call, 200+1024 the second,
    50 is the remainder.  Text elements are skipped and never end a batch."""
    segs = [(T, 10), (M, 300), (T, 4), (M, 800), (M, 200), (T, 1), (M, 1024), (M, 50), (T, 2)]
    assert encoder_batches(segs, 1024) == [[1, 3], [4, 6], [7]]
    assert encoder_batches(segs, 1) == [[1], [3], [4], [6], [7]]
    assert encoder_batches(segs, 10 ** 9) == [[1, 3, 4, 6, 7]]
    assert encoder_batches([(T, 5)], 16) == []


def test_algorithm2_budget_is_shared_in_fifo_order():
    """B = 10: the head request takes what it can, the next ones share the rest; the request that does not fit gets the
    remainder of the budget and nothing behind it is visited."""
    a, b, c, d = (TrackedRequest(i, [(T, n)]) for i, n in enumerate([4, 3, 8, 2]))
    s, q = schedule_round([a, b, c, d], 10)
    assert [(x[0].request_id, x[1], x[2]) for x in s] == [(0, 0, 4), (1, 0, 3), (2, 0, 3)]
    assert [r.request_id for r in q] == [2, 3]            # c is incomplete and returns to the head, d was not visited
    s, q = schedule_round(q, 10)
    assert [(x[0].request_id, x[1], x[2]) for x in s] == [(2, 3, 5), (3, 0, 2)] and q == []


def test_algorithm2_blocked_request_does_not_block_the_queue():
    """Inter-request pipeline: a request waiting for its encoder is visited, contributes nothing and keeps its place."""
    a = TrackedRequest(0, [(M, 6), (T, 2)])
    b = TrackedRequest(1, [(T, 5)])
    s, q = schedule_round([a, b], 8)
    assert [(x[0].request_id, x[2]) for x in s] == [(0, 0), (1, 5)]
    assert [r.request_id for r in q] == [0]
    a.mark_ready(0)
    s, q = schedule_round(q, 8)
    assert [(x[0].request_id, x[1], x[2]) for x in s] == [(0, 0, 8)] and q == []


def random_trace(rng, n_requests=6):
    reqs = []
    for i in range(n_requests):
        segs = [(bool(rng.integers(0, 2)), int(rng.integers(1, 40))) for _ in range(int(rng.integers(1, 7)))]
        reqs.append((100 + i, segs))
    return reqs


@pytest.mark.parametrize("seed", range(8))
def test_oracle_invariants_on_random_traces(seed):
    """Every token is scheduled exactly once, in prompt order, never before it is ready; a round never exceeds B;
    requests leave the queue exactly when their prompt is done; queue order is FIFO among unfinished requests."""
    rng = np.random.default_rng(seed)
    budget = int(rng.integers(5, 60))
    pending = [TrackedRequest(i, s) for i, s in random_trace(rng)]
    arrival = {r.request_id: k for k, r in enumerate(pending)}
    not_ready = [(r, k) for r in pending for k, (mm, _) in enumerate(r.segments) if mm]
    rng.shuffle(not_ready)
    q = []
    seen = {r.request_id: 0 for r in pending}
    length = {r.request_id: r.prompt_length for r in pending}
    rounds = 0
    while pending or q or not_ready:
        rounds += 1
        assert rounds < 10000
        if pending and rng.random() < 0.5:
            q.append(pending.pop(0))
        if not_ready and rng.random() < 0.6:
            r, k = not_ready.pop()
            r.mark_ready(k)
        before = {r.request_id: r.prefilled for r in q}
        ready_before = {r.request_id: list(r.ready) for r in q}
        s, q = schedule_round(q, budget)
        assert sum(n for _, _, n in s) <= budget
        for r, first, n in s:
            assert first == before[r.request_id] == seen[r.request_id]
            assert all(ready_before[r.request_id][first: first + n])
            seen[r.request_id] += n
        ids = [r.request_id for r in q]
        assert all(r.prefilled < r.prompt_length for r in q)
        assert ids == sorted(ids, key=lambda i: arrival[i])
    assert seen == length


@pytest.mark.parametrize("seed", range(6))
def test_algorithm1_invariants(seed):
    rng = np.random.default_rng(100 + seed)
    segs = [(bool(rng.integers(0, 3)), int(rng.integers(1, 700))) for _ in range(int(rng.integers(1, 30)))]
    c = int(rng.integers(1, 1500))
    calls = encoder_batches(segs, c)
    flat = [i for call in calls for i in call]
    assert flat == [i for i, (mm, _) in enumerate(segs) if mm]          # every item once, in order, never split
    for call in calls[:-1]:
        assert sum(segs[i][1] for i in call) >= c                        # full batches
        assert sum(segs[i][1] for i in call[:-1]) < c                    # closed as soon as C is reached
    if calls:
        assert sum(segs[i][1] for i in calls[-1][:-1]) < c


# ------------------------------------------------------------------ library against the oracle
@pytest.mark.parametrize("seed", range(10))
def test_library_matches_oracle_on_random_traces(seed):
    rng = np.random.default_rng(1000 + seed)
    budget = int(rng.integers(5, 80))
    trace = random_trace(rng, n_requests=8)
    lib = Scheduler(budget)
    orc = {i: TrackedRequest(i, s) for i, s in trace}
    pending = list(trace)
    not_ready = [(i, k) for i, s in trace for k, (mm, _) in enumerate(s) if mm]
    rng.shuffle(not_ready)
    q = []
    added = set()
    for step in range(4000):
        if not pending and not q and not not_ready:
            break
        if pending and rng.random() < 0.5:
            i, s = pending.pop(0)
            lib.add_request(i, s)
            q.append(orc[i])
            added.add(i)
        if not_ready and rng.random() < 0.6:
            i, k = not_ready[-1]
            if i in added:
                not_ready.pop()
                lib.mark_ready(i, k)
                orc[i].mark_ready(k)
        for r in q:
            assert lib.schedulable_tokens(r.request_id) == r.schedulable_tokens()
            assert lib.prefilled_tokens(r.request_id) == r.prefilled
        s, q = schedule_round(q, budget)
        got = lib.next_round()
        assert got == [(r.request_id, first, n, r.prefilled == r.prompt_length) for r, first, n in s]
        assert lib.queue_ids() == [r.request_id for r in q]
    else:
        raise AssertionError("trace did not finish")
    for i, s in trace:
        assert lib.prefilled_tokens(i) == lib.prompt_length(i) == sum(n for _, n in s)
        c = int(rng.integers(1, 100))
        assert [list(range(a, b + 1)) for a, b, _, _ in lib.encoder_batches(i, c)] == \
            [list(range(call[0], call[-1] + 1)) for call in encoder_batches(s, c)]
        assert [(n, t) for _, _, n, t in lib.encoder_batches(i, c)] == \
            [(len(call), sum(s[k][1] for k in call)) for call in encoder_batches(s, c)]


def test_library_rejects_bad_calls():
    s = Scheduler(16)
    with pytest.raises(RsError):
        Scheduler(0)
    s.add_request(1, [(T, 3), (M, 4)])
    for bad in (lambda: s.add_request(1, [(T, 1)]), lambda: s.add_request(2, []), lambda: s.add_request(2, [(T, 0)]),
                lambda: s.mark_ready(1, 0), lambda: s.mark_ready(1, 2), lambda: s.mark_ready(9, 0),
                lambda: s.encoder_batches(1, 0), lambda: s.release_request(5)):
        with pytest.raises(RsError) as e:
            bad()
        assert e.value.status_name == "RS_EINVAL"
    assert s.schedulable_tokens(9) == -1 and s.prompt_length(1) == 7
    s.add_request(2, [(T, 30)])
    with pytest.raises(RsError) as e:
        s.next_round(capacity=1)          # two requests would be visited
    assert e.value.status_name == "RS_EWORKSPACE"
    assert s.prefilled_tokens(1) == 0 and s.queue_ids() == [1, 2]      # nothing changed
    assert s.next_round() == [(1, 0, 3, False), (2, 0, 13, False)]
    s.mark_ready(1, 1)
    s.mark_ready(1, 1)                                                 # idempotent
    assert s.next_round() == [(1, 3, 4, True), (2, 13, 12, False)]
    s.release_request(2)
    assert s.queue_length() == 0 and s.next_round() == []
