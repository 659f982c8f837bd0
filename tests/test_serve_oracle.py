"""Pins for the serving-loop model: schedules worked by hand from Algorithm 3 and the rules in
the oracle's header."""
from oracle.serve_oracle import ServeModel


def test_hand_worked_schedule():
    # C = 2, page 4, 6 pages, chunks of 4 rows, 8 rows per pass
    m = ServeModel(2, 1.0, 6, 4, 4, 8)
    m.submit(0, 6, 2)     # 8 rows: prompt 6 (chunks 4 + 2), 2 decode steps
    m.submit(1, 3, 0)     # 3 rows
    m.submit(2, 1, 1)     # 2 rows, waits for a place in the batch
    # pass 0: both prompts start; request 0 takes page 0, request 1 page 1
    mem, fin, pages, nb, nn = m.run_pass(0.0)
    assert mem == [(0, 0, 4), (1, 0, 3)] and fin == [1] and (nb, nn) == (2, 2)
    assert pages == {0: [0], 1: [1]}
    # pass 1: request 1 is gone, request 2 joins (batch start still 0.0, 0.0 + 1.0 > 0.5);
    # request 0's second chunk needs a second page: the returned page 1 is reused first
    mem, fin, pages, nb, nn = m.run_pass(0.5)
    assert mem == [(0, 4, 2), (2, 0, 1)] and fin == [] and (nb, nn) == (2, 1)
    assert pages == {0: [0, 1], 2: [2]}
    # pass 2: both decode; request 2 finishes
    mem, fin, pages, nb, nn = m.run_pass(0.6)
    assert mem == [(0, 6, 1), (2, 1, 1)] and fin == [2]
    # pass 3: last decode row of request 0 (row 7 still fits its two pages)
    mem, fin, pages, nb, nn = m.run_pass(0.7)
    assert mem == [(0, 7, 1)] and fin == [0] and pages == {0: [0, 1]}
    assert sorted(m.free) == [0, 1, 2, 3, 4, 5] and m.req == {}
    assert m.run_pass(0.8)[0] == []


def test_row_budget_and_page_shortage_make_members_wait():
    # 5 rows per pass: the second prompt gets what is left of the pass
    m = ServeModel(4, 1.0, 3, 4, 4, 5)
    m.submit(0, 4, 1)
    m.submit(1, 4, 0)
    mem, fin, pages, _, _ = m.run_pass(0.0)
    assert mem == [(0, 0, 4), (1, 0, 1)]
    # next pass: request 0 decodes (row 4 needs its second page: page 2, the last free one),
    # request 1 continues with rows 1..3 inside its page
    mem, fin, pages, _, _ = m.run_pass(0.1)
    assert mem == [(0, 4, 1), (1, 1, 3)] and sorted(fin) == [0, 1]
    assert pages == {0: [0, 2], 1: [1]}
    # pool of one page: the second request cannot start until the first has finished
    m = ServeModel(4, 1.0, 1, 4, 4, 8)
    m.submit(0, 2, 0)
    m.submit(1, 2, 0)
    assert m.run_pass(0.0)[0] == [(0, 0, 2)]
    assert m.run_pass(0.1)[0] == [(1, 0, 2)]


def test_a_pool_that_cannot_hold_two_whole_requests_serves_them_one_after_the_other():
    """Two requests of three pages each over a pool of three pages.  Handing out pages chunk by chunk would give
    each of them one page in the first pass and leave both waiting for ever; with the pages of the whole
    sequence set aside at the start, request 1 waits until request 0 has finished, and the loop drains."""
    m = ServeModel(2, 1.0, 3, 4, 4, 8)
    m.submit(0, 8, 4)
    m.submit(1, 8, 4)
    assert m.run_pass(0.0)[0] == [(0, 0, 4)] and m.unreserved == 0
    assert m.run_pass(0.1)[0] == [(0, 4, 4)]
    for k in range(4):
        mem, fin, pages, nb, _ = m.run_pass(0.2 + 0.1 * k)
        assert mem == [(0, 8 + k, 1)] and nb == 2 and fin == ([0] if k == 3 else [])
    assert m.unreserved == 3 and sorted(m.free) == [0, 1, 2]
    assert m.run_pass(0.7)[0] == [(1, 0, 4)]
    n = 1
    while m.req:
        assert m.run_pass(0.7 + 0.1 * n)[0]     # every pass makes progress
        n += 1
    assert n == 6 and m.unreserved == 3
