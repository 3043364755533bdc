"""Pins for the iteration-scheduler oracle (oracle/replay.py), CPU only: traces small enough to work through
by hand.  The expected batches below were derived on paper from the rules of Sec. 3.4 / Sec. 4.4 (decode batch
first, one restricted prefill task at a time, chunk = chunk size - decode batch size); the derivation of the
first trace is written out next to it."""
import pytest

from oracle import replay as orp


def test_three_requests_worked_by_hand():
    # chunk size 8, two table rows, every pass takes 1 s (one layer, nothing else):
    #  t=0  R0 (10 in, 3 out) arrives and becomes the prefill task: chunk of 8              -> ctx 8
    #  t=1  R1 arrived at 0.5 and waits (one task at a time); R0's last 2 tokens            -> ctx 10, first token of R0 at t=2
    #  t=2  R2 arrived at 1.5; R1 becomes the task; decode batch {R0} leaves 7, R1 needs 5  -> R0 ctx 11, R1 ctx 5, first token of R1 at t=3
    #  t=3  both rows are taken, R2 waits; decode batch {R0, R1}                            -> ctx 12, 6; R0 has 3 tokens, R1 has 2: both done at t=4
    #  t=4  R2 (4 in, 1 out) is the task                                                    -> ctx 4; first token = last token at t=5
    reqs = [(0.0, 10, 3), (0.5, 5, 2), (1.5, 4, 1)]
    its, first, done = orp.schedule(reqs, chunk_size=8, max_resident=2, num_pages=100, max_pages_per_seq=10,
                                    pass_time=lambda q, c: 1.0, layers=1, other_s=0.0, horizon_s=20.0)
    assert its == [((0,), (8,), (8,)), ((0,), (2,), (10,)), ((0, 1), (1, 5), (11, 5)), ((0, 1), (1, 1), (12, 6)),
                   ((2,), (4,), (4,))]
    assert first == {0: 2.0, 1: 3.0, 2: 5.0}
    assert done == {0: 4.0, 1: 4.0, 2: 5.0}
    ttft = {r: first[r] - reqs[r][0] for r in first}
    assert ttft == {0: 2.0, 1: 2.5, 2: 3.5}


def test_decode_batch_takes_the_chunk_budget_first():
    # chunk size 2: a decode batch of two leaves nothing for the task, a batch of one leaves one token
    reqs = [(0.0, 2, 4), (0.0, 2, 3), (0.0, 3, 1)]
    its, first, done = orp.schedule(reqs, chunk_size=2, max_resident=3, num_pages=100, max_pages_per_seq=10,
                                    pass_time=lambda q, c: 1.0, layers=1, other_s=0.0, horizon_s=20.0)
    assert its == [((0,), (2,), (2,)), ((0, 1), (1, 1), (3, 1)), ((0, 1), (1, 1), (4, 2)), ((0, 1), (1, 1), (5, 3)),
                   ((1, 2), (1, 1), (4, 1)), ((2,), (2,), (3,))]
    assert first == {0: 1.0, 1: 3.0, 2: 6.0} and done == {0: 4.0, 1: 5.0, 2: 6.0}


def test_admission_waits_for_pages_and_time_formula():
    # two pages in the pool: R0 (20 in + 2 out = 2 pages) holds both until it is done; time per iteration =
    # pass time (1 ms per query token) x 2 layers + 10 ms
    reqs = [(0.0, 20, 2), (0.0, 1, 1)]
    its, first, done = orp.schedule(reqs, chunk_size=32, max_resident=4, num_pages=2, max_pages_per_seq=2,
                                    pass_time=lambda q, c: 1e-3 * sum(q), layers=2, other_s=0.01, horizon_s=1.0)
    assert its == [((0,), (20,), (20,)), ((0,), (1,), (21,)), ((1,), (1,), (1,))]
    t1 = 20e-3 * 2 + 0.01
    t2 = t1 + 1e-3 * 2 + 0.01
    t3 = t2 + 1e-3 * 2 + 0.01
    assert first[0] == pytest.approx(t1) and done[0] == pytest.approx(t2)
    assert first[1] == pytest.approx(t3) and done[1] == pytest.approx(t3)
    # a request that can never fit stays at the head of the queue and nothing overtakes it
    its, first, done = orp.schedule([(0.0, 100, 1), (0.0, 1, 1)], chunk_size=32, max_resident=4, num_pages=2,
                                    max_pages_per_seq=2, pass_time=lambda q, c: 1.0, layers=1, other_s=0.0,
                                    horizon_s=5.0)
    assert its == [] and first == {} and done == {}


def test_idle_decoder_jumps_to_the_next_arrival():
    its, first, _ = orp.schedule([(3.25, 4, 2)], chunk_size=8, max_resident=1, num_pages=4, max_pages_per_seq=4,
                                 pass_time=lambda q, c: 0.5, layers=1, other_s=0.0, horizon_s=10.0)
    assert its == [((0,), (4,), (4,)), ((0,), (1,), (5,))]
    assert first == {0: 3.75}
