"""The library's layer-granular swapping control (pure host logic) against the oracle's simulation of the
paper's protocol, decision by decision, under the same timing model (no GPU)."""
import pytest

from oracle import layer_fifo as LF
from paper_2411_09317_amd import binding as B

STATE = {LF.GPU: B.LAYER_GPU, LF.HOST: B.LAYER_HOST, LF.MOVING_OUT: B.LAYER_MOVING_OUT, LF.MOVING_IN: B.LAYER_MOVING_IN}
SKIP = {None: B.SKIP_NOT, "busy": B.SKIP_BUSY, "no_slot": B.SKIP_NO_SLOT, "colder_on_host": B.SKIP_COLDER_ON_HOST,
        "none": B.SKIP_NONE, "room_left": B.SKIP_ROOM_LEFT}


def run_library(n, gpu, host, on_host, n_tokens, t_compute, t_in, t_out, slots_for_token=None):
    """Drives the library's protocol with clocks instead of a GPU: a move started at t completes at t + t_in / t_out."""
    s = B.LayerSched(n, gpu, host, on_host)
    now, in_done, out_done = 0.0, None, None
    records, stall = [], 0.0

    def retire(t):
        nonlocal in_done, out_done
        if out_done is not None and out_done <= t:
            s.complete(1)
            out_done = None
        if in_done is not None and in_done <= t:
            s.complete(0)
            in_done = None

    def started(a, t):
        nonlocal in_done, out_done
        if a.out_layer >= 0:
            out_done = t + t_out
        if a.in_layer >= 0:
            in_done = t + t_in

    for token in range(n_tokens):
        retire(now)
        if slots_for_token is not None and slots_for_token(token) is not None:
            s.set_gpu_slots(slots_for_token(token))
        for k in range(n):
            retire(now)
            t_begin, forced = now, False
            while True:
                a = s.present(k)
                started(a, now)
                forced = forced or bool(a.forced_in)
                if a.wait == B.WAIT_NONE:
                    break
                now = max(now, in_done if a.wait == B.WAIT_IN else out_done)
                retire(now)
            stall += now - t_begin
            a = s.policy(k)
            started(a, now)
            records.append((token, k, t_begin, now, a.out_layer, a.in_layer, a.out_skipped, a.in_skipped, forced))
            now += t_compute
    table = s.table()
    s.close()
    return records, stall, table


CASES = [
    (9, 7, 4, [7, 8], 6, 1.0, 2.0, 2.0),             # the paper's worked example
    (9, 7, 4, [7, 8], 6, 1.0, 2.2, 2.2),             # link too slow: waits and forced moves
    (12, 8, 6, [8, 9, 10, 11], 5, 1.0, 1.5, 2.5),
    (5, 3, 4, [0, 4], 9, 1.0, 0.7, 0.4),
    (16, 10, 8, [1, 5, 9, 12, 13, 15], 5, 1.0, 3.3, 4.1),
    (6, 6, 2, [], 3, 1.0, 2.0, 2.0),                 # nothing in CPU memory: nothing moves
    (8, 3, 7, [0, 1, 2, 3, 4], 4, 1.0, 5.0, 5.0),    # far too little GPU room: victims are evicted
    (4, 1, 4, [1, 2, 3], 3, 1.0, 0.5, 0.5),          # a single GPU slot
]


@pytest.mark.parametrize("n,gpu,host,on_host,tokens,tc,ti,to", CASES)
def test_every_decision_matches_the_oracle(n, gpu, host, on_host, tokens, tc, ti, to):
    ref = LF.simulate(n, gpu, host, on_host, tokens, t_compute=tc, t_in=ti, t_out=to)
    got, stall, table = run_library(n, gpu, host, on_host, tokens, tc, ti, to)
    assert len(got) == len(ref.records)
    for g, r in zip(got, ref.records):
        want = (r.token, r.layer, r.t_begin, r.t_start, -1 if r.out_started is None else r.out_started,
                -1 if r.in_started is None else r.in_started,
                SKIP[r.out_skipped] if r.out_started is None else B.SKIP_NOT,
                SKIP[r.in_skipped] if r.in_started is None else B.SKIP_NOT, r.forced_in)
        assert g == want
    assert stall == pytest.approx(ref.stall)
    for j, (state, gs, hs) in enumerate(table):
        e = ref.table[j]
        assert state == STATE[e.state]
        assert gs == (-1 if e.gpu_slot is None else e.gpu_slot) and hs == (-1 if e.host_slot is None else e.host_slot)


def test_argument_and_state_errors():
    with pytest.raises(B.PieError) as e:
        B.LayerSched(4, 2, 1, [0, 1])                # two layers do not fit one CPU slot
    assert e.value.code == B.ENOMEM
    with pytest.raises(B.PieError) as e:
        B.LayerSched(4, 4, 2, [7])
    assert e.value.code == B.EINVAL
    s = B.LayerSched(4, 3, 2, [3])
    with pytest.raises(B.PieError) as e:
        s.complete(0)                                # nothing in flight
    assert e.value.code == B.ESTATE
    with pytest.raises(B.PieError) as e:
        s.policy(3)                                  # not present
    assert e.value.code == B.ESTATE
    s.close()


SCHEDULES = [
    # all layers on the GPU at first, then slots are taken away and given back between tokens
    (9, 9, 6, [], 14, 2.0, {1: 8, 3: 7, 6: 6, 8: 7, 10: 9, 12: 5}),
    (12, 12, 8, [], 16, 1.3, {0: 10, 2: 8, 5: 6, 9: 12, 11: 7}),
    (6, 5, 7, [5], 10, 0.6, {2: 3, 4: 1, 7: 5}),
]


@pytest.mark.parametrize("n,gpu,host,on_host,tokens,t,sched", SCHEDULES)
def test_changing_the_number_of_gpu_slots_matches_the_oracle(n, gpu, host, on_host, tokens, t, sched):
    ref = LF.simulate(n, gpu, host, on_host, tokens, t_compute=1.0, t_in=t, t_out=t,
                      gpu_slots_for_token=lambda token, stall: sched.get(token))
    got, stall, table = run_library(n, gpu, host, on_host, tokens, 1.0, t, t, slots_for_token=lambda token: sched.get(token))
    for g, r in zip(got, ref.records):
        assert g[:6] == (r.token, r.layer, r.t_begin, r.t_start, -1 if r.out_started is None else r.out_started,
                         -1 if r.in_started is None else r.in_started)
        assert g[8] == r.forced_in
    assert stall == pytest.approx(ref.stall)
    for j, (state, gs, hs) in enumerate(table):
        e = ref.table[j]
        assert state == STATE[e.state]
        assert gs == (-1 if e.gpu_slot is None else e.gpu_slot) and hs == (-1 if e.host_slot is None else e.host_slot)
    # with fewer slots allowed than layers, that many layers are away from the GPU at the end
    last = sched[max(sched)]
    assert sum(1 for st, _, _ in table if st != B.LAYER_GPU) >= n - last
