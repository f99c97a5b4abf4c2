"""The host-side order generator (the paper's update-ordering heuristic, Alg. 1
and Alg. 2 of Sec. 5.1) against the paper's worked example and its stated
properties.  CPU only; control plane, not part of the GPU path."""
import numpy as np

from workloads import scheduler as S

MBPS = 1e6 / 8          # bytes per second


def test_completion_time_integrates_the_residual_bandwidth():
    assert S.completion_time(S.Profile.constant(10.0), 30.0) == 3.0
    # 2 units/s for 5 s, nothing for 3 s, then 10 units/s: 30 units are through at t = 10
    p = S.Profile([0.0, 5.0, 8.0], [2.0, 0.0, 10.0])
    assert S.completion_time(p, 30.0) == 10.0
    assert S.completion_time(p, 10.0) == 5.0
    assert S.completion_time(p, 4.0) == 2.0
    assert S.completion_time(S.Profile([0.0, 1.0], [5.0, 0.0]), 30.0) == S.INF
    assert S.completion_time(p, 0.0) == 0.0


def test_reservation_leaves_the_rest_of_the_link():
    link = S.Profile.constant(100.0)
    used = S.Profile.constant(10.0)
    left = S.reserve(link, used, until=4.0)
    assert left.at_breaks([0.0, 3.9, 4.0, 100.0]) == [90.0, 90.0, 100.0, 100.0]
    both = S.bottleneck(S.Profile([0.0, 2.0], [5.0, 50.0]), S.Profile([0.0, 3.0], [20.0, 7.0]))
    assert both.at_breaks([0.0, 2.5, 3.5]) == [5.0, 20.0, 7.0]


def example_network():
    """Sec. 5.1.3: worker 1 sits behind a 10 Mbps link, the server link has
    100 Mbps; both updates are 100 Mbit."""
    return S.Network(S.Profile.constant(100 * MBPS),
                     {1: S.Profile.constant(10 * MBPS), 2: S.Profile.constant(100 * MBPS)})


def test_paper_example_of_a_preemptive_drop():
    """dl(g1) = 1, dl(g2) = 5.  g1 would take 10 s; with its 10 Mbps reserved, g2
    gets the remaining 90 Mbps and finishes in 1.1 s, before g1: g1 is dropped
    at the worker and g2 is scheduled at once."""
    nw = example_network()
    size = 100e6 / 8
    g1, g2 = S.Update(1, size, version=0), S.Update(2, size, version=4)
    assert nw.t_en(g1) == 10.0
    assert abs(nw.after(g1).t_en(g2) - 100 / 90) < 1e-9          # "1.1 s"
    order, dropped = S.order_updates([g1, g2], nw, tau_max=1, v_init=0)
    assert order == [2] and dropped == [1]


def test_without_deadline_pressure_shortest_transfer_goes_first():
    nw = example_network()
    size = 100e6 / 8
    g1, g2 = S.Update(1, size, version=10), S.Update(2, size, version=10)
    order, dropped = S.order_updates([g1, g2], nw, tau_max=50, v_init=10)
    assert order == [2, 1] and dropped == []
    sjf, finish = S.shortest_transfer_first([g1, g2], nw)
    assert sjf == [2, 1]
    # time sharing: g2 has the server link for 1 s, then g1 trickles in at 10 Mbps
    assert abs(finish[0] - 1.0) < 1e-9 and abs(finish[1] - 11.0) < 1e-9


def test_a_due_update_is_taken_first_when_it_does_not_hold_up_the_next():
    # both links fast: the due update finishes before the next could, so it is kept
    nw = S.Network(S.Profile.constant(100.0), {0: S.Profile.constant(100.0),
                                               1: S.Profile.constant(100.0)})
    big, small = S.Update(0, 300.0, version=0), S.Update(1, 100.0, version=9)
    order, dropped = S.order_updates([big, small], nw, tau_max=1, v_init=0)
    assert order == [0, 1] and dropped == []
    order, _ = S.order_updates([big, small], nw, tau_max=50, v_init=0)
    assert order == [1, 0]                                        # no deadline: shortest first


def test_random_batches_keep_every_update_at_most_once():
    for seed in range(20):
        rng = np.random.default_rng(seed)
        K = int(rng.integers(1, 20))
        access = {j: S.Profile.constant(float(rng.uniform(1, 100))) for j in range(K)}
        nw = S.Network(S.Profile.constant(100.0), access)
        ups = [S.Update(j, float(rng.uniform(10, 500)), int(rng.integers(0, 10))) for j in range(K)]
        order, dropped = S.order_updates(ups, nw, tau_max=int(rng.integers(1, 12)), v_init=10)
        assert sorted(order + dropped) == list(range(K))
        assert len(order) >= 1
        loose, none = S.order_updates(ups, nw, tau_max=10 ** 6, v_init=10)
        assert none == [] and loose == S.shortest_transfer_first(ups, nw)[0]


def test_scheduled_order_has_the_form_the_gpu_calls_take():
    seen_drop = False
    for seed in range(10):
        o = S.scheduled_order(16, seed)
        assert o.dtype == np.int32 and len(set(o.tolist())) == len(o) <= 16
        assert o.min() >= 0 and o.max() < 16
        seen_drop = seen_drop or len(o) < 16
        assert np.array_equal(o, S.scheduled_order(16, seed))    # seeded
    assert seen_drop
