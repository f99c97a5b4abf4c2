"""Host-side generator of commit orders: the paper's update-ordering heuristic.

The GPU library takes the scheduler's decisions (`order`, with dropped workers
left out) as inputs.  The parity tests mostly use seeded permutations; this
module produces orders the way the paper's scheduler would (Sec. 5.1 "Update
Ordering": shortest transfer first, deadlines from the delay bound, look-ahead
drops -- the final ordering algorithm, Alg. 2), so that tests and benchmarks
can also run on sequences with that structure.  It is control-plane code on the
CPU and contains none of the arithmetic of the GPU path.

Network model (the paper defines the completion time t_en and the bandwidth
reservation NetUp by two figures that its text does not contain; this is the
reading used here, and it reproduces the worked example of Sec. 5.1.3):

  * one server; worker j reaches it over its own access link and the server's
    link; each link has a residual bandwidth that is piecewise constant in time;
  * an update of `size` available at t = 0 uses, at every instant, all of the
    bottleneck residual min(access_j(t), server(t)); t_en is the instant its
    bytes are through;
  * NetUp reserves exactly that time-varying rate on both links until t_en.

Deadlines: dl(g) = v(g) + tau_max - v_init, compared with the iteration counter
of the ordering loop as the algorithm is printed (the counter also advances when
an update is dropped).  An update whose deadline has passed counts as due.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

INF = float("inf")


@dataclass
class Profile:
    """Residual bandwidth, piecewise constant: rate[i] on [t[i], t[i+1]), the
    last piece extending to infinity.  t[0] == 0."""
    t: list = field(default_factory=lambda: [0.0])
    rate: list = field(default_factory=lambda: [0.0])

    @staticmethod
    def constant(rate: float) -> "Profile":
        return Profile([0.0], [float(rate)])

    def at_breaks(self, times):
        """Rates on the refinement given by the sorted break times `times`."""
        idx = np.searchsorted(np.asarray(self.t), np.asarray(times), side="right") - 1
        return [self.rate[i] for i in idx]


def bottleneck(a: Profile, b: Profile) -> Profile:
    times = sorted(set(a.t) | set(b.t))
    ra, rb = a.at_breaks(times), b.at_breaks(times)
    return Profile(times, [min(x, y) for x, y in zip(ra, rb)])


def completion_time(path: Profile, size: float) -> float:
    """t_en: when an update of `size` is through, using all of `path`."""
    left = float(size)
    if left <= 0:
        return 0.0
    for i, t0 in enumerate(path.t):
        t1 = path.t[i + 1] if i + 1 < len(path.t) else INF
        r = path.rate[i]
        if r > 0 and (t1 == INF or r * (t1 - t0) >= left):
            return t0 + left / r
        if t1 == INF:
            return INF
        left -= r * (t1 - t0)
    return INF


def reserve(link: Profile, used: Profile, until: float) -> Profile:
    """NetUp on one link: subtract `used` (the transfer's rate) on [0, until)."""
    times = sorted(set(link.t) | set(used.t) | ({until} if until < INF else set()))
    rl, ru = link.at_breaks(times), used.at_breaks(times)
    rate = [max(l - (u if t < until else 0.0), 0.0) for t, l, u in zip(times, rl, ru)]
    return Profile(times, rate)


@dataclass
class Update:
    worker: int
    size: float           # bytes (any unit consistent with the bandwidths)
    version: int          # v(g): model version the update was computed on


@dataclass
class Network:
    server: Profile
    access: dict          # worker -> Profile

    def path(self, g: Update) -> Profile:
        return bottleneck(self.access[g.worker], self.server)

    def t_en(self, g: Update) -> float:
        return completion_time(self.path(g), g.size)

    def after(self, g: Update) -> "Network":
        """NetUp(NW, g, S): the network with g's transfer reserved."""
        used, end = self.path(g), self.t_en(g)
        access = dict(self.access)
        access[g.worker] = reserve(self.access[g.worker], used, end)
        return Network(reserve(self.server, used, end), access)


def _pick(iteration, pending, nw, deadline):
    """ShrtDline: a due update if there is one (the one finishing first among
    several), else the update with the least completion time."""
    if not pending:
        return None
    due = [g for g in pending if deadline[g.worker] <= iteration]
    pool = due if due else pending
    return min(pool, key=lambda g: (nw.t_en(g), g.worker))


def order_updates(updates, nw: Network, tau_max: int, v_init: int):
    """Final ordering algorithm (Alg. 2).  Returns (order, dropped): the workers
    in commit order, and the workers whose updates were dropped."""
    deadline = {g.worker: g.version + tau_max - v_init for g in updates}
    pending = list(updates)
    order, dropped = [], []
    for i in range(1, len(updates) + 1):
        current = _pick(i, pending, nw, deadline)
        if current is None:
            break
        pending = [g for g in pending if g.worker != current.worker]
        reserved = nw.after(current)
        nxt = _pick(i + 1, pending, reserved, deadline)
        if nxt is not None and nw.t_en(current) > reserved.t_en(nxt):
            dropped.append(current.worker)       # "next" would be applied first: drop
            continue
        order.append(current.worker)
        nw = reserved
    return order, dropped


def shortest_transfer_first(updates, nw: Network):
    """Alg. 1: greedy shortest-completion-time ordering without deadlines."""
    pending, order, finish = list(updates), [], []
    while pending:
        g = min(pending, key=lambda u: (nw.t_en(u), u.worker))
        finish.append(nw.t_en(g))
        order.append(g.worker)
        pending = [u for u in pending if u.worker != g.worker]
        nw = nw.after(g)
    return order, finish


def scheduled_order(K: int, seed: int, size: float = 100e6, tau_max=None):
    """A seeded batch of K equal-sized updates on a cluster shaped like the
    paper's (Sec. 6: 10 Gbps links; some workers behind slow links, some updates
    stale) run through Alg. 2.  Returns an int32 order (dropped workers left out),
    the form the GPU calls take."""
    rng = np.random.default_rng(seed)
    server = Profile.constant(10e9 / 8)
    access = {}
    for j in range(K):
        slow = rng.random() < 0.25                       # network stragglers (Sec. 6, N2/N3)
        access[j] = Profile.constant((1e9 if slow else 10e9) / 8 * rng.uniform(0.5, 1.0))
    tau_max = 2 * K if tau_max is None else tau_max
    v_init = 1000
    updates = []
    for j in range(K):
        # most updates are fresh; a quarter come from compute stragglers and are
        # close to the delay bound (Sec. 6, C2/C3), so their deadline falls early
        stale = rng.random() < 0.25
        age = tau_max - int(rng.integers(0, 3)) if stale else int(rng.integers(0, 4))
        updates.append(Update(j, size, v_init - max(age, 0)))
    order, _ = order_updates(updates, Network(server, access), tau_max, v_init)
    return np.asarray(order, dtype=np.int32)
