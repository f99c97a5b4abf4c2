"""Host-side generator of commit orders: the paper's update-ordering heuristic.

The GPU library takes the scheduler's decisions (`order`, with dropped workers
left out) as inputs.  The parity tests mostly use seeded permutations; this
module produces orders the way the paper's scheduler would (Sec. 5.1 "Update
Ordering": shortest transfer first, deadlines from the delay bound, look-ahead
drops -- the final ordering algorithm, Alg. 2), so that tests and benchmarks
can also run on sequences with that structure.  It is control-plane code on the
CPU and contains none of the arithmetic of the GPU path.

Network model (the paper defines the completion time t_en of a transfer and the
reservation of its bandwidth by two figures that its text does not contain; this
is the reading used here, and it reproduces the worked example of Sec. 5.1.3):

  * one server; worker j reaches it over its own access link and the server's
    link; each link has a residual bandwidth that is piecewise constant in time;
  * an update of `size` available at t = 0 uses, at every instant, all of the
    bottleneck residual min(access_j(t), server(t)); t_en is the instant its
    bytes are through;
  * committing a transfer reserves exactly that time-varying rate on both links
    until t_en.

Deadlines: dl(g) = v(g) + tau_max - v_init counts commit slots: every update
that is considered takes one slot, also when it ends up dropped.  An update
whose deadline slot has been reached or passed is due.
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
    """One link after a transfer is committed: `used` (the transfer's rate) is
    taken off on [0, until)."""
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
        """The network with g's transfer reserved on its access link and on the
        server link."""
        used, end = self.path(g), self.t_en(g)
        access = dict(self.access)
        access[g.worker] = reserve(self.access[g.worker], used, end)
        return Network(reserve(self.server, used, end), access)


class CommitRound:
    """One pass of the final ordering (Sec. 5.1, Alg. 2) over a batch: the
    updates still waiting, the residual network after the commits so far, and
    the commit slot being filled."""

    def __init__(self, updates, nw: Network, tau_max: int, v_init: int):
        self.waiting = {g.worker: g for g in updates}
        self.deadline = {g.worker: g.version + tau_max - v_init for g in updates}
        self.nw = nw
        self.slot = 1
        self.order, self.dropped = [], []

    def front_runner(self, slot, nw, skip=None):
        """The update that would take `slot` on network `nw`: among the due ones
        if any is due, else among all that wait, the one whose transfer ends
        first (ties by worker id).  `skip` leaves one worker out."""
        pool = [g for w, g in self.waiting.items() if w != skip]
        if not pool:
            return None
        due = [g for g in pool if self.deadline[g.worker] <= slot]
        return min(due or pool, key=lambda g: (nw.t_en(g), g.worker))

    def overtaken(self, chosen, reserved):
        """Look-ahead: with `chosen` reserved, would the front runner of the
        next slot still be through before `chosen` itself?  Then `chosen` holds
        nobody up by being dropped at its worker (the 10 s / 1.1 s example of
        Sec. 5.1.3)."""
        rival = self.front_runner(self.slot + 1, reserved, skip=chosen.worker)
        return rival is not None and self.nw.t_en(chosen) > reserved.t_en(rival)

    def fill_slot(self):
        chosen = self.front_runner(self.slot, self.nw)
        reserved = self.nw.after(chosen)
        if self.overtaken(chosen, reserved):
            self.dropped.append(chosen.worker)
        else:
            self.order.append(chosen.worker)
            self.nw = reserved
        del self.waiting[chosen.worker]
        self.slot += 1


def order_updates(updates, nw: Network, tau_max: int, v_init: int):
    """Final ordering of a batch (Sec. 5.1, Alg. 2): deadline-forced updates
    first, else the shortest transfer, with the look-ahead drop.  Returns
    (order, dropped): the workers in commit order, and the workers whose updates
    were dropped."""
    rnd = CommitRound(updates, nw, tau_max, v_init)
    while rnd.waiting:
        rnd.fill_slot()
    return rnd.order, rnd.dropped


def shortest_transfer_first(updates, nw: Network):
    """Ordering without deadlines (Sec. 5.1, Alg. 1): always the transfer that
    ends first on what is left of the network."""
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
    stale) run through the final ordering.  Returns an int32 order (dropped workers left out),
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
