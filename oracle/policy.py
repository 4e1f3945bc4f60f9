"""Host-side policies of the paper, restated plainly (test oracle).

selective_handles : Algorithm 1 ("selective memory reclamation", Section 5): k times pick the
                    handle whose not-yet-evicted requests cost least; ties go to the lowest
                    handle index (the paper leaves ties open).
fifo_handles      : the FIFO baseline the paper compares Algorithm 1 with (Section 7.2).
Miad              : the dynamic reservation of Section 5 ("Dynamic MIAD-style memory
                    reservation"): headroom H grows multiplicatively on a pressure event
                    (usage >= 90 % of H), shrinks by one handle every interval T otherwise;
                    T itself rises multiplicatively while the pressure-event rate over a
                    sliding window exceeds the target and falls additively otherwise.  The
                    paper gives no constants besides the 90 %; they are parameters here.
CooldownGate      : the wake-up rule of Section 4.2: offline work is preempted the moment the
                    online tenant turns busy and re-enabled only after it has been idle for
                    T_cool = 2 G without interruption, G being the largest gap seen between
                    two decode iterations of one request.
"""
from __future__ import annotations

import math


def handle_requests(tables, num_blocks: int, blocks_per_handle: int):
    """Reqs(h): for every handle the set of table rows holding a block inside it."""
    reqs = [set() for _ in range(num_blocks // blocks_per_handle)]
    for r, row in enumerate(tables):
        for e in row:
            e = int(e)
            if e >= 0:
                reqs[e // blocks_per_handle].add(r)
    return reqs


def selective_handles(k: int, reqs, cost, candidates=None):
    """Algorithm 1.  reqs[h] = set of requests of handle h, cost[r] = Cost(r).
    Returns (handles in the order picked, evicted request set, total cost)."""
    pool = list(range(len(reqs))) if candidates is None else list(candidates)
    chosen, evicted, total = [], set(), 0
    for _ in range(k):
        best, best_cost = None, None
        for h in pool:
            if h in chosen:
                continue
            c = sum(cost[r] for r in reqs[h] if r not in evicted)
            if best is None or c < best_cost:
                best, best_cost = h, c
        if best is None:
            raise ValueError("fewer candidate handles than k")
        chosen.append(best)
        total += best_cost
        evicted |= reqs[best]
    return chosen, evicted, total


def fifo_handles(k: int, reqs, cost, candidates=None):
    """The comparison policy of Section 7.2 ("evicts offline KV cache blocks in first-in-first-out
    order"): in a pool that hands out its lowest free blocks first, the oldest blocks sit in the lowest
    handles, so FIFO takes the first k candidate handles by index.  Same return as selective_handles."""
    pool = list(range(len(reqs))) if candidates is None else list(candidates)
    if k > len(pool):
        raise ValueError("fewer candidate handles than k")
    chosen = pool[:k]
    evicted = set()
    for h in chosen:
        evicted |= reqs[h]
    return chosen, evicted, sum(cost[r] for r in evicted)


class Miad:
    def __init__(self, h_init, h_min, h_max, alpha, pressure_frac, t_init, t_min, t_max, t_up, t_down,
                 window_s, target_rate):
        self.h, self.h_min, self.h_max = h_init, h_min, h_max
        self.alpha, self.frac = alpha, pressure_frac
        self.t, self.t_min, self.t_max, self.t_up, self.t_down = t_init, t_min, t_max, t_up, t_down
        self.window, self.target = window_s, target_rate
        self.events = []            # times of pressure events inside the window
        self.last_release = None    # time of the last release tick (or of the first observation)

    def _adapt_interval(self, now):
        self.events = [t for t in self.events if t > now - self.window]
        rate = len(self.events) / self.window
        if rate > self.target:
            self.t = min(self.t_max, self.t * self.t_up)
        else:
            self.t = max(self.t_min, self.t - self.t_down)

    def observe(self, now, used):
        """Returns (headroom, grow_by, release, pressure_event, interval)."""
        if self.last_release is None:
            self.last_release = now
        grow = release = event = 0
        if used >= self.frac * self.h:
            event = 1
            new_h = min(self.h_max, max(self.h + 1, int(math.ceil(self.h * self.alpha))))
            grow = new_h - self.h
            self.h = new_h
            self.events.append(now)
            self._adapt_interval(now)
            self.last_release = now
        elif now - self.last_release >= self.t:
            if self.h > self.h_min and self.h - 1 > used:
                self.h -= 1
                release = 1
            self.last_release = now
            self._adapt_interval(now)
        return self.h, grow, release, event, self.t


class CooldownGate:
    def __init__(self, initial_gap):
        self.g = initial_gap
        self.busy = False
        self.idle_since = 0.0
        self.offline_on = True
        self.last_request = None
        self.preemptions = 0

    def online_busy(self, now, request_id):
        """Returns 1 if offline work has to be preempted now."""
        preempt = 0
        if not self.busy:
            if self.last_request is not None and request_id == self.last_request:
                self.g = max(self.g, now - self.idle_since)     # a gap between two iterations of one request
            self.busy = True
        if self.offline_on:
            self.offline_on = False
            self.preemptions += 1
            preempt = 1
        self.last_request = request_id
        return preempt

    def online_idle(self, now):
        if self.busy:
            self.busy = False
            self.idle_since = now

    def poll(self, now):
        """Returns 1 if offline work may run at `now` (re-enabling it if the cooldown has passed)."""
        if not self.offline_on and not self.busy and now - self.idle_since >= 2.0 * self.g:
            self.offline_on = True
        return 1 if self.offline_on else 0
