"""Oracle for FlexLink's two-stage load balancer.

TEST INFRASTRUCTURE, NOT THE PRODUCT: imported only by the test-suite and the
smoke check.  It shares no code with the C++ balancer in the HIP library and
does not import it.

The balancer is a heuristic, so the oracle is the method itself (paper:
Algorithm 1 for Stage 1, Section "Stage 2: Runtime Fine-Grained Adjustment" for
Stage 2), restated here as a small state machine:

    round(state, times) -> state'

One *round* is one measurement of every live path followed by at most one
*transfer* of share units.  Both stages use the same transfer rule and differ
only in how large the transfer is and in what ends them, so the module is
built from three pieces:

    rank_paths      who is slowest / fastest among the live paths
    choose_transfer the rule table below: who gives, who receives
    apply_transfer  move the units, retire a path that reaches zero

Transfer rule (Algorithm 1's choice of source and target, reused by Stage 2):

    slowest path      primary live?   giver      receiver
    ---------------   -------------   --------   ------------------
    an auxiliary      yes             slowest    the primary path
    an auxiliary      no              slowest    the fastest path
    the primary       (it is)         primary    the fastest path

A path is identified by its index; the path the paper calls NVLink (the one the
tuning favours) is `primary`.  Shares are non-negative integers with a fixed
sum.

Parity unpinned against the paper: it prints no worked numerical example of
the balancer, and the load percentages of its Table 2 belong to H800 links.
The pins are hand-executed trajectories, the closed-form balance point of a
pure-bandwidth timing model, and the properties the prose states.

Readings taken where the paper leaves a choice (documented readings, not facts
of the paper):

* Shares and the stride are integers; halving is integer division, never
  below 1.
* Slowest and fastest path: ties go to the lowest path index.
* Starting shares: proportional to the measured per-path bandwidth; every
  auxiliary path gets floor(total * bw_p / sum(bw)) and the primary path the
  rest.  A path that starts with 0 units starts retired, by the same rule that
  retires a path whose share falls to 0.
* Stage 2 looks at a window of the last W calls, every W calls; the per-path
  figure of a window is its median (mean of the two middle values when W is
  even); a retired path stays retired.
* Optional per-path ceiling (`cap`): a receiver is never filled beyond its
  ceiling.  A transfer trimmed to nothing leaves the shares alone; Stage 1
  counts such a round as a calm one.  With cap=None (the default) this module
  is the paper's method unchanged.
"""
import math
from dataclasses import dataclass
from typing import Optional


# ----------------------------------------------------------------- pieces

def initialize_shares(bw, total, primary=0):
    """Bandwidth-proportional starting shares.

    bw[p] is the measured rate of path p when it carries a whole message alone
    (any unit, the same for all paths; <= 0 means the path is unavailable).
    """
    usable = [max(b, 0.0) for b in bw]
    whole = 0.0
    for b in usable:                       # plain left-to-right sum, as the library does
        whole = whole + b
    shares = [0] * len(bw)
    for p, b in enumerate(usable):
        if p != primary and whole > 0:
            shares[p] = int(math.floor(total * b / whole))
    shares[primary] = total - sum(shares)
    return shares


def rank_paths(times, live):
    """(slowest, fastest) among the live paths; the lowest index wins a tie."""
    order = sorted(live)
    slowest = max(order, key=lambda p: (times[p], -p))
    fastest = min(order, key=lambda p: (times[p], p))
    return slowest, fastest


def find_slowest_fastest(times, live):
    return rank_paths(times, live)


def choose_transfer(slowest, fastest, live, primary):
    """The rule table of the module docstring: (giver, receiver)."""
    if slowest != primary and primary in live:
        return slowest, primary
    return slowest, fastest


def apply_transfer(shares, live, giver, receiver, want, cap=None):
    """Move up to `want` units; returns (shares', live', moved)."""
    room = want if cap is None or cap[receiver] is None else max(cap[receiver] - shares[receiver], 0)
    moved = min(want, shares[giver], room)
    out = list(shares)
    out[giver] -= moved
    out[receiver] += moved
    alive = set(live)
    if out[giver] <= 0:
        alive.discard(giver)
    return out, alive, moved


def spread(times, slowest, fastest):
    """Relative gap between the slowest and the fastest live path."""
    return (times[slowest] - times[fastest]) / times[fastest]


def median(values):
    v = sorted(values)
    n = len(v)
    mid = n // 2
    return v[mid] if n % 2 else (v[mid - 1] + v[mid]) / 2.0


# ---------------------------------------------------------------- Stage 1

@dataclass(frozen=True)
class Tuning:
    """State carried from one Stage-1 round to the next."""
    shares: tuple
    live: frozenset
    stride: int                       # units a transfer moves
    calm_rounds: int = 0              # consecutive rounds within the threshold
    last_giver: Optional[int] = None  # slowest path of the last round that moved
    rounds: int = 0
    done: bool = False


def tuning_start(shares, stride, primary=0):
    live = frozenset(p for p, s in enumerate(shares) if s > 0)
    return Tuning(tuple(shares), live, stride, done=(live == {primary}))


def tuning_round(state, times, primary=0, threshold=0.05, calm_needed=3, max_rounds=100, cap=None):
    """One Stage-1 round on the measured `times`.  Returns (state', report)."""
    slowest, fastest = rank_paths(times, state.live)
    gap = spread(times, slowest, fastest)
    shares, live = list(state.shares), set(state.live)
    stride, calm, last = state.stride, state.calm_rounds, state.last_giver
    settled = False
    if gap < threshold:
        calm += 1
        settled = calm >= calm_needed
    else:
        # a bottleneck that changed place means the last transfer overshot
        if last is not None and slowest != last:
            stride = max(stride // 2, 1)
        giver, receiver = choose_transfer(slowest, fastest, live, primary)
        shares, live, moved = apply_transfer(shares, live, giver, receiver, stride, cap)
        calm = 0
        if moved == 0:                # receiver at its ceiling: nothing can change any more
            calm = state.calm_rounds + 1
            settled = calm >= calm_needed
        last = slowest
    rounds = state.rounds + 1
    done = settled or live == {primary} or rounds >= max_rounds
    nxt = Tuning(tuple(shares), frozenset(live), stride, calm, last, rounds, done)
    report = dict(i=rounds, T=list(times), slow=slowest, fast=fastest, imbalance=gap, step=stride,
                  stability_count=calm, S=list(shares), active=sorted(live))
    return nxt, report


def initial_tune(S_init, measure, primary=0, step0=64, threshold=0.05,
                 stability_required=3, max_iters=100, trace=None, cap=None):
    """Stage 1 from start to end.  Returns (shares, live paths).

    S_init  -- starting shares, one per path.
    measure -- measure(shares, live) -> list of per-path completion times; the
               entries of retired paths are ignored.
    trace   -- optional list; one report (dict) per measured round is appended.
    """
    state = tuning_start(S_init, step0, primary)
    while not state.done:
        times = measure(list(state.shares), set(state.live))
        state, report = tuning_round(state, times, primary, threshold, stability_required, max_iters, cap)
        if trace is not None:
            trace.append(report)
    return list(state.shares), set(state.live)


# ---------------------------------------------------------------- Stage 2

class RuntimeAdjuster:
    """Stage 2: the Evaluator's window plus the periodic Load Balancer."""

    def __init__(self, S, C_active, primary=0, window=10, threshold=0.10, step=4, cap=None):
        self.S = list(S)
        self.C_active = set(C_active)
        self.primary = primary
        self.window = window
        self.threshold = threshold
        self.step = step
        self.cap = cap
        self.samples = []           # Evaluator: per-call lists of path times
        self.adjustments = 0

    def observe(self, T):
        """Record one collective call's per-path times.  Returns True when
        this call completed a window and the Load Balancer moved a share."""
        self.samples.append(list(T))
        if len(self.samples) < self.window:
            return False
        batch, self.samples = self.samples, []
        if len(self.C_active) < 2:
            return False
        typical = [median([s[p] for s in batch]) if p in self.C_active else 0.0 for p in range(len(self.S))]
        slowest, fastest = rank_paths(typical, self.C_active)
        if not spread(typical, slowest, fastest) > self.threshold:
            return False
        giver, receiver = choose_transfer(slowest, fastest, self.C_active, self.primary)
        self.S, self.C_active, moved = apply_transfer(self.S, self.C_active, giver, receiver, self.step, self.cap)
        if moved == 0:
            return False
        self.adjustments += 1
        return True
