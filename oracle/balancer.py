"""Oracle for FlexLink's two-stage load balancer.

TEST INFRASTRUCTURE, NOT THE PRODUCT: imported only by the test-suite and the
smoke check.  It shares no code with the C++ balancer in the HIP library and
does not import it.

The balancer is a heuristic, so the oracle is the algorithm itself, taken step
by step in the paper's order and notation:

* Stage 1 is the paper's Algorithm 1 ("Initial Coarse-Grained Load Tuning",
  Section "Stage 1: Initial Coarse-Grained Tuning").
* Stage 2 is the prose of Section "Stage 2: Runtime Fine-Grained Adjustment".

A path is identified by its index in C; the path the paper calls NVLink (the
primary path, which the tuning favours) is passed in as `primary`.  Shares are
non-negative integers that sum to a fixed total.

Parity unpinned against the paper: it prints no worked numerical example of
the balancer, and the load percentages of its Table 2 belong to H800 links.
The pins are hand-executed trajectories of Algorithm 1, the closed-form balance
point of a pure-bandwidth timing model, and the properties the prose states.

Readings taken where the paper leaves a choice (each is a documented reading,
not a fact of the paper):

* Shares and `step` are integers, `step / 2` is integer division (the
  algorithm's max(step / 2, 1) only makes sense for integers).
* Slowest and fastest path: ties go to the lowest path index.
* InitializeShares: proportional to the measured per-path bandwidth; every
  auxiliary path gets floor(total * bw_p / sum(bw)) and the primary path the
  rest, which makes the primary's share the dominant one whenever it is the
  fastest path.  A path whose initial share is 0 starts inactive, by the same
  rule that deactivates a path whose share falls to 0.
* Stage 2 looks at a window of the last W calls, every W calls; the per-path
  figure of a window is its median (mean of the two middle values when W is
  even); the target of a move is chosen by the same primary-first rule as in
  Algorithm 1; a deactivated path stays deactivated.
"""
import math


def initialize_shares(bw, total, primary=0):
    """Bandwidth-proportional starting shares.

    bw[p] is the measured rate of path p when it carries a whole message alone
    (any unit, the same for all paths; <= 0 means the path is unavailable).
    """
    rate = [b if b > 0 else 0.0 for b in bw]
    denom = 0.0
    for b in rate:
        denom = denom + b
    S = [0] * len(bw)
    used = 0
    for p in range(len(bw)):
        if p == primary:
            continue
        S[p] = int(math.floor(total * rate[p] / denom)) if denom > 0 else 0
        used += S[p]
    S[primary] = total - used
    return S


def find_slowest_fastest(T, C_active):
    """Indices of the largest and smallest time among active paths."""
    c_slow = c_fast = None
    for c in sorted(C_active):
        if c_slow is None or T[c] > T[c_slow]:
            c_slow = c
        if c_fast is None or T[c] < T[c_fast]:
            c_fast = c
    return c_slow, c_fast


def initial_tune(S_init, measure, primary=0, step0=64, threshold=0.05,
                 stability_required=3, max_iters=100, trace=None):
    """Algorithm 1.  Returns (S, C_active).

    S_init  -- starting shares, one per path (InitializeShares' result).
    measure -- measure(S, C_active) -> list of per-path completion times; the
               entries of inactive paths are ignored.
    trace   -- optional list; one dict per measured iteration is appended.
    """
    S = list(S_init)
    C_active = {c for c in range(len(S)) if S[c] > 0}
    step = step0
    stability_count = 0
    prev_slowest = None
    for i in range(1, max_iters + 1):
        if C_active == {primary}:
            break                                   # only the primary remains
        T = measure(list(S), set(C_active))
        c_slow, c_fast = find_slowest_fastest(T, C_active)
        imbalance = (T[c_slow] - T[c_fast]) / T[c_fast]
        stable_exit = False
        if imbalance < threshold:
            stability_count += 1
            if stability_count >= stability_required:
                stable_exit = True
        else:
            stability_count = 0
            if c_slow != prev_slowest and prev_slowest is not None:
                step = max(step // 2, 1)            # bottleneck moved: damp
            c_source = c_slow
            if c_slow != primary and primary in C_active:
                c_target = primary                  # favour the primary path
            else:
                c_target = c_fast                   # primary is the bottleneck
            move_amount = min(step, S[c_source])
            S[c_source] -= move_amount
            S[c_target] += move_amount
            if S[c_source] <= 0:
                C_active.discard(c_source)
            prev_slowest = c_slow
        if trace is not None:
            trace.append(dict(i=i, T=list(T), slow=c_slow, fast=c_fast,
                              imbalance=imbalance, step=step,
                              stability_count=stability_count,
                              S=list(S), active=sorted(C_active)))
        if stable_exit:
            break
    return S, C_active


def median(values):
    v = sorted(values)
    n = len(v)
    if n % 2:
        return v[n // 2]
    return (v[n // 2 - 1] + v[n // 2]) / 2.0


class RuntimeAdjuster:
    """Stage 2: Evaluator window plus the periodic Load Balancer."""

    def __init__(self, S, C_active, primary=0, window=10, threshold=0.10, step=4):
        self.S = list(S)
        self.C_active = set(C_active)
        self.primary = primary
        self.window = window
        self.threshold = threshold
        self.step = step
        self.samples = []           # Evaluator: per-call tuples of path times
        self.adjustments = 0

    def observe(self, T):
        """Record one collective call's per-path times.  Returns True when
        this call completed a window and the Load Balancer moved a share."""
        self.samples.append(list(T))
        if len(self.samples) < self.window:
            return False
        samples, self.samples = self.samples, []
        if len(self.C_active) < 2:
            return False
        Tm = [median([s[c] for s in samples]) if c in self.C_active else 0.0
              for c in range(len(self.S))]
        c_slow, c_fast = find_slowest_fastest(Tm, self.C_active)
        gap = (Tm[c_slow] - Tm[c_fast]) / Tm[c_fast]
        if not gap > self.threshold:
            return False
        c_source = c_slow
        if c_slow != self.primary and self.primary in self.C_active:
            c_target = self.primary
        else:
            c_target = c_fast
        move_amount = min(self.step, self.S[c_source])
        self.S[c_source] -= move_amount
        self.S[c_target] += move_amount
        if self.S[c_source] <= 0:
            self.C_active.discard(c_source)
        self.adjustments += 1
        return True
