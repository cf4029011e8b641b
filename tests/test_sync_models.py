"""CPU models of the two cross-workgroup protocols of the library, run under random interleavings.

The kernels themselves cannot be single-stepped, so their synchronisation logic is restated here step by step
(one `yield` per access to memory that other workgroups see) and driven by a scheduler that picks the next
workgroup at random, lets workgroups start late (not resident yet) and lets waits run out.  What is checked is
the protocol, not the arithmetic: that every wait ends, that nothing is consumed before it was produced, that
work is done exactly once, and that the result does not depend on the interleaving.

  * the selection of one unit by several workgroups (kvs_select.hip, select_unit_split): three rendezvous through
    an exchange area, bounded waits, a phase that either completes for every part or fails for every part (a part
    that runs out of time marks the phase counter with a compare-and-swap that only succeeds while the count is
    short), the unit's first part selecting alone when a phase fails or the threshold's bin is too crowded for the
    list;
  * the one-pass score kernel (kvs_score_fused.hip): work items handed out by a ticket counter in unit order, the
    workgroup that publishes a unit's last statistics reduces them to the normalisers, the others wait (bounded) for
    them, and items given up on go to a list that a second launch finishes.
"""

import random

import numpy as np
import pytest

from oracle import kvs_oracle as O


# ------------------------------------------------------------------------------------------------ scheduler
def run_interleaved(workgroups, rng, resident, max_steps=2_000_000):
    """workgroups: generators.  At most `resident` of them run at a time, in index order of admission (as a GPU
    dispatches a grid); the next one is admitted when one finishes.  Returns the number of steps taken."""
    waiting = list(range(len(workgroups)))
    live = []
    steps = 0
    while waiting or live:
        while waiting and len(live) < resident:
            live.append(waiting.pop(0))
        i = rng.choice(live)
        try:
            next(workgroups[i])
        except StopIteration:
            live.remove(i)
        steps += 1
        assert steps < max_steps, "the protocol did not come to an end"
    return steps


# ------------------------------------------------------------------------------------------------ split selection
GAVE_UP = 1 << 16


class Exchange:
    def __init__(self, bins, cand_max):
        self.notmin = 0                 # the area starts from zero: the minimum travels complemented
        self.max = 0
        self.ncand = 0
        self.arrive = [0] * 3
        self.hist = [0] * bins
        self.cand = [None] * cand_max
        self.cand_part = [None] * cand_max
        self.part_low = {}


MASK32 = 0xFFFFFFFF


def single_workgroup_select(keys, r):
    """What one workgroup computes: the r smallest keys, ties to the lower index."""
    order = np.argsort(keys, kind="stable")
    sel = np.zeros(len(keys), dtype=bool)
    sel[order[:r]] = True
    return sel


def select_part(part, P, keys, r, g, out, log, timeout, bins, cand_max):
    """One part of select_unit_split.  `out[t]` receives the selection flags; `log` counts what happened."""
    n = len(keys)
    per = (n + P - 1) // P
    lo, hi = min(n, part * per), min(n, (part + 1) * per)
    mine = keys[lo:hi]

    def arrive(phase):
        g.arrive[phase] += 1
        yield

    def wait(phase):
        waited = 0
        while True:
            v = g.arrive[phase]
            yield                                       # (others move between the load and what follows)
            if v == P:
                return True
            if v & GAVE_UP:
                return False
            if waited >= timeout:
                if g.arrive[phase] == v:                # compare-and-swap: only while the count is still what was read
                    g.arrive[phase] = v | GAVE_UP
                    return False
                continue
            waited += 1

    def give_up(phase):
        log["gave_up"].append((part, phase))
        if part == 0:                                  # the unit's first part selects alone
            log["fallback"] += 1
            sel = single_workgroup_select(keys, r)
            for t in range(n):
                out[t].append(bool(sel[t]))
                if t % 7 == 0:
                    yield

    # phase 0: minimum and maximum
    if len(mine):
        g.notmin = max(g.notmin, (~int(mine.min())) & MASK32)
        yield
        g.max = max(g.max, int(mine.max()))
        yield
    yield from arrive(0)
    if not (yield from wait(0)):
        yield from give_up(0)
        return
    kmin, kmax = (~g.notmin) & MASK32, g.max
    span = max(kmax - kmin, 1)
    digit = lambda k: min(bins - 1, (int(k) - kmin) * bins // (span + 1))
    # phase 1: histogram of the first digit
    for k in mine:
        g.hist[digit(k)] += 1
    yield
    yield from arrive(1)
    if not (yield from wait(1)):
        yield from give_up(1)
        return
    hist = list(g.hist)
    assert sum(hist) == n, "a histogram was read before every part had added to it"
    below, b = 0, 0
    while below + hist[b] < r:
        below += hist[b]
        b += 1
    want = r - below
    if hist[b] > cand_max:                              # every part sees the same histogram and leaves the same way
        log["crowded"] += 1
        yield from give_up(-1)
        return
    # phase 2: the keys of that bin with this part's number, and this part's keys in the bins below
    cands = [int(k) for k in mine if digit(k) == b]
    g.part_low[part] = sum(1 for k in mine if digit(k) < b)
    yield
    base = g.ncand
    g.ncand += len(cands)
    yield
    for i, k in enumerate(cands):
        g.cand[base + i] = k
        g.cand_part[base + i] = part
        if i % 3 == 0:
            yield
    yield from arrive(2)
    if not (yield from wait(2)):
        yield from give_up(2)
        return
    lst = g.cand[:hist[b]]
    tags = g.cand_part[:hist[b]]
    assert None not in lst and None not in tags, "the list was read before every part had written its keys"
    srt = sorted(lst)
    T = srt[want - 1]
    n_equal = srt.count(T)
    want_eq = want - sum(1 for k in srt if k < T)
    simple = n_equal == want_eq
    # what lies before this part: from the list and the parts' counts alone, nothing more is exchanged
    eq_before = 0
    for p in range(part):
        assert p in g.part_low, "a part's count was read before it was written"
        if not simple:
            eq_before += sum(1 for k, tg in zip(lst, tags) if tg == p and k == T)
    selected = lambda k: digit(k) < b or (digit(k) == b and (int(k) < T or (simple and int(k) == T)))
    for t in range(lo, hi):
        k = int(keys[t])
        if selected(k):
            s = True
        elif k == T:
            s = eq_before < want_eq
            eq_before += 1
        else:
            s = False
        out[t].append(s)
        if t % 5 == 0:
            yield
    log["finished"] += 1


@pytest.mark.parametrize("seed", range(40))
def test_split_selection_protocol(seed):
    rng = random.Random(seed)
    nrng = np.random.default_rng(seed)
    n = rng.choice([40, 200, 1000])
    P = rng.choice([2, 3, 8, 16])
    kinds = rng.choice(["spread", "ties", "crowded"])
    if kinds == "spread":
        keys = nrng.integers(1000, 1 << 30, size=n, dtype=np.int64)
    elif kinds == "ties":
        keys = nrng.integers(5, 9, size=n, dtype=np.int64) * 1000
    else:
        keys = 50_000 + nrng.integers(0, 3, size=n, dtype=np.int64)
    r = rng.randint(1, n - 1)
    timeout = rng.choice([0, 3, 50, 10_000])
    resident = rng.choice([1, 2, P, P])                # fewer slots than parts: late parts find the unit given up
    g = Exchange(bins=16, cand_max=64)
    out = [[] for _ in range(n)]
    log = {"gave_up": [], "fallback": 0, "finished": 0, "crowded": 0}
    parts = [select_part(p, P, keys, r, g, out, log, timeout, 16, 64) for p in range(P)]
    run_interleaved(parts, rng, resident)
    ref = single_workgroup_select(keys, r)
    for t in range(n):
        assert out[t], f"token {t} was never written"
        assert all(v == bool(ref[t]) for v in out[t]), f"token {t}: a writer disagrees with the single-workgroup result"
    if not log["gave_up"]:
        assert log["finished"] == P and log["fallback"] == 0
    else:
        # a phase fails for every part or for none: all parts left, at the same phase, and nobody wrote but part 0
        assert len(log["gave_up"]) == P and len({ph for _, ph in log["gave_up"]}) == 1
        assert log["fallback"] == 1 and log["finished"] == 0
    if timeout == 10_000 and resident >= P and not log["crowded"]:
        assert not log["gave_up"], "with every part resident and time to spare nobody gives up"


def test_split_selection_matches_the_oracle_selection():
    """The model's single-workgroup rule is the oracle's selection on the same scores (ties to the lower index)."""
    rng = np.random.default_rng(3)
    a = rng.integers(1, 4, size=300).astype(np.float64)
    a /= a.sum()
    mask, _ = O.select(a.astype(np.float32), 120, 0, 0, sigma_dtype=np.float32)
    sigma = (a.astype(np.float32)[:-1] + a.astype(np.float32)[1:])
    sel = single_workgroup_select(sigma.view(np.uint32).astype(np.int64), 300 - 120)
    assert (sel == (mask[:-1] == 1)).all()    # the mask byte of token m says whether edge (m, m + 1) is selected


# ------------------------------------------------------------------------------------------------ one-pass score
def fused_workgroup(wg, grid, units, sh, log, timeout):
    """One persistent workgroup of score_fused_kernel<SECOND = false>.  units: items per unit."""
    total = sum(units)
    first = np.concatenate([[0], np.cumsum(units)])
    item = sh["ticket"]
    sh["ticket"] += 1
    yield
    while item < total:
        u = int(np.searchsorted(first, item, side="right") - 1)
        chunk = item - first[u]
        yield                                            # phase A
        sh["stats"][item] = True                          # the item's statistics are out before it waits for anything
        yield
        sh["done"][u] += 1
        last = sh["done"][u] == units[u]
        yield
        ok = True
        if last:
            assert all(sh["stats"][first[u]:first[u + 1]]), "normalisers reduced before every chunk's statistics were out"
            assert not sh["c_ready"][u], "a unit's normalisers were reduced twice"
            yield
            sh["c_ready"][u] = True
        else:
            ok = False
            if units[u] - 1 - chunk <= grid // 2:        # otherwise the unit's other chunks cannot all start in time
                for _ in range(timeout + 1):
                    if sh["c_ready"][u]:
                        ok = True
                        break
                    yield
        if not ok:
            sh["deferred"].append(item)
        nxt = sh["ticket"]
        sh["ticket"] += 1
        yield
        if ok:
            assert sh["c_ready"][u]
            log["phase_b"][item] += 1
            yield
        item = nxt


@pytest.mark.parametrize("seed", range(40))
def test_one_pass_score_protocol(seed):
    rng = random.Random(100 + seed)
    grid = rng.choice([1, 2, 5, 16])
    units = [rng.choice([1, 2, 3, 9, 40]) for _ in range(rng.randint(1, 6))]
    timeout = rng.choice([0, 2, 30, 5_000])
    total = sum(units)
    sh = {"ticket": 0, "stats": [False] * total, "done": [0] * len(units), "c_ready": [False] * len(units),
          "deferred": []}
    log = {"phase_b": [0] * total}
    wgs = [fused_workgroup(w, grid, units, sh, log, timeout) for w in range(grid)]
    run_interleaved(wgs, rng, resident=grid)
    # the first launch has ended: every unit's normalisers exist, whatever was given up on
    assert all(sh["c_ready"]) and all(sh["stats"])
    assert len(set(sh["deferred"])) == len(sh["deferred"])
    for item in sh["deferred"]:                           # the second launch finishes the listed items from memory
        log["phase_b"][item] += 1
    assert log["phase_b"] == [1] * total, "every item's alpha_bar phase runs exactly once"
    if grid == 1:
        # one workgroup: an item can only be finished in the first launch when it is its unit's last
        assert len(sh["deferred"]) == total - len(units)
