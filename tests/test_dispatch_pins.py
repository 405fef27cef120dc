"""Pins of the dispatch oracle (oracle/sp_dispatch_oracle.py) against things other than itself: the paper's worked
example, a brute-force formulation without the dictionary, hand-worked controller traces, closed forms of the
dispatcher loop.  CPU only."""
import os

import numpy as np
import pytest

from oracle import sp_dispatch_oracle as O

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "length_aware_buffer_figure.txt")


def test_figure_example_of_the_paper():
    """Section 3.3.2, figure "Length-aware Buffer": 30 tokens joins the not-full element of its bin, 52 tokens finds
    the element of its bin full and goes to the tail."""
    buf = O.LengthAwareBuffer(bin_width=8, max_len=128, max_elem=4, capacity=16)
    for n, line in enumerate(l for l in open(GOLDEN) if l.strip() and not l.startswith("#")):
        parts = line.split()
        length, want = int(parts[0]), parts[1]
        before = [list(e["ids"]) for e in buf.queue]
        joined = buf.push(n, length)
        after = [list(e["ids"]) for e in buf.queue]
        if want == "tail":
            assert not joined and after[:-1] == before and after[-1] == [n], line
        else:
            e = int(parts[2])
            assert joined and len(after) == len(before) and after[e] == before[e] + [n], line
    assert [len(e["ids"]) for e in buf.queue] == [2, 4, 1]
    assert buf.pop()[1] == 32 and buf.pop()[1] == 56 and buf.pop()[1] == 56      # padded lengths of the bins


def test_bins_are_eight_tokens_wide():
    """Appendix: the range 0-128 in 16 bins at every step of 8 tokens; a sample is padded or clipped to the maximum
    length of its bin."""
    buf = O.LengthAwareBuffer()
    assert [buf.bin_of(n) for n in (1, 8, 9, 16, 17, 120, 121, 128)] == [0, 0, 1, 1, 2, 14, 15, 15]
    assert {buf.bin_of(n) for n in range(1, 129)} == set(range(16))
    assert all(buf.bin_len(buf.bin_of(n)) >= n and buf.bin_len(buf.bin_of(n)) - n < 8 for n in range(1, 129))
    assert buf.bin_of(500) == 15 and buf.bin_of(0) == 0                            # clipped


class BruteForceBuffer:
    """The same behaviour stated without a dictionary: a new sample joins the LAST element of its bin in the queue
    if that element has room, else it becomes the tail.  O(queue) per push: a definition, not an implementation."""

    def __init__(self, bin_width, max_len, max_elem):
        self.bw, self.ml, self.me, self.q = bin_width, max_len, max_elem, []

    def push(self, sid, length):
        n = min(max(length, 1), self.ml)
        b = -(-n // self.bw) - 1
        for e in reversed(self.q):
            if e[0] == b:
                if len(e[1]) < self.me:
                    e[1].append(sid)
                    return
                break
        self.q.append((b, [sid]))

    def pop(self):
        return self.q.pop(0)


@pytest.mark.parametrize("seed", range(6))
def test_dictionary_bookkeeping_against_brute_force(seed):
    """Random pushes and pops: the queue of the oracle (dictionary + queue, O(1) operations) always equals the
    brute-force definition.  A wrong deletion rule on dispatch, a stale pointer or a join into an older element of
    the bin fails here."""
    rng = np.random.default_rng(seed)
    me = int(rng.integers(1, 5))
    a = O.LengthAwareBuffer(8, 128, me, capacity=10_000)
    b = BruteForceBuffer(8, 128, me)
    sid = 0
    for _ in range(4000):
        if len(a) and rng.random() < 0.3:
            bin_, bl, ids, lens = a.pop()
            wb, wids = b.pop()
            assert (bin_, ids) == (wb, wids) and bl == 8 * (bin_ + 1) and all(a.bin_of(x) == bin_ for x in lens)
        else:
            length = int(rng.choice([5, 12, 13, 30, 31, 52, 64, 100, 128, 300]))
            a.push(sid, length)
            b.push(sid, length)
            sid += 1
        assert [(e["bin"], e["ids"]) for e in a.queue] == [(x, y) for x, y in b.q]
        # the dictionary holds exactly the bins that are present, each pointing at the last element of its bin
        last = {}
        for e in a.queue:
            last[e["bin"]] = e
        assert set(a.where) == set(last) and all(a.where[k] is last[k] for k in last)


def test_buffer_invariants_and_capacity():
    buf = O.LengthAwareBuffer(8, 128, 4, capacity=3)
    for i, n in enumerate((10, 20, 30)):
        assert not buf.push(i, n)
    assert buf.push(3, 11)                      # joins, needs no new element
    with pytest.raises(O.BufferFull):
        buf.push(4, 40)                         # a fourth element does not fit the storage
    assert len(buf) == 3 and buf.samples() == 4
    assert buf.pop()[2] == [0, 3]               # first in, first out; samples of an element in arrival order
    assert not buf.push(5, 12)                  # the entry of bin 1 went with its element: a new tail element
    assert [e["ids"] for e in buf.queue] == [[1], [2], [5]]


def test_controller_hand_worked_trace():
    """Appendix "Student Number Adaptation": drop one student when the buffer reaches the number of groups; add one
    when the buffer has been empty for the window and the idle groups hold more students than there are occupied
    groups.  8 students, 8 instance slots: k = 8 -> 1 group, 4 -> 2 groups, 2 -> 4, 1 -> 8."""
    c = O.StudentNumberController(total_students=8, slots=8, k_min=1, window_us=100)
    assert (c.k, c.groups()) == (8, 1)
    assert c.on_buffered(1) and c.k == 7 and c.groups() == 1       # 1 element >= 1 group
    assert c.on_buffered(1) and c.k == 6
    for _ in range(2):
        c.on_buffered(5)
    assert (c.k, c.groups()) == (4, 2)
    assert not c.on_buffered(1) and c.k == 4                       # 1 element < 2 groups: nothing happens
    assert c.on_buffered(2) and (c.k, c.groups()) == (3, 2)
    # the buffer empties at t = 1000; both groups idle; the window is 100 us
    assert not c.on_tick(1000, 0, 0) and not c.on_tick(1099, 0, 0)
    assert c.on_tick(1100, 0, 0) and c.k == 4                      # 2 idle groups x 3 students > 0 occupied
    assert not c.on_tick(1150, 0, 0)                               # the window restarted at 1100
    assert not c.on_tick(1160, 1, 2) and not c.on_tick(1300, 0, 2) # non-empty buffer restarts it again (at 1300)
    assert not c.on_tick(1400, 0, 2)                               # elapsed, but no idle group: 0 > 2 is false
    assert c.on_tick(1401, 0, 1) and c.k == 5                      # 1 idle group x 4 students > 1 occupied
    c2 = O.StudentNumberController(total_students=3, slots=3, k_min=2, window_us=0, k_start=2)
    assert not c2.on_buffered(9) and c2.k == 2                     # never below k_min
    assert c2.on_tick(0, 0, 0) and c2.k == 3 and not c2.on_tick(5, 0, 0)   # never above the trained number


KW = dict(total_students=4, slots=4, k_min=1, window_us=10**9, base_us=[0, 100, 110, 120, 130],
          per_token_ns=[0, 1000, 1000, 1000, 1000], bin_width=8, max_len=128, max_elem=4, capacity=64)


def test_dispatcher_sparse_arrivals_go_out_at_once():
    """Closed form: when every sample arrives after the previous one has finished, nothing is ever buffered: each is
    dispatched at its arrival time, alone, with all students, and takes base + length microseconds."""
    lengths = [10, 64, 128, 33]
    arr = [0, 1000, 2000, 3000]
    r = O.simulate(arr, lengths, padded=False, **KW)
    assert r.dispatch_us == arr and r.k_used == [4] * 4 and r.elem_size == [1] * 4
    assert r.done_us == [a + 130 + n for a, n in zip(arr, lengths)]
    rp = O.simulate(arr, lengths, padded=True, **KW)
    assert rp.done_us == [a + 130 + 8 * -(-n // 8) for a, n in zip(arr, lengths)]   # padded to the bin


def test_dispatcher_burst_hand_worked():
    """Six samples at t = 0 with 4 slots and k_min = 2, worked by hand.  Sample 0 goes out alone (k = 4, one group;
    done at 130 + 30 = 160).  Samples 1..5 find the group busy and are buffered.  Sample 1 (30 tokens): new element;
    1 element >= 1 group, so k = 3 (still one group).  Sample 2 (31): same bin, joins; 1 >= 1, so k = 2, two groups:
    the element [1, 2] goes out at t = 0 with k = 2 (110 + 61 = 171).  Sample 3 (52): both groups are busy, new
    element; 1 element < 2 groups.  Sample 4 (100): new element; 2 >= 2 but k is already k_min.  Sample 5 (30): the
    entry of its bin left with [1, 2], so a new element.  Completions: t = 160: [3] goes out (110 + 52 -> 322);
    t = 171: [4] (110 + 100 -> 381); t = 322: [5] (110 + 30 -> 462)."""
    kw = dict(KW, k_min=2)
    r = O.simulate([0] * 6, [30, 30, 31, 52, 100, 30], padded=False, **kw)
    assert r.dispatch_us == [0, 0, 0, 160, 171, 322]
    assert r.done_us == [160, 171, 171, 322, 381, 462]
    assert r.k_used == [4, 2, 2, 2, 2, 2]
    assert r.element == [0, 1, 1, 2, 3, 4] and r.elem_size == [1, 2, 1, 1, 1] and r.elem_tokens == [30, 61, 52, 100, 30]
    assert r.k_trace == [(0, 4), (0, 3), (0, 2)] and r.refused == 0


def test_dispatcher_idle_window_hand_worked():
    """Students come back after an idle window, worked by hand (4 students, 4 slots, window 50 us, 1 us per token).
    t = 0: sample 0 (10 tokens) goes out alone with k = 4 (done 0 + 130 + 10 = 140).  Sample 1 (20) finds the one group
    busy: buffered, 1 element >= 1 group, k = 3 (still one group).  Sample 2 (40, another bin): second element,
    2 >= 1, k = 2: two groups, the idle one takes [1] (done 0 + 110 + 20 = 130).  t = 130: that group finishes and
    takes [2] (130 + 110 + 40 = 280); the buffer is empty from here on.  t = 140: sample 0 done, 10 us of empty buffer.
    t = 280: last group done; 150 us >= the window, two idle groups x 2 students > 0 occupied: k = 3, window restarts.
    t = 1000: sample 3 (16) goes out at once with k = 3 (1000 + 120 + 16 = 1136); the window has elapsed again but the
    only group (4 // 3 = 1) is occupied: 0 x 3 > 1 is false.  t = 1005: sample 4 (8) finds it busy: buffered,
    1 >= 1, k = 2, and the second group that now exists takes it (1005 + 110 + 8 = 1123)."""
    kw = dict(KW, window_us=50)
    r = O.simulate([0, 0, 0, 1000, 1005], [10, 20, 40, 16, 8], padded=False, **kw)
    assert r.dispatch_us == [0, 0, 130, 1000, 1005]
    assert r.done_us == [140, 130, 280, 1136, 1123]
    assert r.k_used == [4, 2, 2, 3, 2]
    assert r.element == [0, 1, 2, 3, 4] and r.elem_size == [1] * 5 and r.elem_tokens == [10, 20, 40, 16, 8]
    assert r.k_trace == [(0, 4), (0, 3), (0, 2), (280, 3), (1005, 2)] and r.refused == 0


@pytest.mark.parametrize("padded", [False, True])
def test_dispatcher_conservation_and_bounds(padded):
    """Properties at any size: every sample is dispatched exactly once, not before it arrives; elements hold one bin
    and at most max_elem samples; never more groups busy than exist for the k in force; k stays in range; the padded
    variant never computes fewer tokens than the packed one for the same element."""
    rng = np.random.default_rng(3)
    n = 3000
    arr = np.cumsum(rng.exponential(40.0, n)).astype(np.int64).tolist()
    lengths = np.clip(np.round(np.exp(rng.normal(np.log(48), 0.6, n))), 8, 256).astype(int).tolist()
    kw = dict(total_students=8, slots=8, k_min=1, window_us=20_000, base_us=[0] + [140 + 5 * k for k in range(1, 9)],
              per_token_ns=[0] + [150 * k for k in range(1, 9)], max_elem=4, capacity=4096)
    r = O.simulate(arr, lengths, padded=padded, **kw)
    assert r.refused == 0 and all(d >= a for d, a in zip(r.dispatch_us, arr)) and all(x > 0 for x in r.k_used)
    assert all(1 <= k <= 8 for _, k in r.k_trace) and all(abs(a[1] - b[1]) == 1 for a, b in zip(r.k_trace, r.k_trace[1:]))
    members = {}
    for s, e in enumerate(r.element):
        members.setdefault(e, []).append(s)
    assert sorted(members) == list(range(len(r.elem_size)))
    for e, ss in members.items():
        assert len(ss) == r.elem_size[e] <= 4
        bins = {-(-min(lengths[s], 128) // 8) for s in ss}
        assert len(bins) == 1 and len({r.dispatch_us[s] for s in ss}) == 1
        true_tokens = sum(min(lengths[s], 128) for s in ss)
        assert r.elem_tokens[e] == (len(ss) * 8 * bins.pop() if padded else true_tokens) >= true_tokens
    # busy groups over time: sweep the dispatch / completion events of the elements
    ev = []
    for e, ss in members.items():
        s = ss[0]
        ev.append((r.dispatch_us[s], 1, 8 // r.k_used[s]))
        ev.append((r.done_us[s], 0, 0))
    busy = 0
    for t, kind, cap in sorted(ev):
        busy += 1 if kind else -1
        assert not kind or busy <= cap
