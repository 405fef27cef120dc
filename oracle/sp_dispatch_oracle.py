"""Plain-Python oracle of the host-side dispatching of Student Parallelism: the length-aware buffer, the
student-number controller and the dispatcher loop that joins them.

TEST INFRASTRUCTURE ONLY: imported by tests/ and by the benchmark's cpu_baseline figure of the dispatch leg.  The
native implementation (csrc/sp_dispatch.cpp) shares no code with this module and never imports it.

What it follows (the algorithm's steps in the paper's order and words, not a listing):
  * length-aware buffer: Section 3.3.2 "Inference Sample Dispatching", its figure, and the appendix section
    "Details about Sample Dispatching based on Length-aware Buffer";
  * student-number controller: the appendix sections "Details about Student Allocation" and "Student Number
    Adaptation" (and Section 3.3.1);
  * dispatcher: steps of the appendix section on the online inference procedure (a sample goes out at once if a
    group is idle and nothing is buffered; otherwise it is buffered; whenever a group becomes idle the first buffer
    element goes out).

Readings where the paper is silent (the native code takes the same ones):
  D1  bins are `bin_width` (8) tokens wide over (0, max_len (128)]: a sample of n tokens belongs to bin
      ceil(n / 8) - 1 and is padded to 8 ceil(n / 8) tokens; longer samples are clipped to max_len, n < 1 counts as 1.
  D2  the dictionary holds, per bin, the position of the most recently appended element of that bin; a new sample can
      only join that element (never an older one of the same bin).
  D3  when the first element is dispatched its dictionary entry is deleted only if the entry still points at it (a newer
      element of the same bin keeps its entry).
  D4  the "maximum buffer size" (the number of student groups) is the controller's threshold; the storage has its own
      fixed capacity and a push that would exceed it is refused (the caller applies back-pressure).
  D5  "reaches the threshold" is evaluated when a sample has been buffered: if the buffer then holds at least as many
      elements as there are groups, one student is dropped (one per buffered sample, never below k_min).
  D6  the buffer-empty window restarts whenever the buffer is non-empty and after every increase; an increase needs
      idle_groups * k > occupied groups at the moment the window has elapsed.
  D7  groups(k) = floor(slots / k): `slots` is the number of student instances the hardware runs concurrently (the
      profiling result the paper calls the optimal student number sharing a GPU, times the GPUs).
  D8  events at the same microsecond: completions first (a group freed at t takes a sample arriving at t), then
      arrivals in input order.
  D9  an element in flight counts as one occupied group whatever student number it was dispatched with: after a
      decrease a new element is admitted while fewer than floor(slots / k_now) elements run, although older ones still
      hold k_old students each until they finish (optimistic during the transition).
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass, field


class BufferFull(Exception):
    pass


class LengthAwareBuffer:
    """Queue of elements (small batches of samples of one length bin) plus a dictionary bin -> element."""

    def __init__(self, bin_width=8, max_len=128, max_elem=4, capacity=64):
        assert bin_width >= 1 and max_len >= bin_width and max_len % bin_width == 0 and max_elem >= 1 and capacity >= 1
        self.bin_width, self.max_len, self.max_elem, self.capacity = bin_width, max_len, max_elem, capacity
        self.queue = deque()          # elements in arrival order of their first sample; element = dict
        self.where = {}               # bin -> the element most recently appended for that bin (D2)

    def bin_of(self, length):
        n = min(max(int(length), 1), self.max_len)              # D1
        return (n + self.bin_width - 1) // self.bin_width - 1

    def bin_len(self, b):
        return (b + 1) * self.bin_width

    def push(self, sample_id, length):
        """Returns True if the sample joined an existing element, False if it became a new tail element."""
        b = self.bin_of(length)
        e = self.where.get(b)
        if e is not None and len(e["ids"]) < self.max_elem:
            e["ids"].append(sample_id)
            e["lengths"].append(min(max(int(length), 1), self.max_len))
            return True
        if len(self.queue) >= self.capacity:
            raise BufferFull()                                  # D4
        e = {"bin": b, "ids": [sample_id], "lengths": [min(max(int(length), 1), self.max_len)]}
        self.queue.append(e)
        self.where[b] = e
        return False

    def pop(self):
        """Removes and returns the first element: (bin, padded length of the bin, sample ids, clipped lengths)."""
        e = self.queue.popleft()
        if self.where.get(e["bin"]) is e:                       # D3
            del self.where[e["bin"]]
        return e["bin"], self.bin_len(e["bin"]), list(e["ids"]), list(e["lengths"])

    def __len__(self):
        return len(self.queue)

    def samples(self):
        return sum(len(e["ids"]) for e in self.queue)


class StudentNumberController:
    """Keeps the number of active students per group, k, between k_min and total_students."""

    def __init__(self, total_students, slots, k_min=1, window_us=120_000_000, k_start=None):
        assert 1 <= k_min <= total_students and slots >= total_students and window_us >= 0
        self.total, self.slots, self.k_min, self.window_us = total_students, slots, k_min, window_us
        self.k = total_students if k_start is None else k_start
        assert k_min <= self.k <= total_students
        self.empty_since = None       # start of the current buffer-empty stretch

    def groups(self):
        return self.slots // self.k                             # D7

    def on_buffered(self, buffer_elements):
        """A sample has just been put into the buffer (D5).  Returns True if a student was dropped."""
        self.empty_since = None
        if buffer_elements >= self.groups() and self.k > self.k_min:
            self.k -= 1
            return True
        return False

    def on_tick(self, now_us, buffer_elements, busy_groups):
        """Any other observation of the system.  Returns True if a student was added (D6)."""
        if buffer_elements > 0:
            self.empty_since = None
            return False
        if self.empty_since is None:
            self.empty_since = now_us
        if now_us - self.empty_since < self.window_us or self.k >= self.total:
            return False
        g = self.groups()
        occupied = min(busy_groups, g)
        idle = g - occupied
        if idle * self.k > occupied:
            self.k += 1
            self.empty_since = now_us
            return True
        return False


@dataclass
class SimResult:
    dispatch_us: list = field(default_factory=list)      # per sample
    done_us: list = field(default_factory=list)
    k_used: list = field(default_factory=list)
    element: list = field(default_factory=list)          # index of the dispatched element the sample was part of
    elem_tokens: list = field(default_factory=list)      # per dispatched element: tokens computed
    elem_size: list = field(default_factory=list)
    k_trace: list = field(default_factory=list)          # (time, k) at every change
    refused: int = 0


def service_us(base_us, per_token_ns, k, tokens):
    """Service-time model shared by both sides as plain integer arithmetic: base[k] + per_token[k] * tokens / 1000."""
    return int(base_us[k]) + (int(per_token_ns[k]) * int(tokens)) // 1000


def simulate(arrival_us, lengths, *, total_students, slots, k_min, window_us, base_us, per_token_ns, padded,
             bin_width=8, max_len=128, max_elem=4, capacity=64, k_start=None):
    """Event-driven run of dispatcher + buffer + controller over a list of arrivals (times non-decreasing, integer
    microseconds).  `padded`: an element costs size * bin length tokens (the paper's padded small batch) instead of the
    sum of its samples' lengths (fully packed).  A refused sample (buffer storage full) is dropped and counted."""
    n = len(arrival_us)
    buf = LengthAwareBuffer(bin_width, max_len, max_elem, capacity)
    ctl = StudentNumberController(total_students, slots, k_min, window_us, k_start)
    res = SimResult([-1] * n, [-1] * n, [0] * n, [-1] * n)
    res.k_trace.append((0, ctl.k))
    running = []                  # completion times of the busy groups (unordered)

    def dispatch(now, bin_len, ids, lens):
        k = ctl.k
        tokens = len(ids) * bin_len if padded else sum(lens)
        done = now + service_us(base_us, per_token_ns, k, tokens)
        e = len(res.elem_tokens)
        res.elem_tokens.append(tokens)
        res.elem_size.append(len(ids))
        for s in ids:
            res.dispatch_us[s], res.done_us[s], res.k_used[s], res.element[s] = now, done, k, e
        running.append(done)

    def drain(now):
        # idle groups take buffer elements, first element first
        while len(buf) > 0 and len(running) < ctl.groups():
            _, bl, ids, lens = buf.pop()
            dispatch(now, bl, ids, lens)

    i = 0
    while i < n or running:
        t_done = min(running) if running else None
        if t_done is not None and (i >= n or t_done <= arrival_us[i]):          # D8
            now = t_done
            running.remove(t_done)
            drain(now)
            if ctl.on_tick(now, len(buf), len(running)):
                res.k_trace.append((now, ctl.k))
            continue
        now = arrival_us[i]
        if len(buf) == 0 and len(running) < ctl.groups():
            b = buf.bin_of(lengths[i])
            dispatch(now, buf.bin_len(b), [i], [min(max(int(lengths[i]), 1), max_len)])
            if ctl.on_tick(now, 0, len(running)):
                res.k_trace.append((now, ctl.k))
        else:
            try:
                buf.push(i, lengths[i])
                if ctl.on_buffered(len(buf)):
                    res.k_trace.append((now, ctl.k))
                    drain(now)                                  # more groups may exist now
            except BufferFull:
                res.refused += 1
        i += 1
    return res
