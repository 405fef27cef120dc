"""Native host-side dispatching (include/sp_dispatch.h, through the binding) against the dispatch oracle, bit for bit:
integer and index work, so every output must be identical.  Host code only: these run without a GPU."""
import numpy as np
import pytest

from oracle import sp_dispatch_oracle as O
from paper_2408_12526_amd import dispatch as D


@pytest.mark.parametrize("seed", range(5))
def test_buffer_operations_bit_exact(seed):
    rng = np.random.default_rng(100 + seed)
    max_elem, cap = int(rng.integers(1, 6)), int(rng.integers(1, 40))
    bw = int(rng.choice([4, 8, 16]))
    a = O.LengthAwareBuffer(bw, 128, max_elem, cap)
    b = D.LengthAwareBuffer(bw, 128, max_elem, cap)
    sid = 0
    for _ in range(6000):
        r = rng.random()
        if r < 0.35:
            if len(a) == 0:
                with pytest.raises(D.DispatchError) as ei:
                    b.pop()
                assert ei.value.code == D.SP_EEMPTY
            else:
                assert a.pop() == b.pop()
        else:
            length = int(rng.integers(-3, 200))
            assert a.bin_of(length) == b.bin_of(length)
            try:
                want = a.push(sid, length)
            except O.BufferFull:
                with pytest.raises(D.DispatchError) as ei:
                    b.push(sid, length)
                assert ei.value.code == D.SP_EFULL
            else:
                assert b.push(sid, length) == want
            sid += 1
        assert len(a) == len(b) and a.samples() == b.samples()
    while len(a):
        assert a.pop() == b.pop()
    assert len(b) == 0 and b.samples() == 0


@pytest.mark.parametrize("seed", range(4))
def test_controller_bit_exact(seed):
    rng = np.random.default_rng(200 + seed)
    total = int(rng.integers(1, 9))
    slots = total * int(rng.integers(1, 4)) + int(rng.integers(0, 3))
    k_min = int(rng.integers(1, total + 1))
    k_start = int(rng.integers(k_min, total + 1))
    window = int(rng.choice([0, 50, 1000]))
    a = O.StudentNumberController(total, slots, k_min, window, k_start)
    b = D.StudentNumberController(total, slots, k_min, window, k_start)
    now = 0
    for _ in range(5000):
        now += int(rng.integers(0, 120))
        if rng.random() < 0.4:
            e = int(rng.integers(1, 12))
            assert a.on_buffered(e) == b.on_buffered(e)
        else:
            e = int(rng.integers(0, 2) * rng.integers(0, 5))
            busy = int(rng.integers(0, slots + 2))
            assert a.on_tick(now, e, busy) == b.on_tick(now, e, busy)
        assert a.k == b.k and a.groups() == b.groups() and k_min <= b.k <= total


def arrivals(rng, n, kind):
    if kind == "poisson":
        gaps = rng.exponential(60.0, n)
    elif kind == "burst":                      # quiet stretches and bursts an order of magnitude denser
        rate = np.where((np.arange(n) // 400) % 2 == 0, 300.0, 12.0)
        gaps = rng.exponential(rate)
    else:                                      # "ties": many equal time stamps
        gaps = rng.integers(0, 3, n) * 40.0
    arr = np.cumsum(gaps).astype(np.int64)
    lengths = np.clip(np.round(np.exp(rng.normal(np.log(48), 0.6, n))), 1, 300).astype(np.int32)
    return arr, lengths


@pytest.mark.parametrize("kind", ["poisson", "burst", "ties"])
@pytest.mark.parametrize("padded", [False, True])
@pytest.mark.parametrize("variant", [0, 1, 2])
def test_dispatcher_loop_bit_exact(kind, padded, variant):
    rng = np.random.default_rng(300 + 10 * ["poisson", "burst", "ties"].index(kind) + 3 * int(padded) + variant)
    n = 4000
    arr, lengths = arrivals(rng, n, kind)
    total, slots, k_min, window, cap, me = [(8, 8, 1, 20_000, 4096, 4), (4, 6, 2, 0, 5, 3), (8, 16, 1, 3_000, 64, 1)][variant]
    kw = dict(total_students=total, slots=slots, k_min=k_min, window_us=window, max_elem=me, capacity=cap,
              base_us=[0] + [140 + 6 * k for k in range(1, total + 1)],
              per_token_ns=[0] + [170 * k + 13 for k in range(1, total + 1)], padded=padded)
    want = O.simulate(arr.tolist(), lengths.tolist(), **kw)
    got = D.simulate(arr, lengths, **kw)
    assert got.refused == want.refused and (variant != 1 or want.refused > 0)       # variant 1 overflows its storage
    assert got.dispatch_us.tolist() == want.dispatch_us and got.done_us.tolist() == want.done_us
    assert got.k_used.tolist() == want.k_used and got.element.tolist() == want.element
    assert got.elem_tokens.tolist() == want.elem_tokens and got.elem_size.tolist() == want.elem_size
    assert got.k_trace == want.k_trace and len(want.k_trace) > 1


def test_native_dispatcher_on_the_hand_worked_traces():
    """The two traces worked by hand in test_dispatch_pins.py (a burst with k_min = 2; students coming back after an idle
    window), given to the native dispatcher directly: its result is pinned to the hand-worked numbers themselves, not only
    to the oracle's."""
    kw = dict(total_students=4, slots=4, k_min=2, window_us=10**9, base_us=[0, 100, 110, 120, 130],
              per_token_ns=[0, 1000, 1000, 1000, 1000], bin_width=8, max_len=128, max_elem=4, capacity=64, padded=False)
    r = D.simulate(np.zeros(6, dtype=np.int64), np.array([30, 30, 31, 52, 100, 30], dtype=np.int32), **kw)
    assert r.dispatch_us.tolist() == [0, 0, 0, 160, 171, 322] and r.done_us.tolist() == [160, 171, 171, 322, 381, 462]
    assert r.k_used.tolist() == [4, 2, 2, 2, 2, 2] and r.element.tolist() == [0, 1, 1, 2, 3, 4]
    assert r.elem_size.tolist() == [1, 2, 1, 1, 1] and r.elem_tokens.tolist() == [30, 61, 52, 100, 30]
    assert r.k_trace == [(0, 4), (0, 3), (0, 2)] and r.refused == 0
    kw.update(k_min=1, window_us=50)
    r = D.simulate(np.array([0, 0, 0, 1000, 1005], dtype=np.int64), np.array([10, 20, 40, 16, 8], dtype=np.int32), **kw)
    assert r.dispatch_us.tolist() == [0, 0, 130, 1000, 1005] and r.done_us.tolist() == [140, 130, 280, 1136, 1123]
    assert r.k_used.tolist() == [4, 2, 2, 3, 2] and r.element.tolist() == [0, 1, 2, 3, 4]
    assert r.elem_size.tolist() == [1] * 5 and r.elem_tokens.tolist() == [10, 20, 40, 16, 8]
    assert r.k_trace == [(0, 4), (0, 3), (0, 2), (280, 3), (1005, 2)] and r.refused == 0


def test_dispatch_argument_errors():
    with pytest.raises(D.DispatchError):
        D.LengthAwareBuffer(bin_width=8, max_len=100)            # not a multiple of the bin width
    with pytest.raises(D.DispatchError):
        D.LengthAwareBuffer(capacity=0)
    with pytest.raises(D.DispatchError):
        D.StudentNumberController(8, 4)                          # fewer instance slots than students
    with pytest.raises(D.DispatchError):
        D.StudentNumberController(8, 8, k_min=9)
    kw = dict(total_students=2, slots=2, k_min=1, window_us=0, base_us=[0, 1, 1], per_token_ns=[0, 1, 1], padded=False)
    with pytest.raises(D.DispatchError):
        D.simulate([5, 3], [10, 10], **kw)                       # arrivals must not go back in time
    r = D.simulate([], [], **kw)
    assert r.refused == 0 and len(r.elem_size) == 0 and r.k_trace == [(0, 2)]
