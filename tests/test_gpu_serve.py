"""Real-time replay of an arrival list on the GPU (sp_serve_replay): dispatcher thread + one worker thread per student
group, each running sp_forward on the elements it is handed.  Dispatch decisions depend on wall-clock timing and are
not reproducible, so what is compared is what is unique: every sample's logits against the oracle at the student number
it was served with, and the structural rules of the buffer."""
import numpy as np
import pytest

from paper_2408_12526_amd import synth

pytestmark = pytest.mark.gpu

SHAPE = synth.StudentShape(K=4, layers=2, hidden=256, heads=4, ffn=512, vocab=500, max_pos=128, classes=3, dtype="bf16")


@pytest.fixture(scope="module")
def loaded():
    import torch
    from paper_2408_12526_amd import sp
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (there is no fallback path)")
    rng = np.random.default_rng(41)
    blob = synth.make_weights(rng, SHAPE, std=0.05, ln_random=True, qk_std=0.1)
    st = sp.Students(sp.config_from_shape(SHAPE), blob)
    n = 300
    arr = synth.make_arrivals(rng, n, 3000.0, 30000.0, 0.02, 0.01)
    lengths = synth.make_lengths(rng, n, ("lognormal", 40, 0.6, 4, 200))      # some longer than max_len: clipped
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    ids = synth.make_ids(rng, int(off[-1]), SHAPE.vocab)
    return st, blob, arr, lengths, off, ids


def check_structure(r, arr, lengths, k_max):
    n = len(arr)
    assert r.refused == 0 and (r.element >= 0).all() and r.elem_size.sum() == n
    assert (r.dispatch_us >= arr).all() and (r.done_us > r.dispatch_us).all()
    assert ((r.k_used >= 1) & (r.k_used <= k_max)).all() and 1 <= r.k_final <= k_max
    clipped = np.minimum(lengths, 128)
    for e in range(len(r.elem_size)):
        members = np.nonzero(r.element == e)[0]
        assert len(members) == r.elem_size[e] <= 4
        assert len({int(-(-clipped[s] // 8)) for s in members}) == 1                 # one length bin per element
        assert len({int(r.dispatch_us[s]) for s in members}) == 1 and len({int(r.k_used[s]) for s in members}) == 1
        assert len({int(r.done_us[s]) for s in members}) == 1


def test_replay_serves_every_sample_with_oracle_logits(loaded, oracle64):
    from oracle.sp_oracle import OracleConfig
    from paper_2408_12526_amd import dispatch
    st, blob, arr, lengths, off, ids = loaded
    r = dispatch.serve_replay(st.handle, SHAPE.classes, arr, ids, off, slots=4, k_min=1, window_us=5000)
    check_structure(r, arr, lengths, SHAPE.K)
    oc = OracleConfig(SHAPE.K, SHAPE.layers, SHAPE.hidden, SHAPE.heads, SHAPE.ffn, SHAPE.vocab, SHAPE.max_pos,
                      SHAPE.classes)
    import torch
    w = torch.from_numpy(blob).to(torch.bfloat16).to(torch.float32).numpy()   # the weights as the bf16 path holds them
    clipped = np.minimum(lengths, 128)
    for k in sorted(set(r.k_used.tolist())):
        pick = np.nonzero(r.k_used == k)[0]
        sub_ids = np.concatenate([ids[off[s]:off[s] + clipped[s]] for s in pick])
        sub_cu = np.concatenate([[0], np.cumsum(clipped[pick])]).astype(np.int32)
        want = oracle64.forward(oc, w, sub_ids, sub_cu, int(k))
        got = r.logits[pick].astype(np.float64)
        err = np.abs(got - want).max() / max(np.abs(want).max(), 1e-3)
        assert err <= 3e-2, (k, err)


def test_replay_padded_variant_and_all_students(loaded):
    from paper_2408_12526_amd import dispatch
    st, blob, arr, lengths, off, ids = loaded
    r = dispatch.serve_replay(st.handle, SHAPE.classes, arr, ids, off, slots=4, k_min=4, window_us=5000, padded=True)
    check_structure(r, arr, lengths, SHAPE.K)
    assert (r.k_used == 4).all() and r.k_final == 4 and np.isfinite(r.logits).all()


def test_replay_argument_errors(loaded):
    from paper_2408_12526_amd import dispatch
    st, blob, arr, lengths, off, ids = loaded
    with pytest.raises(dispatch.DispatchError):
        dispatch.serve_replay(st.handle, SHAPE.classes, arr, ids, off, slots=2, k_min=1, window_us=0)       # slots < K
    with pytest.raises(dispatch.DispatchError):
        dispatch.serve_replay(st.handle, SHAPE.classes, arr, ids, off, slots=4, k_min=1, window_us=0, max_len=256)
    with pytest.raises(dispatch.DispatchError):
        dispatch.serve_replay(st.handle, SHAPE.classes, arr[::-1].copy(), ids, off, slots=4, k_min=1, window_us=0)
