"""sp_forward_static (the entry point that allocates nothing) against sp_forward, through the C ABI.  Needs an MI355X."""
import numpy as np
import pytest
import torch

from paper_2408_12526_amd import synth

pytestmark = pytest.mark.gpu


def _inputs(sp, rng, lengths, vocab):
    lengths = np.array(lengths, dtype=np.int32)
    ids = synth.make_ids(rng, int(lengths.sum()), vocab)
    cu = sp.sp_pack(lengths)
    return torch.from_numpy(ids).cuda(), torch.from_numpy(cu).cuda(), int(lengths.max())


def test_static_workspace_forward_matches_sp_forward_on_two_calls_in_a_row():
    """Two calls in a row on the static workspace, the second with a smaller input (so the array still holds the
    first call's rows beyond the second call's), each against sp_forward on a workspace of its own: the same kernels
    are enqueued, so the logits must agree bit for bit (which is within the bf16 bound of 3e-2 relative a fortiori)."""
    from paper_2408_12526_amd import sp
    w = synth.WORKLOADS[3]                                     # the batch-1 latency group: K = 8, hidden 768
    shape = synth.small_variant(w, vocab=2000).shape
    rng = np.random.default_rng(51)
    st = sp.Students(sp.config_from_shape(shape), synth.make_weights(rng, shape))
    calls = [((70, 33, 128, 25), 8), ((64,), 5)]               # 256 tokens in 4 sequences, then 64 tokens in 1
    for lengths, k in calls:
        d_ids, d_cu, mx = _inputs(sp, rng, lengths, shape.vocab)
        want = st.sp_forward(d_ids, d_cu, mx, k).clone()
        got = torch.full((len(lengths), shape.classes), float("nan"), dtype=torch.float32, device="cuda")
        st.sp_forward_static(d_ids, d_cu, mx, k, got)
        torch.cuda.synchronize()
        assert torch.isfinite(got).all()
        err = (got - want).abs().max().item() / max(want.abs().max().item(), 1e-3)
        assert err <= 3e-2, f"lengths {lengths}, k_active {k}: relative error {err:.3e}"
        assert torch.equal(got, want), f"lengths {lengths}, k_active {k}: not bit-identical"
    # the first input once more: the array now holds the smaller call's contents
    lengths, k = calls[0]
    rng = np.random.default_rng(52)
    d_ids, d_cu, mx = _inputs(sp, rng, lengths, shape.vocab)
    want = st.sp_forward(d_ids, d_cu, mx, k).clone()
    got = torch.empty_like(want)
    st.sp_forward_static(d_ids, d_cu, mx, k, got)
    assert torch.equal(got, want)
    st.close()


def test_static_workspace_refuses_what_does_not_fit():
    from paper_2408_12526_amd import sp
    w = synth.WORKLOADS[3]
    shape = synth.small_variant(w, vocab=2000).shape
    rng = np.random.default_rng(53)
    cfg = sp.config_from_shape(shape)
    st = sp.Students(cfg, synth.make_weights(rng, shape))
    assert sp.sp_static_scratch_bytes() == 64 << 20
    assert sp.sp_workspace_bytes(cfg, 256, 4) <= sp.sp_static_scratch_bytes() < sp.sp_workspace_bytes(cfg, 257, 4)
    d_ids, d_cu, mx = _inputs(sp, rng, (200, 57), shape.vocab)          # 257 tokens
    out = torch.zeros(2, shape.classes, dtype=torch.float32, device="cuda")
    with pytest.raises(sp.SpError) as e:
        st.sp_forward_static(d_ids, d_cu, mx, 8, out)
    assert e.value.code == -8
    torch.cuda.synchronize()
    assert (out == 0).all()                                              # nothing was enqueued
    with pytest.raises(sp.SpError) as e:                                 # sp_forward's own checks still apply
        st.sp_forward_static(d_ids[:64], d_cu[:2].clone().fill_(0), 64, 9, out[:1])
    assert e.value.code == -3
    st.close()
