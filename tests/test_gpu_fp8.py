"""Quantised students (SP_DTYPE_FP8): the fp8 projections against the oracle.  Needs an MI355X.

The oracle stays fp64 and consumes the de-quantised weights: every tensor rounded to bf16 as in the bf16 mode, except
the query/key/value, attention-output, FFN-up and FFN-down matrices of the layers that run on fp8 operands, which are quantised per
output feature to e4m3 by the library conversion (torch.float8_e4m3fn) and multiplied back by their scales.  Activation
quantisation is the HIP path's own rounding, like the bf16 rounding of activations in the bf16 mode.

Tolerances (derived in the design doc): a projection checked on the HIP path's own quantised input carries only the bf16
rounding of its output (1.2e-2 of the tensor's largest magnitude, as in the bf16 stage tests); an fp8 activation is
within 2^-4 relative of the value it encodes (3 mantissa bits, round to nearest); whole-forward logits within 1e-1 of
the largest logit (each fp8 operand pair adds about 4 % of independent noise per projection output, most of which the
residual connections and LayerNorms dilute).
"""
import numpy as np
import pytest
import torch

from oracle.sp_oracle import OracleConfig
from paper_2408_12526_amd import synth

pytestmark = pytest.mark.gpu

FP8_LOGITS_REL = 1e-1
QUANT = ("Wq", "Wk", "Wv", "Wo", "W1", "W2")


def ocfg(s):
    return OracleConfig(s.K, s.layers, s.hidden, s.heads, s.ffn, s.vocab, s.max_pos, s.classes, s.ln_eps)


def rel_err(got, ref):
    return np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-3)


def dequantised_weights(blob, shape, fp8_layers):
    """bf16-rounded blob, with the four projection families of `fp8_layers` per-output-feature e4m3 instead."""
    out = torch.from_numpy(blob).to(torch.bfloat16).to(torch.float32).numpy()
    for m in range(shape.K):
        src, dst = synth.student_views(blob, shape, m), synth.student_views(out, shape, m)
        for l in fp8_layers:
            for name in QUANT:
                w = torch.from_numpy(src[f"l{l}.{name}"])                      # [in][out]
                amax = w.abs().amax(dim=0)
                scale = torch.where(amax > 0, amax / 448.0, torch.ones_like(amax))
                dst[f"l{l}.{name}"][...] = ((w / scale).to(torch.float8_e4m3fn).float() * scale).numpy()
    return out


@pytest.fixture(scope="module")
def sp():
    from paper_2408_12526_amd import sp as binding
    return binding


def make_case(sp, seed, nseq, shape):
    rng = np.random.default_rng(seed)
    lengths = rng.integers(20, 101, size=nseq).astype(np.int32)
    lengths[:3] = (200, 1, 129)
    assert lengths.sum() >= 2048
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.05, ln_random=True, qk_std=0.1)
    cu = sp.sp_pack(lengths)
    return lengths, ids, blob, cu


SHAPE = synth.StudentShape(K=2, layers=2, hidden=256, heads=4, ffn=512, vocab=300, max_pos=320, classes=3, dtype="fp8")


def test_fp8_projections_stage_by_stage(sp, oracle64):
    """Each fp8 projection in isolation, on the HIP path's own quantised input as it left it in the workspace, and
    each quantised activation against the bf16 tensor it was rounded from."""
    shape = SHAPE
    lengths, ids, blob, cu = make_case(sp, 61, 40, shape)
    T, B, k, H = int(cu[-1]), len(lengths), shape.K, shape.hidden
    st = sp.Students(sp.config_from_shape(shape, last_layer_all_tokens=True), blob)
    d_ids, d_cu = torch.from_numpy(ids).cuda(), torch.from_numpy(cu).cuda()
    mx = int(lengths.max())
    ow = dequantised_weights(blob, shape, range(shape.layers))
    tol = 1.2e-2

    def ln_rows(u, g, b):
        return np.stack([oracle64.layernorm(r, g, b, shape.ln_eps) for r in u])

    def check_quantised(q, ref, what):
        # 3 mantissa bits, round to nearest: 2^-4 relative (+ the bf16 rounding of the reference copy), and the
        # subnormal step 2^-9 / 16 below 2^-6 / 16
        bound = (2.0 ** -4 + 2.0 ** -8) * np.abs(ref) + 2.0 ** -14
        worst = (np.abs(q - ref) - bound).max()
        assert worst <= 0, f"{what}: exceeds the e4m3 rounding bound by {worst:.3e}"
        assert np.abs(q).max() > 0.5 * np.abs(ref).max()

    for layer in range(shape.layers):
        ws = st.sp_forward_partial(d_ids, d_cu, mx, k, layer + 1)
        got = {n: st.read_activation(ws, n, T, B, k) for n in ("qkv", "att", "x1", "x", "x1q", "gq", "xq", "attq")}
        if layer == 0:
            ws0 = st.sp_forward_partial(d_ids, d_cu, mx, k, 0)
            x_in, xq_in = st.read_activation(ws0, "x", T, B, k), st.read_activation(ws0, "xq", T, B, k)
            st.sp_forward_partial(d_ids, d_cu, mx, k, layer + 1)
        for m in range(k):
            v = synth.student_views(ow, shape, m)
            p = f"l{layer}."
            check_quantised(xq_in[m], x_in[m], f"layer {layer} student {m}: fp8 copy of the layer input")
            Wqkv = np.concatenate([v[p + "Wq"], v[p + "Wk"], v[p + "Wv"]], axis=1)
            bqkv = np.concatenate([v[p + "bq"], v[p + "bk"], v[p + "bv"]])
            e = rel_err(got["qkv"][m], oracle64.linear(xq_in[m], Wqkv, bqkv))
            assert e < tol, f"layer {layer} student {m}: fp8 q|k|v projection, rel err {e:.3e}"
            check_quantised(got["attq"][m], got["att"][m], f"layer {layer} student {m}: fp8 copy of the attention output")
            want_x1 = ln_rows(x_in[m] + oracle64.linear(got["attq"][m], v[p + "Wo"], v[p + "bo"]), v[p + "ln1_g"],
                              v[p + "ln1_b"])
            e = rel_err(got["x1"][m], want_x1)
            assert e < tol, f"layer {layer} student {m}: fp8 attention output projection + residual + LayerNorm, rel err {e:.3e}"
            check_quantised(got["x1q"][m], got["x1"][m], f"layer {layer} student {m}: fp8 copy of x1")
            want_g = torch.nn.functional.gelu(torch.from_numpy(oracle64.linear(got["x1q"][m], v[p + "W1"], v[p + "b1"]))).numpy()
            bound = 2.0 ** -4 * np.abs(want_g) + 2e-3 * np.abs(want_g).max()
            worst = (np.abs(got["gq"][m] - want_g) - bound).max()
            assert worst <= 0, f"layer {layer} student {m}: fp8 GELU(FFN up), beyond the bound by {worst:.3e}"
            want_x = ln_rows(got["x1"][m] + oracle64.linear(got["gq"][m], v[p + "W2"], v[p + "b2"]), v[p + "ln2_g"],
                             v[p + "ln2_b"])
            e = rel_err(got["x"][m], want_x)
            assert e < tol, f"layer {layer} student {m}: fp8 FFN down + residual + LayerNorm, rel err {e:.3e}"
        x_in, xq_in = got["x"], got["xq"]
    st.close()


def test_gelu_of_the_fp8_epilogue_is_the_erf_form_to_a_thirtieth_of_a_code_step(sp):
    """The fp8 FFN up-projection stores GELU as e4m3 codes and evaluates it through a shorter fit than the bf16 path.
    Before scaling and rounding it must stay within 1e-4 of x (1 + erf(x / sqrt 2)) / 2 everywhere, huge arguments
    included (the fit has no clamp: its exponent keeps falling); the e4m3 step at the function's minimum, -0.17, is
    2^-3 * 2^-3 = 1.6e-2 wide there, so the fit moves no code by more than a hundredth of a step."""
    import math
    grid = np.concatenate([np.linspace(-12, 12, 1_000_001), np.linspace(-1e-3, 1e-3, 2_001),
                           [0.0, -0.0, 1.0, -1.0, 30.0, -30.0, 1e4, -1e4, 1e20, -1e20, 3e38, -3e38]]).astype(np.float32)
    got = sp.sp_probe_gelu_fp8(torch.from_numpy(grid).cuda()).cpu().numpy().astype(np.float64)
    x = grid.astype(np.float64)
    want = 0.5 * x * (1.0 + np.vectorize(math.erf)(x / math.sqrt(2.0)))
    assert np.isfinite(got).all()
    err = np.abs(got - want)
    rel_big = err[np.abs(x) > 12] / np.maximum(np.abs(want[np.abs(x) > 12]), 1.0)
    assert err[np.abs(x) <= 12].max() <= 1e-4, f"max error {err[np.abs(x) <= 12].max():.3e} at x = {x[err.argmax()]}"
    assert rel_big.max() <= 1e-6
    assert got[np.flatnonzero(grid == 0.0)].max() == 0.0


@pytest.mark.parametrize("all_tokens", [True, False])
def test_fp8_forward_against_oracle_with_dequantised_weights(sp, oracle64, all_tokens):
    """Whole forward of quantised students, both last-layer variants (with the first-token last layer only the first
    layer's projections are fp8), every sequence, each k_active, against the fp64 oracle on the de-quantised weights;
    and the bf16 mode of the same students stays within the same bound of the fp8 mode's oracle (sanity: the
    quantisation changes the logits by a few per cent, not more)."""
    shape = SHAPE
    lengths, ids, blob, cu = make_case(sp, 62, 45, shape)
    st = sp.Students(sp.config_from_shape(shape, last_layer_all_tokens=all_tokens), blob)
    d_ids, d_cu = torch.from_numpy(ids).cuda(), torch.from_numpy(cu).cuda()
    fp8_layers = range(shape.layers) if all_tokens else range(shape.layers - 1)
    ow = dequantised_weights(blob, shape, fp8_layers)
    for k in (1, 2):
        got = st.sp_forward(d_ids, d_cu, int(lengths.max()), k).cpu().numpy().astype(np.float64)
        want = oracle64.forward(ocfg(shape), ow, ids, cu, k)
        assert np.isfinite(got).all() and np.abs(want).max() > 5e-2
        e = rel_err(got, want)
        print(f"fp8 all_tokens={all_tokens} k_active={k}: rel err {e:.3e}", flush=True)
        assert e <= FP8_LOGITS_REL, f"all_tokens={all_tokens} k_active={k}: rel err {e:.3e}"
    st.close()


def test_fp8_mode_keeps_small_calls_on_the_bf16_path(sp, oracle64):
    """Calls below 2048 token rows of quantised students run entirely in bf16 (the arena keeps both copies): they
    must meet the bf16 bound against the bf16 oracle weights."""
    shape = SHAPE
    rng = np.random.default_rng(63)
    lengths = np.array([64, 17, 100, 1, 33], dtype=np.int32)
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.05, ln_random=True, qk_std=0.1)
    cu = sp.sp_pack(lengths)
    st = sp.Students(sp.config_from_shape(shape), blob)
    got = st.sp_forward(torch.from_numpy(ids).cuda(), torch.from_numpy(cu).cuda(), int(lengths.max()), shape.K)
    want = oracle64.forward(ocfg(shape), dequantised_weights(blob, shape, ()), ids, cu, shape.K)
    assert rel_err(got.cpu().numpy().astype(np.float64), want) <= 3e-2
    st.close()


def test_fp8_mode_keeps_other_widths_on_the_bf16_path(sp, oracle64):
    """The fp8 kernel's one tile is 256 x 256: quantised students whose widths are not multiples of 256 (hidden 384
    here) run large calls in bf16 as well and must meet the bf16 bound against the bf16 oracle weights."""
    shape = synth.StudentShape(K=2, layers=2, hidden=384, heads=6, ffn=640, vocab=300, max_pos=320, classes=3, dtype="fp8")
    lengths, ids, blob, cu = make_case(sp, 64, 40, shape)
    st = sp.Students(sp.config_from_shape(shape), blob)
    got = st.sp_forward(torch.from_numpy(ids).cuda(), torch.from_numpy(cu).cuda(), int(lengths.max()), shape.K)
    want = oracle64.forward(ocfg(shape), dequantised_weights(blob, shape, ()), ids, cu, shape.K)
    assert rel_err(got.cpu().numpy().astype(np.float64), want) <= 3e-2
    st.close()


def test_fp8_burst_workload_part(sp, oracle64):
    """The burst workload with quantised students (hidden 768, 58 token tiles, reduction depths 768 and 3072): one
    third of the sequences against the oracle at k_active 8 and 2."""
    w = synth.WORKLOADS[4]
    shape = synth.StudentShape(**{**w.shape.__dict__, "dtype": "fp8"})
    batch, blob = synth.make_workload(w)
    cu = sp.sp_pack(batch.lengths)
    st = sp.Students(sp.config_from_shape(shape), blob)
    d_ids, d_cu = torch.from_numpy(batch.ids).cuda(), torch.from_numpy(cu).cuda()
    ow = dequantised_weights(blob, shape, range(shape.layers - 1))     # first-token last layer: bf16
    lo, hi = 171, 256
    sub_cu = (cu[lo:hi + 1] - cu[lo]).astype(np.int32)
    _, terms = oracle64.forward(ocfg(shape), ow, batch.ids[cu[lo]:cu[hi]], sub_cu, shape.K, want_terms=True)
    for k in (8, 2):
        got = st.sp_forward(d_ids, d_cu, int(batch.lengths.max()), k).cpu().numpy().astype(np.float64)
        want = terms[:k].sum(0)
        e = rel_err(got[lo:hi], want)
        print(f"fp8 burst k_active={k}: rel err {e:.3e}", flush=True)
        assert e <= FP8_LOGITS_REL
    st.close()


def test_fp8_call_whose_buffers_pass_four_gib(sp, oracle64):
    """Quantised students on a call of about 177 thousand tokens (the burst batch's lengths twelve times over, fresh
    ids): the one-byte FFN activations (4.3 GB) as well as the bf16 q|k|v buffer lie beyond what 32-bit offsets
    reach.  First, middle and last sequences against the oracle (computed as a batch of their own), the whole call
    finite and repeatable bit for bit."""
    w = synth.WORKLOADS[4]
    shape = synth.StudentShape(**{**w.shape.__dict__, "dtype": "fp8"})
    batch, blob = synth.make_workload(w)
    rng = np.random.default_rng(4097)
    lengths = np.tile(batch.lengths, 12).astype(np.int32)
    B, T = len(lengths), int(lengths.sum())
    assert T * shape.ffn * shape.K > 4 * 2**30
    ids = synth.make_ids(rng, T, shape.vocab)
    cu = sp.sp_pack(lengths)
    st = sp.Students(sp.config_from_shape(shape), blob)
    d_ids, d_cu = torch.from_numpy(ids).cuda(), torch.from_numpy(cu).cuda()
    ow = dequantised_weights(blob, shape, range(shape.layers - 1))
    picks = [0, 1, B // 2, B // 2 + 1, B - 2, B - 1]
    sub_ids = np.concatenate([ids[cu[b]:cu[b + 1]] for b in picks])
    sub_cu = np.concatenate([[0], np.cumsum(lengths[picks])]).astype(np.int32)
    _, terms = oracle64.forward(ocfg(shape), ow, sub_ids, sub_cu, shape.K, want_terms=True)
    for k in (8, 3):
        got = st.sp_forward(d_ids, d_cu, int(lengths.max()), k).cpu().numpy().astype(np.float64)
        assert got.shape == (B, shape.classes) and np.isfinite(got).all()
        e = rel_err(got[picks], terms[:k].sum(0))
        print(f"fp8 {T} tokens k_active={k}: rel err {e:.3e}", flush=True)
        assert e <= FP8_LOGITS_REL
        again = st.sp_forward(d_ids, d_cu, int(lengths.max()), k).cpu().numpy().astype(np.float64)
        assert np.array_equal(got, again)
    st.close()


def test_fp8_large_width(sp, oracle64):
    """Quantised students at the large width (hidden 1024, 16 heads, FFN 4096: reduction depths 1024 and 4096, four and
    sixteen 256-wide feature tiles), sequences of up to 300 tokens, every sequence against the oracle."""
    shape = synth.StudentShape(K=2, layers=2, hidden=1024, heads=16, ffn=4096, vocab=500, max_pos=320, classes=2,
                               dtype="fp8")
    rng = np.random.default_rng(64)
    lengths = rng.integers(30, 301, size=14).astype(np.int32)
    assert 2048 <= lengths.sum()
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.02, ln_random=True, qk_std=float(np.sqrt(1.5 / shape.hidden)))
    cu = sp.sp_pack(lengths)
    st = sp.Students(sp.config_from_shape(shape), blob)
    got = st.sp_forward(torch.from_numpy(ids).cuda(), torch.from_numpy(cu).cuda(), int(lengths.max()), shape.K)
    want = oracle64.forward(ocfg(shape), dequantised_weights(blob, shape, range(shape.layers - 1)), ids, cu, shape.K)
    e = rel_err(got.cpu().numpy().astype(np.float64), want)
    print(f"fp8 hidden 1024: rel err {e:.3e}", flush=True)
    assert e <= FP8_LOGITS_REL
    st.close()
