"""Parity of the HIP path (through the C ABI) against the CPU oracle.  Needs an MI355X."""
import numpy as np
import pytest
import torch

from oracle.sp_oracle import OracleConfig
from paper_2408_12526_amd import synth

pytestmark = pytest.mark.gpu

FP32_MAX_ABS = 1e-3        # fp32 path: max |gpu - oracle| over all logits
BF16_REL = 3e-2            # bf16 path: max |gpu - oracle| / max(max |oracle|, 1e-3)


def ocfg(s):
    return OracleConfig(s.K, s.layers, s.hidden, s.heads, s.ffn, s.vocab, s.max_pos, s.classes, s.ln_eps)


def oracle_weights(blob, shape):
    """What the oracle consumes: in bf16 mode the weights rounded to bf16 once (library conversion), upcast."""
    if shape.dtype == "bf16":
        return torch.from_numpy(blob).to(torch.bfloat16).to(torch.float32).numpy()
    return blob


def rel_err(got, ref):
    return np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-3)


def check_logits(got, ref, shape, what=""):
    assert np.isfinite(got).all(), what
    if shape.dtype == "fp32":
        err = np.abs(got - ref).max()
        assert err <= FP32_MAX_ABS, f"{what}: max abs err {err:.3e}"
    else:
        err = rel_err(got, ref)
        assert err <= BF16_REL, f"{what}: rel err {err:.3e}"
    return err


@pytest.fixture(scope="module")
def sp():
    from paper_2408_12526_amd import sp as binding
    return binding


def gpu_inputs(lengths, ids, sp):
    cu = sp.sp_pack(lengths)
    return (torch.from_numpy(ids).cuda(), torch.from_numpy(cu).cuda(), cu)


# ---- kernel-by-kernel on small shapes ---------------------------------------------------------

STAGE_SHAPES = {
    "fp32": synth.StudentShape(K=2, layers=2, hidden=128, heads=2, ffn=256, vocab=100, max_pos=320, classes=3,
                               dtype="fp32"),
    "bf16": synth.StudentShape(K=3, layers=2, hidden=128, heads=2, ffn=256, vocab=100, max_pos=320, classes=3,
                               dtype="bf16"),
}
STAGE_LENGTHS = (5, 1, 96, 33, 64, 200, 70, 129)   # spans several key tiles, query blocks and a ragged tail
SINGLE_TILE_LENGTHS = (7, 1, 30, 19)                # 57 tokens: the single-tile (latency) code path of the bf16 mode


@pytest.mark.parametrize("dtype,lens", [("fp32", STAGE_LENGTHS), ("bf16", STAGE_LENGTHS),
                                        ("bf16", SINGLE_TILE_LENGTHS), ("bf16", (64,)),
                                        ("bf16", (300, 5, 140, 64, 257)),   # > 256 tokens: the key/value-sharing kernel
                                        ("bf16", (320, 193, 129, 161))])    # its partly filled waves and query blocks
def test_every_stage_against_oracle_pieces(sp, oracle64, dtype, lens):
    """Each kernel in isolation: its output against the oracle's piece applied to the kernel's own input
    (as the HIP path left it in the workspace), so that one kernel's rounding is not charged to the next."""
    shape = STAGE_SHAPES[dtype]
    rng = np.random.default_rng(21)
    lengths = np.array(lens, dtype=np.int32)
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.08, ln_random=True, qk_std=0.25)
    ow = oracle_weights(blob, shape)
    st = sp.Students(sp.config_from_shape(shape), blob)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    T, B, k, H = int(cu[-1]), len(lengths), shape.K, shape.hidden
    mx = int(lengths.max())
    # relative to the tensor's largest magnitude: fp32 reorders sums only; bf16 rounds each output once (2^-9)
    # and, in attention, the probabilities as well
    tol = 2e-5 if dtype == "fp32" else 1.2e-2

    def per_seq(fn, *tensors):
        return np.concatenate([fn(*[t[cu[b]:cu[b + 1]] for t in tensors]) for b in range(B)], axis=0)

    def ln_rows(u, g, b):
        return np.stack([oracle64.layernorm(r, g, b, shape.ln_eps) for r in u])

    def gelu(u):
        return torch.nn.functional.gelu(torch.from_numpy(u)).numpy()

    ws = st.sp_forward_partial(d_ids, d_cu, mx, k, 0)
    x_in = st.read_activation(ws, "x", T, B, k)
    for m in range(k):
        x0 = np.concatenate([oracle64.taps(ocfg(shape), ow, ids, cu, m, b)["x0"] for b in range(B)], axis=0)
        assert rel_err(x_in[m], x0) < tol, f"embedding + LayerNorm, student {m}"
    for layer in range(shape.layers):
        ws = st.sp_forward_partial(d_ids, d_cu, mx, k, layer + 1)
        got = {n: st.read_activation(ws, n, T, B, k) for n in ("qkv", "att", "x1", "g", "x")}
        for m in range(k):
            v = synth.student_views(ow, shape, m)
            p = f"l{layer}."
            Wqkv = np.concatenate([v[p + "Wq"], v[p + "Wk"], v[p + "Wv"]], axis=1)
            bqkv = np.concatenate([v[p + "bq"], v[p + "bk"], v[p + "bv"]])
            want = {
                "qkv": oracle64.linear(x_in[m], Wqkv, bqkv),
                "att": per_seq(lambda a: oracle64.attention(a[:, :H], a[:, H:2 * H], a[:, 2 * H:], shape.heads),
                               got["qkv"][m]),
                "x1": ln_rows(x_in[m] + oracle64.linear(got["att"][m], v[p + "Wo"], v[p + "bo"]), v[p + "ln1_g"],
                              v[p + "ln1_b"]),
                "g": gelu(oracle64.linear(got["x1"][m], v[p + "W1"], v[p + "b1"])),
                "x": ln_rows(got["x1"][m] + oracle64.linear(got["g"][m], v[p + "W2"], v[p + "b2"]), v[p + "ln2_g"],
                             v[p + "ln2_b"]),
            }
            for name in ("qkv", "att", "x1", "g", "x"):
                e = rel_err(got[name][m], want[name])
                assert e < tol, f"layer {layer} student {m} stage {name}: rel err {e:.3e}"
        x_in = got["x"]
    # head in isolation: pooled first-token state through the oracle's linear pieces.  (A whole forward with the last
    # layer on every token: that is the one whose head consumes the rows the partial forward above left in `x`; with the
    # default setting a call of a few sequences recomputes the first-token rows of the last layer another way.)
    st.close()
    st = sp.Students(sp.config_from_shape(shape, last_layer_all_tokens=True), blob)
    logits = st.sp_forward(d_ids, d_cu, mx, k).cpu().numpy().astype(np.float64)
    z = st.read_activation(st.workspace(T, B), "z", T, B, k)
    for m in range(k):
        v = synth.student_views(ow, shape, m)
        pooled = np.tanh(oracle64.linear(x_in[m][cu[:-1]], v["Wp"], v["bp"]))
        assert rel_err(z[m], oracle64.linear(pooled, v["Wc"], v["bc"])) < (2e-5 if dtype == "fp32" else 2e-3)
    np.testing.assert_allclose(logits, z.sum(0), atol=1e-5)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_small_shape_end_to_end(sp, oracle64, dtype):
    """Whole forward on the small shape with non-trivial LayerNorm parameters and sharpened attention."""
    shape = STAGE_SHAPES[dtype]
    rng = np.random.default_rng(22)
    lengths = np.array(STAGE_LENGTHS, dtype=np.int32)
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.05, ln_random=True, qk_std=0.12)
    st = sp.Students(sp.config_from_shape(shape), blob)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    for k in range(1, shape.K + 1):
        got = st.sp_forward(d_ids, d_cu, int(lengths.max()), k).cpu().numpy().astype(np.float64)
        want = oracle64.forward(ocfg(shape), oracle_weights(blob, shape), ids, cu, k)
        assert np.abs(want).max() > 5e-2
        check_logits(got, want, shape, f"small shape {dtype} k_active={k}")


def test_first_token_last_layer_matches_all_tokens(sp, oracle64):
    """Calls with >= 1024 tokens run the last layer on the first-token rows only; a stock all-token last layer must
    give the same logits (up to attention's rounding order), and both must match the oracle."""
    # four heads: the first-token path needs a head count that is a multiple of four (the small stage shape has two
    # and would silently take the all-token path for both settings)
    shape = synth.StudentShape(K=3, layers=2, hidden=256, heads=4, ffn=512, vocab=100, max_pos=320, classes=3,
                               dtype="bf16")
    rng = np.random.default_rng(23)
    lengths = rng.integers(1, 130, size=37).astype(np.int32)
    lengths[:3] = (200, 1, 129)
    assert lengths.sum() >= 1024 and shape.heads % 4 == 0 and lengths.max() <= 512
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.05, ln_random=True, qk_std=0.12)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    want = oracle64.forward(ocfg(shape), oracle_weights(blob, shape), ids, cu, shape.K)
    got = {}
    for all_tokens in (False, True):
        st = sp.Students(sp.config_from_shape(shape, last_layer_all_tokens=all_tokens), blob)
        got[all_tokens] = st.sp_forward(d_ids, d_cu, int(lengths.max()), shape.K).cpu().numpy().astype(np.float64)
        check_logits(got[all_tokens], want, shape, f"all_tokens={all_tokens}")
    assert rel_err(got[False], got[True]) < 1e-2


def test_sequences_longer_than_512_tokens(sp, oracle64):
    """Sequences beyond 512 tokens: three and four 256-query workgroups per (sequence, head) in the key/value-sharing
    attention body, a dozen key tiles per query block; up to 32 tiles of tokens under the running softmax of the folded
    first-token attention in the last layer.  Whole forward against the oracle, every sequence, each k_active, with the
    last layer on the first tokens and on every token; and the attention stage by itself."""
    shape = synth.StudentShape(K=2, layers=2, hidden=256, heads=4, ffn=512, vocab=200, max_pos=1024, classes=3,
                               dtype="bf16")
    rng = np.random.default_rng(29)
    lengths = np.array([700, 513, 40, 1, 1000, 257], dtype=np.int32)
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.05, ln_random=True, qk_std=0.12)
    st = sp.Students(sp.config_from_shape(shape), blob)
    st_all = sp.Students(sp.config_from_shape(shape, last_layer_all_tokens=True), blob)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    ow = oracle_weights(blob, shape)
    for k in (1, 2):
        want = oracle64.forward(ocfg(shape), ow, ids, cu, k)
        for name, students in (("first tokens", st), ("every token", st_all)):
            got = students.sp_forward(d_ids, d_cu, int(lengths.max()), k).cpu().numpy().astype(np.float64)
            check_logits(got, want, shape, f"long sequences, last layer on {name}, k_active={k}")
    st_all.close()
    T, B = int(cu[-1]), len(lengths)
    ws = st.sp_forward_partial(d_ids, d_cu, int(lengths.max()), shape.K, 1)
    qkv, att = st.read_activation(ws, "qkv", T, B, shape.K), st.read_activation(ws, "att", T, B, shape.K)
    for m in range(shape.K):
        for b in range(B):
            rows = slice(int(cu[b]), int(cu[b + 1]))
            a = qkv[m][rows]
            H = shape.hidden
            e = rel_err(att[m][rows], oracle64.attention(a[:, :H], a[:, H:2 * H], a[:, 2 * H:], shape.heads))
            assert e < 1.2e-2, f"student {m}, sequence of {lengths[b]} tokens: attention rel err {e:.3e}"
    st.close()


def test_folded_first_token_attention_against_the_definition(sp, oracle64):
    """The first-token last layer never forms keys and values (the query is folded through the key projection, the
    value projection is applied to the weighted mean of the token rows).  Its attention output is checked against the
    definition: keys and values projected by the oracle from the layer's own input rows as the HIP path left them,
    softmax attention of the HIP path's own first-token queries over them."""
    shape = synth.StudentShape(K=2, layers=2, hidden=256, heads=4, ffn=512, vocab=100, max_pos=320, classes=3,
                               dtype="bf16")
    rng = np.random.default_rng(27)
    lengths = rng.integers(1, 130, size=30).astype(np.int32)
    lengths[:4] = (300, 1, 129, 64)
    assert lengths.sum() >= 1024
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    # score spread about 4 (query/key weights at 0.12): sharp enough that a wrong scale, mask or fold shows; the
    # rounding of the folded query moves a score by about 2^-9 of its size, like the rounding of a key would
    blob = synth.make_weights(rng, shape, std=0.08, ln_random=True, qk_std=0.12)
    ow = oracle_weights(blob, shape)
    st = sp.Students(sp.config_from_shape(shape), blob)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    T, B, k, H = int(cu[-1]), len(lengths), shape.K, shape.hidden
    ws = st.workspace(T, B)
    st.sp_forward(d_ids, d_cu, int(lengths.max()), k, workspace=ws)
    torch.cuda.synchronize()
    x = st.read_activation(ws, "x", T, B, k)               # input of the last layer
    q = st.read_activation(ws, "first_q", T, B, k)
    got = st.read_activation(ws, "first_att", T, B, k)
    p = f"l{shape.layers - 1}."
    for m in range(k):
        v = synth.student_views(ow, shape, m)
        qref = oracle64.linear(x[m][cu[:-1]], v[p + "Wq"], v[p + "bq"])
        assert rel_err(q[m], qref) < 1.2e-2, f"student {m}: first-token queries"
        want = np.empty((B, H))
        for b in range(B):
            xs = x[m][cu[b]:cu[b + 1]]
            keys, vals = oracle64.linear(xs, v[p + "Wk"], v[p + "bk"]), oracle64.linear(xs, v[p + "Wv"], v[p + "bv"])
            qs = np.repeat(q[m][b][None, :], len(xs), axis=0)      # rows are independent: row 0 is the first token's
            want[b] = oracle64.attention(qs, keys, vals, shape.heads)[0]
        e = rel_err(got[m], want)
        assert e < 1.2e-2, f"student {m}: folded first-token attention, rel err {e:.3e}"


FIRST_EDGE_CASES = {
    # the longest sequence the one-query attention kernel takes, the shortest possible ones, a ragged mix
    "len512_and_len1": [512, 1, 1, 2, 257, 33, 128, 129, 64, 7],
    # every sequence is a single token (its own first token): 1100 sequences, not a multiple of any tile
    "all_single_tokens": [1] * 1100,
    # a sequence longer than that kernel's limit: the call must take the all-token last layer and still be right
    "len600_falls_back": [600, 5, 300, 150, 31],
}


@pytest.mark.parametrize("case", list(FIRST_EDGE_CASES))
def test_first_token_edge_cases(sp, oracle64, case):
    """Calls of >= 1024 tokens at the edges of the first-token last layer: longest / shortest sequences, a batch of
    single tokens, and a sequence beyond its length limit (fallback to the all-token layer)."""
    shape = synth.StudentShape(K=2, layers=2, hidden=256, heads=4, ffn=512, vocab=100, max_pos=640, classes=3,
                               dtype="bf16")
    rng = np.random.default_rng(29)
    lengths = np.array(FIRST_EDGE_CASES[case], dtype=np.int32)
    assert lengths.sum() >= 1024
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.05, ln_random=True, qk_std=0.1)
    st = sp.Students(sp.config_from_shape(shape), blob)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    got = st.sp_forward(d_ids, d_cu, int(lengths.max()), shape.K).cpu().numpy().astype(np.float64)
    want = oracle64.forward(ocfg(shape), oracle_weights(blob, shape), ids, cu, shape.K)
    check_logits(got, want, shape, case)


# ---- the other student shapes the paper uses (Table 2: 2L256D, its headline student; 6L768D; 12L1024D) -------------

OTHER_SHAPES = {
    # name: (shape, number of sequences, length range); batches sized so that the fp64 oracle takes seconds
    "2L256D": (synth.StudentShape(K=4, layers=2, hidden=256, heads=4, ffn=1024, vocab=1000, max_pos=128, classes=2,
                                  dtype="bf16"), 28, (8, 100)),       # >= 1024 tokens: first-token last layer, 4 heads
    "6L768D": (synth.StudentShape(K=1, layers=6, hidden=768, heads=12, ffn=3072, vocab=500, max_pos=128, classes=2,
                                  dtype="bf16"), 7, (8, 80)),
    "12L1024D": (synth.StudentShape(K=1, layers=12, hidden=1024, heads=16, ffn=4096, vocab=500, max_pos=128, classes=3,
                                    dtype="bf16"), 4, (8, 48)),
}


@pytest.mark.parametrize("name", list(OTHER_SHAPES))
def test_other_student_shapes(sp, oracle64, name):
    """The kernels are shape-generic (hidden 256 / 768 / 1024 with 64-wide heads) and the layer count is a loop
    bound only: whole forward against the oracle, weights N(0, 0.02) as in the workloads.  The query/key weights are
    spread so that the attention scores have a standard deviation of about 1.5 at every width (far from uniform, so a
    wrong scale or mask shows, but not the near-argmax regime in which twelve layers amplify any rounding chaotically)."""
    shape, nseq, (lo, hi) = OTHER_SHAPES[name]
    rng = np.random.default_rng(31)
    lengths = rng.integers(lo, hi + 1, size=nseq).astype(np.int32)
    if name == "2L256D":
        lengths[:2] = (100, 100)
        assert lengths.sum() >= 1024
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.02, ln_random=True, qk_std=float(np.sqrt(1.5 / shape.hidden)))
    st = sp.Students(sp.config_from_shape(shape), blob)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    got = st.sp_forward(d_ids, d_cu, int(lengths.max()), shape.K).cpu().numpy().astype(np.float64)
    want = oracle64.forward(ocfg(shape), oracle_weights(blob, shape), ids, cu, shape.K)
    check_logits(got, want, shape, name)


LARGE_OTHER = {
    # reduction depths 256 / 1024 and 512 / 1280: with the depths 768 / 3072 of the workloads, the last k-tile of the
    # large-tile projection kernel ends in every position of its five-slot operand ring
    "256D_ffn1024": synth.StudentShape(K=2, layers=2, hidden=256, heads=4, ffn=1024, vocab=1000, max_pos=128,
                                       classes=2, dtype="bf16"),
    "512D_ffn1280": synth.StudentShape(K=2, layers=2, hidden=512, heads=8, ffn=1280, vocab=1000, max_pos=128,
                                       classes=3, dtype="bf16"),
    # reduction depth 128 (two k-tiles): such projections go to the 128 x 128 tile even in large calls; the shortest
    # reduction the large tile meets is depth 256 (four k-tiles: the 256-wide student above)
    "128D_ffn256": synth.StudentShape(K=3, layers=2, hidden=128, heads=2, ffn=256, vocab=1000, max_pos=128,
                                      classes=2, dtype="bf16"),
}


@pytest.mark.parametrize("name", list(LARGE_OTHER))
def test_large_calls_on_other_widths(sp, oracle64, name):
    """Calls of more than 2048 tokens (the 256 x 256 projection tiles, the long-call LayerNorm and embedding paths) on
    widths other than the workloads'.  The oracle checks a sample of the sequences (sequences are independent)."""
    shape = LARGE_OTHER[name]
    rng = np.random.default_rng(37)
    lengths = rng.integers(24, 97, size=40).astype(np.int32)
    assert 2048 < lengths.sum()
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.02, ln_random=True, qk_std=float(np.sqrt(1.5 / shape.hidden)))
    st = sp.Students(sp.config_from_shape(shape), blob)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    got = st.sp_forward(d_ids, d_cu, int(lengths.max()), shape.K).cpu().numpy().astype(np.float64)
    pick = np.sort(rng.choice(len(lengths), size=6, replace=False))
    sub_ids = np.concatenate([ids[cu[b]:cu[b + 1]] for b in pick])
    sub_cu = np.concatenate([[0], np.cumsum(lengths[pick])]).astype(np.int32)
    want = oracle64.forward(ocfg(shape), oracle_weights(blob, shape), sub_ids, sub_cu, shape.K)
    check_logits(got[pick], want, shape, name)
    # and the all-token last layer (the same projections on every row of the last layer as well)
    st2 = sp.Students(sp.config_from_shape(shape, last_layer_all_tokens=True), blob)
    got2 = st2.sp_forward(d_ids, d_cu, int(lengths.max()), shape.K).cpu().numpy().astype(np.float64)
    check_logits(got2[pick], want, shape, name + " all-token last layer")


def test_fp32_large_call(sp, oracle64):
    """The fp32 path on a call large enough for its 64 x 64 projection tile (a grid of at least 1024 such tiles: the
    q|k|v and FFN up-projections here; the two residual projections stay on the 32 x 32 tile), sequences of up to 300
    tokens (several key chunks and query blocks in the fp32 attention kernel), every sequence against the oracle to the
    fp32 bound."""
    shape = synth.StudentShape(K=2, layers=2, hidden=128, heads=2, ffn=512, vocab=1000, max_pos=320, classes=3,
                               dtype="fp32")
    rng = np.random.default_rng(43)
    lengths = rng.integers(1, 301, size=40).astype(np.int32)
    lengths[:3] = (300, 1, 65)
    total = int(lengths.sum())
    assert (shape.ffn // 64) * ((total + 255) // 256 * 4) * shape.K >= 1024, total
    ids = synth.make_ids(rng, total, shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.02, ln_random=True, qk_std=float(np.sqrt(1.5 / shape.hidden)))
    st = sp.Students(sp.config_from_shape(shape), blob)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    want = oracle64.forward(ocfg(shape), blob, ids, cu, shape.K)
    for k in (2, 1):
        got = st.sp_forward(d_ids, d_cu, int(lengths.max()), k).cpu().numpy().astype(np.float64)
        ref = want if k == 2 else oracle64.forward(ocfg(shape), blob, ids, cu, 1)
        err = check_logits(got, ref, shape, f"fp32, {total} tokens, k_active={k}")
        assert err < 1e-4
    st.close()


@pytest.mark.parametrize("nseq", [3, 24])
def test_fp32_deep_reduction_on_small_grids(sp, oracle64, nseq):
    """The fp32 FFN down-projection (reduction depth 512) on calls too small to fill the chip with tiles: the reduction
    range is split over the waves of a workgroup, with 16 x 16 tiles for the smallest calls (3 sequences, about a
    hundred tokens) and 32 x 32 tiles for the next size (24 sequences, about 800 tokens).  Every sequence against the
    oracle."""
    shape = synth.StudentShape(K=2, layers=2, hidden=128, heads=2, ffn=512, vocab=1000, max_pos=64, classes=3,
                               dtype="fp32")
    rng = np.random.default_rng(47 + nseq)
    lengths = rng.integers(20, 49, size=nseq).astype(np.int32)
    total = int(lengths.sum())
    mtile = 256 if total > 256 else (128 if total > 64 else 64)
    tiles = (shape.hidden // 32) * ((total + mtile - 1) // mtile * mtile // 32) * shape.K
    assert (tiles < 128) if nseq == 3 else (128 <= tiles <= 256), (total, tiles)
    ids = synth.make_ids(rng, total, shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.05, ln_random=True, qk_std=0.12)
    st = sp.Students(sp.config_from_shape(shape), blob)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    got = st.sp_forward(d_ids, d_cu, int(lengths.max()), shape.K).cpu().numpy().astype(np.float64)
    want = oracle64.forward(ocfg(shape), blob, ids, cu, shape.K)
    assert np.abs(want).max() > 5e-2
    assert check_logits(got, want, shape, f"fp32, {total} tokens") < 1e-4
    st.close()


BOUNDARY_TOKENS = [63, 64, 65, 127, 128, 129, 255, 256, 257, 1023, 1024, 1025, 2047, 2048, 2049]


@pytest.mark.parametrize("total", BOUNDARY_TOKENS)
def test_call_sizes_at_every_path_boundary(sp, oracle64, total):
    """The forward changes its launch plan with the size of the call: split reductions and the fused head up to 128
    token rows, 64 / 128 / 256-row projection tiles, the first-token last layer from 1024 tokens, two groups of
    students and the long-call LayerNorm from 2048.  One call just below, at and just above each boundary, against the
    oracle (a sample of the sequences for the large ones), with k_active below and at K."""
    shape = synth.StudentShape(K=3, layers=2, hidden=256, heads=4, ffn=1024, vocab=800, max_pos=160, classes=3,
                               dtype="bf16")
    rng = np.random.default_rng(1000 + total)
    lengths = []
    left = total
    while left > 0:
        n = int(min(left, rng.integers(1, 150)))
        lengths.append(n)
        left -= n
    lengths = np.array(lengths, dtype=np.int32)
    assert lengths.sum() == total
    ids = synth.make_ids(rng, total, shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.02, ln_random=True, qk_std=float(np.sqrt(1.5 / shape.hidden)))
    st = sp.Students(sp.config_from_shape(shape), blob)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    pick = np.arange(len(lengths)) if len(lengths) <= 8 else np.sort(rng.choice(len(lengths), size=8, replace=False))
    sub_ids = np.concatenate([ids[cu[b]:cu[b + 1]] for b in pick])
    sub_cu = np.concatenate([[0], np.cumsum(lengths[pick])]).astype(np.int32)
    ow = oracle_weights(blob, shape)
    for k in (2, 3):
        got = st.sp_forward(d_ids, d_cu, int(lengths.max()), k).cpu().numpy().astype(np.float64)
        want = oracle64.forward(ocfg(shape), ow, sub_ids, sub_cu, k)
        check_logits(got[pick], want, shape, f"{total} tokens, k_active={k}")


@pytest.mark.parametrize("lengths", [(64,), (1,), (128,), (17, 3), (60, 1, 67), (30, 31, 32, 33), (1, 1, 1, 1),
                                     (25, 25, 25, 25, 25), (129,), (300,), (100, 90), (128, 128, 128, 128),
                                     (5, 200, 7), (1, 640, 1, 381), (640, 640), (200, 200, 200, 200, 200)])
def test_calls_of_a_few_sequences(sp, oracle64, lengths):
    """Whole forwards of one to four sequences finish their last layer on the first-token rows by per-feature dot
    products: attention-output projection, LayerNorm, FFN, and then either the small-call head on the raw
    down-projection (up to 128 tokens) or the pooler by dot products and the classifier kernel (up to 1023 tokens; from
    1024 on the folded first-token layer takes over); five sequences take the tile path.  Random LayerNorm parameters
    and sharpened attention, every k_active, against the oracle; and the same call with the last layer on every token
    (the tile path) must agree with it to rounding."""
    shape = synth.StudentShape(K=3, layers=2, hidden=256, heads=4, ffn=1024, vocab=500, max_pos=640, classes=3,
                               dtype="bf16")
    rng = np.random.default_rng(500 + sum(lengths) + len(lengths))
    lengths = np.array(lengths, dtype=np.int32)
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.05, ln_random=True, qk_std=0.12)
    st = sp.Students(sp.config_from_shape(shape), blob)
    st_tiles = sp.Students(sp.config_from_shape(shape, last_layer_all_tokens=True), blob)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    ow = oracle_weights(blob, shape)
    for k in range(1, shape.K + 1):
        got = st.sp_forward(d_ids, d_cu, int(lengths.max()), k).cpu().numpy().astype(np.float64)
        tiles = st_tiles.sp_forward(d_ids, d_cu, int(lengths.max()), k).cpu().numpy().astype(np.float64)
        want = oracle64.forward(ocfg(shape), ow, ids, cu, k)
        assert np.abs(want).max() > 5e-2
        check_logits(got, want, shape, f"{len(lengths)} sequences {tuple(lengths)}, k_active={k}")
        check_logits(tiles, want, shape, f"{len(lengths)} sequences {tuple(lengths)}, tile path, k_active={k}")
        # (beyond 128 tokens the tile path rounds the rows before each LayerNorm to bf16 and the dot-product path does
        # not: the two differ by about as much as either differs from the oracle)
        assert rel_err(got, tiles) < (1e-3 if lengths.sum() <= 128 else 3e-2)
    st.close()
    st_tiles.close()


# ---- the five workloads ----------------------------------------------------------------------------

_cache = {}


def loaded(sp, n, **cfg_kw):
    """Students + inputs of workload n, kept for the module (weights are large)."""
    key = (n, tuple(sorted(cfg_kw.items())))
    if key not in _cache:
        _cache.clear()
        w = synth.WORKLOADS[n]
        batch, blob = synth.make_workload(w)
        st = sp.Students(sp.config_from_shape(w.shape, **cfg_kw), blob)
        _cache[key] = (w, batch, oracle_weights(blob, w.shape), st)
    return _cache[key]


def part_range(lengths, part, nparts):
    """Sequences [lo, hi) of part `part` when the batch is cut into `nparts` contiguous runs of about equal token
    counts (the parts together cover every sequence exactly once)."""
    cum = np.concatenate([[0], np.cumsum(lengths.astype(np.int64))])
    cuts = [int(np.searchsorted(cum, cum[-1] * i / nparts)) for i in range(nparts + 1)]
    cuts[0], cuts[-1] = 0, len(lengths)
    return cuts[part], cuts[part + 1]


def run_workload(sp, oracle, n, part=0, nparts=1, **cfg_kw):
    """Every logit of the sequences in one part of workload n (all of it by default), for each of its k_active
    values, against the oracle.  The GPU always runs the whole batch; the oracle runs the part's sequences as a batch
    of their own (samples are independent: pinned by test_each_sample_is_independent_of_its_batch) once with all K
    students and hands out the per-student terms; its logits for k_active are their sum in student order (what its
    own forward does: pinned by test_prefix_sums_and_tail_pruning).  Large workloads are cut into parts so that no
    single test keeps the oracle busy for minutes."""
    w, batch, ow, st = loaded(sp, n, **cfg_kw)
    d_ids, d_cu, cu = gpu_inputs(batch.lengths, batch.ids, sp)
    mx = int(batch.lengths.max())
    lo, hi = part_range(batch.lengths, part, nparts)
    assert hi > lo
    sub_cu = (cu[lo:hi + 1] - cu[lo]).astype(np.int32)
    _, terms = oracle.forward(ocfg(w.shape), ow, batch.ids[cu[lo]:cu[hi]], sub_cu, w.shape.K, want_terms=True)
    errs = {}
    for k in sorted(w.k_actives):
        got = st.sp_forward(d_ids, d_cu, mx, k).cpu().numpy().astype(np.float64)
        want = np.zeros_like(terms[0])
        for m in range(k):
            want = want + terms[m]
        assert got.shape == (len(batch.lengths), w.shape.classes) and want.shape == (hi - lo, w.shape.classes)
        assert np.abs(want).max() > 1e-2
        errs[k] = check_logits(got[lo:hi], want, w.shape, f"{w.name} k_active={k}, sequences {lo}..{hi - 1}")
    return errs


def test_config1_tiny_fp32(sp, oracle64, oracle32):
    errs = run_workload(sp, oracle64, 1)
    run_workload(sp, oracle32, 1)       # the fp32 build the benchmark spec names, same bound
    assert max(errs.values()) < 1e-4    # fp32 arithmetic does far better than the 1e-3 gate


def test_config2_base_width_b32_every_sequence(sp, oracle64):
    run_workload(sp, oracle64, 2)


def test_config3_latency_b1(sp, oracle64):
    run_workload(sp, oracle64, 3)


@pytest.mark.parametrize("part", range(3))
def test_config4_burst_b256_every_sequence(sp, oracle64, part):
    """All 256 sequences, in three parts (58 token tiles of 256 rows: the last block of the token-tile-blocked
    projection order is a partial one, and the last tile is padded)."""
    run_workload(sp, oracle64, 4, part, 3)


@pytest.mark.parametrize("part", range(3))
def test_config4_burst_b256_all_token_last_layer_every_sequence(sp, oracle64, part):
    """The stock variant (every token through the last layer as well) at full size: the second layer's large-tile
    projections, attention kernels and LayerNorm on all 14722 rows."""
    run_workload(sp, oracle64, 4, part, 3, last_layer_all_tokens=True)


@pytest.mark.parametrize("part", range(6))
def test_config5_large_width_b64_every_sequence(sp, oracle64, part):
    """All 64 sequences, in six parts (64 to 512 tokens, hidden 1024, 16 heads: every attention path at that width,
    sequences of more than 256 tokens included, 74 token tiles)."""
    run_workload(sp, oracle64, 5, part, 6)


def test_partial_last_block_of_the_token_tile_order(sp, oracle64):
    """A small shape that reaches the partial last block of the large projection tile's order: hidden 512 (six
    256-wide feature tiles in the query/key/value projection, eight in the FFN up-projection) and 11 token tiles of
    256 rows (blocks of five: 5 + 5 + 1), every sequence against the oracle, both last-layer variants."""
    shape = synth.StudentShape(K=2, layers=2, hidden=512, heads=8, ffn=2048, vocab=1000, max_pos=128, classes=3,
                               dtype="bf16")
    rng = np.random.default_rng(41)
    lengths = rng.integers(20, 101, size=42).astype(np.int32)
    total = int(lengths.sum())
    assert 2560 < total <= 2816, total          # 11 token tiles
    ids = synth.make_ids(rng, total, shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.02, ln_random=True, qk_std=float(np.sqrt(1.5 / shape.hidden)))
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    want = oracle64.forward(ocfg(shape), oracle_weights(blob, shape), ids, cu, shape.K)
    for all_tokens in (False, True):
        st = sp.Students(sp.config_from_shape(shape, last_layer_all_tokens=all_tokens), blob)
        got = st.sp_forward(d_ids, d_cu, int(lengths.max()), shape.K).cpu().numpy().astype(np.float64)
        check_logits(got, want, shape, f"11 token tiles, all_tokens={all_tokens}")
        st.close()


@pytest.mark.parametrize("all_tokens", [False, True])
def test_call_whose_buffers_pass_four_gib(sp, oracle64, all_tokens):
    """A call of about 132 thousand tokens on the burst workload's students (2304 sequences: the burst batch's lengths
    nine times over, fresh ids): the q|k|v buffer (4.9 GB), the FFN activations (6.5 GB) and every student's share of
    them lie beyond what 32-bit element or byte offsets reach, and the grids are nine times those of the burst batch.
    The first, middle and last sequences and the longest one are compared with the oracle, which computes them as a
    batch of their own (samples are independent: pinned by test_each_sample_is_independent_of_its_batch), for all
    eight students and for five (two groups of unequal size); the logits of the whole call must be finite and a second
    call must repeat them bit for bit."""
    w, batch, ow, st = loaded(sp, 4, last_layer_all_tokens=all_tokens)
    rng = np.random.default_rng(4096)
    lengths = np.tile(batch.lengths, 9).astype(np.int32)
    B, T = len(lengths), int(lengths.sum())
    assert T * 3 * w.shape.hidden * 2 * w.shape.K > 4 * 2**30 and T * 3 * w.shape.hidden > 2**28
    ids = synth.make_ids(rng, T, w.shape.vocab)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    mx = int(lengths.max())
    longest = int(np.argmax(lengths[B // 2:])) + B // 2
    picks = sorted({0, 1, B // 2, B // 2 + 1, longest, B - 2, B - 1})
    sub_ids = np.concatenate([ids[cu[b]:cu[b + 1]] for b in picks])
    sub_cu = np.concatenate([[0], np.cumsum(lengths[picks])]).astype(np.int32)
    _, terms = oracle64.forward(ocfg(w.shape), ow, sub_ids, sub_cu, w.shape.K, want_terms=True)
    for k in (8, 5):
        got = st.sp_forward(d_ids, d_cu, mx, k).cpu().numpy().astype(np.float64)
        assert got.shape == (B, w.shape.classes) and np.isfinite(got).all()
        want = np.zeros_like(terms[0])
        for m in range(k):
            want = want + terms[m]
        check_logits(got[picks], want, w.shape, f"{T} tokens, k_active={k}, sequences {picks}")
        again = st.sp_forward(d_ids, d_cu, mx, k).cpu().numpy().astype(np.float64)
        assert np.array_equal(got, again)
    st.release_workspace()


# ---- properties that hold at any size ----------------------------------------------------------------

def test_prefix_property_and_determinism_at_full_size(sp):
    """logits(k) - logits(k-1) is student k-1's term exactly, and two runs agree bit for bit."""
    w, batch, _, st = loaded(sp, 4)
    d_ids, d_cu, cu = gpu_inputs(batch.lengths, batch.ids, sp)
    T, B = int(cu[-1]), len(batch.lengths)
    mx = int(batch.lengths.max())
    full = st.sp_forward(d_ids, d_cu, mx, 8).clone()
    z = torch.from_numpy(st.read_activation(st.workspace(T, B), "z", T, B, 8)).float()
    again = st.sp_forward(d_ids, d_cu, mx, 8)
    assert torch.equal(full, again)
    acc = torch.zeros(B, w.shape.classes)
    for k in range(1, 9):
        acc = acc + z[k - 1]
        if k in (2, 4, 8):
            got = st.sp_forward(d_ids, d_cu, mx, k).cpu()
            assert torch.equal(got, acc), f"k_active={k} is not the fixed-order prefix sum"


def test_two_groups_of_students_bit_identical_to_single_stream(sp):
    """Large calls run the active students as two groups on two streams; the logits are summed over all students in
    ascending order afterwards, so they must equal the single-stream result bit for bit, for even and odd k_active."""
    w, batch, _, st = loaded(sp, 4)
    d_ids, d_cu, cu = gpu_inputs(batch.lengths, batch.ids, sp)
    mx = int(batch.lengths.max())
    _, blob = synth.make_workload(w)
    single = sp.Students(sp.config_from_shape(w.shape, single_stream=True), blob)
    for k in (8, 5, 2):
        a = st.sp_forward(d_ids, d_cu, mx, k).cpu().numpy()
        b = single.sp_forward(d_ids, d_cu, mx, k).cpu().numpy()
        assert np.array_equal(a, b), f"k_active={k}: max diff {np.abs(a - b).max():.3e}"
    single.close()


def test_forward_can_be_captured_in_a_graph(sp):
    """sp_forward only enqueues work (also when it forks to the model's second stream), so it can be captured; every
    replay, with eager calls and synchronisations between them, must reproduce the eager logits bit for bit."""
    w, batch, _, st = loaded(sp, 4)
    d_ids, d_cu, cu = gpu_inputs(batch.lengths, batch.ids, sp)
    mx, B = int(batch.lengths.max()), len(batch.lengths)
    ws = st.workspace(int(cu[-1]), B)
    out = torch.empty(B, w.shape.classes, dtype=torch.float32, device="cuda")
    st.sp_forward(d_ids, d_cu, mx, 8, out, ws)
    torch.cuda.synchronize()
    ref = out.clone()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        st.sp_forward(d_ids, d_cu, mx, 8, out, ws, stream=side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        st.sp_forward(d_ids, d_cu, mx, 8, out, ws, stream=side)
    torch.cuda.synchronize()
    for i in range(3):
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref), f"replay {i}"
        st.sp_forward(d_ids, d_cu, mx, 4, out, ws)     # eager work between the replays
        torch.cuda.synchronize()


def test_small_call_can_be_captured_in_a_graph(sp):
    """The same for the path of a single short sequence (split reductions, per-feature dot products, the small-call
    head: a dozen and a half launches on one stream), at two student numbers."""
    w, batch, _, st = loaded(sp, 3)
    d_ids, d_cu, cu = gpu_inputs(batch.lengths, batch.ids, sp)
    mx, B = int(batch.lengths.max()), len(batch.lengths)
    ws = st.workspace(int(cu[-1]), B)
    side = torch.cuda.Stream()
    for k in (8, 3):
        out = torch.empty(B, w.shape.classes, dtype=torch.float32, device="cuda")
        st.sp_forward(d_ids, d_cu, mx, k, out, ws)
        torch.cuda.synchronize()
        ref = out.clone()
        with torch.cuda.stream(side):
            st.sp_forward(d_ids, d_cu, mx, k, out, ws, stream=side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            st.sp_forward(d_ids, d_cu, mx, k, out, ws, stream=side)
        torch.cuda.synchronize()
        for i in range(3):
            out.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, ref), f"k_active={k}, replay {i}"
            st.sp_forward(d_ids, d_cu, mx, 1, out, ws)     # eager work between the replays
            torch.cuda.synchronize()
        del graph


def test_sample_is_independent_of_batch_mates(sp):
    """A sequence's logits do not depend on where it sits in the packed batch (bitwise in the fp32 path)."""
    w = synth.WORKLOADS[1]
    batch, blob = synth.make_workload(w)
    st = sp.Students(sp.config_from_shape(w.shape), blob)
    d_ids, d_cu, cu = gpu_inputs(batch.lengths, batch.ids, sp)
    full = st.sp_forward(d_ids, d_cu, int(batch.lengths.max()), 2).cpu().numpy()
    order = [2, 0, 3, 1]
    p_ids = np.concatenate([batch.ids[cu[b]:cu[b + 1]] for b in order])
    dp_ids, dp_cu, _ = gpu_inputs(batch.lengths[order], p_ids, sp)
    perm = st.sp_forward(dp_ids, dp_cu, int(batch.lengths.max()), 2).cpu().numpy()
    assert np.array_equal(perm, full[order])


# ---- boundary behaviour --------------------------------------------------------------------------------

def test_error_codes(sp):
    w = synth.WORKLOADS[1]
    batch, blob = synth.make_workload(w)
    cfg = sp.config_from_shape(w.shape)
    st = sp.Students(cfg, blob)
    d_ids, d_cu, cu = gpu_inputs(batch.lengths, batch.ids, sp)
    mx = int(batch.lengths.max())
    for k in (0, 3):
        with pytest.raises(sp.SpError) as e:
            st.sp_forward(d_ids, d_cu, mx, k)
        assert e.value.code == -3
    with pytest.raises(sp.SpError) as e:
        st.sp_forward(d_ids, d_cu, w.shape.max_pos + 1, 2)
    assert e.value.code == -2
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(sp.SpError) as e:
        st.sp_forward(d_ids, d_cu, mx, 2, workspace=small)
    assert e.value.code == -4
    bad = sp.make_config(2, 2, 96, 2, 256, 100, 64, 2, "bf16")     # head width 48: unsupported
    with pytest.raises(sp.SpError) as e:
        sp.Students(bad, np.zeros(sp.sp_blob_floats(bad), np.float32))
    assert e.value.code == -2


def test_input_contents_check(sp):
    """sp_check_inputs flags what sp_forward cannot see without a synchronisation: ids outside the vocabulary,
    offsets that do not start at 0, do not increase, describe a sequence longer than max_seqlen, or do not end at the
    token count."""
    shape = synth.StudentShape(K=1, layers=1, hidden=128, heads=2, ffn=128, vocab=50, max_pos=64, classes=2, dtype="bf16")
    rng = np.random.default_rng(3)
    st = sp.Students(sp.config_from_shape(shape), synth.make_weights(rng, shape))
    lengths = np.array([5, 30, 1, 64, 17], dtype=np.int32)
    ids = synth.make_ids(rng, int(lengths.sum()), shape.vocab)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    assert st.sp_check_inputs(d_ids, d_cu, 64) == 0
    assert st.sp_check_inputs(d_ids, d_cu, 63) == sp.SP_BAD_LENGTH
    bad = d_ids.clone(); bad[40] = shape.vocab
    assert st.sp_check_inputs(bad, d_cu, 64) == sp.SP_BAD_ID
    bad[3] = -1
    assert st.sp_check_inputs(bad, d_cu, 64) == sp.SP_BAD_ID
    c = d_cu.clone(); c[0] = 1
    assert st.sp_check_inputs(d_ids, c, 64) & sp.SP_BAD_CU0
    c = d_cu.clone(); c[2] = c[1]                          # an empty sequence
    assert st.sp_check_inputs(d_ids, c, 64) == sp.SP_BAD_ORDER
    c = d_cu.clone(); c[-1] += 1                           # last sequence 18 tokens, one more than there are ids
    assert st.sp_check_inputs(d_ids, c, 64) == sp.SP_BAD_TOTAL
    with pytest.raises(sp.SpError):
        st.sp_check_inputs(d_ids, d_cu, 65)                # max_seqlen beyond the position table


# ---- pieces that the stage tolerance cannot resolve ------------------------------------------------------

def test_gelu_of_the_bf16_epilogue_is_the_erf_form(sp):
    """The bf16 FFN up-projection evaluates GELU through a fitted complementary error function.  In fp32, before the
    rounding to bf16, it must stay within 5e-7 of x (1 + erf(x / sqrt 2)) / 2 everywhere (a dense grid over the range
    in which the function is not yet x or 0 to fp32 accuracy, plus the tails and the special points); the
    tanh approximation of the same function, which this reading rejects, is up to 5e-4 away."""
    import math
    grid = np.concatenate([np.linspace(-12, 12, 2_000_001), np.linspace(-1e-3, 1e-3, 20_001),
                           [0.0, -0.0, 1.0, -1.0, 30.0, -30.0, 1e4, -1e4, 6.0811, -6.0811]]).astype(np.float32)
    got = sp.sp_probe_gelu(torch.from_numpy(grid).cuda()).cpu().numpy().astype(np.float64)
    x = grid.astype(np.float64)
    want = 0.5 * x * (1.0 + np.vectorize(math.erf)(x / math.sqrt(2.0)))
    err = np.abs(got - want)
    assert err.max() <= 5e-7, f"max |gelu_fast - gelu_erf| = {err.max():.3e} at x = {x[err.argmax()]}"
    assert got[np.flatnonzero(grid == 0.0)].max() == 0.0
    tanh_form = 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))
    assert np.abs(tanh_form - want).max() > 1e-4 > 100 * err.max()       # the test can tell the two forms apart


def test_two_threads_issue_large_calls_on_one_model(sp):
    """Calls of >= 2048 tokens fork to the model's second stream and join again; two host threads issuing such calls
    on one model at the same time (own stream, own workspace, own output each) must both get the single-threaded
    logits bit for bit, every time."""
    import threading
    w, batch, _, st = loaded(sp, 4)
    d_ids, d_cu, cu = gpu_inputs(batch.lengths, batch.ids, sp)
    T, B, mx = int(cu[-1]), len(batch.lengths), int(batch.lengths.max())
    ref = {k: st.sp_forward(d_ids, d_cu, mx, k).clone() for k in (8, 3)}
    torch.cuda.synchronize()
    need = sp.sp_workspace_bytes(st.cfg, T, B)
    results, errors = {}, []

    def worker(i, k):
        try:
            stream = torch.cuda.Stream()
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            out = torch.empty(B, w.shape.classes, dtype=torch.float32, device="cuda")
            bad = 0
            for _ in range(6):
                out.zero_()
                stream.wait_stream(torch.cuda.current_stream())
                st.sp_forward(d_ids, d_cu, mx, k, out, ws, stream=stream)
                stream.synchronize()
                bad += int(not torch.equal(out, ref[k]))
            results[i] = bad
        except Exception as e:          # surfaced below: an exception in a thread would otherwise be lost
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(0, 8)), threading.Thread(target=worker, args=(1, 3))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    assert results == {0: 0, 1: 0}, results


@pytest.mark.parametrize("total", [70, 1500, 2600])
def test_widest_head_and_odd_student_count(sp, oracle64, total):
    """The limits of the head: 16 classes (the most the kernels take), five students with k_active 1, 3 and 5 (odd
    counts split unevenly over the two student groups of a large call), at a small, a medium and a large call size."""
    shape = synth.StudentShape(K=5, layers=2, hidden=256, heads=4, ffn=512, vocab=400, max_pos=256, classes=16,
                               dtype="bf16")
    rng = np.random.default_rng(3000 + total)
    lengths = []
    left = total
    while left > 0:
        n = int(min(left, rng.integers(1, 200)))
        lengths.append(n)
        left -= n
    lengths = np.array(lengths, dtype=np.int32)
    ids = synth.make_ids(rng, total, shape.vocab)
    blob = synth.make_weights(rng, shape, std=0.03, ln_random=True, qk_std=float(np.sqrt(1.5 / shape.hidden)))
    st = sp.Students(sp.config_from_shape(shape), blob)
    d_ids, d_cu, cu = gpu_inputs(lengths, ids, sp)
    _, terms = oracle64.forward(ocfg(shape), oracle_weights(blob, shape), ids, cu, shape.K, want_terms=True)
    for k in (1, 3, 5):
        got = st.sp_forward(d_ids, d_cu, int(lengths.max()), k).cpu().numpy().astype(np.float64)
        assert got.shape == (len(lengths), 16)
        check_logits(got, terms[:k].sum(0), shape, f"{total} tokens, 16 classes, k_active={k}")
    st.close()


def test_degenerate_calls_are_refused(sp):
    """Empty inputs and inconsistent sizes never reach a kernel: an empty batch, fewer tokens than sequences, a
    max_seqlen of 0 or one that cannot hold the tokens."""
    w = synth.WORKLOADS[1]
    batch, blob = synth.make_workload(w)
    st = sp.Students(sp.config_from_shape(w.shape), blob)
    lib = sp.raw_lib()
    ids = torch.zeros(8, dtype=torch.int32, device="cuda")
    cu = torch.tensor([0, 3, 8], dtype=torch.int32, device="cuda")
    ws = st.workspace(8, 2)
    out = torch.zeros(2, w.shape.classes, dtype=torch.float32, device="cuda")

    def call(batch_n, total, max_seqlen, k=1):
        return lib.sp_forward(st.handle, ids.data_ptr(), cu.data_ptr(), batch_n, total, max_seqlen, k, ws.data_ptr(),
                              ws.numel(), out.data_ptr(), None)
    assert call(2, 8, 5) == 0
    assert call(0, 0, 5) == -2            # empty batch
    assert call(0, 8, 5) == -2
    assert call(2, 1, 5) == -2            # fewer tokens than sequences: some sequence would be empty
    assert call(2, 8, 0) == -2
    assert call(2, 8, 3) == -2            # two sequences of at most three tokens cannot hold eight
    assert call(2, 8, w.shape.max_pos + 1) == -2
    torch.cuda.synchronize()
    st.close()
