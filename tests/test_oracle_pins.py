"""Pins for the float64 CPU oracle (CPU only).

Nothing in the paper prints an output value of the operator, so the oracle is
pinned to what the mathematics fixes: a hand-evaluated example, closed forms,
invariants, special cases that reduce to a library GEMM chain, brute force
with a dense Delta W, and an even plainer pure-Python evaluation.
"""
import json
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import oracle
from oracle import tiny
from paper_2411_00915_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _adapters(w):
    return oracle.Adapters(w.adapter_rank, w.adapter_scale, w.A, w.B)


def _small(seed=1, T=23, K=40, N=28, n_a=5, ranks=(1, 2, 3, 4, 8), frac_none=0.2, scales=(0.5, 1.0, 2.0, -1.25, 3.0)):
    return wl.random_case(seed, T, K, N, n_a, ranks, dtype="f32", max_seg=5, frac_none=frac_none,
                          scales=scales, empty_segments=True)


def test_hand_example():
    g = json.load(open(os.path.join(GOLD, "hand_example.json")))
    x, W = np.array(g["x"], float), np.array(g["W"], float)
    A = [np.array(a, float) for a in g["A"]]
    B = [np.array(b, float) for b in g["B"]]
    tok = oracle.token_adapter(3, g["seg_indptr"], g["seg_adapter"])
    assert tok.tolist() == [1, 0, -1]
    ad = oracle.Adapters(g["adapter_rank"], g["adapter_scale"], A, B)
    assert np.array_equal(oracle.base(x, W), np.array(g["xW"], float))
    assert np.array_equal(oracle.shrink(x, tok, ad, apply_scale=False), np.array(g["v_unscaled"], float))
    assert np.array_equal(oracle.forward(x, W, tok, ad), np.array(g["y"], float))
    delta = np.array(g["y"], float) - np.array(g["xW"], float)
    assert np.array_equal(oracle.expand(x, tok, ad, 3), delta)
    assert np.array_equal(oracle.expand(x, tok, ad, 3, literal=True), delta)
    assert np.array_equal(oracle.expand(x, tok, ad, 3, y_in=np.array(g["xW"], float)), np.array(g["y"], float))


def test_zero_adapters_is_exactly_xW():
    w = _small(seed=2)
    ad = _adapters(w)
    base = oracle.base(w.x, w.W)
    # all segments without adapter
    none = np.full(w.T, -1, dtype=np.int32)
    assert np.array_equal(oracle.forward(w.x, w.W, none, ad), base)
    # all ranks zero
    ad0 = oracle.Adapters(np.zeros(w.num_adapters, np.int32), w.adapter_scale,
                          [a[:, :0] for a in w.A], [b[:0, :] for b in w.B])
    assert np.array_equal(oracle.forward(w.x, w.W, w.token_adapter(), ad0), base)
    # B = 0
    adB = oracle.Adapters(w.adapter_rank, w.adapter_scale, w.A, [np.zeros_like(b) for b in w.B])
    assert np.array_equal(oracle.forward(w.x, w.W, w.token_adapter(), adB), base)
    # base product itself against the library GEMM
    ref = w.x.astype(np.float64) @ w.W.astype(np.float64)
    assert np.allclose(base, ref, rtol=1e-12, atol=1e-13)


def test_rank1_closed_form():
    rng = np.random.default_rng(3)
    T, K, N = 9, 31, 17
    x = rng.standard_normal((T, K))
    W = rng.standard_normal((K, N))
    a = rng.standard_normal(K)
    b = rng.standard_normal(N)
    s = 1.75
    ad = oracle.Adapters([1], [s], [a[:, None]], [b[None, :]])
    tok = np.zeros(T, np.int32)
    y = oracle.forward(x, W, tok, ad)
    xw = oracle.base(x, W)
    for t in range(T):
        coef = s * float(np.dot(x[t], a))        # scalar (x.a)
        assert np.allclose(y[t] - xw[t], coef * b, rtol=1e-12, atol=1e-12)


def test_token_permutation_invariance():
    w = _small(seed=4, T=31)
    ad = _adapters(w)
    tok = w.token_adapter()
    y = oracle.forward(w.x, w.W, tok, ad)
    v = oracle.shrink(w.x, tok, ad)
    perm = np.random.default_rng(5).permutation(w.T)
    yp = oracle.forward(w.x[perm], w.W, tok[perm], ad)
    vp = oracle.shrink(w.x[perm], tok[perm], ad)
    assert np.array_equal(yp, y[perm])           # per-token loop: exactly
    assert np.array_equal(vp, v[perm])
    # permuting whole segments through the segment table gives the same map
    S = w.num_segments
    sp = np.random.default_rng(6).permutation(S)
    lens = np.diff(w.seg_indptr)[sp]
    indptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    tok2 = oracle.token_adapter(w.T, indptr, w.seg_adapter[sp])
    rows = np.concatenate([np.arange(w.seg_indptr[s], w.seg_indptr[s + 1]) for s in sp]).astype(np.int64)
    assert np.array_equal(tok2, tok[rows])
    assert np.array_equal(oracle.forward(w.x[rows], w.W, tok2, ad), y[rows])


def test_dense_delta_w_brute_force():
    w = _small(seed=7)
    ad = _adapters(w)
    tok = w.token_adapter()
    y = oracle.forward(w.x, w.W, tok, ad)
    x64, W64 = w.x.astype(np.float64), w.W.astype(np.float64)
    for t in range(w.T):
        a = tok[t]
        Weff = W64.copy()
        if a >= 0:
            dW = w.A[a].astype(np.float64) @ w.B[a].astype(np.float64)
            Weff = W64 + float(w.adapter_scale[a]) * dW
        assert np.allclose(y[t], x64[t] @ Weff, rtol=1e-11, atol=1e-12)


def test_single_adapter_is_gemm_chain():
    # one segment, one adapter: textbook x @ A @ B; first shape is scaled down
    # from the paper's Table 1 inputs (256x4096 . 4096x32) and (8192x4096 . 4096x128)
    for (T, K, r, N) in [(32, 512, 32, 24), (64, 256, 128, 16)]:
        rng = np.random.default_rng(T)
        x = rng.standard_normal((T, K)); A = rng.standard_normal((K, r)); B = rng.standard_normal((r, N))
        ad = oracle.Adapters([r], [1.0], [A], [B])
        tok = oracle.token_adapter(T, [0, T], [0])
        assert np.allclose(oracle.shrink(x, tok, ad), x @ A, rtol=1e-12, atol=1e-12)
        assert np.allclose(oracle.expand(x, tok, ad, N), x @ A @ B, rtol=1e-11, atol=1e-11)


def test_block_independence():
    w = _small(seed=8, frac_none=0.0)
    ad = _adapters(w)
    tok = w.token_adapter()
    y = oracle.forward(w.x, w.W, tok, ad)
    used = set(tok.tolist())
    # change an adapter's weights: rows of other adapters are bit-identical
    victim = int(tok[0])
    A2 = [a.copy() for a in w.A]; B2 = [b.copy() for b in w.B]
    A2[victim] += 1.0; B2[victim] -= 2.0
    y2 = oracle.forward(w.x, w.W, tok, oracle.Adapters(w.adapter_rank, w.adapter_scale, A2, B2))
    other = tok != victim
    assert np.array_equal(y2[other], y[other])
    assert not np.array_equal(y2[~other], y[~other])
    # tokens of one adapter computed alone equal the same tokens in the batch
    rows = np.nonzero(tok == victim)[0]
    alone = oracle.forward(w.x[rows], w.W, tok[rows], ad)
    assert np.array_equal(alone, y[rows])
    # the row-subset interface selects the same rows
    assert np.array_equal(oracle.forward(w.x, w.W, tok, ad, rows=rows), y[rows])
    assert np.array_equal(oracle.shrink(w.x, tok, ad, rows=rows), oracle.shrink(w.x, tok, ad)[rows])
    assert len(used) > 1


def test_scale_linearity_and_zero_scale():
    w = _small(seed=9, scales=(1.0,))
    tok = w.token_adapter()
    one = oracle.Adapters(w.adapter_rank, np.ones(w.num_adapters), w.A, w.B)
    d1 = oracle.expand(w.x, tok, one, w.N)
    for s in (0.0, 2.0, -0.37, 5.5):
        ds = oracle.expand(w.x, tok, oracle.Adapters(w.adapter_rank, np.full(w.num_adapters, s), w.A, w.B), w.N)
        assert np.allclose(ds, s * d1, rtol=1e-14, atol=0)
    z = oracle.Adapters(w.adapter_rank, np.zeros(w.num_adapters), w.A, w.B)
    assert np.array_equal(oracle.forward(w.x, w.W, tok, z), oracle.base(w.x, w.W))
    # scaled v is s * unscaled v
    het = oracle.Adapters(w.adapter_rank, np.arange(1, w.num_adapters + 1) * 0.75, w.A, w.B)
    vs, vu = oracle.shrink(w.x, tok, het, True), oracle.shrink(w.x, tok, het, False)
    for t in range(w.T):
        if tok[t] >= 0:
            assert np.allclose(vs[t], het.scale[tok[t]] * vu[t], rtol=1e-15, atol=0)


def test_rank_zero_padding_invariance():
    w = _small(seed=10)
    tok = w.token_adapter()
    y = oracle.forward(w.x, w.W, tok, _adapters(w))
    pad = 3
    A2 = [np.concatenate([a, np.zeros((w.K, pad), a.dtype)], axis=1) for a in w.A]
    B2 = [np.concatenate([b, np.zeros((pad, w.N), b.dtype)], axis=0) for b in w.B]
    y2 = oracle.forward(w.x, w.W, tok, oracle.Adapters(w.adapter_rank + pad, w.adapter_scale, A2, B2))
    assert np.allclose(y2, y, rtol=1e-14, atol=1e-14)


def test_delora_identity():
    # mixture mode (section 4.4.1): with W_merge = W + s1 A1 B1, running a request of
    # adapter x through W_merge with the de-LoRA branch (-s1 A1 B1) plus its own
    # adapter reproduces x (W + s_x A_x B_x).
    rng = np.random.default_rng(11)
    T, K, N, r1, rx = 7, 24, 19, 4, 3
    x = rng.standard_normal((T, K)); W = rng.standard_normal((K, N))
    A1, B1 = rng.standard_normal((K, r1)), rng.standard_normal((r1, N))
    Ax, Bx = rng.standard_normal((K, rx)), rng.standard_normal((rx, N))
    s1, sx = 0.5, 2.0
    W_merge = W + s1 * (A1 @ B1)
    Acat = np.concatenate([Ax, A1], axis=1)
    Bcat = np.concatenate([sx * Bx, -s1 * B1], axis=0)
    tok = np.zeros(T, np.int32)
    mixed = oracle.forward(x, W_merge, tok, oracle.Adapters([rx + r1], [1.0], [Acat], [Bcat]))
    plain = oracle.forward(x, W, tok, oracle.Adapters([rx], [sx], [Ax], [Bx]))
    assert np.allclose(mixed, plain, rtol=1e-11, atol=1e-11)


def test_merge_mode_switch():
    # mode switch (section 4.4.2): W' = W + s A B.  Pinned to (i) the merged layer reproducing the
    # unmerged operator x W + s (x A) B computed by the C oracle (an independent code path), (ii) a closed
    # form for constant factors, (iii) merge followed by unmerge, (iv) entries worked by hand, with
    # non-square shapes so that a transposed factor cannot pass
    rng = np.random.default_rng(21)
    T, K, N, r, s = 9, 14, 11, 3, 1.75
    x = rng.standard_normal((T, K)); W = rng.standard_normal((K, N))
    A, B = rng.standard_normal((K, r)), rng.standard_normal((r, N))
    Wm = oracle.merge(W, A, B, s)
    tok = np.zeros(T, np.int32)
    unmerged = oracle.forward(x, W, tok, oracle.Adapters([r], [s], [A], [B]))
    assert np.allclose(oracle.base(x, Wm), unmerged, rtol=1e-12, atol=1e-12)
    # constant factors: (A B)[k, n] = r a b
    ones = oracle.merge(np.zeros((K, N)), np.full((K, r), 2.0), np.full((r, N), -0.5), 3.0)
    assert np.array_equal(ones, np.full((K, N), 3.0 * r * 2.0 * -0.5))
    # unmerge undoes merge (float64: to rounding), and sign = -1 is the same as a negated scale
    back = oracle.merge(Wm, A, B, s, sign=-1)
    assert np.allclose(back, W, rtol=0, atol=1e-13)
    assert np.array_equal(oracle.merge(W, A, B, s, sign=-1), oracle.merge(W, A, B, -s))
    # two entries by hand: W'[k, n] = W[k, n] + s sum_j A[k, j] B[j, n]
    for k, n in [(0, 0), (K - 1, N - 2)]:
        hand = W[k, n] + s * sum(A[k, j] * B[j, n] for j in range(r))
        assert abs(Wm[k, n] - hand) < 1e-13


def test_fast_expand_is_bitwise_literal_and_consistent_with_forward():
    w = _small(seed=12)
    ad = _adapters(w)
    tok = w.token_adapter()
    rng = np.random.default_rng(13)
    y_in = rng.standard_normal((w.T, w.N))
    lit = oracle.expand(w.x, tok, ad, w.N, y_in=y_in, literal=True)
    fast = oracle.expand(w.x, tok, ad, w.N, y_in=y_in)
    assert np.array_equal(lit, fast)
    # forward == expand applied onto the base output, bit for bit
    assert np.array_equal(oracle.forward(w.x, w.W, tok, ad),
                          oracle.expand(w.x, tok, ad, w.N, y_in=oracle.base(w.x, w.W)))
    # v feeds expand: delta = s * v_unscaled @ B
    v = oracle.shrink(w.x, tok, ad, apply_scale=False)
    d = oracle.expand(w.x, tok, ad, w.N)
    for t in range(w.T):
        a = tok[t]
        if a >= 0:
            r = w.adapter_rank[a]
            assert np.allclose(d[t], w.adapter_scale[a] * (v[t, :r] @ w.B[a].astype(np.float64)), rtol=1e-12, atol=1e-13)
        else:
            assert not d[t].any() and not v[t].any()


def test_against_pure_python_evaluation():
    w = wl.random_case(14, 6, 5, 4, 3, (1, 2, 3), dtype="f32", max_seg=2, frac_none=0.3,
                       scales=(0.5, 2.0, -1.0))
    tok = tiny.token_adapter(w.T, w.seg_indptr, w.seg_adapter)
    assert tok == oracle.token_adapter(w.T, w.seg_indptr, w.seg_adapter).tolist()
    y_py = np.array(tiny.forward(w.x.tolist(), w.W.tolist(), tok, w.adapter_rank.tolist(),
                                 w.adapter_scale.tolist(), [a.tolist() for a in w.A], [b.tolist() for b in w.B]))
    y_c = oracle.forward(w.x, w.W, np.array(tok, np.int32), _adapters(w))
    assert np.allclose(y_c, y_py, rtol=1e-13, atol=1e-14)


def test_transposed_operand_would_fail():
    # guards the pins themselves: a K x r / r x K mix-up changes the result on
    # a square adapter (where shapes alone would not catch it)
    rng = np.random.default_rng(15)
    T, K = 4, 6
    x = rng.standard_normal((T, K)); A = rng.standard_normal((K, K)); B = rng.standard_normal((K, K))
    tok = np.zeros(T, np.int32)
    good = oracle.expand(x, tok, oracle.Adapters([K], [1.0], [A], [B]), K)
    assert np.allclose(good, x @ A @ B, rtol=1e-12)
    assert not np.allclose(good, x @ A.T @ B, rtol=1e-3)
    assert not np.allclose(good, x @ A @ B.T, rtol=1e-3)
    assert not np.allclose(good, x @ B @ A, rtol=1e-3)


@settings(max_examples=200, deadline=None)
@given(st.lists(st.integers(0, 5), min_size=0, max_size=12), st.data())
def test_segment_arithmetic(lengths, data):
    S = len(lengths)
    T = sum(lengths)
    ads = data.draw(st.lists(st.integers(-1, 6), min_size=S, max_size=S))
    indptr = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32) if S else np.zeros(1, np.int32)
    if S == 0:
        assert oracle.token_adapter(0, indptr, []).shape[0] == 0
        return
    tok = oracle.token_adapter(T, indptr, ads)
    # same map by binary search on the boundaries
    seg = np.searchsorted(indptr, np.arange(T), side="right") - 1
    assert np.array_equal(tok, np.asarray(ads, np.int32)[seg]) if T else tok.shape[0] == 0
    assert tok.tolist() == tiny.token_adapter(T, indptr, ads)


def test_segment_table_errors():
    with pytest.raises(ValueError):
        oracle.token_adapter(4, [0, 2, 3], [0, 1])        # does not reach T
    with pytest.raises(ValueError):
        oracle.token_adapter(4, [0, 3, 2, 4], [0, 1, 2])  # decreasing
    with pytest.raises(ValueError):
        oracle.token_adapter(4, [1, 4], [0])              # does not start at 0


def test_numerical_budget_of_bf16_output():
    # rounding y once to bf16 (nearest-even) stays inside the stated tolerance
    w = wl.random_case(16, 64, 256, 192, 4, (8, 16), dtype="bf16", max_seg=16)
    y = oracle.forward(w.x, w.W, w.token_adapter(), _adapters(w))
    nrm, elem = oracle.error_metrics(wl.round_to_bf16(y.astype(np.float32)), y)
    assert nrm <= 2e-3 and elem <= 2.0 ** -8 * 1.01


def test_error_metrics_hand_worked_values():
    """The two error measures every parity verdict passes through, against values worked by hand.

    Reference [[3, 4], [0, 0.005]]: Frobenius norm sqrt(9 + 16 + 0.000025).  Candidate differs by
    (+0.3, -0.4, +1.0, +0.001): difference norm sqrt(0.09 + 0.16 + 1 + 0.000001).  Entries whose reference is
    at most the 1e-2 threshold (0 and 0.005) are left out of the elementwise measure, whatever their error
    (1.0 and 20 %), so it is max(0.3/3, 0.4/4) = 0.1."""
    ref = np.array([[3.0, 4.0], [0.0, 0.005]])
    got = ref + np.array([[0.3, -0.4], [1.0, 0.001]])
    nrm, elem = oracle.error_metrics(got, ref)
    assert nrm == pytest.approx(np.sqrt(1.250001) / np.sqrt(25.000025), rel=1e-14)
    assert elem == pytest.approx(0.1, rel=1e-12)
    # sign of the difference and of the reference do not matter; the denominator is |reference|, not |candidate|
    nrm2, elem2 = oracle.error_metrics(-got, -ref)
    assert (nrm2, elem2) == (nrm, elem)
    assert oracle.error_metrics(np.array([1.0]), np.array([2.0]))[1] == pytest.approx(0.5)     # not 1/1
    assert oracle.error_metrics(np.array([2.0]), np.array([1.0]))[1] == pytest.approx(1.0)
    # the threshold is strict and applies to |reference|: 0.01 itself is excluded, the next float is included
    above = np.nextafter(0.01, 1.0)
    assert oracle.error_metrics(np.array([0.02]), np.array([0.01]))[1] == 0.0
    assert oracle.error_metrics(np.array([2 * above]), np.array([above]))[1] == pytest.approx(1.0)
    assert oracle.error_metrics(np.array([-0.03]), np.array([-above]))[1] == pytest.approx(2.0, rel=1e-6)
    # an entry just under and just over the 1e-2 elementwise tolerance, at a reference value of 0.5
    _, under = oracle.error_metrics(np.array([0.5 * (1 + 0.0099)]), np.array([0.5]))
    _, over = oracle.error_metrics(np.array([0.5 * (1 - 0.0101)]), np.array([0.5]))
    assert under == pytest.approx(0.0099, rel=1e-9) and under <= 1e-2 < over == pytest.approx(0.0101, rel=1e-9)
    # the same for the normwise tolerance 2e-3: a single wrong entry of 100 equal ones, error e -> e / 10
    ref = np.ones((10, 10))
    got = ref.copy()
    got[3, 7] += 0.0199
    assert oracle.error_metrics(got, ref)[0] == pytest.approx(0.00199, rel=1e-9)
    got[3, 7] = 1.0201
    assert oracle.error_metrics(got, ref)[0] > 2e-3
    # zero-norm reference: the normwise measure falls back to the absolute norm of the difference (no division
    # by zero, and a wrong candidate does not pass as 0); nothing is above the threshold, so elementwise is 0
    nrm0, elem0 = oracle.error_metrics(np.array([[0.0, 3.0], [4.0, 0.0]]), np.zeros((2, 2)))
    assert nrm0 == 5.0 and elem0 == 0.0
    assert oracle.error_metrics(np.zeros((2, 2)), np.zeros((2, 2))) == (0.0, 0.0)
    # float32 / bf16-like inputs are widened, not compared in their own precision
    a32 = np.array([1.0 + 2.0 ** -20], dtype=np.float32)
    assert oracle.error_metrics(a32, np.array([1.0]))[0] == 2.0 ** -20
    # a custom threshold moves the mask only
    assert oracle.error_metrics(np.array([0.002, 1.0]), np.array([0.001, 1.0]), threshold=1e-4)[1] == pytest.approx(1.0)
