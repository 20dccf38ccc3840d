"""Pins for the CPU oracle: everything here checks oracle/ against facts that do not come from it
(closed forms, library routines on special cases, exact rational arithmetic, hand-worked tables,
multilinearity).  The paper prints no worked numeric example of the contraction, so there is no
golden file from it; the formula is LoRA's (cited in Section 1) batched as Section 3.3 describes."""
from fractions import Fraction

import numpy as np
import pytest

from paper_2511_00101_amd import synth

pytestmark = pytest.mark.filterwarnings("ignore")


def f64(bits):
    return synth.bf16_bits_to_f64(bits)


def grid_bits(rng, shape, lo=-128, hi=128, denom=64.0):
    """bf16-exact values k/denom with |k| <= 128 (8 significant bits)."""
    v = rng.integers(lo, hi + 1, size=shape).astype(np.float32) / np.float32(denom)
    bits = synth.f32_to_bf16_bits(v)
    assert np.array_equal(synth.bf16_bits_to_f32(bits), v)
    return bits


def run_forward(oracle_mod, p):
    return oracle_mod.forward(p.x, p.y0, p.A, p.B, p.ranks, p.scales, p.batch.token_adapter, p.batch.token_kind)


# ---------------------------------------------------------------------------------------------
# bf16 decoding inside the oracle, against numpy's reinterpretation of the same bits
# ---------------------------------------------------------------------------------------------
def test_bf16_decode_all_finite_patterns(oracle_mod):
    bits = np.arange(65536, dtype=np.uint32)
    finite = ((bits >> 7) & 0xFF) != 0xFF
    bits = bits[finite].astype(np.uint16)
    T = bits.shape[0]
    one = synth.f32_to_bf16_bits(np.ones((1, 1), np.float32))
    res = oracle_mod.forward(bits.reshape(T, 1), np.zeros((T, 1), np.uint16), [one], [one], [1], [1.0],
                             np.zeros(T, np.int32), np.full(T, 1, np.uint8))
    expect = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.array_equal(res.y[:, 0], expect)


# ---------------------------------------------------------------------------------------------
# closed forms of the forward
# ---------------------------------------------------------------------------------------------
def test_zero_B_leaves_y_unchanged(oracle_mod):
    p = synth.small_mixed(1, T=37, d_in=24, d_out=40, ranks=[4, 8, 3], drop_frac=0.2)
    p.B = [np.zeros_like(b) for b in p.B]
    res = run_forward(oracle_mod, p)
    assert np.array_equal(res.y, f64(p.y0))


def test_single_adapter_equals_dense_matmul(oracle_mod):
    rng = np.random.default_rng(5)
    T, d_in, d_out, r, s = 50, 96, 72, 8, 1.75
    x, y0 = synth.normal_bf16(rng, (T, d_in), 1.0), synth.normal_bf16(rng, (T, d_out), 1.0)
    A, B = synth.normal_bf16(rng, (r, d_in), 0.02), synth.normal_bf16(rng, (r, d_out), 0.02)
    kinds = rng.integers(0, 3, size=T).astype(np.uint8)
    res = oracle_mod.forward(x, y0, [A], [B], [r], [s], np.zeros(T, np.int32), kinds)
    expect = f64(y0) + s * (f64(x) @ f64(A).T) @ f64(B)
    np.testing.assert_allclose(res.y, expect, rtol=1e-12, atol=1e-13)


def test_transposed_operands_would_fail(oracle_mod):
    """Guards the layout reading (A is [r, d_in], B is [r, d_out]) with non-square, non-symmetric shapes:
    the dense form with either operand transposed differently does not even have matching shapes, and
    with d_in == d_out it gives a different answer."""
    rng = np.random.default_rng(6)
    T, d, r = 9, 16, 16
    x, y0 = synth.normal_bf16(rng, (T, d), 1.0), np.zeros((T, d), np.uint16)
    A, B = synth.normal_bf16(rng, (r, d), 1.0), synth.normal_bf16(rng, (r, d), 1.0)
    res = oracle_mod.forward(x, y0, [A], [B], [r], [1.0], np.zeros(T, np.int32), np.ones(T, np.uint8))
    good = (f64(x) @ f64(A).T) @ f64(B)
    bad = (f64(x) @ f64(A)) @ f64(B).T
    np.testing.assert_allclose(res.y, good, rtol=1e-12, atol=1e-12)
    assert np.abs(res.y - bad).max() > 1.0


def test_rank1_is_outer_product(oracle_mod):
    rng = np.random.default_rng(7)
    T, d_in, d_out = 11, 33, 29
    p_x, p_y0 = synth.normal_bf16(rng, (T, d_in), 1.0), synth.normal_bf16(rng, (T, d_out), 1.0)
    a, b = synth.normal_bf16(rng, (1, d_in), 0.5), synth.normal_bf16(rng, (1, d_out), 0.5)
    s = 3.0
    res = oracle_mod.forward(p_x, p_y0, [a], [b], [1], [s], np.zeros(T, np.int32), np.full(T, 2, np.uint8))
    X, Y0, av, bv = f64(p_x), f64(p_y0), f64(a)[0], f64(b)[0]
    for t in range(T):
        dot = sum(X[t, k] * av[k] for k in range(d_in))
        for n in range(d_out):
            assert res.y[t, n] == pytest.approx(Y0[t, n] + s * dot * bv[n], rel=1e-13, abs=1e-14)


def test_token_permutation_invariance_is_bit_exact(oracle_mod):
    p = synth.small_mixed(11, T=61, d_in=48, d_out=56, ranks=[2, 16, 5, 8], drop_frac=0.1)
    base = run_forward(oracle_mod, p)
    rng = np.random.default_rng(12)
    order = rng.permutation(p.n_tokens)
    res = oracle_mod.forward(p.x[order], p.y0[order], p.A, p.B, p.ranks, p.scales,
                             p.batch.token_adapter[order], p.batch.token_kind[order])
    assert np.array_equal(res.y, base.y[order])
    # adapters listed in another order (ids remapped) give the same rows as well
    remap = rng.permutation(p.n_adapters)            # new id of old adapter i is remap[i]
    inv = np.argsort(remap)
    ta = p.batch.token_adapter.copy()
    live = ta >= 0
    ta[live] = remap[ta[live]]
    res2 = oracle_mod.forward(p.x, p.y0, [p.A[i] for i in inv], [p.B[i] for i in inv], p.ranks[inv], p.scales[inv],
                              ta, p.batch.token_kind)
    assert np.array_equal(res2.y, base.y)


def test_exact_rational_brute_force(oracle_mod):
    """Tiny shapes, bf16-exact grid inputs, exact arithmetic with fractions: the fp64 oracle must be
    within a few ulp of the exact value (all products and sums here are in fact exactly representable)."""
    rng = np.random.default_rng(21)
    T, d_in, d_out = 7, 6, 5
    ranks = [1, 3, 2]
    scales = [0.5, 2.0, -1.25]
    x, y0 = grid_bits(rng, (T, d_in)), grid_bits(rng, (T, d_out))
    A = [grid_bits(rng, (r, d_in)) for r in ranks]
    B = [grid_bits(rng, (r, d_out)) for r in ranks]
    ta = np.array([2, 0, -1, 1, 1, 0, 2], np.int32)
    tk = np.array([0, 2, 1, 0, 1, 2, 0], np.uint8)
    res = oracle_mod.forward(x, y0, A, B, ranks, scales, ta, tk)
    Fx = [[Fraction(float(v)) for v in row] for row in synth.bf16_bits_to_f32(x)]
    Fy = [[Fraction(float(v)) for v in row] for row in synth.bf16_bits_to_f32(y0)]
    FA = [[[Fraction(float(v)) for v in row] for row in synth.bf16_bits_to_f32(a)] for a in A]
    FB = [[[Fraction(float(v)) for v in row] for row in synth.bf16_bits_to_f32(b)] for b in B]
    for t in range(T):
        a = int(ta[t])
        for n in range(d_out):
            exact = Fy[t][n]
            if a >= 0:
                upd = Fraction(0)
                for j in range(ranks[a]):
                    hj = sum(Fx[t][k] * FA[a][j][k] for k in range(d_in))
                    upd += hj * FB[a][j][n]
                exact += Fraction(scales[a]) * upd
            assert abs(Fraction(res.y[t, n]) - exact) <= abs(exact) * Fraction(1, 2 ** 50)
    # saved h of the fine-tune tokens, exact as well; layout: (kind 0, adapter 1) rows first, then adapter 2
    #   token 3 -> adapter 1 (rank 3) at offset 0; tokens 0 and 6 -> adapter 2 (rank 2) at offsets 3 and 5
    expect_h = []
    for t, a in ((3, 1), (0, 2), (6, 2)):
        for j in range(ranks[a]):
            expect_h.append(sum(Fx[t][k] * FA[a][j][k] for k in range(d_in)))
    assert res.h.shape[0] == len(expect_h) == 7
    for got, ex in zip(res.h, expect_h):
        assert Fraction(got) == ex


def test_rows_without_adapter_and_empty_batch(oracle_mod):
    p = synth.small_mixed(31, T=20, d_in=16, d_out=24, ranks=[4, 4], drop_frac=0.5)
    res = run_forward(oracle_mod, p)
    dead = p.batch.token_adapter < 0
    assert dead.any() and (~dead).any()
    assert np.array_equal(res.y[dead], f64(p.y0)[dead])
    assert not np.array_equal(res.y[~dead], f64(p.y0)[~dead])
    # adapter ids beyond the table and unknown kinds are treated like "no adapter"
    ta = p.batch.token_adapter.copy()
    tk = p.batch.token_kind.copy()
    ta[0], tk[1] = 2, 3
    ta[1] = 0
    res2 = oracle_mod.forward(p.x, p.y0, p.A, p.B, p.ranks, p.scales, ta, tk)
    assert np.array_equal(res2.y[:2], f64(p.y0)[:2])
    empty = oracle_mod.forward(np.zeros((0, 16), np.uint16), np.zeros((0, 24), np.uint16), p.A, p.B, p.ranks, p.scales,
                               np.zeros(0, np.int32), np.zeros(0, np.uint8))
    assert empty.y.shape == (0, 24) and empty.h.shape == (0,) and empty.segments.n_segments == 0


def test_scale_linearity(oracle_mod):
    p = synth.small_mixed(41, T=33, d_in=40, d_out=24, ranks=[8, 2, 5], scales=[1.0, 0.5, 4.0])
    r1 = run_forward(oracle_mod, p)
    p.scales = p.scales * np.float32(2.0)
    r2 = run_forward(oracle_mod, p)
    y0 = f64(p.y0)
    np.testing.assert_allclose(r2.y - y0, 2.0 * (r1.y - y0), rtol=1e-12, atol=1e-13)
    assert np.array_equal(r1.h, r2.h)          # the saved h is unscaled


def test_saved_h_layout_and_values(oracle_mod):
    """h rows of fine-tune tokens sit at offsets given by an independent reconstruction of the metadata
    (Python's stable sort), with values x A^T from a library matmul."""
    p = synth.small_mixed(51, T=70, d_in=32, d_out=16, ranks=[3, 8, 1, 16], drop_frac=0.15)
    res = run_forward(oracle_mod, p)
    ta, tk = p.batch.token_adapter, p.batch.token_kind
    order = sorted((t for t in range(p.n_tokens) if ta[t] >= 0), key=lambda t: (int(tk[t]), int(ta[t])))
    X = f64(p.x)
    expect = []
    for t in order:
        if tk[t] == synth.KIND_FINETUNE:
            expect.extend((X[t] @ f64(p.A[ta[t]]).T).tolist())
    np.testing.assert_allclose(res.h, np.asarray(expect), rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------------------------------------
# segment metadata
# ---------------------------------------------------------------------------------------------
def python_segments(ta, tk, ranks):
    n_ad = len(ranks)
    live = [t for t in range(len(ta)) if 0 <= ta[t] < n_ad and tk[t] <= 2]
    order = sorted(live, key=lambda t: (int(tk[t]), int(ta[t])))   # sorted() is stable
    starts, sad, skd, hoff = [0], [], [], [0]
    for i, t in enumerate(order):
        if i + 1 == len(order) or (tk[order[i + 1]], ta[order[i + 1]]) != (tk[t], ta[t]):
            sad.append(int(ta[t]))
            skd.append(int(tk[t]))
            length = i + 1 - starts[-1]
            hoff.append(hoff[-1] + (length * int(ranks[ta[t]]) if tk[t] == 0 else 0))
            starts.append(i + 1)
    return order, starts, sad, skd, hoff


def test_segments_hand_worked_example(oracle_mod):
    """Worked by hand from the definition: batch order fine-tune | prefill | decode (Algorithm 1), grouped by
    adapter inside a kind, ties in original token order."""
    #            t: 0  1  2  3  4   5  6  7  8  9 10 11
    ta = np.array([1, 0, 1, -1, 0,  2, 1, 0, 2, 0, 1, 5], np.int32)
    tk = np.array([2, 0, 0, 0,  1,  2, 0, 2, 2, 0, 2, 0], np.uint8)
    ranks = np.array([4, 8, 2], np.int32)     # adapter 5 does not exist -> token 11 is dropped, as is token 3
    seg = oracle_mod.build_segments(ta, tk, ranks)
    assert seg.perm.tolist() == [1, 9, 2, 6, 4, 7, 0, 10, 5, 8]
    assert seg.seg_starts.tolist() == [0, 2, 4, 5, 6, 8, 10]
    assert seg.seg_adapter.tolist() == [0, 1, 0, 0, 1, 2]
    assert seg.seg_kind.tolist() == [0, 0, 1, 2, 2, 2]
    assert seg.h_offsets.tolist() == [0, 8, 24, 24, 24, 24, 24]


@pytest.mark.parametrize("seed", range(6))
def test_segments_match_library_stable_sort(oracle_mod, seed):
    rng = np.random.default_rng(100 + seed)
    T = int(rng.integers(0, 400))
    n_ad = int(rng.integers(1, 40))
    ranks = rng.integers(1, 65, size=n_ad).astype(np.int32)
    ta = rng.integers(-1, n_ad + 1, size=T).astype(np.int32)
    tk = rng.integers(0, 4, size=T).astype(np.uint8)
    seg = oracle_mod.build_segments(ta, tk, ranks)
    order, starts, sad, skd, hoff = python_segments(ta, tk, ranks)
    assert seg.perm.tolist() == order
    assert seg.seg_starts.tolist() == starts
    assert seg.seg_adapter.tolist() == sad
    assert seg.seg_kind.tolist() == skd
    assert seg.h_offsets.tolist() == hoff


def test_config1_structure(oracle_mod):
    p = synth.config1()
    seg = oracle_mod.build_segments(p.batch.token_adapter, p.batch.token_kind, p.ranks)
    assert p.n_tokens == 102
    assert seg.seg_starts[:3].tolist() == [0, 64, 96] and seg.seg_kind[:2].tolist() == [0, 1]
    assert seg.perm[:96].tolist() == list(range(96))
    assert seg.h_offsets[1:].tolist() == [64 * 8] * seg.n_segments
    assert sorted(seg.perm.tolist()) == list(range(102))


# ---------------------------------------------------------------------------------------------
# dynamic per-request scale (Section 3.3): a per-token array that replaces the per-adapter scale
# ---------------------------------------------------------------------------------------------
def test_token_scale_single_adapter_is_dense_matmul_with_a_diagonal(oracle_mod):
    rng = np.random.default_rng(15)
    T, d_in, d_out, r = 45, 80, 56, 8
    x, y0 = synth.normal_bf16(rng, (T, d_in), 1.0), synth.normal_bf16(rng, (T, d_out), 1.0)
    A, B = synth.normal_bf16(rng, (r, d_in), 0.02), synth.normal_bf16(rng, (r, d_out), 0.02)
    ts = rng.uniform(-2.0, 3.0, size=T).astype(np.float32)
    res = oracle_mod.forward(x, y0, [A], [B], [r], [123.0], np.zeros(T, np.int32), np.zeros(T, np.uint8), token_scales=ts)
    expect = f64(y0) + np.diag(ts.astype(np.float64)) @ (f64(x) @ f64(A).T) @ f64(B)
    np.testing.assert_allclose(res.y, expect, rtol=1e-12, atol=1e-12)
    # a transposed or misplaced diagonal (scale indexed by column) gives something else
    wrong = f64(y0) + (f64(x) @ f64(A).T) @ f64(B) * np.resize(ts, d_out).astype(np.float64)[None, :]
    assert np.abs(res.y - wrong).max() > 1e-3
    # the saved h stays unscaled
    np.testing.assert_allclose(res.h.reshape(T, r), f64(x) @ f64(A).T, rtol=1e-12, atol=1e-12)


def test_token_scale_agrees_with_adapter_scale_and_is_row_wise_linear(oracle_mod):
    p = synth.small_mixed(8, T=40, d_in=32, d_out=24, ranks=[4, 8, 2], drop_frac=0.15)
    base = run_forward(oracle_mod, p)
    ta = p.batch.token_adapter
    same = np.where(ta >= 0, p.scales[np.maximum(ta, 0)], 77.0).astype(np.float32)
    res = oracle_mod.forward(p.x, p.y0, p.A, p.B, p.ranks, p.scales, ta, p.batch.token_kind, token_scales=same)
    assert np.array_equal(res.y, base.y) and np.array_equal(res.h, base.h)
    # doubling one token's scale doubles that row's update and leaves every other row alone (powers of two: exact)
    t = int(np.flatnonzero(ta >= 0)[3])
    bumped = same.copy()
    bumped[t] *= 2.0
    res2 = oracle_mod.forward(p.x, p.y0, p.A, p.B, p.ranks, p.scales, ta, p.batch.token_kind, token_scales=bumped)
    y0 = f64(p.y0)
    others = np.arange(p.n_tokens) != t
    assert np.array_equal(res2.y[others], base.y[others])
    np.testing.assert_allclose(res2.y[t] - y0[t], 2.0 * (base.y[t] - y0[t]), rtol=1e-12, atol=1e-15)
    # rows without an adapter ignore their scale
    dead = ta < 0
    assert dead.any() and np.array_equal(res.y[dead], y0[dead])


# ---------------------------------------------------------------------------------------------
# backward
# ---------------------------------------------------------------------------------------------
def loss_of(oracle_mod, x, y0, A, B, ranks, scales, ta, tk, dy, token_scales=None):
    res = oracle_mod.forward(x, y0, A, B, ranks, scales, ta, tk, token_scales=token_scales)
    ft = (tk == 0) & (ta >= 0)
    return float(np.sum(f64(dy)[ft] * res.y[ft]))


@pytest.mark.parametrize("per_token", [False, True])
def test_backward_against_exact_differences(oracle_mod, per_token):
    """L = sum dy*y over fine-tune rows is linear in each single input element, so a one-sided difference
    with a bf16-representable step is exact: L(e + delta) - L(e) = delta * dL/de.  With per_token the scale is
    the dynamic per-token one (values k/8, exact)."""
    rng = np.random.default_rng(61)
    T, d_in, d_out = 10, 7, 6
    ranks = np.array([2, 3], np.int32)
    scales = np.array([0.75, -1.5], np.float32)
    x, y0, dy = grid_bits(rng, (T, d_in), -64, 64), grid_bits(rng, (T, d_out)), grid_bits(rng, (T, d_out), -64, 64)
    A = [grid_bits(rng, (int(r), d_in), -64, 64) for r in ranks]
    B = [grid_bits(rng, (int(r), d_out), -64, 64) for r in ranks]
    ta = np.array([0, 1, 1, 0, -1, 1, 0, 0, 1, 1], np.int32)
    tk = np.array([0, 0, 1, 0, 0, 2, 0, 1, 0, 0], np.uint8)
    ts = (rng.integers(-16, 17, size=T) / 8.0).astype(np.float32) if per_token else None
    bw = oracle_mod.backward(x, dy, None, A, B, ranks, scales, ta, tk, token_scales=ts)
    L0 = loss_of(oracle_mod, x, y0, A, B, ranks, scales, ta, tk, dy, ts)
    delta = 1.0 / 64.0

    def bump(bits, idx):
        v = synth.bf16_bits_to_f32(bits).copy()
        v[idx] += np.float32(delta)
        out = synth.f32_to_bf16_bits(v)
        assert synth.bf16_bits_to_f32(out)[idx] == v[idx]
        return out

    for a in range(2):
        for j in range(int(ranks[a])):
            for k in range(d_in):
                A2 = list(A)
                A2[a] = bump(A[a], (j, k))
                d = loss_of(oracle_mod, x, y0, A2, B, ranks, scales, ta, tk, dy, ts) - L0
                assert d == pytest.approx(delta * bw.dA[a][j, k], rel=1e-9, abs=1e-9)
            for n in range(d_out):
                B2 = list(B)
                B2[a] = bump(B[a], (j, n))
                d = loss_of(oracle_mod, x, y0, A, B2, ranks, scales, ta, tk, dy, ts) - L0
                assert d == pytest.approx(delta * bw.dB[a][j, n], rel=1e-9, abs=1e-9)
    for t in range(T):
        for k in range(d_in):
            d = loss_of(oracle_mod, bump(x, (t, k)), y0, A, B, ranks, scales, ta, tk, dy, ts) - L0
            assert d == pytest.approx(delta * bw.dx[t, k], rel=1e-9, abs=1e-9)
    assert np.abs(bw.dA[0]).max() > 0 and np.abs(bw.dB[1]).max() > 0 and np.abs(bw.dx).max() > 0
    # rows that are not fine-tune rows get no gradient
    assert np.all(bw.dx[(tk != 0) | (ta < 0)] == 0.0)


def test_backward_single_adapter_dense_form(oracle_mod):
    rng = np.random.default_rng(71)
    T, d_in, d_out, r, s = 40, 48, 36, 8, 2.0
    x, dy, dx0 = (synth.normal_bf16(rng, (T, d_in), 1.0), synth.normal_bf16(rng, (T, d_out), 1.0),
                  synth.normal_bf16(rng, (T, d_in), 1.0))
    A, B = synth.normal_bf16(rng, (r, d_in), 0.02), synth.normal_bf16(rng, (r, d_out), 0.02)
    bw = oracle_mod.backward(x, dy, dx0, [A], [B], [r], [s], np.zeros(T, np.int32), np.zeros(T, np.uint8))
    X, DY, Af, Bf = f64(x), f64(dy), f64(A), f64(B)
    G = DY @ Bf.T
    np.testing.assert_allclose(bw.dB[0], s * (X @ Af.T).T @ DY, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(bw.dA[0], s * G.T @ X, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(bw.dx, f64(dx0) + s * G @ Af, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(bw.g, G.reshape(-1), rtol=1e-11, atol=1e-12)


def test_backward_token_scale_single_adapter_dense_form(oracle_mod):
    rng = np.random.default_rng(73)
    T, d_in, d_out, r = 30, 40, 28, 4
    x, dy, dx0 = (synth.normal_bf16(rng, (T, d_in), 1.0), synth.normal_bf16(rng, (T, d_out), 1.0),
                  synth.normal_bf16(rng, (T, d_in), 1.0))
    A, B = synth.normal_bf16(rng, (r, d_in), 0.02), synth.normal_bf16(rng, (r, d_out), 0.02)
    ts = rng.uniform(-1.0, 2.0, size=T).astype(np.float32)
    bw = oracle_mod.backward(x, dy, dx0, [A], [B], [r], [9.0], np.zeros(T, np.int32), np.zeros(T, np.uint8), token_scales=ts)
    X, DY, Af, Bf, S = f64(x), f64(dy), f64(A), f64(B), np.diag(ts.astype(np.float64))
    G = DY @ Bf.T
    np.testing.assert_allclose(bw.dB[0], (X @ Af.T).T @ S @ DY, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(bw.dA[0], G.T @ S @ X, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(bw.dx, f64(dx0) + S @ G @ Af, rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------------------------------------
# LoRA dropout on the fine-tuning rows (training configurations of the appendix: lora_dropout 0.05); the mask is a
# contract of this library (a counter-based hash), so what is pinned is what the mathematics fixes: independent
# Bernoulli(1 - p) elements, the same for the same (seed, row, column), and rows of other kinds untouched
# ---------------------------------------------------------------------------------------------
def test_dropout_mask_statistics(oracle_mod):
    T, d, p = 400, 1024, 0.05
    x = np.full((T, d), 0x3F80, np.uint16)                      # 1.0 everywhere
    ta, tk = np.zeros(T, np.int32), np.zeros(T, np.uint8)
    m = oracle_mod.dropout_rows(x, ta, tk, 1, seed=1234, p=p) != 0
    n = T * d
    sigma = np.sqrt(p * (1 - p) / n)
    assert abs((1.0 - m.mean()) - oracle_mod.dropout_threshold(p) / 65536.0) < 5 * sigma
    # every row and every column has about the same rate (no dead or stuck rows / columns)
    assert np.abs((1 - m.mean(axis=1)) - p).max() < 6 * np.sqrt(p * (1 - p) / d)
    assert np.abs((1 - m.mean(axis=0)) - p).max() < 6 * np.sqrt(p * (1 - p) / T)
    # neighbours are uncorrelated: along a row (also across the two 16-bit fields of a word), down a column, diagonally
    z = (m.astype(np.float64) - m.mean()) / m.std()
    for a, b in ((z[:, :-1], z[:, 1:]), (z[:, :-2], z[:, 2:]), (z[:-1, :], z[1:, :]), (z[:-1, :-1], z[1:, 1:]),
                 (z[:, 0::2], z[:, 1::2])):
        assert abs(float((a * b).mean())) < 5.0 / np.sqrt(a.size)
    # another seed gives another, equally uncorrelated mask
    m2 = oracle_mod.dropout_rows(x, ta, tk, 1, seed=1235, p=p) != 0
    z2 = (m2.astype(np.float64) - m2.mean()) / m2.std()
    assert abs(float((z * z2).mean())) < 5.0 / np.sqrt(n)
    assert (m != m2).mean() > p                                   # (about 2 p (1 - p) of the elements differ)


def test_dropout_rates_and_determinism(oracle_mod):
    T, d = 64, 4096
    x = np.full((T, d), 0x3F80, np.uint16)
    ta, tk = np.zeros(T, np.int32), np.zeros(T, np.uint8)
    for p in (0.0, 0.01, 0.05, 0.5, 0.9):
        m = oracle_mod.dropout_rows(x, ta, tk, 1, seed=7, p=p) != 0
        assert abs((1.0 - m.mean()) - p) < 5 * np.sqrt(max(p * (1 - p), 1e-9) / (T * d)) + 1.0 / 65536
        if p == 0.0:
            assert m.all()
        assert np.array_equal(m, oracle_mod.dropout_rows(x, ta, tk, 1, seed=7, p=p) != 0)
        # the element-wise entry point is the same function
        for (t, k) in ((0, 0), (3, 1), (17, 4095), (63, 2048)):
            assert oracle_mod.dropout_keep(7, t, k, oracle_mod.dropout_threshold(p)) == bool(m[t, k])
    # the mask of a row does not depend on what else is in the batch: row t of a longer batch
    big = oracle_mod.dropout_rows(np.full((2 * T, d), 0x3F80, np.uint16), np.zeros(2 * T, np.int32), np.zeros(2 * T, np.uint8),
                                  1, seed=7, p=0.05) != 0
    assert np.array_equal(big[:T], oracle_mod.dropout_rows(x, ta, tk, 1, seed=7, p=0.05) != 0)


def test_dropout_touches_fine_tune_rows_only_and_keeps_values(oracle_mod):
    p = synth.small_mixed(5, T=60, d_in=64, d_out=8, ranks=[4, 4], drop_frac=0.2)
    out = oracle_mod.dropout_rows(p.x, p.batch.token_adapter, p.batch.token_kind, p.n_adapters, seed=99, p=0.3)
    ft = (p.batch.token_kind == 0) & (p.batch.token_adapter >= 0)
    assert np.array_equal(out[~ft], p.x[~ft])
    kept = out[ft] != 0
    assert np.array_equal(out[ft][kept], p.x[ft][kept])           # kept elements are bit-identical
    assert 0.15 < 1.0 - kept.mean() < 0.45


# ---------------------------------------------------------------------------------------------
# Algorithm 1's row split by kind and concatenation
# ---------------------------------------------------------------------------------------------
def test_kind_offsets_split_and_concat(oracle_mod):
    rng = np.random.default_rng(2)
    ta = np.array([1, 0, -1, 2, 0, 1, 2, 2, 0, -1, 1], np.int32)
    tk = np.array([2, 0, 0, 1, 2, 0, 1, 2, 0, 1, 2], np.uint8)
    seg = oracle_mod.build_segments(ta, tk, np.array([4, 4, 4], np.int32))
    off = oracle_mod.kind_offsets(seg)
    live = ta >= 0
    assert off.tolist() == [0, int((live & (tk == 0)).sum()), int((live & (tk <= 1)).sum()), int(live.sum())]
    src = rng.integers(0, 65536, size=(len(ta), 6)).astype(np.uint16)
    parts = oracle_mod.split_rows(src, seg)
    # every kind's part holds exactly the rows of that kind (by hand: numpy masks), in (adapter, token) order
    for c in range(3):
        want_rows = sorted(np.flatnonzero(live & (tk == c)), key=lambda t: (ta[t], t))
        assert np.array_equal(parts[off[c]: off[c + 1]], src[want_rows])
    # concatenation is the inverse on the live rows and leaves the other rows alone
    dst0 = rng.integers(0, 65536, size=src.shape).astype(np.uint16)
    back = oracle_mod.concat_rows(parts, seg, dst0)
    assert np.array_equal(back[live], src[live]) and np.array_equal(back[~live], dst0[~live])
    # a batch without prefill rows: the prefill part is empty and starts where the decode part starts
    seg2 = oracle_mod.build_segments(ta, np.where(tk == 1, 2, tk).astype(np.uint8), np.array([4, 4, 4], np.int32))
    off2 = oracle_mod.kind_offsets(seg2)
    assert off2[1] == off2[2] and off2[3] == int(live.sum())
