"""Pins for the oracle's dropout on the attention weights (Section 2.2 names a dropout beside the softmax
in the normalisation of the scores; read as softmax, then inverted dropout on the weights).

What fixes the right answer: p = 0 is the pinned no-dropout oracle; the keep decision depends on
positions in the whole sequence, so segments still concatenate to the sequential result (Section
3, Principle 3); the 1/(1-p) scaling makes the output unbiased over seeds; with the mask held
fixed the function is smooth, so central differences fix the backward; and the mask itself has
the statistics of independent coin flips."""
import numpy as np
import pytest

import oracle
from paper_2311_02382_amd import synth


def _inputs(B, l_x, H, d, seed):
    q, k, v, do = synth.make_inputs(B, l_x, H, d, seed)
    return q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), do.astype(np.float64)


def test_p_zero_is_the_plain_oracle():
    q, k, v, do = _inputs(2, 40, 2, 8, 21)
    for s0, l_s in ((0, 40), (13, 9)):
        a = oracle.segment_fwd(q[:, s0:s0 + l_s], k, v, s0, True)
        b = oracle.segment_fwd_dropout(q[:, s0:s0 + l_s], k, v, s0, True, 0.0, 99)
        assert all(np.array_equal(x, y) for x, y in zip(a, b))
        a = oracle.segment_bwd(q[:, s0:s0 + l_s], k, v, do[:, s0:s0 + l_s], s0, True)
        b = oracle.segment_bwd_dropout(q[:, s0:s0 + l_s], k, v, do[:, s0:s0 + l_s], s0, True, 0.0, 99)
        assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert oracle.dropout_mask(0.0, 5, 0, 7, 33, 1, 2).all()


@pytest.mark.parametrize("p", [0.1, 0.25, 0.5, 0.9])
def test_mask_has_the_statistics_of_independent_coin_flips(p):
    B, H, l_x = 2, 3, 512
    m = oracle.dropout_mask(p, 0x1234_5678_9ABC_DEF0, 0, l_x, l_x, B, H).astype(np.float64)
    n = m.size
    sigma = np.sqrt(p * (1 - p) / n)
    assert abs(m.mean() - (1 - p)) < 5 * sigma
    # every row, column, head and batch entry on its own
    for axis, cnt in ((3, l_x), (2, l_x)):
        frac = m.mean(axis=axis)
        assert np.abs(frac - (1 - p)).max() < 6 * np.sqrt(p * (1 - p) / cnt)
    # no correlation between neighbours along any axis
    c = m - m.mean()
    var = (c * c).mean()
    for a, b in ((c[..., 1:], c[..., :-1]), (c[:, :, 1:], c[:, :, :-1]), (c[:, 1:], c[:, :-1]), (c[1:], c[:-1]),
                 (c[:, :, 1:, 1:], c[:, :, :-1, :-1]), (c[:, :, 1:, :-1], c[:, :, :-1, 1:])):
        assert abs((a * b).mean() / var) < 5 / np.sqrt(a.size)
    # transposing the roles of row and column gives another mask
    assert abs((c * c.transpose(0, 1, 3, 2)).mean() / var) < 0.02


@pytest.mark.parametrize("p", [0.1, 0.5, 0.75])
def test_rectangles_of_the_mask_are_not_tied_together(p):
    # The random number of a weight is a mix of (row key + column key): a SEPARABLE input.  If the
    # final mix were weak, the four corners of a rectangle (r1, c1), (r1, c2), (r2, c1), (r2, c2) would
    # be tied -- e.g. keep = f(row) xor g(col) gives parity 0 for every rectangle.  For independent coin
    # flips that keep with probability s = 1 - p, the parity of four of them is odd with probability
    # (1 - (2s - 1)^4) / 2.  Checked over all rectangles built from neighbouring and from distant rows
    # and columns, per (batch, head).
    B, H, l_x = 2, 2, 384
    m = oracle.dropout_mask(p, 0x0BAD_5EED_0000_0042, 0, l_x, l_x, B, H).astype(np.int64)
    s_keep = 1.0 - p
    expect = (1.0 - (2.0 * s_keep - 1.0) ** 4) / 2.0
    for dr, dc in ((1, 1), (1, 7), (5, 1), (64, 64), (191, 3), (2, 190)):
        par = (m[:, :, :-dr, :-dc] + m[:, :, dr:, :-dc] + m[:, :, :-dr, dc:] + m[:, :, dr:, dc:]) & 1
        n = par.size
        # overlapping rectangles share corners, so their parities are only pairwise weakly dependent:
        # allow 8 standard deviations of the independent case
        assert abs(par.mean() - expect) < 8 * np.sqrt(expect * (1 - expect) / n), (dr, dc, par.mean(), expect)
    # and the same for rectangles that span two heads (same rows and columns, other batch*head key)
    par = (m[0, 0, :-1, :-1] + m[0, 0, 1:, 1:] + m[1, 1, :-1, :-1] + m[1, 1, 1:, 1:]) & 1
    assert abs(par.mean() - expect) < 8 * np.sqrt(expect * (1 - expect) / par.size)


def test_mask_depends_on_every_part_of_its_key():
    p, l_x = 0.5, 256
    base = oracle.dropout_mask(p, 7, 0, l_x, l_x, 2, 2)
    for seed in (8, 7 + (1 << 32), 7 + (1 << 63)):           # low and high halves of the seed
        other = oracle.dropout_mask(p, seed, 0, l_x, l_x, 2, 2)
        assert 0.4 < (other != base).mean() < 0.6
    flat = base.reshape(4, l_x, l_x)
    for i in range(4):
        for j in range(i):
            assert 0.4 < (flat[i] != flat[j]).mean() < 0.6    # batch entries and heads differ
    # same seed, same answer; a segment's mask is its rows of the whole sequence's mask
    assert np.array_equal(base, oracle.dropout_mask(p, 7, 0, l_x, l_x, 2, 2))
    seg = oracle.dropout_mask(p, 7, 100, 37, l_x, 2, 2)
    assert np.array_equal(seg, base[:, :, 100:137])
    # a smaller p keeps a superset (one threshold on one random number per position)
    less = oracle.dropout_mask(0.2, 7, 0, l_x, l_x, 2, 2)
    assert np.all(less >= base)


@pytest.mark.parametrize("causal", [True, False])
def test_forward_is_the_dense_formula_with_that_mask(causal):
    B, l_x, H, d, s0, l_s, p, seed = 2, 24, 2, 4, 5, 11, 0.3, 77
    q, k, v, _ = _inputs(B, l_x, H, d, 22)
    out, lse = oracle.segment_fwd_dropout(q[:, s0:s0 + l_s], k, v, s0, causal, p, seed)
    A = oracle.segment_weights(q[:, s0:s0 + l_s], k, s0, causal)             # [B, H, l_s, l_x]
    M = oracle.dropout_mask(p, seed, s0, l_s, l_x, B, H) / (1 - p)
    want = np.einsum("bhrj,bjhc->brhc", A * M, v)
    assert np.allclose(out, want, rtol=1e-12, atol=1e-13)
    assert np.array_equal(lse, oracle.segment_fwd(q[:, s0:s0 + l_s], k, v, s0, causal)[1])
    assert np.abs(out - oracle.segment_fwd(q[:, s0:s0 + l_s], k, v, s0, causal)[0]).max() > 1e-3


def test_segments_concatenate_to_the_sequential_result():
    B, l_x, H, d, p, seed = 1, 48, 2, 8, 0.2, 5
    q, k, v, do = _inputs(B, l_x, H, d, 23)
    full, full_lse = oracle.segment_fwd_dropout(q, k, v, 0, True, p, seed)
    fdq, fdk, fdv = oracle.segment_bwd_dropout(q, k, v, do, 0, True, p, seed)
    cuts = [0, 7, 20, 21, 48]
    dks, dvs = [], []
    for a, b in zip(cuts, cuts[1:]):
        out, lse = oracle.segment_fwd_dropout(q[:, a:b], k, v, a, True, p, seed)
        assert np.allclose(out, full[:, a:b], rtol=1e-13, atol=1e-14)
        assert np.allclose(lse, full_lse[:, :, a:b], rtol=1e-13, atol=1e-14)
        dq, dk, dv = oracle.segment_bwd_dropout(q[:, a:b], k, v, do[:, a:b], a, True, p, seed)
        assert np.allclose(dq, fdq[:, a:b], rtol=1e-12, atol=1e-13)
        assert not np.any(dk[:, b:]) and not np.any(dv[:, b:])
        dks.append(dk); dvs.append(dv)
    assert np.allclose(oracle.reduce_partials(dks), fdk, rtol=1e-12, atol=1e-13)
    assert np.allclose(oracle.reduce_partials(dvs), fdv, rtol=1e-12, atol=1e-13)


def test_output_is_unbiased_over_seeds():
    # E[dropout(A)] = A, so the mean of the outputs over seeds approaches the plain output
    B, l_x, H, d, p, n = 1, 32, 1, 4, 0.5, 4000
    q, k, v, _ = _inputs(B, l_x, H, d, 24)
    plain = oracle.segment_fwd(q, k, v, 0, False)[0]
    acc = np.zeros_like(plain)
    for seed in range(n):
        acc += oracle.segment_fwd_dropout(q, k, v, 0, False, p, seed)[0]
    err = np.abs(acc / n - plain).max()
    spread = np.abs(v).max() * np.sqrt(p / (1 - p) / n)      # a row's weights sum to 1: at most this per draw / sqrt(n)
    assert err < 5 * spread
    assert err > 0


@pytest.mark.parametrize("causal", [True, False])
def test_gradients_by_finite_differences_with_the_mask_held_fixed(causal):
    B, l_x, H, d, s0, l_s, p, seed = 1, 10, 2, 3, 3, 5, 0.4, 11
    q, k, v, do = _inputs(B, l_x, H, d, 25)
    qs, dos = q[:, s0:s0 + l_s].copy(), do[:, s0:s0 + l_s]

    def loss(qq, kk, vv):
        return float((oracle.segment_fwd_dropout(qq, kk, vv, s0, causal, p, seed)[0] * dos).sum())

    dq, dk, dv = oracle.segment_bwd_dropout(qs, k, v, dos, s0, causal, p, seed)
    eps = 1e-6
    for arr, grad, which in ((qs, dq, 0), (k, dk, 1), (v, dv, 2)):
        fd = np.zeros_like(arr)
        for idx in np.ndindex(*arr.shape):
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps; lo[idx] -= eps
            args_hi = [qs, k, v]; args_lo = [qs, k, v]
            args_hi[which], args_lo[which] = hi, lo
            fd[idx] = (loss(*args_hi) - loss(*args_lo)) / (2 * eps)
        assert np.abs(grad - fd).max() <= 2e-8 * max(1.0, np.abs(fd).max()), which
        assert np.abs(fd).max() > 1e-3


def test_bad_probability_is_rejected():
    q, k, v, _ = _inputs(1, 8, 1, 4, 26)
    for p in (-0.1, 1.0, float("nan")):
        with pytest.raises(ValueError):
            oracle.segment_fwd_dropout(q, k, v, 0, True, p, 1)
