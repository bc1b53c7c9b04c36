"""Pins for the oracle's linear maps around the segment attention (fused-communication form,
Section 3, Principle 3; Fig. 2(ii), (iii), (v)): brute-force loops, special weights with a
closed form, the segment/full-sequence relations, and finite differences through the whole
chain x -> (Q_i, K, V) -> E_i, which fix every transpose in the backward maps."""
import numpy as np
import pytest

import oracle
from paper_2311_02382_amd import synth


def _inputs(B, l_x, H, d, seed):
    x, w_q, w_kv = synth.make_projection_inputs(B, l_x, H, d, seed)
    return x.astype(np.float64), w_q.astype(np.float64), w_kv.astype(np.float64)


def test_forward_maps_against_loops():
    B, l_x, H, d, s0, l_s = 2, 7, 2, 3, 2, 4
    E = H * d
    x, w_q, w_kv = _inputs(B, l_x, H, d, 11)
    q, k, v = oracle.project_qkv(x, w_q, w_kv, s0, l_s, H)
    for b in range(B):
        for h in range(H):
            for c in range(d):
                col = h * d + c
                for j in range(l_x):
                    kk = sum(x[b, j, e] * w_kv[e, col] for e in range(E))
                    vv = sum(x[b, j, e] * w_kv[e, E + col] for e in range(E))
                    assert abs(k[b, j, h, c] - kk) < 1e-12 and abs(v[b, j, h, c] - vv) < 1e-12
                for r in range(l_s):
                    qq = sum(x[b, s0 + r, e] * w_q[e, col] for e in range(E))
                    assert abs(q[b, r, h, c] - qq) < 1e-12


def test_backward_maps_against_loops():
    B, l_x, H, d, l_s = 1, 5, 2, 2, 3
    E = H * d
    _, w_q, w_kv = _inputs(B, l_x, H, d, 12)
    g = np.random.default_rng(3)
    dq = g.standard_normal((B, l_s, H, d))
    dk = g.standard_normal((B, l_x, H, d))
    dv = g.standard_normal((B, l_x, H, d))
    dx_q, dx_p = oracle.project_bwd(dq, dk, dv, w_q, w_kv)
    assert dx_q.shape == (B, l_s, E) and dx_p.shape == (B, l_x, E)
    for e in range(E):
        for r in range(l_s):
            want = sum(dq[0, r, c // d, c % d] * w_q[e, c] for c in range(E))
            assert abs(dx_q[0, r, e] - want) < 1e-12
        for j in range(l_x):
            want = sum(dk[0, j, c // d, c % d] * w_kv[e, c] + dv[0, j, c // d, c % d] * w_kv[e, E + c]
                       for c in range(E))
            assert abs(dx_p[0, j, e] - want) < 1e-12


def test_identity_and_selector_weights():
    # W = I returns x itself, split into heads; a weight that swaps two columns swaps them in K only
    B, l_x, H, d = 1, 6, 2, 4
    E = H * d
    x, _, _ = _inputs(B, l_x, H, d, 13)
    eye = np.eye(E)
    q, k, v = oracle.project_qkv(x, eye, np.hstack([eye, 2 * eye]), 1, 3, H)
    assert np.array_equal(q, x[:, 1:4].reshape(B, 3, H, d))
    assert np.array_equal(k, x.reshape(B, l_x, H, d)) and np.array_equal(v, 2 * x.reshape(B, l_x, H, d))
    swap = eye.copy()
    swap[[0, 5]] = swap[[5, 0]]                     # K column 0 <- x column 5 and back
    _, k2, v2 = oracle.project_qkv(x, eye, np.hstack([swap, eye]), 0, l_x, H)
    xs = x.copy()
    xs[..., [0, 5]] = xs[..., [5, 0]]
    assert np.array_equal(k2, xs.reshape(B, l_x, H, d)) and np.array_equal(v2, x.reshape(B, l_x, H, d))
    # backward with the same weights: dK's column 0 lands in dx column 5
    dk = np.zeros((B, l_x, H, d)); dk[0, 2, 0, 0] = 1.0
    _, dx = oracle.project_bwd(np.zeros((B, 1, H, d)), dk, np.zeros_like(dk), eye, np.hstack([swap, eye]))
    want = np.zeros((B, l_x, E)); want[0, 2, 5] = 1.0
    assert np.array_equal(dx, want)


def test_segment_queries_are_rows_of_the_full_projection():
    B, l_x, H, d = 2, 12, 3, 2
    x, w_q, w_kv = _inputs(B, l_x, H, d, 14)
    q_all, k_all, v_all = oracle.project_qkv(x, w_q, w_kv, 0, l_x, H)
    for s0, l_s in ((0, 5), (5, 3), (8, 4)):
        q, k, v = oracle.project_qkv(x, w_q, w_kv, s0, l_s, H)
        assert np.array_equal(q, q_all[:, s0:s0 + l_s])
        assert np.array_equal(k, k_all) and np.array_equal(v, v_all)    # every segment holds the same K, V


@pytest.mark.parametrize("causal", [True, False])
def test_chain_gradient_by_finite_differences(causal):
    # loss(x) = sum_i <dO_i, E_i(x)>.  Its gradient is the segment sum of dx_partial plus each
    # segment's dx_q placed on its own rows; compared with central differences in x.
    B, l_x, H, d = 1, 8, 2, 2
    cuts = [0, 3, 5, 8]
    x, w_q, w_kv = _inputs(B, l_x, H, d, 15)
    w_q, w_kv = 3.0 * w_q, 3.0 * w_kv             # scores of order 1, so the softmax is not flat
    do = np.random.default_rng(5).standard_normal((B, l_x, H, d))

    def loss(xx):
        tot = 0.0
        for a, b in zip(cuts, cuts[1:]):
            q, k, v = oracle.project_qkv(xx, w_q, w_kv, a, b - a, H)
            out, _ = oracle.segment_fwd(q, k, v, a, causal)
            tot += float((out * do[:, a:b]).sum())
        return tot

    grad = np.zeros_like(x)
    parts = []
    for a, b in zip(cuts, cuts[1:]):
        q, k, v = oracle.project_qkv(x, w_q, w_kv, a, b - a, H)
        dq, dk, dv = oracle.segment_bwd(q, k, v, do[:, a:b], a, causal)
        dx_q, dx_p = oracle.project_bwd(dq, dk, dv, w_q, w_kv)
        grad[:, a:b] += dx_q
        parts.append(dx_p)
    grad += oracle.reduce_partials(parts)
    eps = 1e-6
    fd = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps; xm[idx] -= eps
        fd[idx] = (loss(xp) - loss(xm)) / (2 * eps)
    assert np.abs(grad - fd).max() <= 1e-7 * max(1.0, np.abs(fd).max())
    assert np.abs(fd).max() > 1e-3


def test_segment_sum_of_dx_equals_unsegmented_gradient():
    # N segments' dx contributions add up to what one segment spanning the sequence gives
    B, l_x, H, d = 2, 24, 2, 4
    x, w_q, w_kv = _inputs(B, l_x, H, d, 16)
    do = np.random.default_rng(6).standard_normal((B, l_x, H, d))
    q, k, v = oracle.project_qkv(x, w_q, w_kv, 0, l_x, H)
    dq, dk, dv = oracle.segment_bwd(q, k, v, do, 0, True)
    dxq_full, dxp_full = oracle.project_bwd(dq, dk, dv, w_q, w_kv)
    parts, dxq = [], np.zeros_like(dxq_full)
    for s0 in range(0, l_x, 6):
        q, k, v = oracle.project_qkv(x, w_q, w_kv, s0, 6, H)
        dq, dk, dv = oracle.segment_bwd(q, k, v, do[:, s0:s0 + 6], s0, True)
        a, p = oracle.project_bwd(dq, dk, dv, w_q, w_kv)
        dxq[:, s0:s0 + 6] = a
        parts.append(p)
        assert not np.any(p[:, s0 + 6:])            # causal: later rows get nothing from this segment
    assert np.allclose(oracle.reduce_partials(parts), dxp_full, rtol=1e-12, atol=1e-12)
    assert np.allclose(dxq, dxq_full, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("causal", [True, False])
def test_weight_gradients_by_finite_differences(causal):
    # loss(W_q, W_kv) = sum_i <dO_i, E_i>; its gradient is the sum over segments of each segment's
    # contribution (Section 4); compared with central differences in single weights.
    B, l_x, H, d = 2, 8, 2, 2
    E = H * d
    cuts = [0, 3, 5, 8]
    x, w_q, w_kv = _inputs(B, l_x, H, d, 17)
    w_q, w_kv = 3.0 * w_q, 3.0 * w_kv
    do = np.random.default_rng(8).standard_normal((B, l_x, H, d))

    def loss(wq, wkv):
        tot = 0.0
        for a, b in zip(cuts, cuts[1:]):
            q, k, v = oracle.project_qkv(x, wq, wkv, a, b - a, H)
            out, _ = oracle.segment_fwd(q, k, v, a, causal)
            tot += float((out * do[:, a:b]).sum())
        return tot

    g_q, g_kv = np.zeros((E, E)), np.zeros((E, 2 * E))
    for a, b in zip(cuts, cuts[1:]):
        q, k, v = oracle.project_qkv(x, w_q, w_kv, a, b - a, H)
        dq, dk, dv = oracle.segment_bwd(q, k, v, do[:, a:b], a, causal)
        dwq, dwkv = oracle.project_bwd_weight(x, dq, dk, dv, a)
        # the definition, one element each
        assert np.isclose(dwq[1, 2], sum(x[bb, a + r, 1] * dq.reshape(B, b - a, E)[bb, r, 2] for bb in range(B) for r in range(b - a)))
        assert np.isclose(dwkv[3, E + 1], sum(x[bb, r, 3] * dv.reshape(B, l_x, E)[bb, r, 1] for bb in range(B) for r in range(l_x)))
        g_q += dwq
        g_kv += dwkv
    eps = 1e-6
    for idx in np.ndindex(E, E):
        wp, wm = w_q.copy(), w_q.copy()
        wp[idx] += eps; wm[idx] -= eps
        assert np.isclose((loss(wp, w_kv) - loss(wm, w_kv)) / (2 * eps), g_q[idx], rtol=1e-6, atol=1e-7)
    for idx in np.ndindex(E, 2 * E):
        wp, wm = w_kv.copy(), w_kv.copy()
        wp[idx] += eps; wm[idx] -= eps
        assert np.isclose((loss(w_q, wp) - loss(w_q, wm)) / (2 * eps), g_kv[idx], rtol=1e-6, atol=1e-7)
    assert np.abs(g_q).max() > 1e-3 and np.abs(g_kv).max() > 1e-3
