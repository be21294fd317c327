"""Pins of the fp64 CPU oracle against things other than itself.

Each test checks the oracle against a closed form, a library routine, an
invariant of the definition, or a structurally different brute force (the dense
masked form of the paper's Algorithm 1 with its two masks).  CPU only.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import moda_ref as R

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def make(seed, B=1, Hq=2, Hk=2, T=9, d=8, L=3, La=None):
    La = L if La is None else La
    r = np.random.default_rng(seed)
    Q = r.standard_normal((B, Hq, T, d))
    K = r.standard_normal((B, Hk, T, d))
    V = r.standard_normal((B, Hk, T, d))
    Kd = r.standard_normal((B, Hk, T, La, d)) if La else None
    Vd = r.standard_normal((B, Hk, T, La, d)) if La else None
    return Q, K, V, Kd, Vd


# --------------------------------------------------------------------------
# Dense brute force in the paper's flattened form (Algorithm 1; "Group-aware
# depth KV calculation"): query rows of one kv head are flattened so that row
# i_q = t*G + (head within group); keys are [Kseq ; Kdepth.reshape(T*L, d)];
# mask = [floor(i_q/G) >= i_k  |  floor(i_q/G) == floor(j_d/L)].
# --------------------------------------------------------------------------
def alg1_masks(T, G, L, causal=True):
    iq = np.arange(T * G)[:, None]
    ik = np.arange(T)[None, :]
    jd = np.arange(T * L)[None, :]
    seq = (iq // G >= ik) if causal else np.ones((T * G, T), bool)
    dep = (iq // G == jd // max(L, 1)) if L else np.zeros((T * G, 0), bool)
    return seq, dep


def dense_bruteforce(Q, K, V, Kd, Vd, L, causal, scale):
    B, Hq, T, d = Q.shape
    Hk = K.shape[1]
    G = Hq // Hk
    O = np.zeros_like(Q)
    LSE = np.zeros((B, Hq, T))
    seq, dep = alg1_masks(T, G, L, causal)
    mask = np.concatenate([seq, dep], axis=1)
    for b in range(B):
        for g in range(Hk):
            qf = Q[b, g * G:(g + 1) * G].transpose(1, 0, 2).reshape(T * G, d)  # row = t*G + hh
            keys = K[b, g]
            vals = V[b, g]
            if L:
                keys = np.concatenate([keys, Kd[b, g, :, :L].reshape(T * L, d)], 0)
                vals = np.concatenate([vals, Vd[b, g, :, :L].reshape(T * L, d)], 0)
            S = scale * (qf @ keys.T)
            S = np.where(mask, S, -np.inf)
            m = S.max(1, keepdims=True)
            P = np.exp(S - m)
            z = P.sum(1, keepdims=True)
            of = (P / z) @ vals
            O[b, g * G:(g + 1) * G] = of.reshape(T, G, d).transpose(1, 0, 2)
            LSE[b, g * G:(g + 1) * G] = (m + np.log(z)).reshape(T, G).T
    return O, LSE


def test_golden_base_time_example_and_utilisation():
    """The paper's worked index example and its depth-utilisation figures pin
    the mask builder that the brute force uses."""
    vals = {}
    with open(os.path.join(GOLDEN, "alg1_index_facts.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                vals[k.strip()] = float(v)
    # worked example: G=4, rows 8..15 -> base times {2,3}, start 2, end 4
    G = int(vals["example_G"])
    rows = np.arange(int(vals["example_row_first"]), int(vals["example_row_last"]) + 1)
    tb = rows // G
    assert tb.min() == vals["example_t_start"] and tb.max() + 1 == vals["example_t_end"]
    # the mask must give exactly those base times as the depth-visible positions
    T, L = 6, 3
    _, dep = alg1_masks(T, G, L)
    seen = sorted({int(j) // L for r in rows for j in np.nonzero(dep[r])[0]})
    assert seen == [2, 3]
    # flash-compatible layout: utilisation of the dense T x (T*L) depth block is 1/T
    for T in (4, 16):
        _, dep = alg1_masks(T, 1, 5)
        assert dep.sum() / dep.size == pytest.approx(1.0 / T)
    # chunk/group-aware: a chunk of C flattened rows x its (C/G)*L depth span is used G/C
    C = int(vals["chunk_C"])
    for G in (2, 4, 8, 16, 32):
        T, L = 2 * C // G, 2
        _, dep = alg1_masks(T, G, L)
        blk = dep[:C, : (C // G) * L]
        assert blk.sum() / blk.size == pytest.approx(vals["eta_G%d" % G] / 100.0, abs=5e-5)


@pytest.mark.parametrize("G,L,La,causal", [(1, 3, 3, True), (2, 4, 6, True), (4, 1, 1, True),
                                           (1, 0, 0, True), (2, 5, 5, False), (1, 2, 4, False)])
def test_P4_dense_bruteforce(G, L, La, causal):
    Hk = 2
    Q, K, V, Kd, Vd = make(10 + G + L, B=2, Hq=Hk * G, Hk=Hk, T=11, d=6, L=L, La=La)
    scale = 0.37
    O, LSE = R.fwd(Q, K, V, Kd, Vd, depth_count=L, causal=causal, scale=scale)
    O2, LSE2 = dense_bruteforce(Q, K, V, Kd, Vd, L, causal, scale)
    np.testing.assert_allclose(O, O2, rtol=0, atol=1e-12)
    np.testing.assert_allclose(LSE, LSE2, rtol=0, atol=1e-12)


def test_P1_depth0_is_causal_attention_library():
    """depth_count = 0 is Eq. 2; compare with a library SDPA in fp64."""
    Q, K, V, _, _ = make(1, B=2, Hq=3, Hk=3, T=17, d=8, L=0)
    O, _ = R.fwd(Q, K, V, causal=True)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V), is_causal=True)
    np.testing.assert_allclose(O, ref.numpy(), rtol=0, atol=1e-12)
    O, _ = R.fwd(Q, K, V, causal=False)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V), is_causal=False)
    np.testing.assert_allclose(O, ref.numpy(), rtol=0, atol=1e-12)


def test_P1_unused_slots_are_ignored():
    Q, K, V, Kd, Vd = make(2, L=3, La=5)
    O0, L0 = R.fwd(Q, K, V, None, None, depth_count=0)
    O1, L1 = R.fwd(Q, K, V, Kd * 100, Vd * 100, depth_count=0)
    assert np.array_equal(O0, O1) and np.array_equal(L0, L1)
    O2, _ = R.fwd(Q, K, V, Kd, Vd, depth_count=3)
    Kd2, Vd2 = Kd.copy(), Vd.copy()
    Kd2[..., 3:, :] = 99.0
    Vd2[..., 3:, :] = -99.0
    O3, _ = R.fwd(Q, K, V, Kd2, Vd2, depth_count=3)
    assert np.array_equal(O2, O3)


def test_P2_single_token():
    Q, K, V, _, _ = make(3, T=1, d=5, L=0)
    O, LSE = R.fwd(Q, K, V, scale=0.5)
    np.testing.assert_allclose(O, V, atol=1e-15)
    np.testing.assert_allclose(LSE, 0.5 * (Q * K).sum(-1), atol=1e-14)


def test_P3_weights_sum_to_one_and_reproduce_output():
    Q, K, V, Kd, Vd = make(4, T=7, L=4)
    O, _ = R.fwd(Q, K, V, Kd, Vd)
    for (b, h, t) in [(0, 0, 0), (0, 1, 3), (0, 1, 6)]:
        w = R.weights(Q, K, V, Kd, Vd, b, h, t)
        assert len(w) == t + 1 + 4 and (w >= 0).all()
        assert w.sum() == pytest.approx(1.0, abs=1e-14)
        vals = np.concatenate([V[b, h, : t + 1], Vd[b, h, t]], 0)
        np.testing.assert_allclose(w @ vals, O[b, h, t], atol=1e-13)


def test_P5_zero_keys_closed_form():
    Q, K, V, Kd, Vd = make(5, T=6, L=3)
    O, LSE = R.fwd(Q, K * 0, V, Kd * 0, Vd)
    for t in range(6):
        n = t + 1 + 3
        want = (V[:, :, : t + 1].sum(2) + Vd[:, :, t].sum(2)) / n
        np.testing.assert_allclose(O[:, :, t], want, atol=1e-13)
        np.testing.assert_allclose(LSE[:, :, t], math.log(n), atol=1e-13)


def test_P6_duplicate_diagonal_closed_form():
    """Depth slots that repeat the diagonal key/value = causal attention with
    ln(1+L) added to the diagonal logit."""
    Q, K, V, _, _ = make(6, T=8, d=4, L=0)
    L = 3
    Kd = np.repeat(K[:, :, :, None, :], L, 3)
    Vd = np.repeat(V[:, :, :, None, :], L, 3)
    scale = 0.5
    O, LSE = R.fwd(Q, K, V, Kd, Vd, scale=scale)
    S = scale * np.einsum("bhtd,bhsd->bhts", Q, K)
    T = 8
    S = S + np.where(np.tril(np.ones((T, T), bool)), 0.0, -np.inf) + np.eye(T) * math.log(1 + L)
    P = np.exp(S - S.max(-1, keepdims=True))
    want = (P / P.sum(-1, keepdims=True)) @ V
    np.testing.assert_allclose(O, want, atol=1e-13)
    np.testing.assert_allclose(LSE, np.log(np.exp(S).sum(-1)), atol=1e-12)


def test_P7_merge_identity_with_depth_only_attention():
    """Joint softmax = log-sum-exp merge of sequence-only attention and the
    paper's Depth Attention (Eq. 5) computed separately."""
    Q, K, V, Kd, Vd = make(7, T=10, d=4, L=5)
    scale = 1.0 / math.sqrt(4)
    O, LSE = R.fwd(Q, K, V, Kd, Vd)
    Os, Ls = R.fwd(Q, K, V, None, None)
    Sd = scale * np.einsum("bhtd,bhtld->bhtl", Q, Kd)
    Ld = np.log(np.exp(Sd).sum(-1))
    Od = np.einsum("bhtl,bhtld->bhtd", np.exp(Sd - Ld[..., None]), Vd)
    np.testing.assert_allclose(LSE, np.logaddexp(Ls, Ld), atol=1e-13)
    ws = 1.0 / (1.0 + np.exp(Ld - Ls))
    np.testing.assert_allclose(O, ws[..., None] * Os + (1 - ws[..., None]) * Od, atol=1e-13)


def test_P8_invariances():
    Q, K, V, Kd, Vd = make(8, T=6, d=4, L=4)
    O, LSE = R.fwd(Q, K, V, Kd, Vd, scale=0.3)
    perm = [2, 0, 3, 1]
    O2, LSE2 = R.fwd(Q, K, V, Kd[:, :, :, perm], Vd[:, :, :, perm], scale=0.3)
    np.testing.assert_allclose(O, O2, atol=1e-14)
    np.testing.assert_allclose(LSE, LSE2, atol=1e-14)
    c = rnd(80, 4)
    O3, LSE3 = R.fwd(Q, K + c, V, Kd + c, Vd, scale=0.3)
    np.testing.assert_allclose(O, O3, atol=1e-13)
    np.testing.assert_allclose(LSE3 - LSE, 0.3 * (Q @ c), atol=1e-13)
    # T = 1: plain softmax over L + 1 keys
    Q, K, V, Kd, Vd = make(81, T=1, d=3, L=2)
    O, LSE = R.fwd(Q, K, V, Kd, Vd, scale=1.0)
    for b, h in [(0, 0), (0, 1)]:
        keys = np.concatenate([K[b, h], Kd[b, h, 0]], 0)
        vals = np.concatenate([V[b, h], Vd[b, h, 0]], 0)
        s = keys @ Q[b, h, 0]
        p = np.exp(s) / np.exp(s).sum()
        np.testing.assert_allclose(O[b, h, 0], p @ vals, atol=1e-14)


def test_P9_causality_and_position_locality():
    Q, K, V, Kd, Vd = make(9, T=8, L=2)
    O, LSE = R.fwd(Q, K, V, Kd, Vd)
    t = 4
    K2, V2, Kd2, Vd2 = K.copy(), V.copy(), Kd.copy(), Vd.copy()
    K2[:, :, t + 1:] += 5.0
    V2[:, :, t + 1:] -= 3.0
    Kd2[:, :, :t] += 1.0
    Kd2[:, :, t + 1:] -= 1.0
    Vd2[:, :, :t] *= 2.0
    Vd2[:, :, t + 1:] *= -2.0
    O2, LSE2 = R.fwd(Q, K2, V2, Kd2, Vd2)
    assert np.array_equal(O[:, :, t], O2[:, :, t]) and np.array_equal(LSE[:, :, t], LSE2[:, :, t])
    assert not np.allclose(O[:, :, t + 1], O2[:, :, t + 1])
    # without the causal mask the later keys do matter
    O3, _ = R.fwd(Q, K, V, Kd, Vd, causal=False)
    O4, _ = R.fwd(Q, K2, V2, Kd, Vd, causal=False)
    assert not np.allclose(O3[:, :, t], O4[:, :, t])


def test_hand_computed_example():
    """d = 1, T = 2, one depth slot, logits chosen as logs of integers so the
    weights are exact rationals (worked by hand in the fixture's comments)."""
    rows = []
    with open(os.path.join(GOLDEN, "hand_example.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append([float(x) for x in line.split()])
    want_O = np.array(rows[0])
    want_LSE = np.array(rows[1])
    ln = math.log
    Q = np.array([1.0, 2.0]).reshape(1, 1, 2, 1)
    K = np.array([ln(2.0), ln(3.0)]).reshape(1, 1, 2, 1)
    V = np.array([1.0, -1.0]).reshape(1, 1, 2, 1)
    Kd = np.array([ln(6.0), ln(2.0)]).reshape(1, 1, 2, 1, 1)
    Vd = np.array([5.0, 7.0]).reshape(1, 1, 2, 1, 1)
    O, LSE = R.fwd(Q, K, V, Kd, Vd, scale=1.0)
    np.testing.assert_allclose(O.ravel(), want_O, atol=1e-12)
    np.testing.assert_allclose(LSE.ravel(), want_LSE, atol=1e-12)


# ------------------------------ backward ---------------------------------
def loss_from(O, W):
    return float((O * W).sum())


@pytest.mark.parametrize("G,L,La,causal", [(1, 3, 3, True), (2, 2, 3, True), (1, 0, 0, True),
                                           (2, 3, 3, False)])
def test_P10_backward_matches_finite_differences(G, L, La, causal):
    Hk = 2
    Q, K, V, Kd, Vd = make(20 + G + L, B=1, Hq=Hk * G, Hk=Hk, T=5, d=3, L=L, La=La)
    W = rnd(99, *Q.shape)
    scale = 0.7
    grads = R.bwd(Q, K, V, Kd, Vd, W, depth_count=L, causal=causal, scale=scale)
    args = [Q, K, V, Kd, Vd]
    eps = 1e-6
    rng = np.random.default_rng(5)
    for ai, g in enumerate(grads):
        if g is None:
            continue
        x = args[ai]
        idxs = [tuple(rng.integers(0, s) for s in x.shape) for _ in range(25)]
        for idx in idxs:
            old = x[idx]
            x[idx] = old + eps
            lp = loss_from(R.fwd(*args, depth_count=L, causal=causal, scale=scale)[0], W)
            x[idx] = old - eps
            lm = loss_from(R.fwd(*args, depth_count=L, causal=causal, scale=scale)[0], W)
            x[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert g[idx] == pytest.approx(fd, rel=1e-6, abs=1e-8), (ai, idx)
    if La > L:
        assert not grads[3][:, :, :, L:].any() and not grads[4][:, :, :, L:].any()


def test_P10_backward_depth0_matches_library_autograd():
    Q, K, V, _, _ = make(30, B=2, Hq=2, Hk=2, T=9, d=4, L=0)
    dO = rnd(31, *Q.shape)
    dQ, dK, dV, _, _ = R.bwd(Q, K, V, None, None, dO)
    q, k, v = (torch.from_numpy(x).requires_grad_() for x in (Q, K, V))
    out = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
    out.backward(torch.from_numpy(dO))
    np.testing.assert_allclose(dQ, q.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dK, k.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dV, v.grad.numpy(), atol=1e-12)


def test_P10_logit_gradients_sum_to_zero():
    """With every key equal to one vector, dQ = scale * (sum of logit grads) * k = 0."""
    Q, K, V, Kd, Vd = make(32, T=6, d=4, L=2)
    k0 = rnd(33, 4)
    dQ, _, _, _, _ = R.bwd(Q, K * 0 + k0, V, Kd * 0 + k0, Vd, rnd(34, *Q.shape))
    np.testing.assert_allclose(dQ, 0.0, atol=1e-13)


# ------------------------------ backward: rounding-noise scale ---------------------------------
def _dense_backward(Q, K, V, Kd, Vd, dO, L, causal, scale, u=0.0, rng=None):
    """Backward in the dense flattened form (one (b, kv head) at a time), optionally with the
    rounding model of moda_ref_bwd_noise_f64 injected: independent relative errors of standard
    deviation u on every weight, every logit gradient and every element of the forward's output."""
    B, Hq, T, d = Q.shape
    Hk = K.shape[1]
    G = Hq // Hk
    seq, dep = alg1_masks(T, G, L, causal)
    mask = np.concatenate([seq, dep], axis=1)
    noise = (lambda shape: 1.0 + u * rng.standard_normal(shape)) if u else (lambda shape: 1.0)
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    dKd = None if Kd is None else np.zeros_like(Kd)
    dVd = None if Vd is None else np.zeros_like(Vd)
    for b in range(B):
        for g in range(Hk):
            flat = lambda X: X[b, g * G:(g + 1) * G].transpose(1, 0, 2).reshape(T * G, d)
            q, go = flat(Q), flat(dO)
            keys, vals = K[b, g], V[b, g]
            if L:
                keys = np.concatenate([keys, Kd[b, g, :, :L].reshape(T * L, d)])
                vals = np.concatenate([vals, Vd[b, g, :, :L].reshape(T * L, d)])
            logit = np.where(mask, scale * q @ keys.T, -np.inf)
            P = np.exp(logit - logit.max(axis=1, keepdims=True))
            P /= P.sum(axis=1, keepdims=True)
            O = (P @ vals) * noise((T * G, d))
            delta = (go * O).sum(axis=1, keepdims=True)
            E = P * (go @ vals.T - delta) * noise(P.shape)
            Pr = P * noise(P.shape)
            gq = scale * E @ keys
            gk = scale * E.T @ q
            gv = Pr.T @ go
            dQ[b, g * G:(g + 1) * G] = gq.reshape(T, G, d).transpose(1, 0, 2)
            dK[b, g], dV[b, g] = gk[:T], gv[:T]
            if L:
                dKd[b, g, :, :L] = gk[T:].reshape(T, L, d)
                dVd[b, g, :, :L] = gv[T:].reshape(T, L, d)
    return dQ, dK, dV, dKd, dVd


@pytest.mark.parametrize("G,L,La,causal", [(1, 2, 2, True), (2, 3, 4, True), (2, 0, 0, False)])
def test_noise_scale_matches_monte_carlo(G, L, La, causal):
    """moda_ref_bwd_noise_f64 claims to be the standard deviation (per unit relative rounding
    error) of the gradient error under its rounding model: draw that model many times on a dense
    evaluation of the backward and compare the empirical standard deviation."""
    Hk = 2
    Q, K, V, Kd, Vd = make(60 + G + L, B=1, Hq=Hk * G, Hk=Hk, T=6, d=4, L=L, La=La)
    dO = rnd(61, *Q.shape)
    scale = 0.6
    exact = _dense_backward(Q, K, V, Kd, Vd, dO, L, causal, scale)
    ref = R.bwd(Q, K, V, Kd, Vd, dO, depth_count=L, causal=causal, scale=scale)
    for a, r in zip(exact, ref):
        if r is not None:
            np.testing.assert_allclose(a, r, atol=1e-12)
    noise = R.bwd_noise(Q, K, V, Kd, Vd, dO, depth_count=L, causal=causal, scale=scale)
    u, draws = 1e-4, 1500
    rng = np.random.default_rng(7)
    sq = [None if a is None else np.zeros_like(a) for a in exact]
    for _ in range(draws):
        noisy = _dense_backward(Q, K, V, Kd, Vd, dO, L, causal, scale, u=u, rng=rng)
        for s_, n_, a in zip(sq, noisy, exact):
            if s_ is not None:
                s_ += (n_ - a) ** 2
    for name, s_, n_ in zip(("dQ", "dK", "dV", "dKd", "dVd"), sq, noise):
        if s_ is None:
            assert n_ is None
            continue
        sd = np.sqrt(s_ / draws) / u
        # the estimate of a standard deviation from 1500 draws is good to about 2 % (one sigma)
        np.testing.assert_allclose(sd, n_, rtol=0.12, atol=1e-9, err_msg=name)
    if La > L:
        assert not noise[3][:, :, :, L:].any() and not noise[4][:, :, :, L:].any()


def test_noise_scale_single_token_closed_form():
    """T = 1, no depth slots: p = 1 and e = 0, so only the output's rounding is left:
    nV = |g|, nK = scale D |q|, nQ = scale D |k| with D = sqrt(sum_k (g_k v_k)^2)."""
    Q, K, V, _, _ = make(70, B=1, Hq=1, Hk=1, T=1, d=5, L=0)
    dO = rnd(71, *Q.shape)
    nQ, nK, nV, nKd, nVd = R.bwd_noise(Q, K, V, None, None, dO, scale=0.3)
    D = math.sqrt(float(((dO * V) ** 2).sum()))
    np.testing.assert_allclose(nV, np.abs(dO), atol=1e-14)
    np.testing.assert_allclose(nK, 0.3 * D * np.abs(Q), atol=1e-14)
    np.testing.assert_allclose(nQ, 0.3 * D * np.abs(K), atol=1e-14)
    assert nKd is None and nVd is None


def test_noise_scale_rows_variant_matches_full():
    Q, K, V, Kd, Vd = make(72, B=2, Hq=4, Hk=2, T=10, d=4, L=2, La=3)
    dO = rnd(73, *Q.shape)
    rows = np.array([0, 9, 4], np.int32)
    nQ, _, _, nKd, nVd = R.bwd_noise(Q, K, V, Kd, Vd, dO, depth_count=2)
    rQ, rKd, rVd = R.bwd_noise_rows(Q[:, :, rows], K, V, Kd[:, :, rows], Vd[:, :, rows], dO[:, :, rows], rows,
                                    depth_count=2)
    np.testing.assert_allclose(nQ[:, :, rows], rQ, atol=1e-14)
    np.testing.assert_allclose(nKd[:, :, rows], rKd, atol=1e-14)
    np.testing.assert_allclose(nVd[:, :, rows], rVd, atol=1e-14)


def test_rows_variants_match_full():
    Q, K, V, Kd, Vd = make(40, B=2, Hq=4, Hk=2, T=12, d=4, L=3, La=4)
    dO = rnd(41, *Q.shape)
    rows = np.array([0, 5, 11, 7], np.int32)
    O, LSE = R.fwd(Q, K, V, Kd, Vd, depth_count=3)
    Or, Lr = R.fwd_rows(Q[:, :, rows], K, V, Kd[:, :, rows], Vd[:, :, rows], rows, depth_count=3)
    assert np.array_equal(O[:, :, rows], Or) and np.array_equal(LSE[:, :, rows], Lr)
    dQ, _, _, dKd, dVd = R.bwd(Q, K, V, Kd, Vd, dO, depth_count=3)
    dQr, dKdr, dVdr = R.bwd_rows(Q[:, :, rows], K, V, Kd[:, :, rows], Vd[:, :, rows],
                                 dO[:, :, rows], rows, depth_count=3)
    np.testing.assert_allclose(dQ[:, :, rows], dQr, atol=1e-14)
    np.testing.assert_allclose(dKd[:, :, rows], dKdr, atol=1e-14)
    np.testing.assert_allclose(dVd[:, :, rows], dVdr, atol=1e-14)


def test_bad_arguments_are_rejected():
    Q, K, V, Kd, Vd = make(50)
    with pytest.raises(ValueError):
        R.fwd(Q, K, V, Kd, Vd, depth_count=7)  # more slots than allocated
    with pytest.raises(ValueError):
        R.fwd_rows(Q[:, :, :1], K, V, Kd[:, :, :1], Vd[:, :, :1], [99])


def test_depth_append_builds_the_stacked_stream():
    """Write step: appending the layers' K / V one slot at a time to an empty cache gives
    the layers stacked along the slot axis (checked against numpy's own stacking routine),
    and a write never touches another slot."""
    rng = np.random.default_rng(5)
    B, Hk, T, d, La = 2, 3, 7, 4, 5
    Ks = [rng.standard_normal((B, Hk, T, d)) for _ in range(La)]
    Vs = [rng.standard_normal((B, Hk, T, d)) for _ in range(La)]
    Kd = np.full((B, Hk, T, La, d), np.nan)
    Vd = np.full((B, Hk, T, La, d), np.nan)
    for order, slot in enumerate([3, 0, 4, 1, 2]):
        before_k = Kd.copy()
        Kd, Vd = R.depth_append(Kd, Vd, Ks[slot], Vs[slot], slot)
        others = [i for i in range(La) if i != slot]
        assert np.array_equal(Kd[:, :, :, others], before_k[:, :, :, others], equal_nan=True)
    assert np.array_equal(Kd, np.stack(Ks, axis=3)) and np.array_equal(Vd, np.stack(Vs, axis=3))
    with pytest.raises(IndexError):
        R.depth_append(Kd, Vd, Ks[0], Vs[0], La)
