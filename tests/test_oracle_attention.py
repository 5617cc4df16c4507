"""Pins for the oracle's attention and projection primitives (CPU only).

Every check compares the oracle with something that is NOT the oracle: a python-loop
brute force, a closed form, a hand-computed value, or torch's CPU library routine."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import tandem_oracle as orc


def brute_attention(q, K, V, scale):
    """Pure-python softmax attention: no numpy reductions at all."""
    N, dh = len(K), len(q)
    s = [scale * sum(q[d] * K[p][d] for d in range(dh)) for p in range(N)]
    mx = max(s)
    e = [math.exp(x - mx) for x in s]
    Z = sum(e)
    return [sum(e[p] / Z * V[p][d] for p in range(N)) for d in range(dh)]


def test_attention_one_brute_force():
    rng = np.random.default_rng(0)
    for N, dh in [(1, 4), (3, 5), (17, 8), (40, 16)]:
        q, K, V = rng.standard_normal(dh), rng.standard_normal((N, dh)), rng.standard_normal((N, dh))
        got = orc.attention_one(q, K, V, 0.37)
        want = brute_attention(q.tolist(), K.tolist(), V.tolist(), 0.37)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)


def test_attention_one_hand_cases():
    # one key: the output is that key's value row whatever the score is
    np.testing.assert_array_equal(orc.attention_one([5.0, -2.0], [[1.0, 1.0]], [[7.0, 9.0]], 1.0), [7.0, 9.0])
    # equal scores (q = 0): plain mean of V
    V = np.array([[1.0, 2.0], [3.0, 6.0], [5.0, 10.0]])
    np.testing.assert_allclose(orc.attention_one([0.0, 0.0], np.ones((3, 2)), V, 1.0), [3.0, 6.0], rtol=1e-15)
    # two keys with scores ln(3) and 0: weights 3/4 and 1/4
    K = np.array([[math.log(3.0)], [0.0]])
    Vv = np.array([[4.0], [8.0]])
    np.testing.assert_allclose(orc.attention_one([1.0], K, Vv, 1.0), [0.75 * 4 + 0.25 * 8], rtol=1e-14)
    # the scale multiplies the score: scale 2 turns ln(3)/2 into ln(3)
    K2 = np.array([[math.log(3.0) / 2], [0.0]])
    np.testing.assert_allclose(orc.attention_one([1.0], K2, Vv, 2.0), [5.0], rtol=1e-14)
    # a transposed K/V mix-up would break this: V's columns differ from K's
    K3 = np.array([[0.0, 0.0], [50.0, 0.0]])
    V3 = np.array([[1.0, 2.0], [3.0, 4.0]])
    np.testing.assert_allclose(orc.attention_one([1.0, 0.0], K3, V3, 1.0), [3.0, 4.0], rtol=1e-12)


def test_attention_one_rejects_empty():
    with pytest.raises(ValueError):
        orc.attention_one(np.zeros(4), np.zeros((0, 4)), np.zeros((0, 4)), 1.0)


def test_attention_one_shift_and_permutation_invariance():
    rng = np.random.default_rng(1)
    q, K, V = rng.standard_normal(8), rng.standard_normal((33, 8)), rng.standard_normal((33, 8))
    base = orc.attention_one(q, K, V, 0.5)
    perm = rng.permutation(33)
    np.testing.assert_allclose(orc.attention_one(q, K[perm], V[perm], 0.5), base, rtol=1e-12)
    # adding c*q/|q|^2 to every key adds the constant c to every score
    Kc = K + 3.0 * q / (q @ q)
    np.testing.assert_allclose(orc.attention_one(q, Kc, V, 0.5), base, rtol=1e-10)


def test_attention_one_large_scores_do_not_overflow():
    q = np.array([1000.0])
    K = np.array([[1.0], [0.999]])
    V = np.array([[1.0], [0.0]])
    w = 1.0 / (1.0 + math.exp(-1.0))
    np.testing.assert_allclose(orc.attention_one(q, K, V, 1.0), [w], rtol=1e-12)


def sdpa(q, K, V, mask, scale):
    """torch CPU library attention in fp64; q [H, Lq, dh], K/V [H, Lk, dh], mask [Lq, Lk] bool."""
    return F.scaled_dot_product_attention(
        torch.from_numpy(q), torch.from_numpy(K), torch.from_numpy(V), attn_mask=torch.from_numpy(mask), scale=scale
    ).numpy()


@pytest.mark.parametrize("q_len,n", [(1, 0), (1, 9), (4, 13), (3, 0), (7, 5)])
def test_block_attn_vs_torch_sdpa(q_len, n):
    rng = np.random.default_rng(q_len * 100 + n)
    B, Hq, Hkv, dh, T = 2, 4, 2, 8, 24
    Q = rng.standard_normal((B, q_len, Hq, dh))
    Kc = rng.standard_normal((B, Hkv, T, dh))
    Vc = rng.standard_normal((B, Hkv, T, dh))
    nb = np.array([n, n + 2])
    got = orc.block_attn(Q, Kc, Vc, nb, 0.3)
    for b in range(B):
        mask = np.zeros((q_len, T), bool)
        for r in range(q_len):
            mask[r, : nb[b] + r + 1] = True
        Kx = np.repeat(Kc[b], Hq // Hkv, axis=0)  # GQA: query head h reads KV head h // G
        Vx = np.repeat(Vc[b], Hq // Hkv, axis=0)
        want = sdpa(np.ascontiguousarray(Q[b].transpose(1, 0, 2)), Kx, Vx, mask, 0.3).transpose(1, 0, 2)
        np.testing.assert_allclose(got[b], want, rtol=1e-11, atol=1e-13)


def test_block_attn_gamma1_is_causal_decode():
    """q_len = 1: the block pass is ordinary one-token causal decoding over n+1 keys."""
    rng = np.random.default_rng(5)
    B, H, dh, T = 3, 2, 4, 10
    Q = rng.standard_normal((B, 1, H, dh))
    Kc, Vc = rng.standard_normal((B, H, T, dh)), rng.standard_normal((B, H, T, dh))
    n = np.array([0, 4, 9])
    got = orc.block_attn(Q, Kc, Vc, n, 0.5)
    for b in range(B):
        for h in range(H):
            want = brute_attention(Q[b, 0, h].tolist(), Kc[b, h, : n[b] + 1].tolist(), Vc[b, h, : n[b] + 1].tolist(), 0.5)
            np.testing.assert_allclose(got[b, 0, h], want, rtol=1e-12)


def test_block_attn_ignores_rows_past_the_causal_limit():
    rng = np.random.default_rng(6)
    Q = rng.standard_normal((1, 3, 2, 4))
    Kc, Vc = rng.standard_normal((1, 2, 12, 4)), rng.standard_normal((1, 2, 12, 4))
    a = orc.block_attn(Q, Kc, Vc, [5], 1.0)
    Kc2, Vc2 = Kc.copy(), Vc.copy()
    Kc2[:, :, 8:] = 99.0
    Vc2[:, :, 8:] = -99.0
    np.testing.assert_array_equal(a, orc.block_attn(Q, Kc2, Vc2, [5], 1.0))
    # ...and row 0 must not see row n+1, row 1 must not see row n+2
    Kc3 = Kc.copy()
    Kc3[:, :, 7] += 1.0
    b3 = orc.block_attn(Q, Kc3, Vc, [5], 1.0)
    np.testing.assert_array_equal(a[:, :2], b3[:, :2])
    assert np.abs(a[:, 2] - b3[:, 2]).max() > 0


@pytest.mark.parametrize("n_large,n_cur", [(0, 1), (0, 3), (11, 1), (11, 4), (20, 2)])
def test_draft_attn_vs_torch_sdpa_union(n_large, n_cur):
    rng = np.random.default_rng(n_large * 10 + n_cur)
    B, Hq, Hkv, dh, T, g = 2, 4, 2, 8, 20, 4
    q = rng.standard_normal((B, Hq, dh))
    khat, vhat = rng.standard_normal((B, Hkv, T, dh)), rng.standard_normal((B, Hkv, T, dh))
    kcur, vcur = rng.standard_normal((B, Hkv, g, dh)), rng.standard_normal((B, Hkv, g, dh))
    nl = np.array([n_large, max(0, n_large - 3)])
    nc = np.array([n_cur, 1 + (n_cur % g)])
    got = orc.draft_attn(q, khat, vhat, nl, kcur, vcur, nc, 0.25)
    for b in range(B):
        # one library call over all T + g rows with a mask selecting the union
        mask = np.zeros((1, T + g), bool)
        mask[0, : nl[b]] = True
        mask[0, T : T + nc[b]] = True
        Kx = np.repeat(np.concatenate([khat[b], kcur[b]], axis=1), Hq // Hkv, axis=0)
        Vx = np.repeat(np.concatenate([vhat[b], vcur[b]], axis=1), Hq // Hkv, axis=0)
        want = sdpa(q[b][:, None, :].copy(), Kx, Vx, mask, 0.25)[:, 0]
        np.testing.assert_allclose(got[b], want, rtol=1e-11, atol=1e-13)


def test_draft_attn_zero_large_rows_closed_form():
    """K_hat = V_hat = 0 (FF_Tandem == 0, zero biases): every large row scores 0 and adds
    nothing, so o = o_own * Z_own / (n + Z_own) with Z_own = sum over own rows of e^s."""
    rng = np.random.default_rng(9)
    B, H, dh, T, g = 2, 2, 8, 16, 4
    q = rng.standard_normal((B, H, dh))
    kcur, vcur = rng.standard_normal((B, H, g, dh)), rng.standard_normal((B, H, g, dh))
    z = np.zeros((B, H, T, dh))
    nl, nc = np.array([16, 5]), np.array([4, 2])
    got = orc.draft_attn(q, z, z, nl, kcur, vcur, nc, 0.4)
    own_only = orc.draft_attn(q, z, z, np.zeros(B, int), kcur, vcur, nc, 0.4)
    for b in range(B):
        for h in range(H):
            s = 0.4 * kcur[b, h, : nc[b]] @ q[b, h]
            Z = np.exp(s).sum()
            np.testing.assert_allclose(got[b, h], own_only[b, h] * Z / (nl[b] + Z), rtol=1e-12)
            # with the large part removed it is exactly plain attention over the own rows
            want = brute_attention(q[b, h].tolist(), kcur[b, h, : nc[b]].tolist(), vcur[b, h, : nc[b]].tolist(), 0.4)
            np.testing.assert_allclose(own_only[b, h], want, rtol=1e-12)


def test_draft_attn_indicator_probe_mask_is_exact():
    """q = 0 gives uniform weights 1/N; V = indicator of one row makes the output 1/N if
    the row is attended and exactly 0 if it is masked."""
    B, H, dh, T, g = 1, 1, 4, 9, 3
    q = np.zeros((B, H, dh))
    khat, kcur = np.ones((B, H, T, dh)), np.ones((B, H, g, dh))
    for nl in (0, 4, 9):
        for nc in (1, 2, 3):
            N = nl + nc
            for p in range(T + g):
                vhat, vcur = np.zeros((B, H, T, dh)), np.zeros((B, H, g, dh))
                (vhat if p < T else vcur)[0, 0, p if p < T else p - T, 0] = 1.0
                o = orc.draft_attn(q, khat, vhat, [nl], kcur, vcur, [nc], 1.0)[0, 0, 0]
                visible = (p < nl) if p < T else (p - T < nc)
                assert o == (1.0 / N if visible else 0.0)


def test_split_merge_equals_two_pass():
    rng = np.random.default_rng(3)
    q, K, V = rng.standard_normal(16), rng.standard_normal((101, 16)) * 3, rng.standard_normal((101, 16))
    base = orc.attention_one(q, K, V, 0.25)
    for bounds in ([0, 101], [0, 50, 101], [0, 1, 2, 101], [0, 0, 37, 37, 101], [0, 16, 32, 48, 64, 80, 96, 101, 101]):
        np.testing.assert_allclose(orc.attention_one_split(q, K, V, 0.25, bounds), base, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ projection
def test_project_hand_values():
    # linear: y = W x + b with W [out, in]
    X = np.array([[1.0, 2.0, 3.0]])
    W = np.array([[1.0, 0.0, -1.0], [2.0, 1.0, 0.5]])
    b = np.array([10.0, 20.0])
    np.testing.assert_array_equal(orc.project(X, {"W": W, "b": b}), [[8.0, 25.5]])
    # MLP with relu: hidden = relu([-2, 4]) = [0, 4]; out = W2 hidden + b2
    ff = {"W1": np.array([[1.0, 0.0, -1.0], [0.0, 2.0, 0.0]]), "b1": np.zeros(2), "W2": np.array([[3.0, 0.5]]), "b2": np.array([1.0]), "act": "relu"}
    np.testing.assert_array_equal(orc.project(X, ff), [[3.0]])


def test_gelu_erf_known_values():
    # Phi(1) = 0.841344746068543, Phi(-1) = 0.158655253931457, Phi(2) = 0.977249868051821
    x = np.array([0.0, 1.0, -1.0, 2.0])
    np.testing.assert_allclose(orc.gelu_erf(x), [0.0, 0.841344746068543, -0.158655253931457, 2 * 0.977249868051821], rtol=1e-13)
    # and it is NOT the tanh approximation
    t = torch.tensor([1.0], dtype=torch.float64)
    assert abs(float(orc.gelu_erf(np.array([1.0]))[0]) - float(F.gelu(t, approximate="tanh"))) > 1e-5


def test_project_vs_torch_library():
    rng = np.random.default_rng(4)
    X = rng.standard_normal((5, 12))
    ff = {"W1": rng.standard_normal((20, 12)), "b1": rng.standard_normal(20), "W2": rng.standard_normal((7, 20)), "b2": rng.standard_normal(7), "act": "gelu"}
    t = lambda a: torch.from_numpy(a)
    want = F.linear(F.gelu(F.linear(t(X), t(ff["W1"]), t(ff["b1"]))), t(ff["W2"]), t(ff["b2"])).numpy()
    np.testing.assert_allclose(orc.project(X, ff), want, rtol=1e-12, atol=1e-13)
    lin = {"W": rng.standard_normal((7, 12)), "b": None}
    np.testing.assert_allclose(orc.project(X, lin), F.linear(t(X), t(lin["W"])).numpy(), rtol=1e-12)


def test_rmsnorm_hand_and_library():
    x = np.array([[3.0, 4.0]])
    g = np.array([2.0, 0.5])
    # mean square = 12.5
    np.testing.assert_allclose(orc.rmsnorm(x, g, 0.0), [[6.0 / math.sqrt(12.5), 2.0 / math.sqrt(12.5)]], rtol=1e-15)
    rng = np.random.default_rng(2)
    x = rng.standard_normal((4, 16))
    g = rng.standard_normal(16)
    want = F.rms_norm(torch.from_numpy(x), (16,), torch.from_numpy(g), eps=1e-6).numpy()
    np.testing.assert_allclose(orc.rmsnorm(x, g, 1e-6), want, rtol=1e-12)


def test_block_attn_shared_equals_block_attn_on_materialised_caches():
    """Shared-prompt attention == ordinary block attention on per-sample caches that hold a copy of the prompt
    rows followed by the sample's own rows (the pinned block_attn, and torch's SDPA through it)."""
    rng = np.random.default_rng(11)
    B, ns, q_len, Hq, Hkv, dh, Ts, To = 2, 3, 2, 4, 2, 8, 9, 6
    Q = rng.standard_normal((B, ns, q_len, Hq, dh))
    Ks, Vs = rng.standard_normal((B, Hkv, Ts, dh)), rng.standard_normal((B, Hkv, Ts, dh))
    Ko, Vo = rng.standard_normal((B * ns, Hkv, To, dh)), rng.standard_normal((B * ns, Hkv, To, dh))
    n_shared = np.array([9, 0])
    n_own = np.array([0, 3, 4, 1, 0, 2])
    scale = dh ** -0.5
    got = orc.block_attn_shared(Q, Ks, Vs, n_shared, Ko, Vo, n_own, scale)
    Kc = np.zeros((B * ns, Hkv, Ts + To, dh))
    Vc = np.zeros_like(Kc)
    n = np.zeros(B * ns, dtype=np.int64)
    for b in range(B):
        for s_ in range(ns):
            i = b * ns + s_
            m = n_shared[b]
            Kc[i, :, :m], Vc[i, :, :m] = Ks[b, :, :m], Vs[b, :, :m]
            Kc[i, :, m : m + To], Vc[i, :, m : m + To] = Ko[i], Vo[i]
            n[i] = m + n_own[i]
    want = orc.block_attn(Q.reshape(B * ns, q_len, Hq, dh), Kc, Vc, n, scale).reshape(Q.shape)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def _mixed_case(seed, B, q_len, Hq, Hkv, dh, T):
    rng = np.random.default_rng(seed)
    mk = lambda *sh: rng.standard_normal(sh)
    return mk(B, q_len, Hq, dh), mk(B, Hkv, T, dh), mk(B, Hkv, T, dh), mk(B, Hkv, T, dh), mk(B, Hkv, T, dh)


def test_mixed_attn_equals_masked_sdpa_over_both_caches():
    """Library special case: torch SDPA over the keys [all hat rows ; all own rows] with the boolean mask
    'hat row j visible iff j < k(i); own row j visible iff k(i) <= j <= i' written out independently."""
    B, q_len, Hq, Hkv, dh, T, gamma = 2, 7, 4, 2, 8, 23, 3
    Q, Kh, Vh, Ko, Vo = _mixed_case(3, B, q_len, Hq, Hkv, dh, T)
    n = np.array([16, 2])
    got = orc.mixed_attn(Q, Kh, Vh, Ko, Vo, n, gamma, dh ** -0.5)
    G = Hq // Hkv
    for b in range(B):
        pos = n[b] + np.arange(q_len)
        j = np.arange(T)
        kb = (pos // gamma) * gamma
        mask = np.concatenate([j[None, :] < kb[:, None], (j[None, :] >= kb[:, None]) & (j[None, :] <= pos[:, None])], axis=1)
        K = np.repeat(np.concatenate([Kh[b], Ko[b]], axis=1), G, axis=0)
        V = np.repeat(np.concatenate([Vh[b], Vo[b]], axis=1), G, axis=0)
        want = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(Q[b].transpose(1, 0, 2)), torch.from_numpy(K), torch.from_numpy(V),
            attn_mask=torch.from_numpy(mask)[None], scale=dh ** -0.5).numpy().transpose(1, 0, 2)
        np.testing.assert_allclose(got[b], want, rtol=1e-11, atol=1e-12)


def test_mixed_attn_block_length_one_and_infinite():
    """gamma = 1: every completed position is read from the hat rows, only the query's own row is its own
    (draft_attn with one own row).  gamma > sequence length: no block is ever complete, ordinary causal
    attention over the own rows (block_attn)."""
    B, q_len, Hq, Hkv, dh, T = 2, 4, 4, 2, 8, 19
    Q, Kh, Vh, Ko, Vo = _mixed_case(4, B, q_len, Hq, Hkv, dh, T)
    n = np.array([15, 0])
    scale = dh ** -0.5
    got = orc.mixed_attn(Q, Kh, Vh, Ko, Vo, n, 1, scale)
    for r in range(q_len):
        pos = n + r
        kc = np.stack([Ko[b, :, pos[b]:pos[b] + 1] for b in range(B)])
        vc = np.stack([Vo[b, :, pos[b]:pos[b] + 1] for b in range(B)])
        want = orc.draft_attn(Q[:, r], Kh, Vh, pos, kc, vc, np.ones(B, int), scale)
        np.testing.assert_allclose(got[:, r], want, rtol=1e-12, atol=1e-13)
    got = orc.mixed_attn(Q, Kh, Vh, Ko, Vo, n, 1000, scale)
    np.testing.assert_allclose(got, orc.block_attn(Q, Ko, Vo, n, scale), rtol=1e-12, atol=1e-13)


def test_mixed_attn_is_the_attention_inside_tandem_forward():
    """The teacher-forced Tandem forward (pinned on its own) uses exactly this attention in its small layers:
    feeding its layer-0 queries and rows to mixed_attn in chunks reproduces its attention output."""
    import math
    from paper_2402_08644_amd import inputs

    T_ = inputs.as_f64(inputs.tiny_tandem(seed=2, dtype="f32"))
    gamma, S = 3, 11
    toks = inputs.token_ids(5, (S,), 1000)
    eps = T_["eps"]
    MS = T_["S"]
    lay = MS["layers"][0]
    xs = orc.decoder_forward(T_["L"], toks, eps)
    yhat = orc.project(xs[T_["ell"][0]], T_["ff"][0])
    y = np.asarray(MS["emb"], np.float64)[toks]
    Hq, Hkv, dh = MS["Hq"], MS["Hkv"], MS["dh"]
    hn, hh = orc.rmsnorm(y, lay["g_attn"], eps), orc.rmsnorm(yhat, lay["g_attn"], eps)
    q = orc.linear(hn, lay["Wq"]).reshape(S, Hq, dh)
    ko = orc.linear(hn, lay["Wk"]).reshape(S, Hkv, dh).transpose(1, 0, 2)
    vo = orc.linear(hn, lay["Wv"]).reshape(S, Hkv, dh).transpose(1, 0, 2)
    kh = orc.linear(hh, lay["Wk"]).reshape(S, Hkv, dh).transpose(1, 0, 2)
    vh = orc.linear(hh, lay["Wv"]).reshape(S, Hkv, dh).transpose(1, 0, 2)
    a = np.concatenate([orc.mixed_attn(q[None, s0:s0 + 4], kh[None], vh[None], ko[None], vo[None], [s0], gamma,
                                       1.0 / math.sqrt(dh))[0] for s0 in range(0, S, 4)])
    y1 = y + orc.linear(a.reshape(S, Hq * dh), lay["Wo"])
    y1 = y1 + orc.mlp(orc.rmsnorm(y1, lay["g_mlp"], eps), lay)
    if len(MS["layers"]) == 1:
        np.testing.assert_allclose(y1, orc.tandem_forward(T_, toks, gamma)["y"], rtol=1e-10, atol=1e-12)
    else:
        # compare through a one-small-layer copy of the model
        T1 = dict(T_)
        T1["S"] = dict(MS, layers=[lay])
        T1["ff"], T1["ell"] = T_["ff"][:1], T_["ell"][:1]
        np.testing.assert_allclose(y1, orc.tandem_forward(T1, toks, gamma)["y"], rtol=1e-10, atol=1e-12)


def test_block_prefix_attn_mask():
    """Deep Tandem's mask (Eq. (3)): against torch SDPA with the mask 'key j visible iff j < floor(i / gamma) gamma'
    written from the 0-indexed form (rows of the first block: zero), and against the paper's 1-indexed formula
    spelled out for gamma = 3 with uniform weights."""
    B, q_len, Hq, Hkv, dh, T, gamma = 2, 6, 4, 2, 8, 20, 3
    Q, K, V, _, _ = _mixed_case(8, B, q_len, Hq, Hkv, dh, T)
    n = np.array([11, 0])
    scale = dh ** -0.5
    got = orc.block_prefix_attn(Q, K, V, n, gamma, scale)
    G = Hq // Hkv
    for b in range(B):
        pos = n[b] + np.arange(q_len)
        kb = (pos // gamma) * gamma
        for r in range(q_len):
            if kb[r] == 0:
                assert (got[b, r] == 0).all()
                continue
            mask = (np.arange(T) < kb[r])[None, None, :]
            want = torch.nn.functional.scaled_dot_product_attention(
                torch.from_numpy(Q[b, r][:, None, :]), torch.from_numpy(np.repeat(K[b], G, axis=0)),
                torch.from_numpy(np.repeat(V[b], G, axis=0)), attn_mask=torch.from_numpy(mask), scale=scale).numpy()[:, 0]
            np.testing.assert_allclose(got[b, r], want, rtol=1e-11, atol=1e-12)
    # paper's 1-indexed formula, spelled out for gamma = 3: positions 1..3 see nothing, 4..6 see x_1..x_3, 7..9 x_1..x_6
    one = orc.block_prefix_attn(np.ones((1, 9, 1, 2)), np.zeros((1, 1, 9, 2)), np.arange(18.0).reshape(1, 1, 9, 2), [0], 3, 1.0)
    want_rows = [None] * 3 + [3] * 3 + [6] * 3
    V1 = np.arange(18.0).reshape(9, 2)
    for i, m in enumerate(want_rows):
        np.testing.assert_allclose(one[0, i, 0], 0.0 if m is None else V1[:m].mean(0), rtol=1e-13)


def test_draft_attn_shared_equals_draft_attn_on_materialised_caches():
    """Shared-prompt draft attention == the pinned draft_attn on per-sample K_hat caches that hold a copy of the
    prompt's rows followed by the sample's own completed rows."""
    rng = np.random.default_rng(12)
    B, ns, Hq, Hkv, dh, Ts, To, gmax = 2, 3, 4, 2, 8, 9, 6, 4
    mk = lambda *sh: rng.standard_normal(sh)
    q = mk(B, ns, Hq, dh)
    Khs, Vhs, Kho, Vho = mk(B, Hkv, Ts, dh), mk(B, Hkv, Ts, dh), mk(B * ns, Hkv, To, dh), mk(B * ns, Hkv, To, dh)
    kc, vc = mk(B * ns, Hkv, gmax, dh), mk(B * ns, Hkv, gmax, dh)
    n_shared, n_own, n_cur = np.array([9, 0]), np.array([0, 3, 6, 1, 0, 2]), np.array([1, 4, 2, 3, 1, 4])
    scale = dh ** -0.5
    got = orc.draft_attn_shared(q, Khs, Vhs, n_shared, Kho, Vho, n_own, kc, vc, n_cur, scale)
    Kc, Vc = np.zeros((B * ns, Hkv, Ts + To, dh)), np.zeros((B * ns, Hkv, Ts + To, dh))
    n = np.zeros(B * ns, dtype=np.int64)
    for b in range(B):
        for s_ in range(ns):
            i, m = b * ns + s_, n_shared[b]
            Kc[i, :, :m], Vc[i, :, :m] = Khs[b, :, :m], Vhs[b, :, :m]
            Kc[i, :, m:m + To], Vc[i, :, m:m + To] = Kho[i], Vho[i]
            n[i] = m + n_own[i]
    want = orc.draft_attn(q.reshape(B * ns, Hq, dh), Kc, Vc, n, kc, vc, n_cur, scale).reshape(q.shape)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
