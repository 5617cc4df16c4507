"""Pins for the oracle's Deep Tandem forward (Sec. 5, Eq. (3) and Eq. (4)).  CPU only: a mask-based batched torch
formulation, the limits that reduce it to the plain small model, and the block structure of its dependencies."""
import copy

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import tandem_oracle as orc
from paper_2402_08644_amd import inputs


def deep_pair(seed=0, d_hidden=24, gain_std=0.3, bias_std=0.2, w_std=0.3):
    W = inputs.tandem_weights(
        seed, vocab=40, large=dict(d=32, n_layers=3, Hq=4, Hkv=2, dh=8, d_ff=48),
        small=dict(d=16, n_layers=2, Hq=2, Hkv=2, dh=8, d_ff=32), ell=(1, 3), d_hidden=d_hidden, dtype="f32", w_std=w_std,
        gain_std=gain_std, bias_std=bias_std, deep=True)
    return inputs.as_f64(W)


def test_visible_rows_of_eq3_index_algebra():
    """k = ceil((i - gamma) / gamma) in 1-indexed rows: row i sees rows 1 .. k gamma, i.e. exactly the blocks
    completed before its own; written out for gamma = 2 and checked against the closed form for others."""
    ceil_div = lambda a, b: -((-a) // b)
    seen = {i: max(ceil_div(i - 2, 2), 0) * 2 for i in range(1, 8)}
    assert seen == {1: 0, 2: 0, 3: 2, 4: 2, 5: 4, 6: 4, 7: 6}
    for gamma in (1, 2, 3, 5):
        for i in range(1, 40):
            k = max(ceil_div(i - gamma, gamma), 0)
            assert k * gamma == ((i - 1) // gamma) * gamma  # rows of the blocks before the block of row i
            assert k * gamma < i                              # never the row itself


def torch_deep_forward(T, tokens, gamma):
    """Batched formulation with torch CPU fp64 library ops: one SDPA per layer with an explicit mask."""
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    eps = T["eps"]
    S = len(tokens)
    tok = torch.from_numpy(np.asarray(tokens))

    def block(M, lay, x, mask):
        n = x.shape[0]
        Hq, Hkv, dh = M["Hq"], M["Hkv"], M["dh"]
        hn = F.rms_norm(x, (x.shape[-1],), t(lay["g_attn"]), eps=eps)
        q = F.linear(hn, t(lay["Wq"])).view(n, Hq, dh).transpose(0, 1)
        k = F.linear(hn, t(lay["Wk"])).view(n, Hkv, dh).transpose(0, 1).repeat_interleave(Hq // Hkv, 0)
        v = F.linear(hn, t(lay["Wv"])).view(n, Hkv, dh).transpose(0, 1).repeat_interleave(Hq // Hkv, 0)
        empty = ~mask.any(dim=1)
        safe = mask.clone()
        safe[empty] = True  # rows that see nothing: any mask, their output is replaced by zero
        a = F.scaled_dot_product_attention(q, k, v, attn_mask=safe, scale=dh**-0.5).transpose(0, 1).reshape(n, Hq * dh)
        a = a * (~empty)[:, None]
        x = x + F.linear(a, t(lay["Wo"]))
        hm = F.rms_norm(x, (x.shape[-1],), t(lay["g_mlp"]), eps=eps)
        return x + F.linear(F.gelu(F.linear(hm, t(lay["W1"]), t(lay["b1"]))), t(lay["W2"]), t(lay["b2"]))

    i = torch.arange(1, S + 2)  # rows of M_L, 1-indexed
    src = i - gamma             # token index of the row's input
    x = t(T["L"]["emb"])[tok[(src - 1).clamp(min=0)]] * (src >= 1)[:, None]
    seen = torch.div(i - 1, gamma, rounding_mode="floor") * gamma  # rows 1 .. seen are visible
    mask = i[None, :] <= seen[:, None]
    for lay in T["L"]["layers"]:
        x = block(T["L"], lay, x, mask)
    ff = T["ff_deep"]
    if "W" in ff:
        sk = F.linear(x, t(ff["W"]), t(ff["b"]))
    else:
        sk = F.linear(F.gelu(F.linear(x, t(ff["W1"]), t(ff["b1"]))), t(ff["W2"]), t(ff["b2"]))
    y = t(T["S"]["emb"])[tok] + sk[1:]  # rows i = 2 .. S+1 read token i-1 and sketch row i
    causal = torch.tril(torch.ones(S, S, dtype=torch.bool))
    for lay in T["S"]["layers"]:
        y = block(T["S"], lay, y, causal)
    lg = F.linear(F.rms_norm(y, (y.shape[-1],), t(T["S"]["g_final"]), eps=eps), t(T["S"]["W_out"]))
    return x.numpy(), y.numpy(), lg.numpy()


@pytest.mark.parametrize("gamma,d_hidden", [(1, 24), (2, 24), (3, 0), (4, 24), (20, 24)])
def test_deep_forward_vs_torch_mask_formulation(gamma, d_hidden):
    T = deep_pair(seed=gamma, d_hidden=d_hidden)
    toks = inputs.token_ids(gamma, (13,), 40)
    got = orc.deep_tandem_forward(T, toks, gamma)
    sk, y, lg = torch_deep_forward(T, toks, gamma)
    np.testing.assert_allclose(got["sketch"], sk, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(got["y"], y, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(got["logits"], lg, rtol=1e-9, atol=1e-11)


def test_zero_ff_deep_tandem_is_the_plain_small_model():
    """Eq. (4) with FF_DeepTandem = 0: y_i^(0) = Emb_S(x_{i-1}) and M_S is an ordinary causal decoder over the tokens."""
    T = deep_pair(seed=5)
    for k in ("W2", "b2"):
        T["ff_deep"][k] = np.zeros_like(T["ff_deep"][k])
    toks = inputs.token_ids(5, (12,), 40)
    got = orc.deep_tandem_forward(T, toks, 3)["y"]
    want = orc.decoder_forward(T["S"], toks, T["eps"])[-1]
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)


def test_block_longer_than_the_sequence_gives_a_constant_sketch():
    """gamma beyond the sequence: no row of M_L has an input token or a visible key, so every sketch row is the same
    vector c, and the model is M_S with FF_DeepTandem(c) added to every input embedding."""
    T = deep_pair(seed=6)
    toks = inputs.token_ids(6, (9,), 40)
    out = orc.deep_tandem_forward(T, toks, 50)
    sk = out["sketch"]
    np.testing.assert_allclose(sk, np.broadcast_to(sk[0], sk.shape), rtol=0, atol=0)
    MS = copy.deepcopy(T["S"])
    MS["emb"] = np.asarray(MS["emb"]) + orc.project(sk[0], T["ff_deep"])
    want = orc.decoder_forward(MS, toks, T["eps"])[-1]
    np.testing.assert_allclose(out["y"], want, rtol=1e-12, atol=1e-14)


def test_sketch_of_a_block_depends_only_on_completed_blocks():
    """Changing token x_t (1-indexed) leaves every sketch row that does not read it, directly (its own input is token
    i - gamma) or through a visible row, untouched; M_S's rows up to t are untouched as well (row i reads x_{i-1})."""
    T = deep_pair(seed=7)
    gamma, S = 3, 13
    toks = inputs.token_ids(7, (S,), 40)
    a = orc.deep_tandem_forward(T, toks, gamma)
    for t in (1, 4, 7, S):  # 1-indexed position of the changed token
        toks2 = toks.copy()
        toks2[t - 1] = (toks2[t - 1] + 1) % 40
        b = orc.deep_tandem_forward(T, toks2, gamma)
        rows = np.arange(1, S + 2)
        # row i reads token i - gamma itself and, through its keys, the inputs of rows <= floor((i-1)/gamma) gamma
        direct = rows - gamma == t
        via_keys = ((rows - 1) // gamma) * gamma - gamma >= t
        touched = direct | via_keys
        same = np.all(a["sketch"] == b["sketch"], axis=1)
        assert (same == ~touched).all(), (t, same, touched)
        np.testing.assert_array_equal(a["y"][: t - 1], b["y"][: t - 1])  # rows i = 2 .. t
        if t <= S:
            assert np.abs(a["y"][t - 1] - b["y"][t - 1]).max() > 1e-9  # row i = t + 1 reads token t


def test_forward_is_prefix_consistent():
    """Row i of the forward reads tokens below i only: appending tokens leaves the earlier rows' sketches,
    and representations bit for bit the same (the logits to rounding) - what makes greedy decoding by re-evaluation well defined."""
    T = deep_pair(seed=8)
    toks = inputs.token_ids(8, (14,), 40)
    full = orc.deep_tandem_forward(T, toks, 3)
    for S in (1, 2, 5, 9):
        part = orc.deep_tandem_forward(T, toks[:S], 3)
        np.testing.assert_array_equal(part["sketch"], full["sketch"][: S + 1])
        np.testing.assert_array_equal(part["y"], full["y"][:S])
        # the head is one matrix product over all rows: its rounding depends on the number of rows
        np.testing.assert_allclose(part["logits"], full["logits"][:S], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("gamma,S0", [(1, 3), (3, 1), (3, 6), (4, 5)])
def test_greedy_generation_vs_block_schedule(gamma, S0):
    """Greedy decoding by definition (forward re-evaluated for every token) against the schedule an implementation
    would run: whenever gamma new tokens are due, M_L's next gamma rows are computed at once from the tokens known
    so far (their sketches do not depend on the tokens about to be sampled), then M_S samples token by token on top
    of them.  Here that schedule is emulated with the mask-based torch forward on a sequence padded with wrong
    tokens where the future ones would be: the sketches of the gamma rows and each next-token distribution must not
    see the padding."""
    T = deep_pair(seed=20 + gamma)
    prompt = inputs.token_ids(9, (S0,), 40)
    n_new = 2 * gamma + 1
    want = orc.deep_tandem_generate(T, prompt, gamma, n_new)
    assert want["tokens"].shape == (S0 + n_new,)
    np.testing.assert_array_equal(want["tokens"][:S0], prompt)
    toks = [int(t) for t in prompt]
    got_logits = []
    while len(toks) < S0 + n_new:
        S = len(toks)
        # M_L rows S + 1 .. S + gamma (1-indexed) from the S known tokens, padded with garbage future tokens
        padded = np.asarray(toks + [39 - (t % 7) for t in range(gamma)])
        sk, _, _ = torch_deep_forward(T, padded, gamma)
        sketch_rows = sk[S : S + gamma]  # rows S + 1 .. S + gamma
        for t in range(gamma):
            if len(toks) == S0 + n_new:
                break
            cur = np.asarray(toks + [0] * (gamma - t))  # the tokens sampled so far in this block are real
            sk2, _, lg = torch_deep_forward(T, cur, gamma)
            np.testing.assert_allclose(sk2[S + t], sketch_rows[t], rtol=1e-10, atol=1e-12)  # computed before sampling
            row = lg[len(toks) - 1]  # M_S row that reads the last real token
            got_logits.append(row)
            toks.append(int(np.argmax(row)))
    np.testing.assert_array_equal(np.asarray(toks), want["tokens"])
    np.testing.assert_allclose(np.stack(got_logits), want["logits"], rtol=1e-8, atol=1e-10)


def test_generated_tokens_are_the_argmax_of_the_teacher_forced_rows():
    """Scoring the generated sequence reproduces it: token S0 + t is the highest logit of row S0 + t - 1."""
    T = deep_pair(seed=31)
    prompt = inputs.token_ids(10, (4,), 40)
    out = orc.deep_tandem_generate(T, prompt, 2, 7)
    lg = orc.deep_tandem_forward(T, out["tokens"][:-1], 2)["logits"]
    np.testing.assert_array_equal(np.argmax(lg[3:], axis=1), out["tokens"][4:])
    np.testing.assert_allclose(lg[3:], out["logits"], rtol=1e-12, atol=1e-14)
