"""fp64 CPU oracle for the Tandem Transformer hot path.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition of everything the HIP library computes.
It is written from the paper (Tandem Transformers, Sec. 3, Eq. (1) and Eq. (2),
Sec. 3.1, Fig. 2 and Fig. 4) and shares no code, table or helper with the HIP
path.  Only tests, the smoke check and the benchmark's CPU-baseline leg may
import it; the product path never does.

Everything is numpy float64, two-pass softmax, no tiling, no online softmax, no
fusion: every function is the definition written out so it can be checked
against the paper by eye.  Library primitives used as steps: numpy matmul,
numpy exp, scipy erf.

Conventions (chosen where the paper is silent; each is listed with its reason
in the design notes of the repository):
  * positions are 0-indexed; block of position i is floor(i/gamma); the
    boundary of Eq. (2) is k(i) = floor(i/gamma)*gamma; the large-derived set
    is {p < k(i)} and the own set is {k(i) <= p <= i} (never empty).  This is
    the reading of Eq. (2) that agrees with the two bullets of the Training
    paragraph and with Fig. 2 / Fig. 4.
  * x^(l(j)) is the residual stream after l(j) large layers, l(j) in [0, L_L].
  * a linear map is y = W x + b with W stored [out, in].
  * blocks are pre-norm RMSNorm (eps inside the square root), residual around
    attention and around the MLP, MLP = W2 gelu_erf(W1 x + b1) + b2,
    attention scale 1/sqrt(d_h), no positional encoding, untied output head
    after a final RMSNorm.
  * FF_Tandem is either linear (paper, Sec. 3 last sentence of the Tandem
    paragraph and Sec. 4) or a 2-layer MLP with erf-GELU.
  * SPEED acceptance is greedy: a draft token is accepted iff it equals the
    argmax of M_L's logits for that position; ties go to the lowest id.

Parity pins (tests/test_oracle_*.py): brute-force python-loop softmax, hand
cases, torch CPU scaled_dot_product_attention with an explicit mask, closed
forms (zero FF_Tandem), block-by-block == causal forward, gamma=1 == causal
decode, gamma -> inf == small model alone, incremental == teacher-forced,
SPEED stream == greedy M_L stream, integer schedules of Fig. 2 / Fig. 4; Deep Tandem (Sec. 5) against a
mask-based torch formulation and its limits (zero FF_DeepTandem == plain M_S; block length beyond the sequence ==
a constant sketch); its greedy decoding is the definition (forward re-evaluated per token), checked for prefix
consistency of the forward it relies on.
Parity unpinned by the paper (it prints no tensor values): the block internals
listed above (norm, activation, eps, head) and the MLP form of FF_Tandem; they
are pinned only by the configuration text this build was given.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# ----------------------------------------------------------------------------
# O1  attention primitive: softmax(q.K^T * scale) V, two-pass, one query.
#     (textbook definition behind Atn in Eq. (1) / Eq. (2))
# ----------------------------------------------------------------------------
def attention_one(q, K, V, scale):
    """q [dh], K [N, dh], V [N, dh] -> o [dh].  N >= 1."""
    q = np.asarray(q, F64)
    K = np.asarray(K, F64)
    V = np.asarray(V, F64)
    if K.shape[0] < 1:
        raise ValueError("attention over an empty key set")
    s = (K @ q) * scale
    e = np.exp(s - s.max())
    w = e / e.sum()
    return w @ V


# ----------------------------------------------------------------------------
# O2  large-model block-mode attention (Sec. 1 step 3, Sec. 3 "Inference",
#     Eq. (1) restricted to the q_len new rows).  The K/V rows of the new
#     tokens are already in the cache at [n, n + q_len).  Row r sees cache rows
#     0 .. n + r inclusive.
# ----------------------------------------------------------------------------
def block_attn(Q, Kc, Vc, n, scale):
    """Q [B, q_len, Hq, dh]; Kc, Vc [B, Hkv, T, dh]; n [B] ints -> O like Q."""
    Q = np.asarray(Q, F64)
    B, q_len, Hq, dh = Q.shape
    Hkv = Kc.shape[1]
    G = Hq // Hkv
    O = np.zeros_like(Q)
    for b in range(B):
        for r in range(q_len):
            last = int(n[b]) + r  # inclusive
            for h in range(Hq):
                kv = h // G
                O[b, r, h] = attention_one(Q[b, r, h], Kc[b, kv, : last + 1], Vc[b, kv, : last + 1], scale)
    return O


# ----------------------------------------------------------------------------
# O3  mixed-source small-model attention, Eq. (2) second line: one softmax
#     over the union of the large-derived rows for completed blocks and the
#     small model's own rows for the current block.
# ----------------------------------------------------------------------------
def draft_attn(q, khat, vhat, n_large, kcur, vcur, n_cur, scale):
    """q [B, Hq, dh]; khat, vhat [B, Hkv, T, dh]; kcur, vcur [B, Hkv, g, dh];
    n_large, n_cur [B] ints (n_cur >= 1) -> o [B, Hq, dh]."""
    q = np.asarray(q, F64)
    B, Hq, dh = q.shape
    Hkv = khat.shape[1]
    G = Hq // Hkv
    o = np.zeros_like(q)
    for b in range(B):
        nl, nc = int(n_large[b]), int(n_cur[b])
        for h in range(Hq):
            kv = h // G
            K = np.concatenate([np.asarray(khat[b, kv, :nl], F64), np.asarray(kcur[b, kv, :nc], F64)], axis=0)
            V = np.concatenate([np.asarray(vhat[b, kv, :nl], F64), np.asarray(vcur[b, kv, :nc], F64)], axis=0)
            o[b, h] = attention_one(q[b, h], K, V, scale)
    return o


# ----------------------------------------------------------------------------
# dense pieces
# ----------------------------------------------------------------------------
def gelu_erf(x):
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def relu(x):
    return np.maximum(x, 0.0)


def linear(x, W, b=None):
    """y = x W^T + b, W stored [out, in]."""
    y = np.asarray(x, F64) @ np.asarray(W, F64).T
    if b is not None:
        y = y + np.asarray(b, F64)
    return y


def rmsnorm(x, g, eps):
    x = np.asarray(x, F64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * np.asarray(g, F64)


_ACTS = {"gelu": gelu_erf, "relu": relu}


# ----------------------------------------------------------------------------
# O4  FF_Tandem, Eq. (2) first line: y_hat = FF_Tandem(x^(l(j))).
#     ff = {"W": [d_S, d_L], "b": opt}                      (linear form), or
#     ff = {"W1": [d_h, d_L], "b1", "W2": [d_S, d_h], "b2", "act": "gelu"|"relu"}
# ----------------------------------------------------------------------------
def project(X, ff):
    if "W" in ff:
        return linear(X, ff["W"], ff.get("b"))
    h = _ACTS[ff.get("act", "gelu")](linear(X, ff["W1"], ff.get("b1")))
    return linear(h, ff["W2"], ff.get("b2"))


def mlp(x, lay):
    return linear(gelu_erf(linear(x, lay["W1"], lay.get("b1"))), lay["W2"], lay.get("b2"))


def _heads(x, H, dh):
    return x.reshape(x.shape[0], H, dh)


# ----------------------------------------------------------------------------
# Eq. (1): the standard causal decoder, run by M_L over a whole sequence.
# Returns the residual stream after every layer: xs[j] = x^(j), j = 0..L.
# ----------------------------------------------------------------------------
def decoder_forward(M, tokens, eps):
    x = np.asarray(M["emb"], F64)[np.asarray(tokens)]
    S = x.shape[0]
    Hq, Hkv, dh = M["Hq"], M["Hkv"], M["dh"]
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(dh)
    xs = [x]
    for lay in M["layers"]:
        hn = rmsnorm(x, lay["g_attn"], eps)
        q = _heads(linear(hn, lay["Wq"]), Hq, dh)
        k = _heads(linear(hn, lay["Wk"]), Hkv, dh)
        v = _heads(linear(hn, lay["Wv"]), Hkv, dh)
        a = np.zeros((S, Hq, dh), F64)
        for i in range(S):
            for h in range(Hq):
                a[i, h] = attention_one(q[i, h], k[: i + 1, h // G], v[: i + 1, h // G], scale)
        x = x + linear(a.reshape(S, Hq * dh), lay["Wo"])
        x = x + mlp(rmsnorm(x, lay["g_mlp"], eps), lay)
        xs.append(x)
    return xs


def logits_of(M, x, eps):
    return linear(rmsnorm(x, M["g_final"], eps), M["W_out"])


def argmax_lowest(v):
    """argmax with ties resolved to the lowest index (numpy's rule)."""
    return int(np.argmax(v))


# ----------------------------------------------------------------------------
# O5  teacher-forced Tandem forward, Eq. (2), every position at once.
#     Returns dict with y (final small representations y^(L_S), [S, d_S]),
#     xs (large residual streams), yhat (per small layer), logits_S, logits_L.
# ----------------------------------------------------------------------------
def tandem_forward(T, tokens, gamma):
    eps = T["eps"]
    ML, MS = T["L"], T["S"]
    tokens = np.asarray(tokens)
    S = tokens.shape[0]
    xs = decoder_forward(ML, tokens, eps)
    yhat = [project(xs[T["ell"][j]], T["ff"][j]) for j in range(len(MS["layers"]))]
    Hq, Hkv, dh = MS["Hq"], MS["Hkv"], MS["dh"]
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(dh)
    y = np.asarray(MS["emb"], F64)[tokens]
    for j, lay in enumerate(MS["layers"]):
        hn = rmsnorm(y, lay["g_attn"], eps)
        q = _heads(linear(hn, lay["Wq"]), Hq, dh)
        k_own = _heads(linear(hn, lay["Wk"]), Hkv, dh)
        v_own = _heads(linear(hn, lay["Wv"]), Hkv, dh)
        hh = rmsnorm(yhat[j], lay["g_attn"], eps)
        k_hat = _heads(linear(hh, lay["Wk"]), Hkv, dh)
        v_hat = _heads(linear(hh, lay["Wv"]), Hkv, dh)
        a = np.zeros((S, Hq, dh), F64)
        for i in range(S):
            kb = (i // gamma) * gamma  # Eq. (2): k = floor(i/gamma)*gamma, 0-indexed reading
            for h in range(Hq):
                kv = h // G
                K = np.concatenate([k_hat[:kb, kv], k_own[kb : i + 1, kv]], axis=0)
                V = np.concatenate([v_hat[:kb, kv], v_own[kb : i + 1, kv]], axis=0)
                a[i, h] = attention_one(q[i, h], K, V, scale)
        y = y + linear(a.reshape(S, Hq * dh), lay["Wo"])
        y = y + mlp(rmsnorm(y, lay["g_mlp"], eps), lay)
    return {
        "y": y,
        "xs": xs,
        "yhat": yhat,
        "logits_S": logits_of(MS, y, eps),
        "logits_L": logits_of(ML, xs[-1], eps),
    }


def attended_sets(i, gamma):
    """Integer form of Eq. (2)'s context split for query position i (0-indexed):
    returns (large_positions, own_positions)."""
    kb = (i // gamma) * gamma
    return list(range(0, kb)), list(range(kb, i + 1))


# ----------------------------------------------------------------------------
# O6a  adaptive block length (Sec. 3.1 "Adaptive Block Length"; Sec. 4: tau = 0.8).  After every draft token a
#      2-layer router MLP looks at M_S's output distribution and decides whether M_S may go on drafting.
#      Features, in this order: the entropy of the distribution over the vocabulary (nats), the k largest
#      probabilities in descending order (equal values: lowest id first), and M_S's embedding rows of those k
#      tokens.  Readings (the paper fixes neither): hidden activation ReLU, output sigmoid = predicted
#      probability that M_L accepts the current draft token; drafting continues iff it is >= tau.
#      R = {"k": int, "W1": [H, 1 + k + k*d], "b1": [H], "w2": [H], "b2": scalar}
# ----------------------------------------------------------------------------
def router_features(logits, emb, k):
    lg = np.asarray(logits, F64)
    z = lg - lg.max()
    e = np.exp(z)
    Z = e.sum()
    prob = e / Z
    nz = prob > 0.0
    entropy = -(prob[nz] * np.log(prob[nz])).sum()
    ids = []
    for _ in range(k):
        best = -1
        for t in range(len(lg)):  # lowest id wins among equal logits
            if t in ids:
                continue
            if best < 0 or lg[t] > lg[best]:
                best = t
        ids.append(best)
    feats = [np.array([entropy]), prob[ids]] + [np.asarray(emb, F64)[t] for t in ids]
    return np.concatenate(feats), ids


def router_prob(R, logits, emb):
    f, _ = router_features(logits, emb, R["k"])
    h = relu(np.asarray(R["W1"], F64) @ f + np.asarray(R["b1"], F64))
    z = float(np.asarray(R["w2"], F64) @ h + float(np.asarray(R["b2"], F64).reshape(-1)[0]))
    return 1.0 / (1.0 + math.exp(-z))


# ----------------------------------------------------------------------------
# O6  one Tandem + SPEED decode step on caller-provided caches (Sec. 3.1,
#     Sec. 1 steps 2-4, Table 6: one step = gamma small runs + one large run).
#
# state = {
#   "KL","VL": list over large layers of [B, Hkv_L, T, dh] float64 arrays,
#   "Khat","Vhat": list over small layers of [B, Hkv_S, T, dh],
#   "n": [B] ints (positions that already have large-model rows),
#   "pending": [B] token ids (token at position n[b], no large rows yet) }
#
# forced: optional [B, gamma] token ids that replace the draft tokens
# d_1..d_gamma as the *inputs* of the following small runs and that are all
# treated as accepted (teacher forcing).  The state is updated in place.
# ----------------------------------------------------------------------------
def decode_step(T, state, gamma, forced=None, free_token=False, router=None, tau=0.8):
    """router: with it, gamma is the largest block length; sequence b stops drafting after the first draft token
    whose router probability is below tau (n_drafted[b] tokens, at least one) and M_L verifies that many (+ 1 with
    the free token); rows of the outputs beyond a sequence's own block length stay at their initial values."""
    assert router is None or forced is None
    eps = T["eps"]
    ML, MS = T["L"], T["S"]
    B = len(state["n"])
    LS, LL = len(MS["layers"]), len(ML["layers"])
    # rows M_L processes: the block [pending, d_1 .. d_{gamma-1}], plus d_gamma when the bonus ("free")
    # token of Sec. 3.1 / Fig. 2 is wanted
    nq = gamma + 1 if free_token else gamma
    out = {
        "draft": np.zeros((B, gamma), np.int64),
        "verify": np.zeros((B, nq), np.int64),
        "n_accepted": np.zeros(B, np.int64),
        "tokens": -np.ones((B, nq), np.int64),
        "n_emitted": np.zeros(B, np.int64),
        "y_small": np.zeros((B, gamma, MS["emb"].shape[1]), F64),
        "x_large": np.zeros((B, nq, ML["emb"].shape[1]), F64),
        "logits_S": np.zeros((B, gamma, MS["W_out"].shape[0]), F64),
        "logits_L": np.zeros((B, nq, ML["W_out"].shape[0]), F64),
        "n_drafted": np.full(B, gamma, np.int64),
        "router_p": np.full((B, gamma), np.nan, F64),
    }
    gamma_max, nq_max = gamma, nq
    for b in range(B):
        gamma, nq = gamma_max, nq_max
        n = int(state["n"][b])
        # ---- draft: gamma autoregressive runs of M_S (Sec. 3.1) ------------
        Hq, Hkv, dh = MS["Hq"], MS["Hkv"], MS["dh"]
        G = Hq // Hkv
        scale = 1.0 / math.sqrt(dh)
        kcur = [np.zeros((Hkv, 0, dh), F64) for _ in range(LS)]
        vcur = [np.zeros((Hkv, 0, dh), F64) for _ in range(LS)]
        inputs = [int(state["pending"][b])]
        for r in range(gamma):
            y = np.asarray(MS["emb"], F64)[inputs[r]]
            for j, lay in enumerate(MS["layers"]):
                hn = rmsnorm(y, lay["g_attn"], eps)
                q = linear(hn, lay["Wq"]).reshape(Hq, dh)
                k = linear(hn, lay["Wk"]).reshape(Hkv, 1, dh)
                v = linear(hn, lay["Wv"]).reshape(Hkv, 1, dh)
                kcur[j] = np.concatenate([kcur[j], k], axis=1)
                vcur[j] = np.concatenate([vcur[j], v], axis=1)
                a = np.zeros((Hq, dh), F64)
                for h in range(Hq):
                    kv = h // G
                    K = np.concatenate([state["Khat"][j][b, kv, :n], kcur[j][kv]], axis=0)
                    V = np.concatenate([state["Vhat"][j][b, kv, :n], vcur[j][kv]], axis=0)
                    a[h] = attention_one(q[h], K, V, scale)
                y = y + linear(a.reshape(Hq * dh), lay["Wo"])
                y = y + mlp(rmsnorm(y, lay["g_mlp"], eps), lay)
            out["y_small"][b, r] = y
            lg = logits_of(MS, y, eps)
            out["logits_S"][b, r] = lg
            d = argmax_lowest(lg)
            out["draft"][b, r] = d
            inputs.append(int(forced[b][r]) if forced is not None else d)
            if router is not None:
                pr = router_prob(router, lg, MS["emb"])
                out["router_p"][b, r] = pr
                if pr < tau:  # M_L is unlikely to accept this token: verify now
                    gamma = r + 1
                    break
        nq = gamma + 1 if free_token else gamma
        out["n_drafted"][b] = gamma
        # ---- verify: M_L in block mode on the first nq tokens of [pending, d_1 .. d_gamma] ----
        Hq, Hkv, dh = ML["Hq"], ML["Hkv"], ML["dh"]
        G = Hq // Hkv
        scale = 1.0 / math.sqrt(dh)
        x = np.asarray(ML["emb"], F64)[np.asarray(inputs[:nq])]
        xs = [x]
        for j, lay in enumerate(ML["layers"]):
            hn = rmsnorm(x, lay["g_attn"], eps)
            qh = _heads(linear(hn, lay["Wq"]), Hq, dh)
            k = _heads(linear(hn, lay["Wk"]), Hkv, dh)
            v = _heads(linear(hn, lay["Wv"]), Hkv, dh)
            state["KL"][j][b, :, n : n + nq] = k.transpose(1, 0, 2)
            state["VL"][j][b, :, n : n + nq] = v.transpose(1, 0, 2)
            a = np.zeros((nq, Hq, dh), F64)
            for r in range(nq):
                for h in range(Hq):
                    kv = h // G
                    a[r, h] = attention_one(
                        qh[r, h], state["KL"][j][b, kv, : n + r + 1], state["VL"][j][b, kv, : n + r + 1], scale
                    )
            x = x + linear(a.reshape(nq, Hq * dh), lay["Wo"])
            x = x + mlp(rmsnorm(x, lay["g_mlp"], eps), lay)
            xs.append(x)
        out["x_large"][b, :nq] = x
        lgL = logits_of(ML, x, eps)
        out["logits_L"][b, :nq] = lgL
        tL = [argmax_lowest(lgL[r]) for r in range(nq)]
        out["verify"][b, :nq] = tL
        # ---- FF_Tandem on the new rows, then the small layer's own norm and
        #      W_K / W_V turn y_hat into cached K_hat / V_hat (Eq. (2) line 1,
        #      Training paragraph second bullet) --------------------------
        for j, lay in enumerate(MS["layers"]):
            yh = project(xs[T["ell"][j]], T["ff"][j])
            hh = rmsnorm(yh, lay["g_attn"], eps)
            kh = _heads(linear(hh, lay["Wk"]), MS["Hkv"], MS["dh"])
            vh = _heads(linear(hh, lay["Wv"]), MS["Hkv"], MS["dh"])
            state["Khat"][j][b, :, n : n + nq] = kh.transpose(1, 0, 2)
            state["Vhat"][j][b, :, n : n + nq] = vh.transpose(1, 0, 2)
        # ---- accept (Sec. 3.1: first location where the draft is wrong) ----
        # Without the free token M_L has not seen d_gamma, so a fully accepted block emits gamma tokens and
        # d_gamma stays pending.  With it, M_L's token after the accepted prefix is always emitted: a + 1
        # tokens, the last of them the bonus token when all gamma drafts were right (Fig. 2).
        if forced is not None:
            a_cnt = gamma
            emitted = [int(t) for t in forced[b][:gamma]]
            if free_token:
                emitted.append(tL[gamma])
            new_pending = emitted[-1]
            n_new = n + nq
        else:
            a_cnt = 0
            while a_cnt < gamma and out["draft"][b, a_cnt] == tL[a_cnt]:
                a_cnt += 1
            if a_cnt < gamma or free_token:
                emitted = [int(t) for t in out["draft"][b, :a_cnt]] + [tL[a_cnt]]
            else:
                emitted = [int(t) for t in out["draft"][b, :gamma]]
            new_pending = emitted[-1]
            n_new = n + (a_cnt + 1 if free_token else min(a_cnt + 1, gamma))
        out["n_accepted"][b] = a_cnt
        out["n_emitted"][b] = len(emitted)
        out["tokens"][b, : len(emitted)] = emitted
        state["n"][b] = n_new
        state["pending"][b] = new_pending
    return out


def prefill_block(T, state, tokens, emit=False):
    """Prompt ingestion (Sec. 1 steps 1 and 3 for tokens that are already known; Sec. 3 "Inference"):
    for every sequence b, M_L processes tokens[b, 0:q] at positions n[b] .. n[b]+q-1 in block mode
    (Eq. (1): row r attends cache rows 0 .. n+r), which appends its K/V rows; FF_Tandem of x^(l(j))
    followed by small layer j's own norm and W_K / W_V appends the K_hat / V_hat rows (Eq. (2) line 1,
    Training paragraph second bullet).  M_S itself does not run: of its own rows only those of the block
    being drafted are ever attended (Eq. (2) line 2).  n[b] += q.  With emit, pending[b] becomes M_L's
    greedy token after the last row (the first generated token); otherwise pending is left alone.
    Returns x^(L_L) of the q rows and, with emit, the emitted tokens."""
    eps = T["eps"]
    ML, MS = T["L"], T["S"]
    tokens = np.asarray(tokens)
    B, nq = tokens.shape
    Hq, Hkv, dh = ML["Hq"], ML["Hkv"], ML["dh"]
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(dh)
    out = {"x_large": np.zeros((B, nq, ML["emb"].shape[1]), F64), "next": -np.ones(B, np.int64)}
    for b in range(B):
        n = int(state["n"][b])
        x = np.asarray(ML["emb"], F64)[tokens[b]]
        xs = [x]
        for j, lay in enumerate(ML["layers"]):
            hn = rmsnorm(x, lay["g_attn"], eps)
            qh = _heads(linear(hn, lay["Wq"]), Hq, dh)
            k = _heads(linear(hn, lay["Wk"]), Hkv, dh)
            v = _heads(linear(hn, lay["Wv"]), Hkv, dh)
            state["KL"][j][b, :, n : n + nq] = k.transpose(1, 0, 2)
            state["VL"][j][b, :, n : n + nq] = v.transpose(1, 0, 2)
            a = np.zeros((nq, Hq, dh), F64)
            for r in range(nq):
                for h in range(Hq):
                    kv = h // G
                    a[r, h] = attention_one(
                        qh[r, h], state["KL"][j][b, kv, : n + r + 1], state["VL"][j][b, kv, : n + r + 1], scale
                    )
            x = x + linear(a.reshape(nq, Hq * dh), lay["Wo"])
            x = x + mlp(rmsnorm(x, lay["g_mlp"], eps), lay)
            xs.append(x)
        out["x_large"][b] = x
        for j, lay in enumerate(MS["layers"]):
            yh = project(xs[T["ell"][j]], T["ff"][j])
            hh = rmsnorm(yh, lay["g_attn"], eps)
            kh = _heads(linear(hh, lay["Wk"]), MS["Hkv"], MS["dh"])
            vh = _heads(linear(hh, lay["Wv"]), MS["Hkv"], MS["dh"])
            state["Khat"][j][b, :, n : n + nq] = kh.transpose(1, 0, 2)
            state["Vhat"][j][b, :, n : n + nq] = vh.transpose(1, 0, 2)
        if emit:
            t = argmax_lowest(logits_of(ML, x[-1], eps))
            out["next"][b] = t
            state["pending"][b] = t
        state["n"][b] = n + nq
    return out


def empty_state(T, B, T_max):
    ML, MS = T["L"], T["S"]
    z = lambda M: np.zeros((B, M["Hkv"], T_max, M["dh"]), F64)
    return {
        "KL": [z(ML) for _ in ML["layers"]],
        "VL": [z(ML) for _ in ML["layers"]],
        "Khat": [z(MS) for _ in MS["layers"]],
        "Vhat": [z(MS) for _ in MS["layers"]],
        "n": np.zeros(B, np.int64),
        "pending": np.zeros(B, np.int64),
    }


def greedy_decode_large(ML, prompt, n_new, eps):
    """Plain greedy decoding with M_L alone (the stream SPEED must reproduce)."""
    toks = [int(t) for t in prompt]
    for _ in range(n_new):
        xs = decoder_forward(ML, np.asarray(toks), eps)
        toks.append(argmax_lowest(logits_of(ML, xs[-1][-1], eps)))
    return toks[len(prompt):]


# ----------------------------------------------------------------------------
# Several samples per prompt (Sec. 4 "num-samples"; footnote of Table 2): the
# samples of one prompt share the prompt's K/V rows; each has its own rows
# for what it generated.  Block-mode attention (Eq. (1) on the new rows) of
# sample s over [shared rows of its prompt ; its own rows], one softmax.
# ----------------------------------------------------------------------------
def block_attn_shared(Q, Ks, Vs, n_shared, Ko, Vo, n_own, scale):
    """Q [B, ns, q_len, Hq, dh]; Ks, Vs [B, Hkv, Ts, dh] with n_shared[b] valid rows, visible to every
    row of every sample of prompt b; Ko, Vo [B*ns, Hkv, To, dh], sample (b, s) = sequence b*ns + s, whose
    query row r sees own rows 0 .. n_own[b*ns+s] + r (its block's rows are already in place)."""
    Q = np.asarray(Q, F64)
    B, ns, q_len, Hq, dh = Q.shape
    Hkv = np.asarray(Ks).shape[1]
    G = Hq // Hkv
    out = np.zeros_like(Q)
    for b in range(B):
        for s in range(ns):
            i = b * ns + s
            for r in range(q_len):
                for h in range(Hq):
                    kv = h // G
                    K = np.concatenate([np.asarray(Ks, F64)[b, kv, : n_shared[b]], np.asarray(Ko, F64)[i, kv, : n_own[i] + r + 1]])
                    V = np.concatenate([np.asarray(Vs, F64)[b, kv, : n_shared[b]], np.asarray(Vo, F64)[i, kv, : n_own[i] + r + 1]])
                    out[b, s, r, h] = attention_one(Q[b, s, r, h], K, V, scale)
    return out


def draft_attn_shared(q, Khs, Vhs, n_shared, Kho, Vho, n_own, kcur, vcur, n_cur, scale):
    """The small model's draft attention (Eq. (2), second line) when `ns` samples continue one prompt: q
    [B, ns, Hq, dh]; Khs, Vhs [B, Hkv, Ts, dh] hold the K_hat / V_hat rows of the prompt, once per prompt; Kho, Vho
    [B*ns, Hkv, To, dh] those of each sample's completed blocks after the prompt; kcur, vcur [B*ns, Hkv, gmax, dh] the
    sample's own rows of the block being drafted.  Sample (b, s) = sequence i = b*ns + s attends, in one softmax,
    Khs[b, :, :n_shared[b]], Kho[i, :, :n_own[i]] and kcur[i, :, :n_cur[i]]."""
    q = np.asarray(q, F64)
    B, ns, Hq, dh = q.shape
    Hkv = np.asarray(Khs).shape[1]
    G = Hq // Hkv
    out = np.zeros_like(q)
    for b in range(B):
        for s in range(ns):
            i = b * ns + s
            for h in range(Hq):
                kv = h // G
                K = np.concatenate([np.asarray(Khs, F64)[b, kv, : n_shared[b]], np.asarray(Kho, F64)[i, kv, : n_own[i]],
                                    np.asarray(kcur, F64)[i, kv, : n_cur[i]]])
                V = np.concatenate([np.asarray(Vhs, F64)[b, kv, : n_shared[b]], np.asarray(Vho, F64)[i, kv, : n_own[i]],
                                    np.asarray(vcur, F64)[i, kv, : n_cur[i]]])
                out[b, s, h] = attention_one(q[b, s, h], K, V, scale)
    return out


# ----------------------------------------------------------------------------
# a4'  the small model's attention at EVERY position of a known sequence (Eq. (2), second line, with the
#      block boundary k = floor(i / gamma) * gamma of the query's own position i, 0-indexed; Sec. 3
#      "Training": this is the form used for training and for teacher-forced scoring).  One call handles
#      q_len consecutive positions n[b] .. n[b] + q_len - 1 of every sequence.
# ----------------------------------------------------------------------------
def mixed_attn(Q, Khat, Vhat, Kown, Vown, n, gamma, scale):
    """Q [B, q_len, Hq, dh]; Khat, Vhat (rows derived from M_L through FF_Tandem) and Kown, Vown (rows M_S
    computed itself) [B, Hkv, T, dh], all indexed by absolute position.  The query at position
    i = n[b] + r attends Khat/Vhat[0 : k) and Kown/Vown[k : i + 1) in one softmax, k = (i // gamma) * gamma."""
    Q = np.asarray(Q, F64)
    B, q_len, Hq, dh = Q.shape
    Hkv = np.asarray(Khat).shape[1]
    G = Hq // Hkv
    out = np.zeros_like(Q)
    for b in range(B):
        for r in range(q_len):
            i = int(n[b]) + r
            large, own = attended_sets(i, gamma)
            for h in range(Hq):
                kv = h // G
                K = np.concatenate([np.asarray(Khat, F64)[b, kv, large], np.asarray(Kown, F64)[b, kv, own]])
                V = np.concatenate([np.asarray(Vhat, F64)[b, kv, large], np.asarray(Vown, F64)[b, kv, own]])
                out[b, r, h] = attention_one(Q[b, r, h], K, V, scale)
    return out


# ----------------------------------------------------------------------------
# a3'  Deep Tandem's large-model attention (Eq. (3)): the query at position i attends only the positions of the
#      blocks completed before its own block, keys x_{<= k gamma} with k = ceil((i - gamma) / gamma) in the
#      paper's 1-indexed positions - 0-indexed: keys j < floor(i / gamma) * gamma.  Queries of the first block see
#      no key at all; their output is defined as zero here (the paper does not say).
# ----------------------------------------------------------------------------
def block_prefix_attn(Q, Kc, Vc, n, gamma, scale):
    """Q [B, q_len, Hq, dh] for positions n[b] .. n[b] + q_len - 1; Kc, Vc [B, Hkv, T, dh] indexed by position."""
    Q = np.asarray(Q, F64)
    B, q_len, Hq, dh = Q.shape
    Hkv = np.asarray(Kc).shape[1]
    G = Hq // Hkv
    out = np.zeros_like(Q)
    for b in range(B):
        for r in range(q_len):
            i1 = int(n[b]) + r + 1                     # the paper's 1-indexed position
            k = -((-(i1 - gamma)) // gamma)            # ceil((i - gamma) / gamma)
            visible = max(k, 0) * gamma                # keys x_1 .. x_{k gamma}
            if visible == 0:
                continue
            for h in range(Hq):
                kv = h // G
                out[b, r, h] = attention_one(Q[b, r, h], np.asarray(Kc, F64)[b, kv, :visible],
                                             np.asarray(Vc, F64)[b, kv, :visible], scale)
    return out


# ----------------------------------------------------------------------------
# Deep Tandem (Sec. 5, Eq. (3) and Eq. (4)): M_L predicts a sketch of the next block in parallel, M_S samples
# autoregressively on top of it.  Written in the paper's 1-indexed notation: tokens x_1 .. x_S, block length gamma.
#
#   Eq. (3), for every row i >= 1 and k = ceil((i - gamma) / gamma):
#     x_i^(0)   = Emb_L(x_{i - gamma})                                   (the formula's reading, see below)
#     x~_i^(j+1) = Atn_L^(j+1)( x_i^(j) | x_{<= k gamma}^(j) ),   x_i^(j+1) = FF_L^(j+1)(x~_i^(j+1))
#   Eq. (4), for every row i >= 2:
#     y_i^(0)   = Emb_S(x_{i-1}) + FF_DeepTandem(x_i^(L_L))
#     y~_i^(j+1) = Atn_S^(j+1)( y_i^(j) | y_{<= i}^(j) ),         y_i^(j+1) = FF_S^(j+1)(y~_i^(j+1))
#   y_i^(L_S) is the model's prediction of token i.
#
# Readings (the paper is at odds with itself or silent; each is listed in the design notes):
#   * the input of row i: the displayed formula gives Emb_L of token i - gamma, the sentence after it the
#     (ceil((i - gamma) / gamma) gamma)-th token.  The formula is taken: with the sentence's reading all gamma rows
#     of a block would get the same input and - there being no positional encoding here - the same sketch.
#   * rows i <= gamma have no token i - gamma and see no key (k = 0): x_i^(0) = 0 and the attention output is 0
#     (the layers' residual and MLP still act on them).
#   * keys and values of a visible row are that row's own x^(j) under the layer's norm and W_K / W_V, as in Eq. (1).
#   * M_S has no input for i = 1 (there is no x_0): its rows are i = 2 .. S + 1; row i reads M_L's row i.
#   * blocks, norms, MLPs, heads as in the Tandem forward above.
# T["ff_deep"]: FF_DeepTandem, d_L -> d_S, same forms as FF_Tandem.
# ----------------------------------------------------------------------------
def deep_tandem_forward(T, tokens, gamma):
    """tokens: x_1 .. x_S.  Returns {"sketch": x^(L_L) of rows i = 1 .. S+1, "y": y^(L_S) of rows i = 2 .. S+1
    (S rows; row i predicts token i), "logits": M_S's logits of those rows}."""
    eps = T["eps"]
    ML, MS = T["L"], T["S"]
    x_tok = {i + 1: int(t) for i, t in enumerate(np.asarray(tokens))}  # 1-indexed tokens
    S = len(x_tok)
    rows = list(range(1, S + 2))  # rows of M_L
    dL = np.asarray(ML["emb"]).shape[1]
    x = {i: (np.asarray(ML["emb"], F64)[x_tok[i - gamma]] if i - gamma >= 1 else np.zeros(dL, F64)) for i in rows}
    Hq, Hkv, dh = ML["Hq"], ML["Hkv"], ML["dh"]
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(dh)
    for lay in ML["layers"]:
        hn = {i: rmsnorm(x[i], lay["g_attn"], eps) for i in rows}
        q = {i: linear(hn[i], lay["Wq"]).reshape(Hq, dh) for i in rows}
        kk = {i: linear(hn[i], lay["Wk"]).reshape(Hkv, dh) for i in rows}
        vv = {i: linear(hn[i], lay["Wv"]).reshape(Hkv, dh) for i in rows}
        nxt = {}
        for i in rows:
            k = -((-(i - gamma)) // gamma)  # ceil((i - gamma) / gamma)
            vis = list(range(1, max(k, 0) * gamma + 1))  # rows x_1 .. x_{k gamma}
            a = np.zeros((Hq, dh), F64)
            if vis:
                for h in range(Hq):
                    K = np.stack([kk[p][h // G] for p in vis])
                    V = np.stack([vv[p][h // G] for p in vis])
                    a[h] = attention_one(q[i][h], K, V, scale)
            xt = x[i] + linear(a.reshape(Hq * dh), lay["Wo"])
            nxt[i] = xt + mlp(rmsnorm(xt, lay["g_mlp"], eps), lay)
        x = nxt
    sketch = np.stack([x[i] for i in rows])
    srows = list(range(2, S + 2))  # rows of M_S
    y = {i: np.asarray(MS["emb"], F64)[x_tok[i - 1]] + project(x[i], T["ff_deep"]) for i in srows}
    Hq, Hkv, dh = MS["Hq"], MS["Hkv"], MS["dh"]
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(dh)
    for lay in MS["layers"]:
        hn = {i: rmsnorm(y[i], lay["g_attn"], eps) for i in srows}
        q = {i: linear(hn[i], lay["Wq"]).reshape(Hq, dh) for i in srows}
        kk = {i: linear(hn[i], lay["Wk"]).reshape(Hkv, dh) for i in srows}
        vv = {i: linear(hn[i], lay["Wv"]).reshape(Hkv, dh) for i in srows}
        nxt = {}
        for i in srows:
            vis = [p for p in srows if p <= i]
            a = np.zeros((Hq, dh), F64)
            for h in range(Hq):
                K = np.stack([kk[p][h // G] for p in vis])
                V = np.stack([vv[p][h // G] for p in vis])
                a[h] = attention_one(q[i][h], K, V, scale)
            yt = y[i] + linear(a.reshape(Hq * dh), lay["Wo"])
            nxt[i] = yt + mlp(rmsnorm(yt, lay["g_mlp"], eps), lay)
        y = nxt
    yo = np.stack([y[i] for i in srows])
    return {"sketch": sketch, "y": yo, "logits": logits_of(MS, yo, eps)}


def deep_tandem_generate(T, tokens, gamma, n_new):
    """Greedy decoding with the Deep Tandem model (Sec. 5): the next token is the highest-logit token of the model's
    prediction for the next row given all tokens so far (ties to the lowest id), n_new times.  Written as the
    definition: the whole forward of Eq. (3)-(4) is evaluated again for every new token; nothing is cached.
    (M_L's rows of a block read only tokens at least gamma positions back, which is what lets an implementation
    compute the sketch of a whole block before M_S samples it - that structure is not used here.)
    Returns {"tokens": prompt followed by the n_new new tokens, "logits": the n_new logit rows they came from}."""
    toks = [int(t) for t in np.asarray(tokens)]
    rows = []
    for _ in range(n_new):
        lg = deep_tandem_forward(T, np.asarray(toks), gamma)["logits"][-1]  # row S + 1: the prediction of token S + 1
        rows.append(lg)
        toks.append(argmax_lowest(lg))
    return {"tokens": np.asarray(toks, np.int64), "logits": np.stack(rows)}


# ----------------------------------------------------------------------------
# a5  split-K re-association of the softmax (exact in real arithmetic):
#     per split (m_s, l_s, O_s) with O_s un-normalised; merged in split order.
# ----------------------------------------------------------------------------
def attention_one_split(q, K, V, scale, bounds):
    """Same result as attention_one, computed over the key ranges
    [bounds[s], bounds[s+1]) separately and merged; empty ranges allowed."""
    q = np.asarray(q, F64)
    parts = []
    for s in range(len(bounds) - 1):
        lo, hi = bounds[s], bounds[s + 1]
        if hi <= lo:
            parts.append((-np.inf, 0.0, np.zeros(V.shape[1], F64)))
            continue
        sc = (np.asarray(K[lo:hi], F64) @ q) * scale
        m = sc.max()
        e = np.exp(sc - m)
        parts.append((m, e.sum(), e @ np.asarray(V[lo:hi], F64)))
    m = max(p[0] for p in parts)
    l = sum(p[1] * math.exp(p[0] - m) for p in parts if p[1] > 0.0)
    o = sum(p[2] * math.exp(p[0] - m) for p in parts if p[1] > 0.0)
    return o / l


# ----------------------------------------------------------------------------
# Integer schedules of the two inference configurations (Sec. 3 "Inference",
# Fig. 2: with the free token; Fig. 4: representations only).  Positions are
# 0-indexed; the prompt has P tokens at positions 0..P-1.  Each event is
#   ("L", processed_positions, emitted_position_or_None)   one M_L block run
#   ("S", input_position, large_visible, own_visible, emitted_position)
# ----------------------------------------------------------------------------
def inference_schedule(P, gamma, n_blocks, free_token):
    ev = []
    if free_token:
        ev.append(("L", list(range(0, P)), P))
        n = P  # positions < n have large representations; position n is M_L's token
    else:
        ev.append(("L", list(range(0, P - 1)), None))
        n = P - 1
    for blk in range(n_blocks):
        for r in range(gamma):
            i = n + r
            ev.append(("S", i, list(range(0, n)), list(range(n, i + 1)), i + 1))
        if free_token:
            ev.append(("L", list(range(n, n + gamma + 1)), n + gamma + 1))
            n += gamma + 1
        else:
            ev.append(("L", list(range(n, n + gamma)), None))
            n += gamma
    return ev
