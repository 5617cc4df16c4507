"""Seeded synthetic input generators.

This module holds NO arithmetic of the method: it only draws seeded random
tensors with the shapes and value distributions of the benchmark configurations
and rounds them to the storage type.  It is the one module that both the test
oracle and the HIP path are fed from, so it imports neither.

Host generators return numpy arrays.  bf16 tensors are represented on the host
as a pair: ``bits`` (uint16, the storage the GPU receives) and ``f64`` (the very
same values widened exactly, which the oracle receives).
"""
from __future__ import annotations

import math

import numpy as np


# ---------------------------------------------------------------- bf16 storage
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit pattern (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float64."""
    u = bits.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


class HostTensor:
    """A host tensor in its storage dtype plus the exact float64 view of it."""

    __slots__ = ("dtype", "store", "f64")

    def __init__(self, values_f32: np.ndarray, dtype: str):
        self.dtype = dtype
        if dtype == "bf16":
            self.store = f32_to_bf16_bits(values_f32)
            self.f64 = bf16_bits_to_f64(self.store)
        elif dtype == "f32":
            self.store = np.ascontiguousarray(values_f32, dtype=np.float32)
            self.f64 = self.store.astype(np.float64)
        else:
            raise ValueError(dtype)

    @property
    def shape(self):
        return self.store.shape

    def to_torch(self, device="cuda"):
        import torch

        if self.dtype == "bf16":
            t = torch.from_numpy(self.store.view(np.int16).copy()).view(torch.bfloat16)
        else:
            t = torch.from_numpy(self.store.copy())
        return t.to(device)


def normal(rng: np.random.Generator, shape, std: float, dtype: str) -> HostTensor:
    return HostTensor((rng.standard_normal(shape, dtype=np.float32) * np.float32(std)), dtype)


def zeros(shape, dtype: str) -> HostTensor:
    return HostTensor(np.zeros(shape, np.float32), dtype)


def ones(shape, dtype: str) -> HostTensor:
    return HostTensor(np.ones(shape, np.float32), dtype)


def torch_to_f64(t) -> np.ndarray:
    """Device/host torch tensor (bf16 or f32) -> float64 numpy, exact."""
    return t.detach().to("cpu").double().numpy()


# ------------------------------------------------------- attention-only cases
def draft_attn_case(seed, B, Hq, Hkv, dh, T_max, gamma_max, n_large, n_cur, dtype="bf16", kv_std=None, q_std=1.0):
    """Inputs of one mixed-source small-model attention call.

    q ~ N(0, q_std); K/V rows ~ N(0, kv_std) (default 1/sqrt(dh)); ``n_large`` and
    ``n_cur`` may be ints or per-sequence lists."""
    rng = np.random.default_rng(seed)
    kv_std = (1.0 / math.sqrt(dh)) if kv_std is None else kv_std
    case = {
        "q": normal(rng, (B, Hq, dh), q_std, dtype),
        "khat": normal(rng, (B, Hkv, T_max, dh), kv_std, dtype),
        "vhat": normal(rng, (B, Hkv, T_max, dh), kv_std, dtype),
        "kcur": normal(rng, (B, Hkv, gamma_max, dh), kv_std, dtype),
        "vcur": normal(rng, (B, Hkv, gamma_max, dh), kv_std, dtype),
        "n_large": np.broadcast_to(np.asarray(n_large, np.int32), (B,)).copy(),
        "n_cur": np.broadcast_to(np.asarray(n_cur, np.int32), (B,)).copy(),
        "scale": 1.0 / math.sqrt(dh),
    }
    return case


def block_attn_case(seed, B, q_len, Hq, Hkv, dh, T_max, n_prefix, dtype="bf16", std=1.0):
    """Inputs of one large-model block-mode attention call (Q/K/V ~ N(0, std))."""
    rng = np.random.default_rng(seed)
    return {
        "q": normal(rng, (B, q_len, Hq, dh), std, dtype),
        "k": normal(rng, (B, Hkv, T_max, dh), std, dtype),
        "v": normal(rng, (B, Hkv, T_max, dh), std, dtype),
        "n": np.broadcast_to(np.asarray(n_prefix, np.int32), (B,)).copy(),
        "scale": 1.0 / math.sqrt(dh),
    }


def shared_attn_case(seed, B, samples, q_len, Hq, Hkv, dh, T_shared, T_own, n_shared, n_own, dtype="bf16", std=1.0):
    """Inputs of one block-mode attention call in which `samples` sequences continue each of B prompts: the
    prompt rows once per prompt, each sample's later rows in a cache of its own (Q/K/V ~ N(0, std))."""
    rng = np.random.default_rng(seed)
    return {
        "q": normal(rng, (B, samples, q_len, Hq, dh), std, dtype),
        "ks": normal(rng, (B, Hkv, T_shared, dh), std, dtype),
        "vs": normal(rng, (B, Hkv, T_shared, dh), std, dtype),
        "ko": normal(rng, (B * samples, Hkv, T_own, dh), std, dtype),
        "vo": normal(rng, (B * samples, Hkv, T_own, dh), std, dtype),
        "n_shared": np.broadcast_to(np.asarray(n_shared, np.int32), (B,)).copy(),
        "n_own": np.broadcast_to(np.asarray(n_own, np.int32), (B * samples,)).copy(),
        "scale": 1.0 / math.sqrt(dh),
    }


def shared_draft_case(seed, B, samples, Hq, Hkv, dh, T_shared, T_own, gmax, n_shared, n_own, n_cur, dtype="bf16", std=1.0):
    """Inputs of one draft-attention call in which `samples` sequences continue each of B prompts."""
    rng = np.random.default_rng(seed)
    nseq = B * samples
    return {
        "q": normal(rng, (B, samples, Hq, dh), std, dtype),
        "khs": normal(rng, (B, Hkv, T_shared, dh), std, dtype),
        "vhs": normal(rng, (B, Hkv, T_shared, dh), std, dtype),
        "kho": normal(rng, (nseq, Hkv, T_own, dh), std, dtype),
        "vho": normal(rng, (nseq, Hkv, T_own, dh), std, dtype),
        "kcur": normal(rng, (nseq, Hkv, gmax, dh), std, dtype),
        "vcur": normal(rng, (nseq, Hkv, gmax, dh), std, dtype),
        "n_shared": np.broadcast_to(np.asarray(n_shared, np.int32), (B,)).copy(),
        "n_own": np.broadcast_to(np.asarray(n_own, np.int32), (nseq,)).copy(),
        "n_cur": np.broadcast_to(np.asarray(n_cur, np.int32), (nseq,)).copy(),
        "scale": 1.0 / math.sqrt(dh),
    }


def mixed_attn_case(seed, B, q_len, Hq, Hkv, dh, T_max, n_prefix, dtype="bf16", std=1.0):
    """Inputs of one all-positions small-model attention call: queries for q_len consecutive positions and the
    two caches (rows derived from the large model; the small model's own rows), Q/K/V ~ N(0, std)."""
    rng = np.random.default_rng(seed)
    return {
        "q": normal(rng, (B, q_len, Hq, dh), std, dtype),
        "khat": normal(rng, (B, Hkv, T_max, dh), std, dtype),
        "vhat": normal(rng, (B, Hkv, T_max, dh), std, dtype),
        "kown": normal(rng, (B, Hkv, T_max, dh), std, dtype),
        "vown": normal(rng, (B, Hkv, T_max, dh), std, dtype),
        "n": np.broadcast_to(np.asarray(n_prefix, np.int32), (B,)).copy(),
        "scale": 1.0 / math.sqrt(dh),
    }


def project_case(seed, M, d_L, d_hidden, d_S, dtype="bf16", x_std=1.0, w_std=0.02, bias_std=0.0):
    """Inputs of one FF_Tandem call.  d_hidden == 0 gives the linear form.
    Weights are stored [out, in]."""
    rng = np.random.default_rng(seed)
    case = {"x": normal(rng, (M, d_L), x_std, dtype)}
    if d_hidden == 0:
        case["W"] = normal(rng, (d_S, d_L), w_std, dtype)
        case["b"] = normal(rng, (d_S,), bias_std, dtype)
    else:
        case["W1"] = normal(rng, (d_hidden, d_L), w_std, dtype)
        case["b1"] = normal(rng, (d_hidden,), bias_std, dtype)
        case["W2"] = normal(rng, (d_S, d_hidden), w_std, dtype)
        case["b2"] = normal(rng, (d_S,), bias_std, dtype)
    return case


# ------------------------------------------------------------- model weights
def _gain(rng, shape, gain_std, dtype):
    """RMSNorm gain: ones, or 1 + gain_std * N(0, 1) when gain_std > 0."""
    if gain_std == 0.0:
        return ones(shape, dtype)
    return HostTensor(np.float32(1.0) + rng.standard_normal(shape, dtype=np.float32) * np.float32(gain_std), dtype)


def _bias(rng, shape, bias_std, dtype):
    return zeros(shape, dtype) if bias_std == 0.0 else normal(rng, shape, bias_std, dtype)


def decoder_weights(rng, vocab, d, n_layers, Hq, Hkv, dh, d_ff, dtype, w_std=0.02, gain_std=0.0, bias_std=0.0):
    """gain_std / bias_std = 0 give the benchmark configurations' gains 1 and biases 0 (no random numbers drawn for
    them, so the weights of a seed do not depend on the option); > 0 gives gains 1 + gain_std N(0,1), biases
    N(0, bias_std)."""
    def lay():
        return {
            "g_attn": _gain(rng, (d,), gain_std, dtype),
            "Wq": normal(rng, (Hq * dh, d), w_std, dtype),
            "Wk": normal(rng, (Hkv * dh, d), w_std, dtype),
            "Wv": normal(rng, (Hkv * dh, d), w_std, dtype),
            "Wo": normal(rng, (d, Hq * dh), w_std, dtype),
            "g_mlp": _gain(rng, (d,), gain_std, dtype),
            "W1": normal(rng, (d_ff, d), w_std, dtype),
            "b1": _bias(rng, (d_ff,), bias_std, dtype),
            "W2": normal(rng, (d, d_ff), w_std, dtype),
            "b2": _bias(rng, (d,), bias_std, dtype),
        }

    return {
        "emb": normal(rng, (vocab, d), w_std, dtype),
        "layers": [lay() for _ in range(n_layers)],
        "g_final": _gain(rng, (d,), gain_std, dtype),
        "W_out": normal(rng, (vocab, d), w_std, dtype),
        "Hq": Hq,
        "Hkv": Hkv,
        "dh": dh,
        "d": d,
        "d_ff": d_ff,
        "vocab": vocab,
    }


def tandem_weights(seed, vocab, large, small, ell, d_hidden, dtype, act="gelu", w_std=0.02, eps=1e-6, gain_std=0.0,
                   bias_std=0.0, deep=False):
    """A random-init Tandem pair.  ``large``/``small`` are dicts with keys
    d, n_layers, Hq, Hkv, dh, d_ff.  ``ell[j]`` in [0, L_L] is the large layer whose
    output small layer j reads.  d_hidden == 0 gives linear FF_Tandem maps.
    gain_std / bias_std: see decoder_weights; they also apply to the FF_Tandem biases."""
    rng = np.random.default_rng(seed)
    L = decoder_weights(rng, vocab, dtype=dtype, w_std=w_std, gain_std=gain_std, bias_std=bias_std, **large)
    S = decoder_weights(rng, vocab, dtype=dtype, w_std=w_std, gain_std=gain_std, bias_std=bias_std, **small)
    ff = []
    for _ in range(small["n_layers"]):
        if d_hidden == 0:
            ff.append({"W": normal(rng, (small["d"], large["d"]), w_std, dtype),
                       "b": _bias(rng, (small["d"],), bias_std, dtype)})
        else:
            ff.append(
                {
                    "W1": normal(rng, (d_hidden, large["d"]), w_std, dtype),
                    "b1": _bias(rng, (d_hidden,), bias_std, dtype),
                    "W2": normal(rng, (small["d"], d_hidden), w_std, dtype),
                    "b2": _bias(rng, (small["d"],), bias_std, dtype),
                    "act": act,
                }
            )
    out = {"L": L, "S": S, "ell": list(ell), "ff": ff, "eps": eps, "dtype": dtype}
    if deep:
        # FF_DeepTandem (Sec. 5): one more map d_L -> d_S, drawn after everything else so that the other weights of a
        # seed do not depend on the option
        if d_hidden == 0:
            out["ff_deep"] = {"W": normal(rng, (small["d"], large["d"]), w_std, dtype),
                              "b": _bias(rng, (small["d"],), bias_std, dtype)}
        else:
            out["ff_deep"] = {"W1": normal(rng, (d_hidden, large["d"]), w_std, dtype),
                              "b1": _bias(rng, (d_hidden,), bias_std, dtype),
                              "W2": normal(rng, (small["d"], d_hidden), w_std, dtype),
                              "b2": _bias(rng, (small["d"],), bias_std, dtype), "act": act}
    return out


def tiny_tandem(seed=0, dtype="f32", gain_std=0.0, bias_std=0.0):
    """The tiny full-forward configuration: vocab 1000; large 4 layers d=256, 4 heads
    of 64, MLP 1024; small 2 layers d=128, 2 heads of 64, MLP 512, reading large
    layers 2 and 4 through a 256->512->128 MLP; weights N(0, 0.02), biases 0, gains 1
    (gain_std / bias_std > 0: the same shapes with random gains and biases, for tests)."""
    return tandem_weights(
        seed,
        vocab=1000,
        large=dict(d=256, n_layers=4, Hq=4, Hkv=4, dh=64, d_ff=1024),
        small=dict(d=128, n_layers=2, Hq=2, Hkv=2, dh=64, d_ff=512),
        ell=(2, 4),
        d_hidden=512,
        dtype=dtype,
        gain_std=gain_std,
        bias_std=bias_std,
    )


def router_weights(seed, k, d, hidden, dtype="f32", w_std=0.05, out_std=None):
    """Random-init router MLP of the adaptive block length: input 1 + k + k*d features, `hidden` units, one output
    (first layer N(0, w_std), output layer N(0, out_std), default 10 w_std; the trained router of the paper is
    not available)."""
    rng = np.random.default_rng(seed)
    out_std = 10 * w_std if out_std is None else out_std
    return {
        "k": k,
        "W1": normal(rng, (hidden, 1 + k + k * d), w_std, dtype),
        "b1": normal(rng, (hidden,), w_std, dtype),
        "w2": normal(rng, (hidden,), out_std, dtype),
        "b2": normal(rng, (1,), w_std, dtype),
    }


def as_f64(tree):
    """Map a weight tree of HostTensors to the float64 tree the oracle takes."""
    if isinstance(tree, HostTensor):
        return tree.f64
    if isinstance(tree, dict):
        return {k: as_f64(v) for k, v in tree.items()}
    if isinstance(tree, (list, tuple)):
        return [as_f64(v) for v in tree]
    return tree


def token_ids(seed, shape, vocab):
    return np.random.default_rng(seed).integers(0, vocab, size=shape, dtype=np.int64)


# ------------------------------------------------------------ device tensors
def device_normal(shape, seed, std=1.0, dtype="bf16", device="cuda", chunk_elems=1 << 28):
    """Seeded N(0, std) tensor generated directly in device memory (for inputs too
    large to stage through the host).  Filled in chunks so the fp32 staging stays
    small."""
    import torch

    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    out = torch.empty(shape, dtype=tdt, device=device)
    flat = out.view(-1)
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    total = flat.numel()
    for lo in range(0, total, chunk_elems):
        hi = min(total, lo + chunk_elems)
        tmp = torch.randn(hi - lo, generator=g, device=device, dtype=torch.float32)
        if std != 1.0:
            tmp.mul_(std)
        flat[lo:hi].copy_(tmp)
        del tmp
    return out
