"""GPU parity of tandem_score - the teacher-forced pass of the small model (Eq. (2) at every position) - through the
C ABI: after tandem_prefill has ingested the same tokens, chunked calls must reproduce the oracle's teacher-forced
Tandem forward (every position at once) at every position."""
import math

import numpy as np
import pytest

from oracle import tandem_oracle as orc
from paper_2402_08644_amd import inputs
from parity import assert_rows_close
from test_gpu_decode_step import small_bf16_pair, tokens_ok

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tb():
    import torch

    from paper_2402_08644_amd import binding

    assert torch.cuda.is_available()
    binding.lib()
    return torch, binding


def run_score(tb, W, toks, gamma, chunks, T_max):
    """Prefill all tokens, then score them chunk by chunk; returns (logits, y, greedy) over all positions."""
    torch, binding = tb
    B, S = toks.shape
    model = binding.TandemModel(W)
    gst = binding.TandemState(model, B, T_max, 4)
    dev_toks = torch.tensor(toks, dtype=torch.int32).cuda()
    for s0 in range(0, S, 32):
        binding.tandem_prefill(model, gst, dev_toks[:, s0:s0 + 32].contiguous())
    ko, vo = binding.own_caches(model, gst)
    lg, ys, gr = [], [], []
    s0 = 0
    for q in chunks:
        pos = torch.full((B,), s0, dtype=torch.int32, device="cuda")
        out = binding.tandem_score(model, gst, ko, vo, pos, dev_toks[:, s0:s0 + q].contiguous(), gamma, logits=True,
                                   y_small=True)
        lg.append(inputs.torch_to_f64(out["logits"]))
        ys.append(inputs.torch_to_f64(out["y_small"]))
        gr.append(out["greedy"].cpu().numpy())
        s0 += q
    torch.cuda.synchronize()
    assert s0 == S
    return np.concatenate(lg, 1), np.concatenate(ys, 1), np.concatenate(gr, 1)


@pytest.mark.parametrize("gamma,chunks,gains", [(2, [32, 32, 32, 32], False), (3, [7, 32, 1, 24], True)])
def test_score_tiny_config_fp32_equals_teacher_forced_forward(tb, gamma, chunks, gains):
    W = inputs.tiny_tandem(seed=0, dtype="f32", gain_std=0.3 if gains else 0.0, bias_std=0.02 if gains else 0.0)
    T = inputs.as_f64(W)
    S = sum(chunks)
    toks = inputs.token_ids(1, (1, S), 1000)
    ref = orc.tandem_forward(T, toks[0], gamma)
    lg, y, greedy = run_score(tb, W, toks, gamma, chunks, 128)
    e = assert_rows_close(y[0], ref["y"], tol=2e-3, what="y^(L_S)")
    assert_rows_close(lg[0], ref["logits_S"], tol=2e-3, what="small logits")
    assert tokens_ok(greedy[0], ref["logits_S"], margin=1e-4)
    print(f"score tiny gamma={gamma}: max rel err {e[0]:.2e}")


def test_score_bf16_batch_equals_teacher_forced_forward(tb):
    """bf16, two sequences, 40 tokens, gamma = 4, chunks that cut through blocks."""
    W = small_bf16_pair(90)
    T = inputs.as_f64(W)
    gamma, chunks = 4, [10, 17, 13]
    toks = inputs.token_ids(2, (2, 40), 512)
    lg, y, greedy = run_score(tb, W, toks, gamma, chunks, 64)
    tol = 2e-2  # rows pass the large layers, FF_Tandem and the small layers; observed 9e-3
    for b in range(2):
        ref = orc.tandem_forward(T, toks[b], gamma)
        assert_rows_close(y[b], ref["y"], tol=tol, what=f"y^(L_S) of sequence {b}")
        assert_rows_close(lg[b], ref["logits_S"], tol=tol, what=f"small logits of sequence {b}")
        assert tokens_ok(greedy[b], ref["logits_S"], margin=2 * tol)


def test_score_error_codes(tb):
    torch, binding = tb
    W = inputs.tiny_tandem(seed=1, dtype="f32")
    model = binding.TandemModel(W)
    gst = binding.TandemState(model, 1, 16, 2)
    ko, vo = binding.own_caches(model, gst)
    pos = torch.zeros(1, dtype=torch.int32, device="cuda")
    toks = torch.zeros((1, 33), dtype=torch.int32, device="cuda")
    with pytest.raises(binding.TandemError):
        binding.tandem_score(model, gst, ko, vo, pos, toks, 2)
    toks = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    with pytest.raises(binding.TandemError):
        binding.tandem_score(model, gst, ko, vo, pos, toks, 0)
    with pytest.raises(binding.TandemError):
        binding.tandem_score(model, gst, ko, vo, pos, toks, 2, ws=torch.zeros(256, dtype=torch.uint8, device="cuda"))
    binding.tandem_score(model, gst, ko, vo, pos, toks, 2)
    torch.cuda.synchronize()
