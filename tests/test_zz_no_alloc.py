"""GPU: tandem_draft_attn_static (the entry point that allocates nothing: split partials in the library's static
device scratch) against tandem_draft_attn (caller's workspace) and the fp64 oracle, through the C ABI.  Two calls in a
row on the shared scratch, the second with a smaller input whose partial table has another shape."""
import ctypes as C

import numpy as np
import pytest

from oracle import tandem_oracle as orc
from paper_2402_08644_amd import inputs
from parity import assert_rows_close

pytestmark = pytest.mark.gpu


def _run_pair(torch, binding, seed, B, Hq, Hkv, T_max, gmax, n_large, n_cur):
    case = inputs.draft_attn_case(seed, B, Hq, Hkv, 128, T_max, gmax, n_large, n_cur, dtype="bf16", kv_std=1.0)
    dev = {k: case[k].to_torch() for k in ("q", "khat", "vhat", "kcur", "vcur")}
    nl = torch.from_numpy(case["n_large"]).cuda()
    nc = torch.from_numpy(case["n_cur"]).cuda()
    L = binding.lib()
    d = binding.attn_desc(B, Hq, Hkv, 128, T_max, gmax, case["scale"], binding.BF16)
    need = binding.tandem_draft_attn_workspace(d)
    assert 0 < need <= binding.STATIC_SCRATCH_BYTES, need  # the case really uses the scratch
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    ref = torch.empty_like(dev["q"])
    got = torch.full_like(dev["q"], float("nan"))
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t: C.c_void_p(t.data_ptr())
    rc = L.tandem_draft_attn(C.byref(d), p(dev["q"]), p(dev["khat"]), p(dev["vhat"]), p(nl), p(dev["kcur"]), p(dev["vcur"]),
                             p(nc), p(ref), p(ws), need, st)
    assert rc == binding.OK
    rc = L.tandem_draft_attn_static(C.byref(d), p(dev["q"]), p(dev["khat"]), p(dev["vhat"]), p(nl), p(dev["kcur"]),
                                    p(dev["vcur"]), p(nc), p(got), st)
    assert rc == binding.OK
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), ref.view(torch.int16)), "static-scratch result differs from the workspace result"
    want = orc.draft_attn(case["q"].f64, case["khat"].f64, case["vhat"].f64, case["n_large"], case["kcur"].f64,
                          case["vcur"].f64, case["n_cur"], case["scale"])
    assert_rows_close(inputs.torch_to_f64(got), want, what="draft_attn_static")


def test_draft_attn_static_matches_workspace_entry_point_two_calls_in_a_row():
    import torch

    from paper_2402_08644_amd import binding

    assert torch.cuda.is_available()
    binding.lib()
    # 4 sequences x 8 KV heads over 1024 + 4 rows: four context splits in wide workgroups, two partial slots per row
    _run_pair(torch, binding, 5, 4, 8, 8, 1024, 4, [1020, 700, 3, 1024], [4, 1, 2, 3])
    # smaller: 3 sequences x 4 KV heads, grouped queries, three (odd) splits - another table shape in the same scratch
    _run_pair(torch, binding, 6, 3, 8, 4, 800, 2, [800, 311, 0], [1, 2, 2])


def test_draft_attn_static_rejects_oversized_requests():
    import torch

    from paper_2402_08644_amd import binding

    L = binding.lib()
    # one sequence, 64 query heads on 8 KV heads, long context: 64 splits x 64 rows x 520 B = 2.1 MB of partials
    big = binding.attn_desc(1, 64, 8, 128, 1 << 20, 4, 0.1, binding.BF16)
    assert binding.tandem_draft_attn_workspace(big) > binding.STATIC_SCRATCH_BYTES
    x = torch.zeros(16, device="cuda")
    p = C.c_void_p(x.data_ptr())
    assert L.tandem_draft_attn_static(C.byref(big), p, p, p, p, p, p, p, p, None) == binding.ERR_WORKSPACE
    torch.cuda.synchronize()
