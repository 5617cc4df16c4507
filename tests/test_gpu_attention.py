"""GPU parity: tandem_draft_attn and tandem_block_attn (through the C ABI) against the fp64
oracle on the same seeded inputs, element by element."""
import math

import numpy as np
import pytest

from oracle import tandem_oracle as orc
from paper_2402_08644_amd import inputs
from parity import assert_rows_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tb():
    import torch

    from paper_2402_08644_amd import binding

    assert torch.cuda.is_available()
    binding.lib()
    return torch, binding


def run_draft(tb, case, scale=None):
    torch, binding = tb
    dev = {k: case[k].to_torch() for k in ("q", "khat", "vhat", "kcur", "vcur")}
    nl = torch.from_numpy(case["n_large"]).cuda()
    nc = torch.from_numpy(case["n_cur"]).cuda()
    out = binding.tandem_draft_attn(dev["q"], dev["khat"], dev["vhat"], nl, dev["kcur"], dev["vcur"], nc, scale=case["scale"])
    torch.cuda.synchronize()
    return inputs.torch_to_f64(out)


def oracle_draft(case):
    return orc.draft_attn(case["q"].f64, case["khat"].f64, case["vhat"].f64, case["n_large"], case["kcur"].f64,
                          case["vcur"].f64, case["n_cur"], case["scale"])


def run_block(tb, case):
    torch, binding = tb
    out = binding.tandem_block_attn(case["q"].to_torch(), case["k"].to_torch(), case["v"].to_torch(),
                                    torch.from_numpy(case["n"]).cuda(), scale=case["scale"])
    torch.cuda.synchronize()
    return inputs.torch_to_f64(out)


def oracle_block(case):
    return orc.block_attn(case["q"].f64, case["k"].f64, case["v"].f64, case["n"], case["scale"])


# --------------------------------------------------------------------------- draft
@pytest.mark.parametrize(
    "B,Hq,Hkv,dh,T_max,gmax,n_large,n_cur,dtype",
    [
        (3, 4, 2, 128, 300, 4, [0, 37, 300], [1, 4, 2], "bf16"),       # ragged, empty large part, full cache
        (2, 8, 8, 128, 1111, 8, [1111, 1000], [8, 3], "bf16"),          # MHA, several splits, ragged tail
        (2, 8, 1, 128, 700, 4, [513, 64], [4, 1], "bf16"),              # G = 8
        (2, 4, 1, 128, 520, 4, [500, 17], [2, 4], "bf16"),              # G = 4
        (2, 4, 2, 64, 400, 4, [400, 129], [3, 1], "bf16"),              # dh = 64
        (2, 2, 2, 64, 130, 2, [128, 5], [2, 1], "f32"),                 # the tiny config's small model shape
        (1, 2, 1, 128, 64, 4, [15], [1], "f32"),
        (2, 2, 2, 128, 16, 4, [0, 0], [1, 4], "bf16"),                  # no completed block at all: own rows only
    ],
)
def test_draft_attn_parity_small(tb, B, Hq, Hkv, dh, T_max, gmax, n_large, n_cur, dtype):
    case = inputs.draft_attn_case(11, B, Hq, Hkv, dh, T_max, gmax, n_large, n_cur, dtype=dtype, kv_std=1.0)
    got = run_draft(tb, case)
    want = oracle_draft(case)
    e = assert_rows_close(got, want, what="draft")
    print(f"draft small {B,Hq,Hkv,dh,T_max,dtype}: max rel err {e[0]:.2e}")


def test_attention_parity_long_context_many_splits(tb):
    """One sequence, one KV head, long context: the largest split count (64) with a ragged last split."""
    case = inputs.draft_attn_case(12, 1, 1, 1, 128, 17001, 4, [16999], [3], dtype="bf16", kv_std=1.0)
    assert_rows_close(run_draft(tb, case), oracle_draft(case), what="draft long context")
    blk = inputs.block_attn_case(13, 1, 4, 4, 1, 128, 17001, [16990], dtype="bf16")
    assert_rows_close(run_block(tb, blk), oracle_block(blk), what="block long context")


def test_draft_attn_parity_config1_full(tb):
    """The single-kernel benchmark configuration: batch 8, 8 heads of 128, 2044 large rows + 4 own rows."""
    case = inputs.draft_attn_case(1, 8, 8, 8, 128, 2044, 4, 2044, 4, dtype="bf16")
    got = run_draft(tb, case)
    e = assert_rows_close(got, oracle_draft(case), what="draft config 1")
    print(f"draft config1: max rel err {e[0]:.2e}")
    # ragged variant
    rng = np.random.default_rng(5)
    case["n_large"] = rng.integers(1800, 2045, size=8).astype(np.int32)
    case["n_cur"] = rng.integers(1, 5, size=8).astype(np.int32)
    assert_rows_close(run_draft(tb, case), oracle_draft(case), what="draft config 1 ragged")


def test_draft_attn_lengths_are_clamped(tb):
    """Lengths beyond the capacities are clamped to them (no out-of-bounds read)."""
    case = inputs.draft_attn_case(3, 2, 2, 2, 128, 100, 4, [1000, -5], [9, 2], dtype="bf16")
    got = run_draft(tb, case)
    case["n_large"] = np.array([100, 0], np.int32)
    case["n_cur"] = np.array([4, 2], np.int32)
    assert_rows_close(got, oracle_draft(case), what="draft clamped")


def test_draft_attn_indicator_probe_exact_mask(tb):
    """q = 0 makes every visible row weigh exactly 1/N; V = e_0 on exactly one row.  The output is
    exactly 0 iff that row is masked.  Sweeps every row of both sources for ragged lengths that
    straddle split and tile boundaries."""
    torch, binding = tb
    B, H, dh, T_max, gmax = 4, 1, 128, 600, 4
    n_large = np.array([0, 255, 256, 600], np.int32)
    n_cur = np.array([1, 4, 2, 3], np.int32)
    q = torch.zeros((B, H, dh), dtype=torch.bfloat16, device="cuda")
    ones_hat = torch.ones((B, H, T_max, dh), dtype=torch.bfloat16, device="cuda")
    ones_cur = torch.ones((B, H, gmax, dh), dtype=torch.bfloat16, device="cuda")
    # V row p carries the value (p mod 251) + 1 in element 0 ... decode which rows contributed through
    # two probes: indicator of "row index in set A" sums to |visible in A| / N.
    for probe in range(3):
        vhat = torch.zeros((B, H, T_max, dh), dtype=torch.float32)
        vcur = torch.zeros((B, H, gmax, dh), dtype=torch.float32)
        if probe == 0:  # all rows flagged: output must be exactly 1 (N/N) - every visible row counted once
            vhat[..., 0] = 1.0
            vcur[..., 0] = 1.0
        elif probe == 1:  # only rows that must be masked are flagged: output must be exactly 0
            for b in range(B):
                vhat[b, :, n_large[b]:, 0] = 1.0
                vcur[b, :, n_cur[b]:, 0] = 1.0
        else:  # only the last visible row of each source is flagged: output 2/N (or 1/N if no large rows)
            for b in range(B):
                if n_large[b] > 0:
                    vhat[b, :, n_large[b] - 1, 0] = 1.0
                vcur[b, :, n_cur[b] - 1, 0] = 1.0
        out = binding.tandem_draft_attn(q, ones_hat, vhat.to(torch.bfloat16).cuda(), torch.from_numpy(n_large).cuda(),
                                        ones_cur, vcur.to(torch.bfloat16).cuda(), torch.from_numpy(n_cur).cuda(), scale=1.0)
        got = out.float().cpu().numpy()[:, 0, 0]
        for b in range(B):
            N = int(n_large[b] + n_cur[b])
            if probe == 0:
                assert abs(got[b] - 1.0) <= 2 ** -7, (b, got[b])
            elif probe == 1:
                assert got[b] == 0.0, (b, got[b])
            else:
                want = (2.0 if n_large[b] > 0 else 1.0) / N
                assert abs(got[b] - want) <= want * 2 ** -7, (b, got[b], want)


def test_draft_attn_single_row_positions_exact(tb):
    """Moves a single flagged V row across every position around split/tile boundaries: the output is
    nonzero exactly when the position is visible."""
    torch, binding = tb
    B, H, dh, T_max, gmax = 1, 1, 128, 1040, 4
    q = torch.zeros((B, H, dh), dtype=torch.bfloat16, device="cuda")
    ones_hat = torch.ones((B, H, T_max, dh), dtype=torch.bfloat16, device="cuda")
    ones_cur = torch.ones((B, H, gmax, dh), dtype=torch.bfloat16, device="cuda")
    for n_large, n_cur in [(1037, 3), (256, 1), (15, 4)]:
        nl = torch.tensor([n_large], dtype=torch.int32, device="cuda")
        nc = torch.tensor([n_cur], dtype=torch.int32, device="cuda")
        positions = sorted(set(list(range(0, 40)) + list(range(240, 280)) + list(range(500, 530)) + list(range(1000, 1040))))
        for p in positions + [T_max + i for i in range(gmax)]:
            vhat = torch.zeros((B, H, T_max, dh), dtype=torch.bfloat16, device="cuda")
            vcur = torch.zeros((B, H, gmax, dh), dtype=torch.bfloat16, device="cuda")
            if p < T_max:
                vhat[0, 0, p, 5] = 1.0
                visible = p < n_large
            else:
                vcur[0, 0, p - T_max, 5] = 1.0
                visible = (p - T_max) < n_cur
            out = binding.tandem_draft_attn(q, ones_hat, vhat, nl, ones_cur, vcur, nc, scale=1.0)
            v = float(out[0, 0, 5])
            if visible:
                want = 1.0 / (n_large + n_cur)
                assert abs(v - want) <= want * 2 ** -7, (n_large, n_cur, p, v)
            else:
                assert v == 0.0, (n_large, n_cur, p, v)
            assert float(out.float().abs().sum()) == abs(v)


def test_draft_attn_is_deterministic(tb):
    torch, binding = tb
    case = inputs.draft_attn_case(2, 4, 8, 8, 128, 1500, 4, [1500, 900, 33, 1024], [4, 1, 2, 3], dtype="bf16")
    dev = {k: case[k].to_torch() for k in ("q", "khat", "vhat", "kcur", "vcur")}
    nl, nc = torch.from_numpy(case["n_large"]).cuda(), torch.from_numpy(case["n_cur"]).cuda()
    a = binding.tandem_draft_attn(dev["q"], dev["khat"], dev["vhat"], nl, dev["kcur"], dev["vcur"], nc).clone()
    b = binding.tandem_draft_attn(dev["q"], dev["khat"], dev["vhat"], nl, dev["kcur"], dev["vcur"], nc)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_draft_attn_never_writes_the_caches(tb):
    torch, binding = tb
    case = inputs.draft_attn_case(4, 2, 4, 4, 128, 300, 4, [300, 10], [4, 1], dtype="bf16")
    dev = {k: case[k].to_torch() for k in ("q", "khat", "vhat", "kcur", "vcur")}
    before = {k: v.clone() for k, v in dev.items()}
    binding.tandem_draft_attn(dev["q"], dev["khat"], dev["vhat"], torch.from_numpy(case["n_large"]).cuda(), dev["kcur"],
                              dev["vcur"], torch.from_numpy(case["n_cur"]).cuda())
    torch.cuda.synchronize()
    for k in dev:
        assert torch.equal(before[k].view(torch.int16), dev[k].view(torch.int16)), k


# --------------------------------------------------------------------------- block
@pytest.mark.parametrize(
    "B,q_len,Hq,Hkv,dh,T_max,n,dtype",
    [
        (2, 4, 8, 2, 128, 300, [296, 0], "bf16"),        # G=4, R=16: one row tile; full cache and empty prefix
        (3, 8, 8, 2, 128, 700, [692, 100, 31], "bf16"),  # R=32: two row tiles
        (2, 1, 4, 4, 128, 260, [259, 7], "bf16"),        # block length 1 = ordinary causal decode, G=1 (15 padded rows)
        (2, 5, 4, 1, 128, 530, [525, 64], "bf16"),       # R=20: ragged row tile
        (1, 32, 8, 2, 128, 300, [200], "bf16"),          # R=128: two passes of four row tiles
        (2, 7, 8, 1, 128, 200, [193, 50], "bf16"),       # G=8, R=56: four row tiles with padding
        (2, 12, 4, 1, 128, 333, [321, 0], "bf16"),       # R=48: three wavefronts, one row tile each
        (1, 24, 8, 2, 128, 777, [753], "bf16"),          # R=96: six
        (2, 28, 4, 1, 128, 150, [122, 31], "bf16"),      # R=112: seven
        (1, 18, 8, 1, 128, 1100, [1082], "bf16"),        # G=8, R=144: two passes of five row tiles, ragged
        (2, 3, 4, 2, 64, 100, [97, 10], "bf16"),         # dh=64 generic path
        (1, 2, 4, 4, 64, 130, [126], "f32"),             # the tiny config's large model shape
        (2, 4, 4, 2, 128, 90, [80, 0], "f32"),
    ],
)
def test_block_attn_parity_small(tb, B, q_len, Hq, Hkv, dh, T_max, n, dtype):
    case = inputs.block_attn_case(21, B, q_len, Hq, Hkv, dh, T_max, n, dtype=dtype)
    got = run_block(tb, case)
    e = assert_rows_close(got, oracle_block(case), what="block")
    print(f"block small {B,q_len,Hq,Hkv,dh,T_max,dtype}: max rel err {e[0]:.2e}")


def test_block_attn_parity_config2_full(tb):
    """Large GQA layer: batch 16, 32/8 heads of 128, prefix 4096 + 4 block-causal queries."""
    case = inputs.block_attn_case(2, 16, 4, 32, 8, 128, 4100, 4096, dtype="bf16")
    got = run_block(tb, case)
    e = assert_rows_close(got, oracle_block(case), what="block config 2")
    print(f"block config2: max rel err {e[0]:.2e}")


def test_block_attn_causal_mask_exact(tb):
    """Q = 0 (uniform weights) and V flagged on exactly one cache row: row r of the block must give
    exactly 0 when the flagged row is past n + r, and 1/(n + r + 1) otherwise."""
    torch, binding = tb
    B, q_len, Hq, Hkv, dh, T_max = 1, 4, 4, 1, 128, 400
    q = torch.zeros((B, q_len, Hq, dh), dtype=torch.bfloat16, device="cuda")
    k = torch.ones((B, Hkv, T_max, dh), dtype=torch.bfloat16, device="cuda")
    for n in (0, 29, 60, 252, 396):
        nn = torch.tensor([n], dtype=torch.int32, device="cuda")
        for p in sorted(set([0, 1, n - 1, n, n + 1, n + 2, n + 3, n + 4, n + 5, 31, 32, 33, 255, 256, T_max - 1])):
            if p < 0 or p >= T_max:
                continue
            v = torch.zeros((B, Hkv, T_max, dh), dtype=torch.bfloat16, device="cuda")
            v[0, 0, p, 77] = 1.0
            out = binding.tandem_block_attn(q, k, v, nn, scale=1.0).float().cpu().numpy()
            for r in range(q_len):
                for h in range(Hq):
                    if p <= n + r:
                        want = 1.0 / (n + r + 1)
                        assert abs(out[0, r, h, 77] - want) <= want * 2 ** -6, (n, p, r, h, out[0, r, h, 77])
                    else:
                        assert out[0, r, h, 77] == 0.0, (n, p, r, h)
            assert np.count_nonzero(out[..., :77]) == 0 and np.count_nonzero(out[..., 78:]) == 0


def _with_dominant_keys(case, kname, positions, dtype, c=48.5):
    """Query component 0 = c in every row and key component 0 = c at the given positions: those keys score
    c * c * scale (about 300 in base-2 units at d_h = 128) above keys whose scores are of order one, so a
    running maximum that misses one of them overflows the exponentials."""
    q = case["q"].f64.astype(np.float32).copy()
    k = case[kname].f64.astype(np.float32).copy()
    q[..., 0] = c
    k[..., 0] = 0.0
    for pos in positions:
        k[:, :, pos, 0] = c
    case["q"] = inputs.HostTensor(q, dtype)
    case[kname] = inputs.HostTensor(k, dtype)
    return case


@pytest.mark.parametrize(
    "B,q_len,Hq,Hkv,T_max,n",
    [
        (2, 4, 4, 1, 700, 690),     # one row tile per KV head: the key-split kernel, several tiles per wavefront
        (2, 4, 8, 1, 700, 690),     # two row tiles
        (1, 16, 8, 2, 600, 580),    # 64 rows per KV head: the row-split kernel
    ],
)
@pytest.mark.parametrize("offset", [0, 5, 10, 15, 20, 25, 30])
def test_block_attn_dominant_key_in_every_lane_group(tb, B, q_len, Hq, Hkv, T_max, n, offset):
    """The running maximum of a query column is shared by four lanes that hold different keys of a tile (keys
    4g .. 4g+3 and 16+4g .. 16+4g+3 in lane group g).  One key per tile position class that dominates all others
    by far: a lane group whose maximum does not reach the others gives infinities instead of weights."""
    case = inputs.block_attn_case(61 + offset, B, q_len, Hq, Hkv, 128, T_max, n, dtype="bf16")
    positions = [32 * t + offset for t in (0, 3, 7, 12)]   # four dominant keys, all visible
    case = _with_dominant_keys(case, "k", positions, "bf16")
    got = run_block(tb, case)
    want = oracle_block(case)
    assert_rows_close(got, want, what=f"block, dominant keys at tile offset {offset}")
    assert np.abs(got).max() < 10.0


@pytest.mark.parametrize("offset", [0, 5, 10, 15, 20, 25, 30])
def test_draft_attn_dominant_key(tb, offset):
    case = inputs.draft_attn_case(71 + offset, 2, 4, 2, 128, 900, 4, [870, 333], [3, 1], dtype="bf16")
    case = _with_dominant_keys(case, "khat", [32 * t + offset for t in (0, 2, 9)], "bf16")
    got = run_draft(tb, case)
    assert_rows_close(got, oracle_draft(case), what=f"draft, dominant keys at offset {offset}")


def test_block_attn_is_deterministic_and_readonly(tb):
    torch, binding = tb
    case = inputs.block_attn_case(8, 3, 4, 8, 2, 128, 1000, [996, 500, 3], dtype="bf16")
    q, k, v = case["q"].to_torch(), case["k"].to_torch(), case["v"].to_torch()
    k0, v0 = k.clone(), v.clone()
    n = torch.from_numpy(case["n"]).cuda()
    a = binding.tandem_block_attn(q, k, v, n).clone()
    b = binding.tandem_block_attn(q, k, v, n)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert torch.equal(k.view(torch.int16), k0.view(torch.int16)) and torch.equal(v.view(torch.int16), v0.view(torch.int16))


def test_block_attn_gamma1_equals_draft_with_own_row(tb):
    """A block of one token is ordinary causal decoding: the block pass over n+1 cache rows equals the
    mixed-source kernel fed n large rows plus the (n+1)-th row as its single own row."""
    torch, binding = tb
    case = inputs.block_attn_case(9, 2, 1, 8, 8, 128, 400, [399, 100], dtype="bf16")
    q, k, v = case["q"].to_torch(), case["k"].to_torch(), case["v"].to_torch()
    n = torch.from_numpy(case["n"]).cuda()
    blk = binding.tandem_block_attn(q, k, v, n)
    idx = n.long()
    kcur = torch.stack([k[b, :, idx[b]] for b in range(2)])[:, :, None, :].contiguous()
    vcur = torch.stack([v[b, :, idx[b]] for b in range(2)])[:, :, None, :].contiguous()
    one = torch.ones(2, dtype=torch.int32, device="cuda")
    drf = binding.tandem_draft_attn(q[:, 0].contiguous(), k, v, n, kcur, vcur, one)
    assert_rows_close(inputs.torch_to_f64(blk[:, 0]), inputs.torch_to_f64(drf), tol=1e-2, what="gamma=1")


# --------------------------------------------------------------------------- several samples per prompt
def run_shared(tb, case):
    torch, binding = tb
    out = binding.tandem_block_attn_shared(case["q"].to_torch(), case["ks"].to_torch(), case["vs"].to_torch(),
                                           torch.from_numpy(case["n_shared"]).cuda(), case["ko"].to_torch(),
                                           case["vo"].to_torch(), torch.from_numpy(case["n_own"]).cuda(),
                                           scale=case["scale"])
    torch.cuda.synchronize()
    return inputs.torch_to_f64(out)


def oracle_shared(case):
    return orc.block_attn_shared(case["q"].f64, case["ks"].f64, case["vs"].f64, case["n_shared"], case["ko"].f64,
                                 case["vo"].f64, case["n_own"], case["scale"])


@pytest.mark.parametrize(
    "B,ns,q_len,Hq,Hkv,dh,Ts,To,n_shared,n_own,dtype",
    [
        (2, 4, 4, 8, 2, 128, 300, 40, [300, 37], [0, 36, 7, 20, 1, 2, 3, 30], "bf16"),   # R=64 shared rows: 4 row tiles
        (1, 4, 5, 4, 1, 128, 700, 64, [650], [59, 0, 13, 31], "bf16"),                   # R=80: two passes, ragged
        (2, 2, 1, 4, 4, 128, 260, 20, [0, 259], [19, 0, 5, 7], "bf16"),                  # an empty prompt; G=1, q_len=1
        (3, 1, 3, 8, 2, 128, 100, 300, [100, 5, 64], [297, 0, 100], "bf16"),             # one sample: prompt + own = a plain split
        (1, 8, 4, 8, 1, 128, 1200, 33, [1111], [29, 0, 1, 2, 3, 4, 5, 6], "bf16"),       # G=8, 256 rows on the prompt
        (2, 3, 2, 4, 2, 64, 90, 12, [90, 10], [10, 0, 3, 4, 5, 6], "bf16"),              # dh=64 generic path
        (2, 2, 3, 4, 4, 64, 50, 16, [17, 50], [0, 13, 7, 2], "f32"),
        (1, 4, 2, 4, 2, 128, 600, 70, [555], [68, 1, 30, 0], "f32"),
    ],
)
def test_block_attn_shared_parity_small(tb, B, ns, q_len, Hq, Hkv, dh, Ts, To, n_shared, n_own, dtype):
    case = inputs.shared_attn_case(31, B, ns, q_len, Hq, Hkv, dh, Ts, To, n_shared, n_own, dtype=dtype)
    got = run_shared(tb, case)
    e = assert_rows_close(got.reshape(-1, Hq, dh), oracle_shared(case).reshape(-1, Hq, dh), what="shared")
    print(f"shared small {B,ns,q_len,Hq,Hkv,dh,Ts,To,dtype}: max rel err {e[0]:.2e}")


@pytest.mark.parametrize(
    "B,ns,Hq,Hkv,dh,Ts,To,gmax,n_shared,n_own,n_cur,dtype",
    [
        (2, 4, 8, 8, 128, 700, 40, 4, [700, 37], [0, 36, 7, 40, 1, 2, 3, 30], [1, 4, 2, 3, 4, 1, 2, 3], "bf16"),  # small-model shape
        (1, 8, 8, 2, 128, 1300, 64, 8, [1234], [5, 0, 64, 31, 2, 9, 50, 17], [8, 1, 2, 3, 4, 5, 6, 7], "bf16"),    # G=4: 32 rows
        (3, 1, 4, 1, 128, 100, 300, 4, [100, 0, 64], [297, 0, 100], [1, 2, 4], "bf16"),                            # one sample
        (2, 12, 4, 1, 128, 260, 20, 2, [0, 259], 7, 2, "bf16"),                                                    # 48 rows, an empty prompt
        (2, 3, 4, 2, 64, 90, 12, 4, [90, 10], [10, 0, 3, 4, 5, 6], [1, 2, 3, 4, 1, 2], "bf16"),                    # dh=64 generic path
        (2, 2, 2, 2, 64, 50, 16, 2, [17, 50], [0, 13, 7, 2], [2, 1, 2, 1], "f32"),
    ],
)
def test_draft_attn_shared_parity_small(tb, B, ns, Hq, Hkv, dh, Ts, To, gmax, n_shared, n_own, n_cur, dtype):
    torch, binding = tb
    c = inputs.shared_draft_case(61, B, ns, Hq, Hkv, dh, Ts, To, gmax, n_shared, n_own, n_cur, dtype=dtype)
    dev = lambda k: torch.from_numpy(c[k]).cuda() if k.startswith("n_") else c[k].to_torch()
    out = binding.tandem_draft_attn_shared(dev("q"), dev("khs"), dev("vhs"), dev("n_shared"), dev("kho"), dev("vho"),
                                           dev("n_own"), dev("kcur"), dev("vcur"), dev("n_cur"), scale=c["scale"])
    torch.cuda.synchronize()
    want = orc.draft_attn_shared(c["q"].f64, c["khs"].f64, c["vhs"].f64, c["n_shared"], c["kho"].f64, c["vho"].f64,
                                 c["n_own"], c["kcur"].f64, c["vcur"].f64, c["n_cur"], c["scale"])
    e = assert_rows_close(inputs.torch_to_f64(out).reshape(-1, Hq, dh), want.reshape(-1, Hq, dh), what="shared draft")
    print(f"shared draft small {B,ns,Hq,Hkv,dh,Ts,To,dtype}: max rel err {e[0]:.2e}")


def test_draft_attn_shared_error_codes(tb):
    torch, binding = tb
    import ctypes as C

    L = binding.lib()
    d = binding.attn_desc(2, 4, 2, 128, 64, 4, 0.1, binding.BF16)
    t = torch.zeros(2 * 4 * 4 * 64 * 128, dtype=torch.bfloat16, device="cuda")
    n = torch.zeros(8, dtype=torch.int32, device="cuda")
    p, pn = C.c_void_p(t.data_ptr()), C.c_void_p(n.data_ptr())
    ws = torch.zeros(1 << 22, dtype=torch.uint8, device="cuda")
    pw = C.c_void_p(ws.data_ptr())
    call = lambda ns, To, q=p, w=pw, wb=ws.numel(): L.tandem_draft_attn_shared(
        C.byref(d), ns, To, q, p, p, pn, p, p, pn, p, p, pn, p, w, wb, None)
    assert call(0, 16) == binding.ERR_SHAPE
    assert call(4, 0) == binding.ERR_SHAPE
    assert call(4, 16, q=None) == binding.ERR_NULL
    assert call(4, 16, w=None) == binding.ERR_NULL
    need = int(L.tandem_draft_attn_shared_workspace(C.byref(d), 4, 16))
    assert need > 0
    assert call(4, 16, wb=need - 1) == binding.ERR_WORKSPACE
    assert call(4, 16, wb=need) == binding.OK
    torch.cuda.synchronize()


def test_block_attn_shared_equals_block_attn_on_copied_prompts(tb):
    """At the latency evaluation's shape (4 samples per prompt, long prompt, short continuations) the shared
    form agrees with tandem_block_attn on per-sample caches holding a copy of the prompt rows, and with the
    oracle on sampled output rows."""
    torch, binding = tb
    B, ns, q_len, Hq, Hkv, dh, Ts, To = 4, 4, 5, 32, 8, 128, 4096, 256
    rng = np.random.default_rng(5)
    n_shared = np.array([4096, 3000, 17, 2049], np.int32)
    n_own = rng.integers(0, To - q_len + 1, size=B * ns).astype(np.int32)
    case = inputs.shared_attn_case(32, B, ns, q_len, Hq, Hkv, dh, Ts, To, n_shared, n_own, dtype="bf16")
    got = run_shared(tb, case)
    ks, vs, ko, vo = (case[k].to_torch() for k in ("ks", "vs", "ko", "vo"))
    kc = torch.zeros(B * ns, Hkv, Ts + To, dh, dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    n = np.zeros(B * ns, np.int32)
    for b in range(B):
        for s_ in range(ns):
            i, m = b * ns + s_, int(n_shared[b])
            kc[i, :, :m], vc[i, :, :m] = ks[b, :, :m], vs[b, :, :m]
            kc[i, :, m:m + To], vc[i, :, m:m + To] = ko[i], vo[i]
            n[i] = m + n_own[i]
    ref = binding.tandem_block_attn(case["q"].to_torch().view(B * ns, q_len, Hq, dh), kc, vc,
                                    torch.from_numpy(n).cuda(), scale=case["scale"])
    torch.cuda.synchronize()
    assert_rows_close(got.reshape(-1, Hq, dh), inputs.torch_to_f64(ref).reshape(-1, Hq, dh), what="shared vs copied")
    q64, ks64, vs64, ko64, vo64 = (case[k].f64 for k in ("q", "ks", "vs", "ko", "vo"))
    G = Hq // Hkv
    for _ in range(24):
        b, s_, r, h = (int(rng.integers(0, x)) for x in (B, ns, q_len, Hq))
        i, kv = b * ns + s_, h // G
        K = np.concatenate([ks64[b, kv, : n_shared[b]], ko64[i, kv, : n_own[i] + r + 1]])
        V = np.concatenate([vs64[b, kv, : n_shared[b]], vo64[i, kv, : n_own[i] + r + 1]])
        want = orc.attention_one(q64[b, s_, r, h], K, V, case["scale"])
        assert_rows_close(got[b, s_, r, h][None], want[None], what=f"shared sampled row {b,s_,r,h}")


def test_block_attn_shared_error_codes(tb):
    torch, binding = tb
    import ctypes as C

    L = binding.lib()
    d = binding.attn_desc(2, 4, 2, 128, 64, 0, 0.1, binding.BF16)
    t = torch.zeros(2 * 4 * 4 * 64 * 128, dtype=torch.bfloat16, device="cuda")
    n = torch.zeros(8, dtype=torch.int32, device="cuda")
    p, pn = C.c_void_p(t.data_ptr()), C.c_void_p(n.data_ptr())
    ws = torch.zeros(1 << 22, dtype=torch.uint8, device="cuda")
    pw = C.c_void_p(ws.data_ptr())
    call = lambda desc, ns, To, ql, q=p, w=pw, wb=ws.numel(): L.tandem_block_attn_shared(
        C.byref(desc), ns, To, q, p, p, pn, p, p, pn, ql, p, w, wb, None)
    assert call(d, 0, 16, 2) == binding.ERR_SHAPE
    assert call(d, 4, 16, 0) == binding.ERR_SHAPE
    assert call(d, 4, 16, 33) == binding.ERR_SHAPE
    assert call(d, 16, 64, 32) == binding.ERR_SHAPE          # samples * q_len above the limit
    assert call(d, 4, 1, 2) == binding.ERR_SHAPE             # own cache shorter than the block
    assert call(d, 4, 16, 2, q=None) == binding.ERR_NULL
    assert call(d, 4, 16, 2, w=None) == binding.ERR_NULL
    need = binding.tandem_block_attn_shared_workspace(d, 4, 16, 2)
    assert need > 0
    assert call(d, 4, 16, 2, wb=need - 1) == binding.ERR_WORKSPACE
    assert call(d, 4, 16, 2, wb=need) == binding.OK
    assert binding.tandem_block_attn_shared_workspace(d, 0, 16, 2) == 0
    torch.cuda.synchronize()


# --------------------------------------------------------------------------- all positions of the small model
def run_mixed(tb, case, gamma):
    torch, binding = tb
    dev = {k: case[k].to_torch() for k in ("q", "khat", "vhat", "kown", "vown")}
    out = binding.tandem_mixed_attn(dev["q"], dev["khat"], dev["vhat"], dev["kown"], dev["vown"],
                                    torch.from_numpy(case["n"]).cuda(), gamma, scale=case["scale"])
    torch.cuda.synchronize()
    return inputs.torch_to_f64(out)


def oracle_mixed(case, gamma):
    return orc.mixed_attn(case["q"].f64, case["khat"].f64, case["vhat"].f64, case["kown"].f64, case["vown"].f64,
                          case["n"], gamma, case["scale"])


@pytest.mark.parametrize(
    "B,q_len,Hq,Hkv,dh,T_max,n,gamma,dtype",
    [
        (2, 32, 8, 8, 128, 700, [668, 0], 4, "bf16"),     # the small model's shape (G=1): 32 rows, two wavefronts
        (3, 8, 8, 2, 128, 300, [292, 100, 3], 4, "bf16"),  # G=4: 32 rows; block boundaries inside the chunk
        (2, 5, 4, 4, 128, 530, [525, 64], 3, "bf16"),      # chunk not aligned with the blocks, one wavefront
        (1, 32, 8, 2, 128, 1300, [1200], 8, "bf16"),       # 128 rows: eight wavefronts, several context splits
        (2, 18, 8, 1, 128, 400, [382, 5], 5, "bf16"),      # G=8, 144 rows: two passes
        (2, 6, 4, 2, 128, 200, [194, 0], 1, "bf16"),       # block length 1: only the query's own row is its own
        (2, 6, 4, 2, 128, 200, [194, 0], 1000, "bf16"),    # no block ever completes: causal over the own rows
        (2, 7, 4, 2, 64, 150, [143, 10], 4, "bf16"),       # dh=64 generic path
        (2, 4, 2, 2, 64, 130, [126, 0], 2, "f32"),         # the tiny config's small model shape
        (1, 9, 4, 1, 128, 600, [555], 4, "f32"),
    ],
)
def test_mixed_attn_parity_small(tb, B, q_len, Hq, Hkv, dh, T_max, n, gamma, dtype):
    case = inputs.mixed_attn_case(41, B, q_len, Hq, Hkv, dh, T_max, n, dtype=dtype)
    got = run_mixed(tb, case, gamma)
    e = assert_rows_close(got.reshape(-1, Hq, dh), oracle_mixed(case, gamma).reshape(-1, Hq, dh), what="mixed")
    print(f"mixed small {B,q_len,Hq,Hkv,dh,T_max,gamma,dtype}: max rel err {e[0]:.2e}")


def test_mixed_attn_reads_the_right_cache_exactly(tb):
    """Q = 0 (uniform weights); V of the hat cache is 1 everywhere, V of the own cache 2: the query at position i
    must give exactly (k + 2 (i + 1 - k)) / (i + 1) with k = floor(i / gamma) * gamma - any key taken from the
    wrong cache, hidden or counted twice changes the value."""
    torch, binding = tb
    B, q_len, Hq, Hkv, dh, T_max, gamma = 1, 32, 8, 8, 128, 400, 4
    q = torch.zeros(B, q_len, Hq, dh, dtype=torch.bfloat16, device="cuda")
    k = torch.randn(B, Hkv, T_max, dh, device="cuda").to(torch.bfloat16)
    vh = torch.ones(B, Hkv, T_max, dh, dtype=torch.bfloat16, device="cuda")
    vo = 2 * vh
    for n0 in (0, 37, 368):
        n = torch.tensor([n0], dtype=torch.int32, device="cuda")
        out = binding.tandem_mixed_attn(q, k, vh, k, vo, n, gamma, scale=1.0).float().cpu().numpy()
        for r in range(q_len):
            i = n0 + r
            kb = i // gamma * gamma
            want = (kb + 2.0 * (i + 1 - kb)) / (i + 1)
            assert np.allclose(out[0, r], want, rtol=4e-3), (n0, r, out[0, r, 0, 0], want)


def test_mixed_attn_full_size_sampled(tb):
    """C3's small-model layer shape at context 8192 (the bench configuration): sampled output rows against the
    oracle's single-row definition."""
    torch, binding = tb
    B, q_len, Hq, Hkv, dh, T_max, gamma = 32, 32, 8, 8, 128, 8192, 4
    g = torch.Generator(device="cuda").manual_seed(7)
    mk = lambda *sh: torch.randn(*sh, device="cuda", generator=g).to(torch.bfloat16)
    q, kh, vh, ko, vo = mk(B, q_len, Hq, dh), mk(B, Hkv, T_max, dh), mk(B, Hkv, T_max, dh), mk(B, Hkv, T_max, dh), mk(B, Hkv, T_max, dh)
    n_host = np.full(B, T_max - q_len, np.int32)
    n_host[1], n_host[2] = 1000, 0
    out = binding.tandem_mixed_attn(q, kh, vh, ko, vo, torch.from_numpy(n_host).cuda(), gamma)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    f = inputs.torch_to_f64
    for _ in range(24):
        b, r, h = int(rng.integers(0, B)), int(rng.integers(0, q_len)), int(rng.integers(0, Hq))
        i = int(n_host[b]) + r
        kb = i // gamma * gamma
        K = np.concatenate([f(kh[b, h, :kb]), f(ko[b, h, kb:i + 1])])
        V = np.concatenate([f(vh[b, h, :kb]), f(vo[b, h, kb:i + 1])])
        want = orc.attention_one(f(q[b, r, h]), K, V, 1.0 / math.sqrt(dh))
        assert_rows_close(f(out[b, r, h])[None], want[None], what=f"mixed sampled row {b,r,h}")


@pytest.mark.parametrize(
    "B,q_len,Hq,Hkv,dh,T_max,n,gamma,dtype",
    [
        (3, 8, 8, 2, 128, 300, [292, 100, 0], 4, "bf16"),   # 32 rows; the third sequence's first block sees nothing
        (1, 32, 8, 2, 128, 1300, [1200], 8, "bf16"),        # 128 rows: the row-split kernel
        (2, 5, 4, 4, 128, 530, [525, 2], 3, "bf16"),
        (2, 7, 4, 2, 64, 150, [143, 1], 4, "bf16"),         # generic path
        (2, 6, 4, 4, 64, 130, [124, 0], 2, "f32"),
    ],
)
def test_block_prefix_attn_parity_small(tb, B, q_len, Hq, Hkv, dh, T_max, n, gamma, dtype):
    torch, binding = tb
    case = inputs.block_attn_case(51, B, q_len, Hq, Hkv, dh, T_max, n, dtype=dtype)
    out = binding.tandem_block_prefix_attn(case["q"].to_torch(), case["k"].to_torch(), case["v"].to_torch(),
                                           torch.from_numpy(case["n"]).cuda(), gamma, scale=case["scale"])
    torch.cuda.synchronize()
    want = orc.block_prefix_attn(case["q"].f64, case["k"].f64, case["v"].f64, case["n"], gamma, case["scale"])
    got = inputs.torch_to_f64(out)
    for b in range(B):
        for r in range(q_len):
            if (case["n"][b] + r) // gamma == 0:
                assert (got[b, r] == 0).all()   # no visible key: exactly zero
    seen = np.abs(want).reshape(B * q_len, -1).max(1) > 0
    e = assert_rows_close(got.reshape(B * q_len, Hq, dh)[seen], want.reshape(B * q_len, Hq, dh)[seen], what="prefix")
    print(f"prefix small {B,q_len,Hq,Hkv,dh,T_max,gamma,dtype}: max rel err {e[0]:.2e}")


def test_mixed_attn_error_codes(tb):
    torch, binding = tb
    import ctypes as C

    L = binding.lib()
    d = binding.attn_desc(2, 4, 2, 128, 64, 0, 0.1, binding.BF16)
    t = torch.zeros(2 * 4 * 64 * 128, dtype=torch.bfloat16, device="cuda")
    n = torch.zeros(2, dtype=torch.int32, device="cuda")
    p, pn = C.c_void_p(t.data_ptr()), C.c_void_p(n.data_ptr())
    ws = torch.zeros(1 << 22, dtype=torch.uint8, device="cuda")
    pw = C.c_void_p(ws.data_ptr())
    call = lambda ql, g, q=p, w=pw, wb=ws.numel(): L.tandem_mixed_attn(C.byref(d), q, p, p, p, p, pn, ql, g, p, w, wb, None)
    assert call(0, 4) == binding.ERR_SHAPE
    assert call(33, 4) == binding.ERR_SHAPE
    assert call(4, 0) == binding.ERR_SHAPE
    assert call(4, 4, q=None) == binding.ERR_NULL
    need = binding.tandem_mixed_attn_workspace(d, 4)
    assert need > 0
    assert call(4, 4, w=None) == binding.ERR_NULL
    assert call(4, 4, wb=need - 1) == binding.ERR_WORKSPACE
    assert call(4, 4, wb=need) == binding.OK
    torch.cuda.synchronize()


# --------------------------------------------------------------------------- error paths
def test_attention_error_codes(tb):
    torch, binding = tb
    import ctypes as C

    L = binding.lib()
    d = binding.attn_desc(2, 4, 2, 128, 64, 4, 0.1, binding.BF16)
    t = torch.zeros(2 * 4 * 64 * 128 * 2, dtype=torch.bfloat16, device="cuda")
    n = torch.zeros(2, dtype=torch.int32, device="cuda")
    p = C.c_void_p(t.data_ptr())
    pn = C.c_void_p(n.data_ptr())
    ws = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    pw = C.c_void_p(ws.data_ptr())
    assert L.tandem_draft_attn(C.byref(d), None, p, p, pn, p, p, pn, p, pw, ws.numel(), None) == binding.ERR_NULL
    assert L.tandem_block_attn(C.byref(d), p, p, p, pn, 0, p, pw, ws.numel(), None) == binding.ERR_SHAPE
    assert L.tandem_block_attn(C.byref(d), p, p, p, pn, 33, p, pw, ws.numel(), None) == binding.ERR_SHAPE
    bad = binding.attn_desc(2, 4, 3, 128, 64, 4, 0.1, binding.BF16)
    assert L.tandem_block_attn(C.byref(bad), p, p, p, pn, 2, p, pw, ws.numel(), None) == binding.ERR_SHAPE
    bad = binding.attn_desc(2, 4, 2, 96, 64, 4, 0.1, binding.BF16)
    assert L.tandem_draft_attn(C.byref(bad), p, p, p, pn, p, p, pn, p, pw, ws.numel(), None) == binding.ERR_UNSUPPORTED
    big = binding.attn_desc(2, 4, 2, 128, 1 << 16, 4, 0.1, binding.BF16)
    need = binding.tandem_draft_attn_workspace(big)
    assert need > 0
    assert L.tandem_draft_attn(C.byref(big), p, p, p, pn, p, p, pn, p, pw, need - 1, None) == binding.ERR_WORKSPACE
    torch.cuda.synchronize()
