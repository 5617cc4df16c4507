"""GPU parity of the adaptive block length (Sec. 3.1): the router alone (tandem_router_eval) and the decode step
that uses it (tandem_decode_step_adaptive), through the C ABI, against the fp64 oracle.

The router's arithmetic is fp32 on the GPU whatever the storage type: p is compared at 1e-4 relative (of the smaller
of p and 1 - p, beyond the fp32 spacing next to 1) on inputs the oracle reads at exactly the stored values.  Its decision p >= tau is an integer taken from floating point:
the step tests put tau in the middle of the widest gap between the oracle's probabilities, and require that gap
to be far above the arithmetic's resolution."""
import numpy as np
import pytest

from oracle import tandem_oracle as orc
from paper_2402_08644_amd import inputs
from parity import assert_rows_close
from test_gpu_decode_step import oracle_state_from, upload_state

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tb():
    import torch

    from paper_2402_08644_amd import binding

    assert torch.cuda.is_available()
    binding.lib()
    return torch, binding


def dev_router(R):
    return {k: (v if k == "k" else v.to_torch()) for k, v in R.items()}


@pytest.mark.parametrize(
    "rows,vocab,d,k,hidden,dtype",
    [
        (5, 1000, 128, 4, 32, "f32"),      # the tiny configuration's small model
        (3, 777, 48, 1, 7, "f32"),         # odd sizes, a single top token, fewer units than wavefronts
        (4, 4096, 256, 8, 100, "bf16"),    # the largest k
        (32, 32768, 1024, 4, 256, "bf16"),  # C3's small model: one call of the decode step
        (3, 40000, 32, 3, 8, "f32"),        # more than 32768 tokens: the logits row does not fit the registers
        (3, 70001, 16, 8, 20, "bf16"),
    ],
)
def test_router_eval_parity(tb, rows, vocab, d, k, hidden, dtype):
    torch, binding = tb
    rng = np.random.default_rng(rows + vocab)
    lg = rng.standard_normal((rows, vocab)).astype(np.float32) * 3.0
    lg[0, 5] = lg[0, 900 % vocab] = lg[0].max() + 0.5   # a tie at the top
    lg[1] = 0.0                                          # uniform: every probability ties
    lg[2, 17] = 60.0                                     # nearly all mass on one token
    logits = inputs.HostTensor(lg, dtype)
    emb = inputs.normal(rng, (vocab, d), 1.0, dtype)
    R = inputs.router_weights(7, k, d, hidden, dtype=dtype, w_std=0.05, out_std=0.3)
    got = binding.tandem_router_eval(dev_router(R), logits.to_torch(), emb.to_torch())
    torch.cuda.synchronize()
    R64 = inputs.as_f64(R)
    n_check = rows if vocab <= 4096 or rows <= 4 else 4   # the oracle's top-k scan is a Python loop
    want = np.array([orc.router_prob(R64, logits.f64[i], emb.f64) for i in range(n_check)])
    got = got.cpu().numpy().astype(np.float64)[:n_check]
    assert np.isfinite(got).all()
    # 1e-4 of the smaller of p and 1 - p, plus the spacing of fp32 numbers next to 1 (p itself is an fp32 number)
    err = (np.abs(got - want) - 5e-7) / np.minimum(want, 1 - want)
    assert err.max() <= 1e-4, (got, want)
    assert want.std() > 1e-3  # the cases do not all give the same number
    print(f"router {rows,vocab,d,k,hidden,dtype}: max rel err beyond fp32 spacing {max(err.max(), 0.0):.2e}")


def _drafted(p, tau):
    """Block lengths that follow from the probabilities p [B, gamma] of a run that never stopped."""
    return [next((r + 1 for r in range(p.shape[1]) if p[b, r] < tau), p.shape[1]) for b in range(p.shape[0])]


def _tau_between_probabilities(p, min_gap):
    """A threshold in the middle of a gap of at least min_gap between the probabilities, chosen so that the
    sequences stop at as many different block lengths as possible."""
    v = np.sort(np.asarray(p).reshape(-1))
    cands = [0.5 * (v[i] + v[i + 1]) for i in range(len(v) - 1) if v[i + 1] - v[i] > min_gap]
    assert cands
    return float(max(cands, key=lambda t: len(set(_drafted(p, t)))))


@pytest.mark.parametrize("free", [False, True])
def test_adaptive_step_tiny_config_fp32(tb, free):
    """Tiny configuration, fp32, gamma_max = 4, batch of 4 on random caches: block lengths, tokens, state and the
    cache rows below the new n are the oracle's."""
    torch, binding = tb
    W = inputs.tiny_tandem(seed=0, dtype="f32", gain_std=0.3, bias_std=0.02)  # random gains, non-zero biases
    T = inputs.as_f64(W)
    B, T_max, gmax = 4, 64, 4
    n, pending = [40, 7, 0, 21], [3, 500, 77, 999]
    R = inputs.router_weights(12, 4, 128, 32, dtype="f32", w_std=2.0, out_std=0.05)
    R64 = inputs.as_f64(R)
    probe_state, host = oracle_state_from(T, B, T_max, 9, n, pending, "f32")
    probe = orc.decode_step(T, probe_state, gmax, free_token=free, router=R64, tau=0.0)
    tau = _tau_between_probabilities(probe["router_p"], 1e-3)
    ost, _ = oracle_state_from(T, B, T_max, 9, n, pending, "f32")
    want = orc.decode_step(T, ost, gmax, free_token=free, router=R64, tau=tau)
    assert len(set(want["n_drafted"])) > 1 and list(want["n_drafted"]) == _drafted(probe["router_p"], tau)
    model = binding.TandemModel(W)
    gst = upload_state(tb, model, B, T_max, gmax, host, n, pending)
    got = binding.tandem_decode_step(model, gst, gmax, free_token=free, router=dev_router(R), tau=tau, aux=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got["n_drafted"].cpu().numpy(), want["n_drafted"])
    np.testing.assert_array_equal(got["n_accepted"].cpu().numpy(), want["n_accepted"])
    np.testing.assert_array_equal(got["tokens"].cpu().numpy(), want["tokens"])
    np.testing.assert_array_equal(gst.n.cpu().numpy(), ost["n"])
    np.testing.assert_array_equal(gst.pending.cpu().numpy(), ost["pending"])
    gp = got["router_p"].cpu().numpy().astype(np.float64)
    for b in range(B):
        g = int(want["n_drafted"][b])
        np.testing.assert_allclose(gp[b, :g], want["router_p"][b, :g], rtol=2e-3)
        for key, M in (("KL", T["L"]), ("Khat", T["S"]), ("VL", T["L"]), ("Vhat", T["S"])):
            for j in range(len(M["layers"])):
                rows = int(ost["n"][b])
                g_rows = inputs.torch_to_f64(getattr(gst, key)[j][b, :, :rows]).reshape(-1, M["dh"])
                assert_rows_close(g_rows, ost[key][j][b, :, :rows].reshape(-1, M["dh"]), tol=2e-3, what=f"{key}[{j}][{b}]")


def test_adaptive_step_thresholds_zero_and_above_one_equal_fixed_steps(tb):
    """tau = 0 never stops (the fixed-gamma step); tau > 1 always stops after one draft token (what a gamma = 1
    step emits).  GPU against GPU, bit for bit, bf16."""
    torch, binding = tb
    from test_gpu_decode_step import small_bf16_pair

    W = small_bf16_pair(70)
    T = inputs.as_f64(W)
    B, T_max, gmax = 3, 128, 4
    n, pending = [40, 7, 0], [3, 500, 77]
    _, host = oracle_state_from(T, B, T_max, 5, n, pending, "bf16")
    R = dev_router(inputs.router_weights(3, 2, 256, 16, dtype="bf16", w_std=0.1, out_std=0.2))
    model = binding.TandemModel(W)
    for tau, g_fixed in ((0.0, gmax), (1.5, 1)):
        for free in (False, True):
            sa = upload_state(tb, model, B, T_max, gmax, host, n, pending)
            sf = upload_state(tb, model, B, T_max, gmax, host, n, pending)
            a = binding.tandem_decode_step(model, sa, gmax, free_token=free, router=R, tau=tau)
            f = binding.tandem_decode_step(model, sf, g_fixed, free_token=free)
            torch.cuda.synchronize()
            q = g_fixed + (1 if free else 0)
            assert a["n_drafted"].cpu().tolist() == [g_fixed] * B
            assert torch.equal(a["tokens"][:, :q], f["tokens"]) and bool((a["tokens"][:, q:] == -1).all())
            assert torch.equal(a["n_accepted"], f["n_accepted"])
            assert torch.equal(sa.n, sf.n) and torch.equal(sa.pending, sf.pending)


def test_adaptive_step_skips_the_runs_after_every_sequence_has_stopped(tb):
    """bf16: once no sequence drafts any more, the kernels of the remaining draft runs return at once - their greedy
    tokens are never written - and the step's results are still the oracle's.  Two thresholds: every sequence stops
    after the first token; and one chosen from the probabilities so that the last one stops after the second."""
    torch, binding = tb
    from test_gpu_decode_step import small_bf16_pair, tokens_ok

    W = small_bf16_pair(71)
    T = inputs.as_f64(W)
    B, T_max, gmax = 4, 128, 4
    n, pending = [40, 7, 0, 90], [3, 500, 77, 12]
    Rh = inputs.router_weights(4, 2, 256, 16, dtype="bf16", w_std=0.1, out_std=0.2)
    R, R64 = dev_router(Rh), inputs.as_f64(Rh)
    probe_state, host = oracle_state_from(T, B, T_max, 6, n, pending, "bf16")
    probe = orc.decode_step(T, probe_state, gmax, router=R64, tau=0.0)["router_p"]
    # above every probability of run 0: all stop at once; above the largest of run 1 only: the last ones stop there
    # (kept 0.01 away from every probability, so that bf16 logits cannot move a decision across it)
    second = next(t for t in float(probe[:, 1].max()) + 0.011 + 0.003 * np.arange(200) if np.abs(probe - t).min() > 0.01)
    assert second < 1.5
    model = binding.TandemModel(W)
    for tau in (1.5, second):
        ost, _ = oracle_state_from(T, B, T_max, 6, n, pending, "bf16")
        want = orc.decode_step(T, ost, gmax, router=R64, tau=tau)
        last = int(max(want["n_drafted"]))
        assert last < gmax
        gst = upload_state(tb, model, B, T_max, gmax, host, n, pending)
        dev = gst.n.device
        out = dict(tokens=torch.empty((B, gmax), dtype=torch.int32, device=dev),
                   n_accepted=torch.empty((B,), dtype=torch.int32, device=dev),
                   draft=torch.full((B, gmax), -7, dtype=torch.int32, device=dev),
                   verify=torch.empty((B, gmax), dtype=torch.int32, device=dev),
                   y_small=torch.empty((B, gmax, model.S.d), dtype=model.dtype, device=dev),
                   x_large=torch.empty((B, gmax, model.L.d), dtype=model.dtype, device=dev),
                   logits_S=torch.empty((B, gmax, model.S.vocab), dtype=model.dtype, device=dev),
                   logits_L=torch.empty((B, gmax, model.L.vocab), dtype=model.dtype, device=dev))
        got = binding.tandem_decode_step(model, gst, gmax, router=R, tau=tau, out=out)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(got["n_drafted"].cpu().numpy(), want["n_drafted"])
        draft = got["draft"].cpu().numpy()
        assert (draft[:, :last] >= 0).all()      # the runs somebody needed ran
        assert (draft[:, last:] == -7).all()     # the later ones wrote no token
        # tokens: the oracle's, or within the arithmetic's resolution of its logits where the GPU's drafts agree
        if np.array_equal(draft[:, :last], np.asarray(want["draft"])[:, :last]):
            np.testing.assert_array_equal(got["n_accepted"].cpu().numpy(), want["n_accepted"])
            np.testing.assert_array_equal(gst.n.cpu().numpy(), ost["n"])
        for b in range(B):
            g = int(want["n_drafted"][b])
            assert tokens_ok(draft[b, :g], np.asarray(want["logits_S"])[b, :g])


def test_adaptive_step_gate_with_many_sequences(tb):
    """40 sequences (M_S's products run the 64-row kernels): with a threshold above every probability all stop after
    the first token, the later runs write nothing, and the step equals the gamma = 1 step bit for bit."""
    torch, binding = tb
    from test_gpu_decode_step import small_bf16_pair

    W = small_bf16_pair(72)
    B, T_max, gmax = 40, 64, 4
    model = binding.TandemModel(W)
    R = dev_router(inputs.router_weights(6, 2, 256, 16, dtype="bf16", w_std=0.1, out_std=0.2))
    fill = lambda *s: torch.randn(s, device="cuda", generator=torch.Generator("cuda").manual_seed(5)).to(torch.bfloat16)
    sa = binding.TandemState(model, B, T_max, gmax, fill=fill)
    sf = binding.TandemState(model, B, T_max, gmax, fill=fill)
    for st in (sa, sf):
        st.n.copy_(torch.arange(B, dtype=torch.int32) % 50)
        st.pending.copy_((torch.arange(B, dtype=torch.int32) * 7) % 512)
    dev = sa.n.device
    out = dict(tokens=torch.empty((B, gmax), dtype=torch.int32, device=dev),
               n_accepted=torch.empty((B,), dtype=torch.int32, device=dev),
               draft=torch.full((B, gmax), -7, dtype=torch.int32, device=dev),
               verify=torch.empty((B, gmax), dtype=torch.int32, device=dev),
               y_small=torch.empty((B, gmax, model.S.d), dtype=model.dtype, device=dev),
               x_large=torch.empty((B, gmax, model.L.d), dtype=model.dtype, device=dev),
               logits_S=torch.empty((B, gmax, model.S.vocab), dtype=model.dtype, device=dev),
               logits_L=torch.empty((B, gmax, model.L.vocab), dtype=model.dtype, device=dev))
    a = binding.tandem_decode_step(model, sa, gmax, router=R, tau=1.5, out=out)
    f = binding.tandem_decode_step(model, sf, 1)
    torch.cuda.synchronize()
    assert a["n_drafted"].cpu().tolist() == [1] * B
    assert bool((a["draft"][:, 0] >= 0).all()) and bool((a["draft"][:, 1:] == -7).all())
    assert torch.equal(a["tokens"][:, :1], f["tokens"]) and bool((a["tokens"][:, 1:] == -1).all())
    assert torch.equal(a["n_accepted"], f["n_accepted"])
    assert torch.equal(sa.n, sf.n) and torch.equal(sa.pending, sf.pending)


def test_router_error_codes(tb):
    torch, binding = tb
    import ctypes as C

    L = binding.lib()
    R = dev_router(inputs.router_weights(1, 2, 16, 4, dtype="f32"))
    lg = torch.zeros(2, 50, device="cuda")
    emb = torch.zeros(50, 16, device="cuda")
    out = torch.zeros(2, device="cuda")
    p = lambda t: C.c_void_p(t.data_ptr())
    rd = binding.router_desc(R)
    assert L.tandem_router_eval(C.byref(rd), p(lg), p(emb), 2, 50, 16, p(out), None) == binding.OK
    assert L.tandem_router_eval(C.byref(rd), None, p(emb), 2, 50, 16, p(out), None) == binding.ERR_NULL
    assert L.tandem_router_eval(C.byref(rd), p(lg), p(emb), 0, 50, 16, p(out), None) == binding.ERR_SHAPE
    assert L.tandem_router_eval(C.byref(rd), p(lg), p(emb), 2, 1, 16, p(out), None) == binding.ERR_SHAPE
    bad = binding.router_desc(R)
    bad.k = 9
    assert L.tandem_router_eval(C.byref(bad), p(lg), p(emb), 2, 50, 16, p(out), None) == binding.ERR_SHAPE
    bad = binding.router_desc(R)
    bad.k = 8  # 1 + 8 * (4096 + 1) floats do not fit the 64 KB of LDS
    assert L.tandem_router_eval(C.byref(bad), p(lg), p(emb), 2, 50, 4096, p(out), None) == binding.ERR_UNSUPPORTED
    torch.cuda.synchronize()
