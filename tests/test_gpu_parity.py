"""GPU parity tests: the HIP path, called through the C ABI, against the CPU
oracle on the same seeded inputs.  Protocol and tolerances: tests/parity.py."""
import numpy as np
import pytest
import torch

from synth_inputs import CONFIGS, SwitchShape, make_inputs

pytestmark = pytest.mark.gpu


def _dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return "cuda:0"


def _report(name, errs):
    print("\n[parity] %s: %s" % (name, {k: (("%.2e" % v) if isinstance(v, float) else v)
                                        for k, v in errs.items()}), flush=True)


# ----------------------------------------------------------------- fp32 path
def test_tiny_fp32_full_parity():
    from parity import compare_full
    s = CONFIGS["tiny"]
    inp = make_inputs(s, _dev())
    errs, gpu, fwd, _ = compare_full(s, inp, d_aux=1.0)
    _report("tiny", errs)
    assert fwd["capacity"] == 80


@pytest.mark.parametrize("T,d,f,E,cf,bias", [
    (300, 20, 36, 3, 0.7, True),      # ragged everything, drops, router bias
    (1000, 64, 128, 8, 1.0, False),   # several token blocks
    (64, 32, 64, 1, 1.0, False),      # single expert: dense FFN, gate 1
    (257, 16, 32, 5, 4.0, False),     # no drops
])
def test_fp32_shapes_full_parity(T, d, f, E, cf, bias):
    from parity import compare_full
    s = SwitchShape("t", T, d, f, E, cf, dtype="f32", zipf_bias=bias, seed_index=31)
    inp = make_inputs(s, _dev())
    errs, gpu, fwd, _ = compare_full(s, inp, d_aux=0.7)
    _report("fp32 %s" % ((T, d, f, E, cf, bias),), errs)
    if E == 1:
        assert np.all(gpu["gate"] == 1.0)
        assert np.abs(gpu["dW_r"]).max() == 0.0


# ----------------------------------------------------------------- bf16 path
@pytest.mark.parametrize("T,d,f,E,cf,bias", [
    (2000, 264, 520, 5, 1.5, False),   # 3 ragged token tiles, K tail (264 = 4*64 + 8), ragged p tiles
    (4096, 128, 256, 16, 1.0, True),   # Zipf bias: overflow and empty experts
    (1024, 64, 64, 1, 1.0, False),     # single expert, 4 full token tiles
    (777, 72, 136, 7, 0.5, False),     # heavy dropping, odd sizes
    (3000, 512, 768, 4, 1.25, False),  # several k steps and 3 x 2 p tiles
])
@pytest.mark.parametrize("in_gemm", [False, True])   # dispatch / combine as passes, or inside the GEMMs
def test_bf16_shapes_full_parity(T, d, f, E, cf, bias, in_gemm):
    from parity import compare_full
    s = SwitchShape("t", T, d, f, E, cf, dtype="bf16", zipf_bias=bias, seed_index=41,
                    fused_dispatch=in_gemm)
    inp = make_inputs(s, _dev())
    errs, gpu, fwd, _ = compare_full(s, inp, d_aux=1.0)
    _report("bf16 %s%s" % ((T, d, f, E, cf, bias), ", in the GEMMs" if in_gemm else ""), errs)
    if bias:
        assert fwd["dropped"].sum() > 0 and (fwd["expert_counts"] == 0).any()


@pytest.mark.parametrize("T,d,f,E,cf,n,bias,ffn,rate,rounds", [
    (2000, 264, 520, 5, 1.5, 1, False, "relu", 0.0, 0),    # ragged tiles everywhere
    (4096, 128, 256, 16, 1.0, 2, True, "relu", 0.1, 1),    # groups, skew, dropout, re-routing
    (3000, 512, 768, 4, 1.25, 1, False, "geglu", 0.0, 0),  # gated-GELU experts
])
def test_bf16_dispatch_inside_the_gemms_agrees_with_the_passes(T, d, f, E, cf, n, bias, ffn, rate, rounds):
    """Dispatch and combine as passes of their own (the default) and inside the GEMMs (on
    request): each against the oracle, and against each other to rounding."""
    from parity import compare_full
    s = SwitchShape("t", T, d, f, E, cf, dtype="bf16", zipf_bias=bias, seed_index=43, n_groups=n,
                    ffn=ffn, expert_dropout=rate, noise_seed=5, ntlb_rounds=rounds)
    inp = make_inputs(s, _dev())
    errs, sep, _, _ = compare_full(s, inp, d_aux=0.9)
    _report("bf16 separate passes %s" % ((T, d, f, E, cf, n, ffn),), errs)
    errs, fused, _, _ = compare_full(s.with_(fused_dispatch=True), inp, d_aux=0.9)
    _report("bf16 inside the GEMMs %s" % ((T, d, f, E, cf, n, ffn),), errs)
    for k in ("expert_index", "gate", "position_in_expert", "dropped", "expert_counts", "aux_loss",
              "router_logits"):
        assert np.array_equal(sep[k], fused[k]), k
    for k in ("y", "dx", "dW_in", "dW_out"):
        a, b = sep[k].astype(np.float64), fused[k].astype(np.float64)
        assert np.linalg.norm(a - b) <= 1e-2 * np.linalg.norm(b), k


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_capacity_zero_everything_dropped(dtype):
    from parity import compare_full
    s = SwitchShape("t", 5, 64, 64, 8, 1.0, dtype=dtype, seed_index=51)
    inp = make_inputs(s, _dev())
    errs, gpu, fwd, bwd = compare_full(s, inp)
    assert fwd["capacity"] == 0 and gpu["dropped"].all()
    assert np.all(gpu["y"] == 0) and np.all(gpu["dW_in"] == 0) and np.all(gpu["dW_out"] == 0)
    assert np.abs(gpu["dx"]).max() > 0          # the auxiliary loss still reaches x


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T,E,cf", [
    (1, 4, 4.0),     # a single token, capacity 1
    (7, 16, 4.0),    # more experts than tokens, capacity 1
    (7, 16, 1.0),    # ... and capacity floor(7/16) = 0
    (255, 3, 1.0),   # one short token block
    (257, 3, 1.0),   # one token into the second block
])
def test_few_tokens(dtype, T, E, cf):
    from parity import compare_full
    s = SwitchShape("t", T, 64, 72, E, cf, dtype=dtype, seed_index=54)
    inp = make_inputs(s, _dev())
    # With a handful of kept tokens all of dW_r and db_r is a few gate gradients
    # <dy_t, o_t> times fixed vectors: their error is measured against the scale of those dot
    # products' terms (parity.router_grad_scales), as for every other case.
    errs, gpu, fwd, _ = compare_full(s, inp, d_aux=0.3)
    _report("few tokens %s %s" % (dtype, (T, E, cf)), errs)
    assert fwd["capacity"] == int(np.floor(T / E * cf))


@pytest.mark.parametrize("T,d,f,E,cf", [
    (1500, 96, 64, 128, 2.0),    # the widest router the matrix-core kernel takes
    (1500, 96, 64, 124, 2.0),    # four experts short of it
    (3000, 64, 64, 132, 1.0),    # one step wider: vector-ALU router, bf16 tokens
    (3000, 64, 64, 256, 1.0),    # two experts per lane in the softmax kernels
    (2048, 72, 64, 126, 1.0),    # E not a multiple of 4: vector-ALU router
])
def test_bf16_router_widths(T, d, f, E, cf):
    from parity import compare_full
    s = SwitchShape("t", T, d, f, E, cf, dtype="bf16", seed_index=55)
    inp = make_inputs(s, _dev())
    errs, gpu, fwd, _ = compare_full(s, inp, d_aux=1.0)
    _report("bf16 router E=%d" % E, errs)


@pytest.mark.parametrize("dtype,T,d,f,E,cf,n", [
    ("f32", 600, 32, 48, 4, 1.0, 2),       # 300 tokens per group: blocks of 256 + 44
    ("f32", 90, 16, 24, 3, 0.9, 5),        # groups smaller than a token block
    ("bf16", 4096, 128, 256, 16, 1.0, 8),  # groups of two full blocks
    ("bf16", 3000, 96, 136, 12, 1.25, 3),  # 1000 tokens per group
    ("bf16", 2100, 64, 72, 7, 0.5, 7),     # heavy dropping in every group, vector-ALU router
])
def test_routing_groups(dtype, T, d, f, E, cf, n):
    """Capacity, positions and the loss fractions per routing group; shared experts."""
    from parity import compare_full
    s = SwitchShape("t", T, d, f, E, cf, dtype=dtype, seed_index=57, n_groups=n)
    inp = make_inputs(s, _dev())
    if dtype == "bf16":   # also with dispatch / combine inside the GEMMs
        errs = compare_full(s.with_(fused_dispatch=True), inp, d_aux=0.8)[0]
        _report("groups %s, in the GEMMs" % ((dtype, T, E, cf, n),), errs)
    errs, gpu, fwd, _ = compare_full(s, inp, d_aux=0.8)
    _report("groups %s" % ((dtype, T, E, cf, n),), errs)
    assert fwd["capacity"] == int(np.floor(T / n / E * cf))
    # positions restart in every group
    Tg = T // n
    first = np.array([np.flatnonzero(gpu["expert_index"][g * Tg:(g + 1) * Tg] ==
                                     gpu["expert_index"][g * Tg])[0] for g in range(n)])
    assert np.all(first == 0) and np.all(gpu["position_in_expert"][::Tg] == 0)


def test_routing_groups_full_size():
    """Switch-Base shape as eight routing groups (capacity 64 per expert and group)."""
    from parity import compare_sampled
    s = CONFIGS["base_cf1.0"].with_(n_groups=8)
    inp = make_inputs(s, _dev())
    errs = compare_sampled(s, inp, n_experts=2, n_tokens=24)
    _report("base_cf1.0 x 8 groups", errs)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_empty_batch(dtype):
    """T = 0: counts and loss zero, weight gradients zero, nothing else touched."""
    import torch
    import oracle
    from paper_2101_03961_amd.layer import SwitchLayer
    s = SwitchShape("t", 0, 64, 72, 4, 1.0, dtype=dtype, seed_index=56)
    inp = make_inputs(s, _dev())
    layer = SwitchLayer(0, 64, 72, 4, 1.0, s.alpha, dtype, device=_dev())
    layer.expert_counts.fill_(7)
    layer.aux_loss.fill_(7.0)
    layer.forward(inp["x"], inp["W_r"], inp["W_in"], inp["W_out"], None)
    layer.alloc_grads(with_bias=True)
    for g in (layer.dW_r, layer.db_r, layer.dW_in, layer.dW_out):
        g.fill_(1.0)
    layer.backward(inp["dy"], inp["x"], inp["W_r"], inp["W_in"], inp["W_out"], None, 1.0)
    torch.cuda.synchronize()
    to_np = lambda t: t.float().cpu().numpy()
    ref = oracle.forward(to_np(inp["x"]), to_np(inp["W_r"]), to_np(inp["W_in"]),
                         to_np(inp["W_out"]), 1.0, s.alpha)
    assert ref["aux_loss"] == 0.0 and ref["capacity"] == 0 and ref["y"].shape == (0, 64)
    assert float(layer.aux_loss[0]) == ref["aux_loss"]
    assert layer.expert_counts.tolist() == ref["expert_counts"].tolist() == [0, 0, 0, 0]
    for g in (layer.dW_r, layer.db_r, layer.dW_in, layer.dW_out):
        assert float(g.float().abs().max()) == 0.0


def test_exact_ties_go_to_expert_zero():
    from parity import run_gpu
    s = SwitchShape("t", 300, 64, 64, 6, 1.0, dtype="bf16", seed_index=52)
    inp = make_inputs(s, _dev())
    inp["W_r"].zero_()
    _, gpu = run_gpu(s, inp, backward=False)
    assert np.all(gpu["expert_index"] == 0)
    assert np.all(gpu["gate"] == np.float32(1.0) / np.float32(6.0))
    assert gpu["expert_counts"].tolist() == [300, 0, 0, 0, 0, 0]
    assert np.array_equal(gpu["position_in_expert"], np.arange(300))
    assert np.array_equal(gpu["dropped"], (np.arange(300) >= 50).astype(np.uint8))
    assert abs(float(gpu["aux_loss"][0]) - 0.01) < 1e-7      # P uniform => loss = alpha


@pytest.mark.parametrize("in_gemm", [False, True])
def test_run_to_run_determinism(in_gemm):
    from parity import run_gpu
    s = SwitchShape("t", 5000, 256, 512, 12, 1.0, dtype="bf16", seed_index=53, fused_dispatch=in_gemm)
    inp = make_inputs(s, _dev())
    _, a = run_gpu(s, inp)
    _, b = run_gpu(s, inp)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


@pytest.mark.parametrize("dtype,in_gemm", [("f32", False), ("bf16", False), ("bf16", True)])
def test_scaling_and_expert_permutation_properties(dtype, in_gemm):
    """Properties of the GPU path alone.  Doubling W_out doubles y exactly (a power of two
    changes no rounding).  Renumbering the experts (columns of W_r, blocks of W_in / W_out)
    renumbers expert_index and the counts and leaves every token's slot; gate and output move
    only by the rounding of the softmax sum taken in another order (and what follows from it)."""
    from parity import run_gpu
    s = SwitchShape("t", 3000, 128, 264, 12, 1.0, dtype=dtype, seed_index=92, fused_dispatch=in_gemm)
    inp = make_inputs(s, _dev())
    _, a = run_gpu(s, inp, backward=False)
    doubled = dict(inp, W_out=inp["W_out"] * 2)
    _, b = run_gpu(s, doubled, backward=False)
    assert np.array_equal(b["y"], 2 * a["y"])
    for k in ("expert_index", "gate", "dropped", "position_in_expert", "aux_loss"):
        assert np.array_equal(a[k], b[k]), k
    perm = torch.randperm(s.E, generator=torch.Generator().manual_seed(5)).to(_dev())
    shuffled = dict(inp, W_r=inp["W_r"][:, perm].contiguous(), W_in=inp["W_in"][perm].contiguous(),
                    W_out=inp["W_out"][perm].contiguous())
    _, c = run_gpu(s, shuffled, backward=False)
    p = perm.cpu().numpy()
    assert np.array_equal(p[c["expert_index"]], a["expert_index"])
    assert np.array_equal(c["expert_counts"], a["expert_counts"][p])
    for k in ("dropped", "position_in_expert"):
        assert np.array_equal(a[k], c[k]), k
    np.testing.assert_allclose(c["gate"], a["gate"], rtol=5e-7, atol=0)
    # one rounding step of the storage type; with the combine inside the GEMMs also: the gate
    # scales the hidden activations before they are rounded, so a gate that moves by one fp32 ulp
    # flips the rounding of a few of them: a row may move by a small share of its RMS
    ulp = 2.0 ** -7 if dtype == "bf16" else 1e-6
    rms = np.sqrt(np.mean(a["y"].astype(np.float64) ** 2, axis=1, keepdims=True))
    floor = 2.0 ** -9 * rms if in_gemm else 1e-30
    assert np.all(np.abs(c["y"].astype(np.float64) - a["y"]) <= ulp * np.abs(a["y"]) + floor)
    assert abs(float(a["aux_loss"][0]) - float(c["aux_loss"][0])) <= 1e-6 * abs(float(a["aux_loss"][0]))


@pytest.mark.parametrize("dtype,T,d,f,E,cf,n", [
    ("bf16", 16384, 64, 64, 4096, 2.0, 1),  # the largest expert count the library takes
    ("f32", 3000, 32, 48, 1000, 3.0, 1),
    ("bf16", 6000, 72, 64, 513, 1.0, 2),    # nine experts per lane in the softmax kernels
])
def test_many_experts(dtype, T, d, f, E, cf, n):
    from parity import compare_full
    s = SwitchShape("t", T, d, f, E, cf, dtype=dtype, seed_index=59, n_groups=n)
    inp = make_inputs(s, _dev())
    errs, gpu, fwd, _ = compare_full(s, inp, d_aux=0.5)
    _report("E=%d" % E, errs)


@pytest.mark.parametrize("T,d,f,E,cf,n,bias,eps,rounds", [
    (4096, 128, 72, 256, 2.0, 1, False, 0.0, 0),      # two full expert tiles
    (3000, 200, 64, 200, 1.0, 2, True, 0.0, 1),       # second tile partly filled, ragged d
    (2048, 776, 64, 1024, 4.0, 1, False, 0.01, 0),    # eight tiles, jittered input planes
    (5000, 96, 64, 132, 1.5, 1, True, 0.0, 2),        # four experts in the second tile
])
def test_bf16_router_on_matrix_cores_beyond_128_experts(T, d, f, E, cf, n, bias, eps, rounds):
    """More than 128 experts (a multiple of 4): the logits come from the matrix-core kernel, one
    tile of 128 experts per block, softmax and the rest from the vector-ALU path's kernel."""
    from parity import compare_full
    s = SwitchShape("t", T, d, f, E, cf, dtype="bf16", seed_index=62, n_groups=n, zipf_bias=bias,
                    jitter_eps=eps, noise_seed=17, ntlb_rounds=rounds)
    errs = compare_full(s, make_inputs(s, _dev()), d_aux=0.5)[0]
    _report("bf16 router, E=%d" % E, errs)


def test_fp32_long_reduction():
    """One expert holding 17 576 tokens: each weight-gradient element is a sum over all of them,
    which the fp32 path takes in two levels (a single fp32 chain drifts past 1e-5 here)."""
    from parity import compare_full
    s = SwitchShape("t", 17576, 292, 152, 1, 1.25, dtype="f32", seed_index=61, n_groups=8)
    errs = compare_full(s, make_inputs(s, _dev()), d_aux=0.5)[0]
    _report("fp32, 17576 tokens in one expert", errs)
    assert errs["dW_in"] < 2e-6 and errs["dW_out"] < 2e-6


def test_random_shapes():
    """Seeded sweep over token counts, widths, expert counts, capacity factors, group counts
    and both storage types: every tile edge and kernel variant at sizes the full oracle takes
    a fraction of a second for."""
    from parity import compare_full
    rng = np.random.default_rng(20210111)
    for case in range(36):
        dtype = "bf16" if rng.random() < 0.75 else "f32"
        mult = 8 if dtype == "bf16" else 4
        E = int(rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 20, 32, 64]))
        n = int(rng.choice([1, 1, 1, 2, 3, 4]))
        T = int(rng.integers(200, 1400)) * n
        hi_d, hi_f = (640, 800) if dtype == "bf16" else (400, 400)
        d = int(rng.integers(32 // mult, hi_d // mult)) * mult
        f = int(rng.integers(32 // mult, hi_f // mult)) * mult
        cf = float(rng.choice([0.7, 1.0, 1.25, 2.0, 8.0]))
        in_gemm = dtype == "bf16" and case % 2 == 1
        s = SwitchShape("t", T, d, f, E, cf, dtype=dtype, seed_index=300 + case, n_groups=n,
                        fused_dispatch=in_gemm)
        print("[random shape %d] %s T=%d d=%d f=%d E=%d cf=%g groups=%d in_gemm=%d" %
              (case, dtype, T, d, f, E, cf, n, in_gemm), flush=True)
        inp = make_inputs(s, _dev())
        compare_full(s, inp, d_aux=0.5)


def test_random_shapes_with_options():
    """The same sweep with the optional parts switched on at random: gated-GELU experts,
    expert dropout, input jitter, re-routing stages, router bias."""
    from parity import compare_full
    rng = np.random.default_rng(20210112)
    for case in range(30):
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        mult = 8 if dtype == "bf16" else 4
        E = int(rng.choice([2, 3, 4, 6, 8, 16, 32, 128]))
        n = int(rng.choice([1, 1, 2, 4]))
        T = int(rng.integers(300, 1400)) * n
        hi_d, hi_f = (520, 400) if dtype == "bf16" else (300, 200)
        d = int(rng.integers(32 // mult, hi_d // mult)) * mult
        f = int(rng.integers(32 // mult, hi_f // mult)) * mult
        cf = float(rng.choice([0.7, 1.0, 1.25, 2.0]))
        ffn = "geglu" if rng.random() < 0.5 else "relu"
        rate = float(rng.choice([0.0, 0.1, 0.4]))
        eps = float(rng.choice([0.0, 0.0, 0.01, 0.1]))
        rounds = int(rng.choice([0, 0, 1, 2, 4]))
        bias = bool(rng.random() < 0.4)
        s = SwitchShape("t", T, d, f, E, cf, dtype=dtype, seed_index=400 + case, n_groups=n,
                        ffn=ffn, expert_dropout=rate, jitter_eps=eps,
                        noise_seed=int(rng.integers(0, 2 ** 62)), ntlb_rounds=rounds, zipf_bias=bias,
                        fused_dispatch=dtype == "bf16" and case % 2 == 0)
        print("[random options %d] %s T=%d d=%d f=%d E=%d cf=%g groups=%d %s drop=%g jitter=%g "
              "stages=%d bias=%d in_gemm=%d" % (case, dtype, T, d, f, E, cf, n, ffn, rate, eps, rounds,
                                                bias, s.fused_dispatch), flush=True)
        inp = make_inputs(s, _dev())
        compare_full(s, inp, d_aux=0.5)


def test_relu_decision_at_a_zero_preactivation():
    """In this seeded case one pre-activation is -7.5e-9 in fp64 (RMS of its row: 1) and the
    fp32 sum of the same exact products comes out positive: the unit's gate is a coin flip,
    the protocol follows the GPU's decision for that one (token, unit) pair."""
    from parity import compare_full
    s = SwitchShape("t", 1206, 208, 712, 1, 2.0, dtype="bf16", seed_index=152)
    inp = make_inputs(s, _dev())
    errs, gpu, fwd, _ = compare_full(s, inp, d_aux=0.5)
    _report("zero pre-activation", errs)
    import oracle
    npi = {k: (None if v is None else v.float().cpu().numpy()) for k, v in inp.items()}
    near = oracle.hidden_near_zero(npi["x"], npi["W_in"], fwd["expert_index"], fwd["dropped"], 1e-6)
    assert (252, 515) in [(t, j) for t, j, _ in near] and len(near) <= 4, near
    assert all(abs(h) < 1e-5 for _, _, h in near)


@pytest.mark.parametrize("options", [
    {},
    dict(fused_dispatch=True),
    dict(ffn="geglu", expert_dropout=0.1, jitter_eps=0.01, noise_seed=3, ntlb_rounds=2),
    dict(ffn="geglu", expert_dropout=0.1, jitter_eps=0.01, noise_seed=3, ntlb_rounds=2,
         fused_dispatch=True),
])
def test_step_can_be_captured_in_a_graph(options):
    """Forward + backward recorded once and replayed: every replay, with eager work and
    synchronisation between them, reproduces the eager result bit for bit (the library launches
    only kernels: no allocation, no memset node, no host synchronisation)."""
    import torch
    from paper_2101_03961_amd.layer import SwitchLayer
    s = SwitchShape("t", 3000, 256, 512, 12, 1.0, dtype="bf16", seed_index=58, n_groups=2,
                    **options)
    inp = make_inputs(s, _dev())
    layer = SwitchLayer(s.T, s.d_model, s.d_ff, s.E, s.capacity_factor, s.alpha, s.dtype,
                        device=_dev(), n_groups=s.n_groups, ffn=s.ffn,
                        expert_dropout=s.expert_dropout, jitter_eps=s.jitter_eps,
                        seed=s.noise_seed, ntlb_rounds=s.ntlb_rounds, fused_dispatch=s.fused_dispatch)
    layer.alloc_grads(with_bias=False)
    names = ("y", "dx", "dW_r", "dW_in", "dW_out", "aux_loss", "expert_counts", "gate", "dropped")

    def step():
        layer.forward(inp["x"], inp["W_r"], inp["W_in"], inp["W_out"], None)
        layer.backward(inp["dy"], inp["x"], inp["W_r"], inp["W_in"], inp["W_out"], None, 1.0)

    step()
    torch.cuda.synchronize()
    eager = {k: getattr(layer, k).clone() for k in names}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(3):
        for k in names:
            getattr(layer, k).fill_(3)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in names:
            assert torch.equal(getattr(layer, k), eager[k]), k
        assert float(layer.y.float().abs().sum()) > 0   # eager work between replays


# ------------------------------------------- training-time noise (Sec. 2.4, App. C)
@pytest.mark.parametrize("dtype,T,d,f,E,cf,n,bias,rate,eps,seed", [
    ("f32", 700, 96, 200, 6, 1.0, 1, False, 0.1, 0.01, 0x123456789ABC),     # both, 48-bit seed
    ("f32", 1024, 64, 136, 8, 0.75, 4, True, 0.4, 0.0, 5),                  # dropout only, groups
    ("f32", 515, 72, 64, 5, 2.0, 1, False, 0.0, 0.25, 2 ** 63 + 11),        # jitter only
    ("bf16", 1500, 256, 520, 6, 1.25, 1, False, 0.4, 0.1, 7),
    ("bf16", 2048, 128, 264, 128, 1.5, 2, True, 0.0, 0.01, 99),             # would take the MFMA router
    ("bf16", 3000, 776, 304, 16, 1.0, 3, False, 0.1, 0.0, 2 ** 40),         # MFMA router + dropout
])
def test_training_noise(dtype, T, d, f, E, cf, n, bias, rate, eps, seed):
    from parity import compare_full
    s = SwitchShape("t", T, d, f, E, cf, dtype=dtype, seed_index=70, n_groups=n, zipf_bias=bias,
                    expert_dropout=rate, jitter_eps=eps, noise_seed=seed)
    inp = make_inputs(s, _dev())
    if dtype == "bf16":   # also with dispatch / combine inside the GEMMs
        errs = compare_full(s.with_(fused_dispatch=True), inp, d_aux=0.8)[0]
        _report("noise %s rate %.2f eps %.2f, in the GEMMs" % (dtype, rate, eps), errs)
    errs, gpu, fwd, _ = compare_full(s, inp, d_aux=0.8)
    _report("noise %s rate %.2f eps %.2f" % (dtype, rate, eps), errs)
    # the noise did something: outputs differ from the noise-free layer's
    _, plain = run_gpu_plain(s, inp)
    assert not np.array_equal(plain["y"], gpu["y"])
    if eps > 0:
        assert not np.array_equal(plain["router_logits"], gpu["router_logits"])
    else:
        assert np.array_equal(plain["router_logits"], gpu["router_logits"])
        assert np.array_equal(plain["expert_index"], gpu["expert_index"])


def run_gpu_plain(s, inp):
    from parity import run_gpu
    return run_gpu(s.with_(expert_dropout=0.0, jitter_eps=0.0), inp, backward=False)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_training_noise_depends_on_the_seed_only(dtype):
    from parity import run_gpu
    s = SwitchShape("t", 2000, 128, 256, 8, 1.25, dtype=dtype, seed_index=71, expert_dropout=0.3,
                    jitter_eps=0.05, noise_seed=1)
    inp = make_inputs(s, _dev())
    _, a = run_gpu(s, inp)
    _, b = run_gpu(s, inp)
    _, c = run_gpu(s.with_(noise_seed=2), inp)
    _, hi = run_gpu(s.with_(noise_seed=1 + (1 << 32)), inp)
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    for other in (c, hi):
        assert not np.array_equal(a["y"], other["y"])
        assert not np.array_equal(a["router_logits"], other["router_logits"])
    # zero rates: the seed is not looked at
    z0 = run_gpu(s.with_(expert_dropout=0.0, jitter_eps=0.0, noise_seed=0), inp)[1]
    z1 = run_gpu(s.with_(expert_dropout=0.0, jitter_eps=0.0, noise_seed=12345), inp)[1]
    for k in z0:
        assert np.array_equal(z0[k], z1[k]), k
    # dropout keeps about 1 - rate of the active hidden units: dW_out rows of dropped units
    # are zero for a token; count exact zeros of y instead -- none expected for kept tokens
    kept = a["dropped"] == 0
    assert np.all(np.abs(a["y"][kept]).sum(axis=1) > 0)


def test_training_noise_full_size_sampled():
    """Switch-Base shape with the fine-tuning expert dropout of Table 4 and jitter."""
    from parity import compare_sampled
    s = CONFIGS["base_cf1.25"].with_(expert_dropout=0.4, jitter_eps=0.01, noise_seed=20210111)
    inp = make_inputs(s, _dev())
    errs = compare_sampled(s, inp, n_experts=2, n_tokens=24)
    _report("base_cf1.25 + noise", errs)


# ------------------------------------------- gated-GELU experts (model tables, FFN_GEGLU)
@pytest.mark.parametrize("dtype,T,d,f,E,cf,n,rate,eps", [
    ("f32", 700, 96, 100, 6, 1.0, 1, 0.0, 0.0),
    ("f32", 1024, 64, 36, 8, 0.75, 4, 0.25, 0.05),
    ("bf16", 1500, 256, 520, 6, 1.25, 1, 0.0, 0.0),     # ragged tiles in every GEMM
    ("bf16", 4096, 128, 264, 16, 1.0, 2, 0.1, 0.0),
    ("bf16", 3000, 776, 128, 5, 2.0, 1, 0.0, 0.01),
    ("bf16", 600, 64, 8, 3, 1.0, 1, 0.0, 0.0),          # the narrowest hidden layer
])
def test_geglu_experts(dtype, T, d, f, E, cf, n, rate, eps):
    from parity import compare_full
    s = SwitchShape("t", T, d, f, E, cf, dtype=dtype, seed_index=80, n_groups=n, ffn="geglu",
                    expert_dropout=rate, jitter_eps=eps, noise_seed=31)
    inp = make_inputs(s, _dev())
    assert inp["W_in"].shape == (E, d, 2 * f)
    if dtype == "bf16":   # also with dispatch / combine inside the GEMMs
        errs = compare_full(s.with_(fused_dispatch=True), inp, d_aux=0.8)[0]
        _report("geglu %s f=%d, in the GEMMs" % (dtype, f), errs)
    errs, gpu, fwd, _ = compare_full(s, inp, d_aux=0.8)
    assert gpu["dW_in"].shape == (E, d, 2 * f)
    _report("geglu %s f=%d" % (dtype, f), errs)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_geglu_capacity_zero_and_empty_batch(dtype):
    from parity import run_gpu
    from paper_2101_03961_amd.layer import SwitchLayer
    s = SwitchShape("t", 64, 64, 72, 128, 1.0, dtype=dtype, seed_index=81, ffn="geglu")  # capacity 0
    inp = make_inputs(s, _dev())
    _, gpu = run_gpu(s, inp)
    assert np.all(gpu["dropped"] == 1) and np.all(gpu["y"] == 0)
    assert np.all(gpu["dW_in"] == 0) and np.all(gpu["dW_out"] == 0)
    layer = SwitchLayer(0, 64, 72, 4, 1.0, s.alpha, dtype, device=_dev(), ffn="geglu")
    e = lambda *shape: torch.empty(shape, dtype=layer.act, device=_dev())
    W_r = torch.zeros((64, 4), device=_dev())
    layer.forward(e(0, 64), W_r, e(4, 64, 144), e(4, 72, 64))
    layer.alloc_grads(with_bias=False)
    layer.dW_in.fill_(1.0)
    layer.dW_out.fill_(1.0)
    g = layer.backward(e(0, 64), e(0, 64), W_r, e(4, 64, 144), e(4, 72, 64))
    torch.cuda.synchronize()
    assert g["dW_in"].shape == (4, 64, 144) and float(g["dW_in"].float().abs().sum()) == 0.0
    assert float(g["dW_out"].float().abs().sum()) == 0.0


def test_layer_refuses_wrong_weight_shape():
    """The ReLU layout handed to a gated-GELU layer must not reach the kernels."""
    from paper_2101_03961_amd.layer import SwitchLayer
    s = SwitchShape("t", 256, 64, 72, 4, 1.0, dtype="bf16", seed_index=82)
    inp = make_inputs(s, _dev())
    layer = SwitchLayer(s.T, s.d_model, s.d_ff, s.E, 1.0, s.alpha, "bf16", device=_dev(), ffn="geglu")
    with pytest.raises(ValueError):
        layer.forward(inp["x"], inp["W_r"], inp["W_in"], inp["W_out"])


def test_geglu_switch_base_sampled():
    from parity import compare_sampled
    s = CONFIGS["base_geglu"]
    inp = make_inputs(s, _dev())
    errs = compare_sampled(s, inp, n_experts=2, n_tokens=24)
    _report("base_geglu", errs)


# ------------------------------------------- No-Token-Left-Behind (App. B)
@pytest.mark.parametrize("dtype,T,d,f,E,cf,n,bias,rounds,ffn", [
    ("f32", 700, 64, 96, 6, 1.0, 1, True, 1, "relu"),
    ("f32", 1024, 64, 40, 8, 0.75, 4, True, 3, "geglu"),
    ("bf16", 3000, 128, 264, 16, 1.0, 1, False, 1, "relu"),     # MFMA router, mild overflow
    ("bf16", 4096, 128, 264, 128, 1.0, 2, True, 2, "relu"),     # heavy skew, 128 experts
    ("bf16", 2500, 72, 64, 513, 2.0, 1, False, 2, "relu"),      # nine experts per lane, ragged
    ("f32", 600, 32, 32, 3, 1.0, 1, True, 16, "relu"),          # more rounds than experts
])
def test_no_token_left_behind(dtype, T, d, f, E, cf, n, bias, rounds, ffn):
    from parity import compare_full, run_gpu
    s = SwitchShape("t", T, d, f, E, cf, dtype=dtype, seed_index=90, n_groups=n, zipf_bias=bias,
                    ntlb_rounds=rounds, ffn=ffn)
    inp = make_inputs(s, _dev())
    if dtype == "bf16":   # also with dispatch / combine inside the GEMMs
        errs = compare_full(s.with_(fused_dispatch=True), inp, d_aux=0.7)[0]
        _report("ntlb %s E=%d rounds=%d, in the GEMMs" % (dtype, E, rounds), errs)
    errs, gpu, fwd, _ = compare_full(s, inp, d_aux=0.7)
    _, plain = run_gpu(s.with_(ntlb_rounds=0), inp, backward=False)
    rescued = int(plain["dropped"].sum()) - int(gpu["dropped"].sum())
    errs["rescued"], errs["still_dropped"] = rescued, int(gpu["dropped"].sum())
    _report("ntlb %s E=%d rounds=%d" % (dtype, E, rounds), errs)
    assert rescued > 0
    # tokens that had a slot keep it; the loss and the counts do not change
    k1 = plain["dropped"] == 0
    assert np.array_equal(plain["expert_index"][k1], gpu["expert_index"][k1])
    assert np.array_equal(plain["position_in_expert"][k1], gpu["position_in_expert"][k1])
    assert np.array_equal(plain["expert_counts"], gpu["expert_counts"])
    assert np.array_equal(plain["aux_loss"], gpu["aux_loss"])
    # no (group, expert) pair exceeds its capacity
    kept = gpu["dropped"] == 0
    key = (np.arange(T) // (T // n))[kept] * E + gpu["expert_index"][kept]
    assert np.bincount(key, minlength=n * E).max() <= fwd["capacity"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_groups_of_two_tokens(dtype):
    """The smallest routing groups: two tokens each, one slot per (group, expert); with a
    re-routing stage the second token of a pair that collides moves to the other expert."""
    from parity import compare_full
    s = SwitchShape("t", 2048, 64, 72, 2, 1.0, dtype=dtype, seed_index=91, n_groups=1024)
    inp = make_inputs(s, _dev())
    errs, gpu, fwd, _ = compare_full(s, inp, d_aux=0.6)
    assert fwd["capacity"] == 1 and 0 < gpu["dropped"].sum() < 1024
    _report("groups of two", errs)
    errs, gpu2, _, _ = compare_full(s.with_(ntlb_rounds=1), inp, d_aux=0.6)
    assert gpu2["dropped"].sum() == 0          # two tokens, two experts with one slot each
    _report("groups of two + re-routing", errs)


def test_no_token_left_behind_full_size():
    from parity import compare_sampled
    s = CONFIGS["base_cf1.0"].with_(ntlb_rounds=2)
    inp = make_inputs(s, _dev())
    errs = compare_sampled(s, inp, n_experts=2, n_tokens=24)
    _report("base_cf1.0 + 2 re-routing stages", errs)


# ------------------------------------------- full sizes
# The metric's own workload (Switch-Base, capacity factor 1.0: 65 536 tokens, 128 experts)
# against the complete fp64 oracle, forward and backward: every row of y and dx, every expert's
# weight gradients, the router's.  The oracle takes the experts sixteen at a time (the GEMMs'
# eight tile ranges); each range is a test of its own, so that the run reports every twenty
# seconds instead of staying silent for minutes, and the router's gradients, which need every
# range, come last.
_BASE_FULL = {}


def _base_full():
    from parity import FullByExperts
    if "run" not in _BASE_FULL:
        s = CONFIGS["base_cf1.0"]
        _BASE_FULL["run"] = FullByExperts(s, make_inputs(s, _dev()), n_chunks=8, d_aux=1.0)
    return _BASE_FULL["run"]


@pytest.mark.parametrize("c", range(8))
def test_switch_base_full_oracle_parity_experts(c):
    run = _base_full()
    print("\n" + run.chunk(c), flush=True)
    assert run.fwd["capacity"] == 512 and int(run.fwd["dropped"].sum()) > 0


def test_switch_base_full_oracle_parity_router():
    run = _base_full()
    if len(run.done) < run.n_chunks:
        pytest.skip("needs every expert range of test_switch_base_full_oracle_parity_experts")
    errs = run.router()
    _BASE_FULL.clear()          # the tensors are large
    _report("base_cf1.0, full oracle", errs)


@pytest.mark.parametrize("name,n_experts", [
    ("base_cf1.25", 18), ("base_zipf", 18), ("large", 12), ("c_share", 6), ("base_e256", 12),
])
def test_full_size_sampled_parity(name, n_experts):
    """The other full-size workloads: all outputs finite, routing on every token, and the
    experts at the edges of the GEMMs' tile ranges (plus the fullest and the emptiest) against
    the oracle."""
    from parity import compare_sampled
    s = CONFIGS[name]
    inp = make_inputs(s, _dev())
    errs = compare_sampled(s, inp, n_experts=n_experts, n_tokens=24)
    _report(name, errs)


@pytest.mark.parametrize("name,n_experts", [("base_cf1.0", 18), ("base_cf1.25", 10)])
def test_full_size_sampled_parity_inside_the_gemms(name, n_experts):
    """The full-size workloads with dispatch and combine inside the GEMMs (gathered operand
    loads, scattered output rows, at 3072+ tiles per launch): same checks as above."""
    from parity import compare_sampled
    s = CONFIGS[name].with_(fused_dispatch=True)
    inp = make_inputs(s, _dev())
    errs = compare_sampled(s, inp, n_experts=n_experts, n_tokens=24)
    _report(name + ", in the GEMMs", errs)


def test_xxl_sampled_parity():
    """Largest shape: the first, the last, the fullest and the emptiest expert plus single
    tokens; the fp64 oracle needs about 0.5 GFLOP per token here."""
    from parity import compare_sampled
    s = CONFIGS["xxl"]
    inp = make_inputs(s, _dev())
    errs = compare_sampled(s, inp, n_experts=4, n_tokens=16)
    _report("xxl", errs)
