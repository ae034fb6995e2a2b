"""GPU parity, second part: every kernel variant on the shapes it is timed on, every row of the prefill
configuration, guard bands around everything a call writes, and a seeded sweep over random shapes.

All comparisons are element by element against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import mdbf_oracle as orc
from paper_2512_24545_amd import synth

pytestmark = pytest.mark.gpu

TOL = 2e-3
TOL_PRECISE = 2e-5


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2512_24545_amd import binding as mb
    mb.lib()
    return torch, mb


def _oracle_args(L):
    return (L["SA"], L["SB"], L["A"], L["Q"], L["G"], L["B"])


def _to_dev(torch, X, dtype="f16"):
    t = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}[dtype]
    return torch.from_numpy(np.ascontiguousarray(X)).to("cuda:0").to(t).contiguous()


# ---------------------------------------------------------------- the block-scaled kernel where it is timed
@pytest.mark.parametrize("which", ["gate", "down"])
@pytest.mark.parametrize("T", [1, 16])
def test_block_scaled_mlp_projections(gpu, which, T):
    """11008 x 4096 and 4096 x 11008 with k = 4096 (32 and 86 contraction blocks, 256 and 688 row tiles):
    the shapes of the bench's MLP plan, forced onto the block-scaled kernel as single calls."""
    torch, mb = gpu
    L, X = synth.config_mlp_decode(which, T=T)
    ref = orc.forward_factored(*_oracle_args(L), X)
    Y = mb.mdbf_forward(mb.DeviceLayer.from_host(L), _to_dev(torch, X), y_dtype="f32", block_scaled=True)
    torch.cuda.synchronize()
    assert orc.max_rel_error(Y.cpu().numpy(), ref) <= TOL


@pytest.mark.parametrize("budget", ["1.0", "1.5", "2.0"])
@pytest.mark.parametrize("mat", [0, 4, 6])
def test_block_scaled_stack_matrices(gpu, budget, mat):
    """q, gate and down of the decoder stack at every budget (k = 1856 / 2816 with rank 8, 2656 / 4096 and
    3616 / 5536 with rank 16; the down projection contracts 86 blocks in factor 1 and 22, 32 or 44 in factor
    2) through the block-scaled kernel, one token."""
    torch, mb = gpu
    L, X = synth.stack_matrix(budget, 3, mat, T=1)
    ref = orc.forward_factored(*_oracle_args(L), X)
    Y = mb.mdbf_forward(mb.DeviceLayer.from_host(L), _to_dev(torch, X), y_dtype="f32", block_scaled=True)
    torch.cuda.synchronize()
    assert orc.max_rel_error(Y.cpu().numpy(), ref) <= TOL


def test_auto_selected_block_scaled_plan_of_mlp_projections(gpu):
    """A plan large enough for the library to pick the block-scaled kernel by itself (64 MLP projections:
    16 384 and more row tiles per factor), as the bench's MLP plan does: eight distinct layers, each listed
    eight times with its own activations; every output of every entry is compared with the oracle."""
    torch, mb = gpu
    hosts, devs = [], []
    for i in range(8):
        m, n = ((11008, 4096), (11008, 4096), (4096, 11008))[i % 3]
        L = synth.make_layer(m, n, 4096, 16, seed=6100 + i, env_dtype="f16", env_kind="llama", signed_env=(i % 2 == 1))
        hosts.append(L)
        devs.append(mb.DeviceLayer.from_host(L))
    layers, Xs, Ys, Xh, which = [], [], [], [], []
    for rep in range(8):
        for i in range(8):
            X = synth.make_activations(hosts[i]["n"], 1, seed=6200 + 8 * rep + i, x_dtype="f16")
            layers.append(devs[i])
            Xs.append(_to_dev(torch, X))
            Ys.append(torch.zeros((1, hosts[i]["m"]), dtype=torch.float16, device="cuda:0"))
            Xh.append(X)
            which.append(i)
    plan = mb.BatchPlan(layers, Xs, Ys)
    assert plan.kernel(1) == "stage_mx_kernel" and plan.kernel(2) == "stage_mx_kernel"
    plan.run()
    torch.cuda.synchronize()
    for i in range(8):
        idx = [j for j in range(64) if which[j] == i]
        ref = orc.forward_factored(*_oracle_args(hosts[i]), np.concatenate([Xh[j] for j in idx]))
        got = np.concatenate([Ys[j].float().cpu().numpy() for j in idx])
        assert orc.max_rel_error(got, ref) <= TOL + 2.0 ** -11   # fp16 outputs, as in the bench


def test_small_plans_report_the_fp16_kernel(gpu):
    """Seven stack matrices are too few row tiles for the block-scaled kernel: the plan says which kernel it
    runs, and MDBF_FLAG_FP16_STAGED keeps a large plan off the block-scaled kernel as well."""
    torch, mb = gpu
    L = synth.make_layer(530, 2104, 1104, 16, seed=77, env_dtype="f16", env_kind="llama")
    dl = mb.DeviceLayer.from_host(L)
    X = _to_dev(torch, synth.make_activations(2104, 1, seed=78))
    Y = torch.zeros((1, 530), dtype=torch.float32, device="cuda:0")
    small = mb.BatchPlan([dl] * 3, [X] * 3, [Y] * 3)
    assert small.kernel(1) == "stage_fast_kernel" and small.kernel(2) == "stage_fast_kernel"
    forced = mb.BatchPlan([dl] * 3, [X] * 3, [Y] * 3, block_scaled=True)
    assert forced.kernel(1) == "stage_mx_kernel"
    ref = orc.forward_factored(*_oracle_args(L), synth.make_activations(2104, 1, seed=78))
    Ya = mb.mdbf_forward(dl, X, y_dtype="f32", fp16_staged=True)
    torch.cuda.synchronize()
    assert orc.max_rel_error(Ya.cpu().numpy(), ref) <= TOL


# ---------------------------------------------------------------- prefill: every row
@pytest.mark.parametrize("x_dtype", ["f16", "bf16"])
def test_prefill_every_token_against_the_dense_oracle(gpu, x_dtype):
    """4096 x 4096, k = 2656, l = 16, 2048 tokens: What is reconstructed once (Eq. "me-dbf-basis") and all
    2048 x 4096 outputs are compared, so every token-slab position of both kernel instantiations is covered.
    The factored oracle confirms the dense one on a strided sample of rows."""
    torch, mb = gpu
    L, X = synth.config_prefill(T=2048, x_dtype=x_dtype)
    ref = orc.forward_dense(*_oracle_args(L), X)
    rows = list(range(0, 2048, 171))
    np.testing.assert_allclose(orc.forward_factored(*_oracle_args(L), X[rows]), ref[rows], rtol=1e-9, atol=1e-6)
    Y = mb.mdbf_forward(mb.DeviceLayer.from_host(L), _to_dev(torch, X, x_dtype), y_dtype="f32")
    torch.cuda.synchronize()
    Yh = Y.cpu().numpy().astype(np.float64)
    assert orc.max_rel_error(Yh, ref) <= TOL
    # per token as well: no row may hide behind the largest one
    per_row = np.abs(Yh - ref).max(axis=1) / np.abs(ref).max(axis=1)
    assert per_row.max() <= TOL, int(per_row.argmax())


# ---------------------------------------------------------------- guard bands
GUARD = 4096          # bytes of sentinel on each side
SENTINELS = (0x00, 0xFF)


def _embedded(torch, src, fill):
    """A copy of the flat uint8 view of `src` inside a larger buffer filled with `fill`; returns (view, whole)."""
    raw = src.contiguous().view(torch.uint8).reshape(-1)
    whole = torch.full((raw.numel() + 2 * GUARD,), fill, dtype=torch.uint8, device=src.device)
    whole[GUARD:GUARD + raw.numel()] = raw
    view = whole[GUARD:GUARD + raw.numel()].view(src.dtype).reshape(src.shape)
    return view, whole


def _margins_intact(whole, nbytes, fill):
    w = whole.cpu().numpy()
    return bool((w[:GUARD] == fill).all() and (w[GUARD + nbytes:] == fill).all())


GUARD_CASES = [
    # m, n, k, l, T, variant
    (530, 2104, 1104, 16, 1, "auto"),
    (530, 2104, 1104, 16, 1, "block_scaled"),
    (1037, 1030, 2105, 16, 3, "block_scaled"),
    (100, 1030, 200, 8, 2, "block_scaled"),
    (77, 300, 70, 5, 1, "auto"),
    (130, 129, 257, 3, 3, "auto"),
    (300, 1160, 648, 16, 7, "auto"),
    (530, 2100, 1100, 16, 40, "auto"),
    (96, 200, 150, 5, 2, "precise"),
    (4096, 4096, 2656, 16, 1, "block_scaled"),
]


@pytest.mark.parametrize("m,n,k,l,T,variant", GUARD_CASES)
def test_nothing_is_written_outside_the_outputs(gpu, m, n, k, l, T, variant):
    """Y and the workspace sit inside larger buffers filled with a sentinel, the inputs (packed signs, envelope
    factors, activations) likewise: after the call the margins of Y and of the workspace are untouched, and
    the result does not depend on what surrounds the inputs (the kernels over-read on purpose: clamped
    addresses, tiles past an item's end) -- two runs with different sentinels agree bit for bit and with the
    oracle."""
    torch, mb = gpu
    L = synth.make_layer(m, n, k, l, seed=m + n + k + l, env_dtype="f16", env_kind="llama", signed_env=True)
    X = synth.make_activations(n, T, seed=5 + T, x_dtype="f16")
    ref = orc.forward_factored(*_oracle_args(L), X)
    base = mb.DeviceLayer.from_host(L)
    kw = dict(precise=(variant == "precise"), block_scaled=(variant == "block_scaled"))
    results = []
    for fill in SENTINELS:
        parts = [_embedded(torch, t, fill) for t in (base.SA_packed, base.SB_packed, base.A, base.Q, base.G, base.B)]
        dl = mb.DeviceLayer(m, n, k, l, *[p[0] for p in parts])
        Xd, _ = _embedded(torch, _to_dev(torch, X), fill)
        d = dl.desc("f16", "f32", **kw)
        ws_bytes = mb.mdbf_workspace_bytes(d, T)
        ws_whole = torch.full((ws_bytes + 2 * GUARD,), fill, dtype=torch.uint8, device="cuda:0")
        Y_whole = torch.full((T * m * 4 + 2 * GUARD,), fill, dtype=torch.uint8, device="cuda:0")
        Y = Y_whole[GUARD:GUARD + T * m * 4].view(torch.float32).reshape(T, m)
        mb.mdbf_forward(dl, Xd, y_dtype="f32", Y=Y, workspace=ws_whole[GUARD:GUARD + ws_bytes], **kw)
        torch.cuda.synchronize()
        assert _margins_intact(Y_whole, T * m * 4, fill), "Y margins"
        assert _margins_intact(ws_whole, ws_bytes, fill), "workspace margins"
        results.append(Y.clone())
    assert torch.equal(results[0], results[1])
    assert orc.max_rel_error(results[0].cpu().numpy(), ref) <= (TOL_PRECISE if variant == "precise" else TOL)


@pytest.mark.parametrize("block_scaled,T", [(True, 1), (False, 1), (False, 6)])
def test_plans_write_nothing_outside_their_outputs(gpu, block_scaled, T):
    """The same for a plan of ragged layers: each Y with a leading dimension larger than m inside a
    sentinel-filled buffer, the plan's workspace inside another; gaps and margins stay untouched."""
    torch, mb = gpu
    fill = 0xA5
    specs = [(530, 2104, 1104), (37, 300, 2105), (1037, 1030, 130), (272, 1032, 4096)]
    layers, Xs, Ys, wholes, refs = [], [], [], [], []
    for i, (m, n, k) in enumerate(specs):
        L = synth.make_layer(m, n, k, 16, seed=8100 + i, env_dtype="f16", env_kind="llama", signed_env=True)
        X = synth.make_activations(n, T, seed=8200 + i, x_dtype="f16")
        layers.append(mb.DeviceLayer.from_host(L))
        Xs.append(_to_dev(torch, X))
        ld = m + 24
        whole = torch.full((GUARD // 4 + T * ld + GUARD // 4,), 0, dtype=torch.float32, device="cuda:0")
        whole.view(torch.uint8).fill_(fill)
        wholes.append(whole)
        Ys.append(whole[GUARD // 4:GUARD // 4 + T * ld].view(T, ld)[:, :m])
        refs.append(orc.forward_factored(*_oracle_args(L), X))
    ws_bytes = mb.BatchPlan(layers, Xs, Ys, block_scaled=block_scaled).workspace_bytes
    ws_whole = torch.full((ws_bytes + 2 * GUARD,), fill, dtype=torch.uint8, device="cuda:0")
    plan = mb.BatchPlan(layers, Xs, Ys, block_scaled=block_scaled, workspace=ws_whole[GUARD:GUARD + ws_bytes])
    plan.run()
    torch.cuda.synchronize()
    assert _margins_intact(ws_whole, ws_bytes, fill)
    for (m, n, k), whole, Y, ref in zip(specs, wholes, Ys, refs):
        assert orc.max_rel_error(Y.cpu().numpy(), ref) <= TOL
        w = whole.cpu().numpy().view(np.uint8).reshape(-1)
        ld = m + 24
        body = w[GUARD:GUARD + T * ld * 4].reshape(T, ld * 4)
        assert (w[:GUARD] == fill).all() and (w[GUARD + T * ld * 4:] == fill).all()
        assert (body[:, m * 4:] == fill).all(), "gap between rows"


# ---------------------------------------------------------------- seeded sweep over random shapes
def _sweep_cases():
    rng = np.random.default_rng(20251224)
    cases = []
    ranks = [1, 2, 3, 4, 8, 16]
    tokens = [1, 2, 5, 16, 17]
    for i in range(96):
        l = ranks[i % 6]
        T = tokens[(i // 6) % 5]
        big = i % 4 == 0
        m = int(rng.integers(1, 1500 if big else 300))
        n = int(rng.integers(1, 2600 if big else 700))
        k = int(rng.integers(1, 2300 if big else 500))
        if i % 7 == 0:
            n += (-n) % 128 + int(rng.choice([1, 7, 9, 127]))     # one past / short of a block boundary
        if i % 5 == 0:
            k += (-k) % 8 + int(rng.choice([1, 3, 5]))            # not a multiple of 8
        env_dtype = ("f16", "f16", "f16", "bf16", "f32")[i % 5]
        x_dtype = ("f16", "f16", "bf16", "f32")[i % 4]
        cases.append((m, n, k, l, T, env_dtype, x_dtype))
    return cases


def test_random_shape_sweep(gpu):
    """96 seeded shapes: every envelope rank in {1, 2, 3, 4, 8, 16}, token counts {1, 2, 5, 16, 17}, contraction
    lengths off the 8- and 128-column boundaries, all input types; each through the library's own choice of
    kernel, through the block-scaled kernel where it applies, and every sixth through the fp32 path.  Stops
    at the first failure and names the case."""
    torch, mb = gpu
    worst = 0.0
    for idx, (m, n, k, l, T, env_dtype, x_dtype) in enumerate(_sweep_cases()):
        L = synth.make_layer(m, n, k, l, seed=40000 + idx, env_dtype=env_dtype, env_kind="llama", signed_env=True)
        X = synth.make_activations(n, T, seed=50000 + idx, x_dtype=x_dtype)
        ref = orc.forward_factored(*_oracle_args(L), X)
        dl = mb.DeviceLayer.from_host(L)
        Xd = _to_dev(torch, X, x_dtype)
        variants = [("auto", {})]
        if l in (8, 16) and env_dtype == "f16" and T <= 16 and n > 128 and k > 128:
            variants.append(("block_scaled", dict(block_scaled=True)))
        if idx % 6 == 0:
            variants.append(("precise", dict(precise=True)))
        for name, kw in variants:
            Y = mb.mdbf_forward(dl, Xd, y_dtype="f32", **kw)
            torch.cuda.synchronize()
            err = orc.max_rel_error(Y.cpu().numpy(), ref)
            worst = max(worst, err if name != "precise" else 0.0)
            assert err <= (TOL_PRECISE if name == "precise" else TOL), (idx, name, (m, n, k, l, T, env_dtype, x_dtype), err)
    assert worst > 0.0


def test_plan_whose_last_round_is_cut_into_pieces(gpu):
    """160 equal layers with 128 row tiles each: 320 work items in the second factor = 1.25 rounds of 256
    workgroups, so the 64 items of the last round are cut into 16-tile pieces (one per workgroup).  Every
    output of every layer is compared with the oracle."""
    torch, mb = gpu
    layers, Xs, Ys, refs = [], [], [], []
    for i in range(160):
        L = synth.make_layer(2048, 384, 256, 16, seed=9100 + i, env_dtype="f16", env_kind="llama", signed_env=True)
        X = synth.make_activations(384, 1, seed=9300 + i, x_dtype="f16")
        layers.append(mb.DeviceLayer.from_host(L))
        Xs.append(_to_dev(torch, X))
        Ys.append(torch.zeros((1, 2048), dtype=torch.float32, device="cuda:0"))
        refs.append(orc.forward_factored(*_oracle_args(L), X))
    plan = mb.BatchPlan(layers, Xs, Ys, block_scaled=True)
    assert plan.kernel(2) == "stage_mx_kernel"
    for _ in range(2):
        plan.run()
    torch.cuda.synchronize()
    for Yb, ref in zip(Ys, refs):
        assert orc.max_rel_error(Yb.cpu().numpy(), ref) <= TOL


def test_plan_whose_first_factor_is_cut_into_pieces_and_writes_the_next_records(gpu):
    """320 equal layers with 64 row tiles in the first factor: 320 work items = 1.25 rounds of 256 workgroups, so the
    last round's items are cut into 16-tile pieces, each of which writes the two 128-column blocks of the second
    factor's activation records that its rows make up (three launches per run).  Every output against the oracle."""
    torch, mb = gpu
    layers, Xs, Ys, refs = [], [], [], []
    for i in range(320):
        L = synth.make_layer(256, 384, 1024, 16, seed=9500 + i, env_dtype="f16", env_kind="llama", signed_env=True)
        X = synth.make_activations(384, 1, seed=9900 + i, x_dtype="f16")
        layers.append(mb.DeviceLayer.from_host(L))
        Xs.append(_to_dev(torch, X))
        Ys.append(torch.zeros((1, 256), dtype=torch.float32, device="cuda:0"))
        refs.append(orc.forward_factored(*_oracle_args(L), X))
    plan = mb.BatchPlan(layers, Xs, Ys, block_scaled=True)
    assert plan.kernel(1) == "stage_mx_kernel" and plan.kernel(2) == "stage_mx_kernel" and plan.launches() == 3
    for _ in range(2):
        plan.run()
    torch.cuda.synchronize()
    for Yb, ref in zip(Ys, refs):
        assert orc.max_rel_error(Yb.cpu().numpy(), ref) <= TOL
