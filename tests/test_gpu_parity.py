"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Gates: sign pack/unpack bit-exact; y within max|Y-Y*|/max|Y*| <= 2e-3 (fp16 staging, fp32
accumulation); the fp32 ("precise") path within 2e-5; exact-integer inputs bit-for-bit."""
import numpy as np
import pytest

from oracle import mdbf_oracle as orc
from paper_2512_24545_amd import synth
from helpers import concat_terms

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


def _to_dev(torch, X, dtype):
    t = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}[dtype]
    return torch.from_numpy(np.ascontiguousarray(X)).to("cuda:0").to(t).contiguous()


def _run(gpu, L, X, x_dtype, y_dtype="f32", precise=False, block_scaled=False):
    torch, mb = gpu
    dl = mb.DeviceLayer.from_host(L)
    Xd = _to_dev(torch, X, x_dtype)
    Y = mb.mdbf_forward(dl, Xd, y_dtype=y_dtype, precise=precise, block_scaled=block_scaled)
    torch.cuda.synchronize()
    return Y.float().cpu().numpy().astype(np.float64)


# ---------------------------------------------------------------- pack / unpack
@pytest.mark.parametrize("rows,cols", [(1, 1), (16, 128), (17, 129), (5, 31), (33, 500), (100, 1000),
                                       (256, 128), (2656, 4096), (4096, 2656)])
def test_pack_unpack_bit_exact(gpu, rows, cols):
    torch, mb = gpu
    rng = np.random.default_rng(rows * 7919 + cols)
    S = synth.random_signs(rng, rows, cols)
    Sd = torch.from_numpy(S).to("cuda:0")
    packed = mb.mdbf_pack(Sd)
    assert packed.numel() == mb.mdbf_packed_bytes(rows, cols)
    back = mb.mdbf_unpack(packed, rows, cols).cpu().numpy()
    np.testing.assert_array_equal(back, S)
    # the logical bits agree with the oracle's reference packing of the same matrix
    np.testing.assert_array_equal(orc.unpack_ref(orc.pack_ref(S), cols), back)
    # one bit per entry, padding bits are zero: population count equals the number of -1 entries
    pc = int(np.unpackbits(packed.cpu().numpy()).sum())
    assert pc == int((S < 0).sum())


def test_pack_zero_is_plus_and_strided_input(gpu):
    torch, mb = gpu
    rng = np.random.default_rng(5)
    big = rng.integers(-3, 4, size=(40, 300)).astype(np.int8)   # includes zeros and |v| > 1
    view = torch.from_numpy(big).to("cuda:0")[:, 10:210]          # leading dimension 300 > cols 200
    packed = mb.mdbf_pack(view)
    back = mb.mdbf_unpack(packed, 40, 200).cpu().numpy()
    np.testing.assert_array_equal(back, orc.sign_pm1(big[:, 10:210]))


# ---------------------------------------------------------------- forward: small and ragged
SMALL = [
    # m, n, k, l, T
    (16, 128, 16, 16, 1),
    (256, 256, 128, 4, 1),
    (40, 300, 70, 16, 2),
    (130, 129, 257, 3, 3),
    (1, 1, 1, 1, 1),
    (100, 1030, 200, 8, 1),
    (530, 2100, 1100, 16, 2),
    (77, 64, 2656, 2, 1),
]


@pytest.mark.parametrize("nbytes,waves", [(16, 4), (16 * 1000, 4), (16 * 65537, 64), (1 << 22, 8192), ((1 << 22) + 48, 1028)])
def test_stream_read_folds_every_word_once(gpu, nbytes, waves):
    """The bandwidth yardstick reads every 16-byte element exactly once: the XOR of its per-wave words equals
    the XOR of all 32-bit words of the buffer, for sizes below, equal to and far above one trip of the launch."""
    torch, mb = gpu
    rng = np.random.default_rng(nbytes % 1000 + waves)
    host = rng.integers(0, 2 ** 32, size=nbytes // 4, dtype=np.uint32)
    src = torch.from_numpy(host.view(np.int32)).to("cuda:0")
    sink = torch.full((waves,), 0x5A5A5A5A, dtype=torch.int32, device="cuda:0")
    mb.mdbf_stream_read(src, sink)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
    assert got == np.bitwise_xor.reduce(host)


@pytest.mark.parametrize("m,n,k,l,T", SMALL)
@pytest.mark.parametrize("precise", [False, True])
def test_forward_small_shapes(gpu, m, n, k, l, T, precise):
    L = synth.make_layer(m, n, k, l, seed=m + 3 * n + 5 * k + l, env_dtype="f16", env_kind="unit", signed_env=True)
    X = synth.make_activations(n, T, seed=99 + m, x_dtype="f16")
    ref = orc.forward_factored(*_oracle_args(L), X)
    got = _run(gpu, L, X, "f16", "f32", precise)
    err = orc.max_rel_error(got, ref)
    assert err <= (TOL_PRECISE if precise else TOL), err


@pytest.mark.parametrize("env_dtype,x_dtype,y_dtype", [("f32", "f32", "f32"), ("bf16", "bf16", "f32"),
                                                         ("f16", "f16", "f16"), ("f16", "bf16", "bf16"),
                                                         ("f32", "f16", "f32")])
def test_forward_dtypes(gpu, env_dtype, x_dtype, y_dtype):
    L = synth.make_layer(96, 200, 150, 5, seed=17, env_dtype=env_dtype, env_kind="llama", signed_env=True)
    X = synth.make_activations(200, 2, seed=18, x_dtype=x_dtype)
    ref = orc.forward_factored(*_oracle_args(L), X)
    got = _run(gpu, L, X, x_dtype, y_dtype)
    # a 16-bit output adds its own rounding: half an ulp of the largest element
    slack = {"f32": 0.0, "f16": 2.0 ** -11, "bf16": 2.0 ** -8}[y_dtype]
    assert orc.max_rel_error(got, ref) <= TOL + slack


def test_toy_config(gpu):
    """256x256, k=128, l=4, fp32 envelopes and activations."""
    L, X = synth.config_toy()
    ref = orc.forward_dense(*_oracle_args(L), X)
    np.testing.assert_allclose(orc.forward_factored(*_oracle_args(L), X), ref, rtol=1e-10, atol=1e-9)
    for precise, tol in ((False, TOL), (True, TOL_PRECISE)):
        got = _run(gpu, L, X, "f32", "f32", precise)
        assert orc.max_rel_error(got, ref) <= tol


# ---------------------------------------------------------------- exact-integer inputs: zero tolerance
@pytest.mark.parametrize("m,n,k,l", [(64, 256, 96, 4), (530, 2100, 1100, 16), (4096, 4096, 2656, 4)])
def test_exact_integer_inputs_bit_for_bit(gpu, m, n, k, l):
    """All-ones envelopes and x in {-1,0,1}: every intermediate is an integer that fp16 staging and
    fp32 accumulation represent exactly, so the result must equal the oracle in any summation order."""
    L = synth.make_layer(m, n, k, l, seed=31 + m, env_dtype="f16", env_kind="ones")
    X = synth.make_activations(n, 1, seed=32, x_dtype="f16", kind="ternary")
    ref = orc.forward_factored(*_oracle_args(L), X)
    assert np.max(np.abs(ref)) < 2 ** 24
    got = _run(gpu, L, X, "f16", "f32")
    np.testing.assert_array_equal(got, ref)


# ---------------------------------------------------------------- the block-scaled variant, forced
# (without the flag the library takes it only for launches that fill the device: the bench-sized plans)
BLOCK_SCALED = [
    # m, n, k, T: ragged K, one or many stages, partial tile groups, several items per matrix
    (16, 128, 16, 1),
    (40, 300, 70, 2),
    (530, 2100, 1100, 3),
    (1100, 1030, 2105, 1),
    (2064, 520, 4100, 16),
    (4096, 4096, 2656, 1),
]


@pytest.mark.parametrize("m,n,k,T", BLOCK_SCALED)
def test_block_scaled_shapes(gpu, m, n, k, T):
    L = synth.make_layer(m, n, k, 16, seed=m + 3 * n + 5 * k, env_dtype="f16", env_kind="unit", signed_env=True)
    X = synth.make_activations(n, T, seed=77 + m, x_dtype="f16")
    ref = orc.forward_factored(*_oracle_args(L), X)
    got = _run(gpu, L, X, "f16", "f32", block_scaled=True)
    assert orc.max_rel_error(got, ref) <= TOL


@pytest.mark.parametrize("m,n,k,T", [(40, 300, 70, 2), (1100, 1030, 2105, 1), (4096, 4096, 1856, 1), (2064, 520, 4100, 16)])
def test_block_scaled_rank_8(gpu, m, n, k, T):
    """Rank-8 envelopes (the 1.0 bits-per-weight budget) through the block-scaled kernel: the 16-wide
    matrix-core tile carries two limbs of every mode side by side."""
    L = synth.make_layer(m, n, k, 8, seed=m + 3 * n + 5 * k + 8, env_dtype="f16", env_kind="unit", signed_env=True)
    X = synth.make_activations(n, T, seed=78 + m, x_dtype="f16")
    ref = orc.forward_factored(*_oracle_args(L), X)
    got = _run(gpu, L, X, "f16", "f32", block_scaled=True)
    assert orc.max_rel_error(got, ref) <= TOL


@pytest.mark.parametrize("x_dtype,y_dtype", [("bf16", "bf16"), ("f32", "f32"), ("f16", "f16")])
def test_block_scaled_dtypes(gpu, x_dtype, y_dtype):
    L = synth.make_layer(300, 700, 450, 16, seed=23, env_dtype="f16", env_kind="llama", signed_env=True)
    X = synth.make_activations(700, 2, seed=24, x_dtype=x_dtype)
    ref = orc.forward_factored(*_oracle_args(L), X)
    got = _run(gpu, L, X, x_dtype, y_dtype, block_scaled=True)
    slack = {"f32": 0.0, "f16": 2.0 ** -11, "bf16": 2.0 ** -8}[y_dtype]
    assert orc.max_rel_error(got, ref) <= TOL + slack


@pytest.mark.parametrize("m,n,k", [(64, 256, 96), (530, 2100, 1100), (4096, 4096, 2656)])
def test_block_scaled_exact_integer_inputs(gpu, m, n, k):
    """All-ones envelopes (l = 16) and x in {-1,0,1}: the scaled activations are small integers times a
    power of two, which three fp6 limbs under a shared exponent hold exactly; fp32 accumulation is exact
    below 2^24.  The result must equal the oracle bit for bit."""
    L = synth.make_layer(m, n, k, 16, seed=41 + m, env_dtype="f16", env_kind="ones")
    X = synth.make_activations(n, 1, seed=42, x_dtype="f16", kind="ternary")
    ref = orc.forward_factored(*_oracle_args(L), X)
    assert np.max(np.abs(ref)) < 2 ** 24
    got = _run(gpu, L, X, "f16", "f32", block_scaled=True)
    np.testing.assert_array_equal(got, ref)


def test_block_scaled_batch_equals_single_calls(gpu):
    torch, mb = gpu
    specs = [(530, 2104, 1104, 2), (4096, 4096, 2656, 1), (272, 1032, 4096, 16), (1100, 1030, 2105, 1)]
    layers, Xs, Ys, refs, singles = [], [], [], [], []
    for i, (m, n, k, T) in enumerate(specs):
        L = synth.make_layer(m, n, k, 16, seed=300 + i, env_dtype="f16", env_kind="llama", signed_env=True)
        X = synth.make_activations(n, T, seed=400 + i, x_dtype="f16")
        dl = mb.DeviceLayer.from_host(L)
        Xd = _to_dev(torch, X, "f16")
        layers.append(dl)
        Xs.append(Xd)
        Ys.append(torch.zeros((T, m), dtype=torch.float32, device="cuda:0"))
        refs.append(orc.forward_factored(*_oracle_args(L), X))
        singles.append(mb.mdbf_forward(dl, Xd, y_dtype="f32", block_scaled=True))
    plan = mb.BatchPlan(layers, Xs, Ys, block_scaled=True)
    plan.run()
    torch.cuda.synchronize()
    for (m, n, k, T), Yb, Y1, ref in zip(specs, Ys, singles, refs):
        assert orc.max_rel_error(Yb.cpu().numpy(), ref) <= TOL
        if T == 1:
            # a single call with one token splits the contraction across workgroups: fp32 partial sums added
            # in another (fixed) order, so z differs in its last bits and a few of its limbs round the other way
            assert orc.max_rel_error(Yb.cpu().numpy(), Y1.cpu().numpy().astype(np.float64)) <= 5e-4
        else:
            assert torch.equal(Yb, Y1)


# ---------------------------------------------------------------- LLaMA-7B shaped layers
def test_attention_projection_decode(gpu):
    """4096x4096, k=2656, l=16, one fp16 token (about 1.5 bits per weight)."""
    L, X = synth.config_attn_decode()
    ref = orc.forward_factored(*_oracle_args(L), X)
    got = _run(gpu, L, X, "f16", "f32")
    assert orc.max_rel_error(got, ref) <= TOL
    got16 = _run(gpu, L, X, "f16", "f16")
    assert orc.max_rel_error(got16, ref) <= TOL + 2.0 ** -11


@pytest.mark.parametrize("which", ["gate", "down"])
@pytest.mark.parametrize("T", [1, 16])
def test_mlp_projections_decode(gpu, which, T):
    L, X = synth.config_mlp_decode(which, T=T)
    ref = orc.forward_factored(*_oracle_args(L), X)
    got = _run(gpu, L, X, "f16", "f32")
    assert orc.max_rel_error(got, ref) <= TOL


def test_determinism(gpu):
    torch, mb = gpu
    L, X = synth.config_attn_decode(seed=7, T=2)
    dl = mb.DeviceLayer.from_host(L)
    Xd = _to_dev(torch, X, "f16")
    Y1 = mb.mdbf_forward(dl, Xd).clone()
    Y2 = mb.mdbf_forward(dl, Xd)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)


def test_determinism_of_the_split_contraction(gpu):
    """One token: the contraction of each factor is split across workgroups and the partial sums are added in a
    fixed order (by the reader for the first factor, by the last workgroup to finish for the second), so
    repeated calls give the same bits, whichever workgroup finishes last."""
    torch, mb = gpu
    for seed, (m, n, k, l) in enumerate([(4096, 4096, 2656, 16), (1100, 1030, 2105, 16), (530, 2104, 1104, 8)]):
        L = synth.make_layer(m, n, k, l, seed=70 + seed, env_dtype="f16", env_kind="llama", signed_env=True)
        X = synth.make_activations(n, 1, seed=80 + seed, x_dtype="f16")
        dl = mb.DeviceLayer.from_host(L)
        Xd = _to_dev(torch, X, "f16")
        first = mb.mdbf_forward(dl, Xd, y_dtype="f32").clone()
        for _ in range(20):
            again = mb.mdbf_forward(dl, Xd, y_dtype="f32")
            assert torch.equal(first, again)
        ref = orc.forward_factored(*_oracle_args(L), X)
        assert orc.max_rel_error(first.cpu().numpy(), ref) <= TOL


# ---------------------------------------------------------------- many layers in one launch pair
def _batch_case(gpu, specs, tokens=lambda i: 1 + (i % 2)):
    torch, mb = gpu
    layers, Xs, Ys, singles, refs = [], [], [], [], []
    for i, (m, n, k, l) in enumerate(specs):
        L = synth.make_layer(m, n, k, l, seed=400 + i, env_dtype="f16", env_kind="llama")
        X = synth.make_activations(n, tokens(i), seed=500 + i, x_dtype="f16")
        dl = mb.DeviceLayer.from_host(L)
        Xd = _to_dev(torch, X, "f16")
        layers.append(dl)
        Xs.append(Xd)
        Ys.append(torch.zeros((Xd.shape[0], m), dtype=torch.float32, device="cuda:0"))
        singles.append(mb.mdbf_forward(dl, Xd))
        refs.append(orc.forward_factored(*_oracle_args(L), X))
    plan = mb.BatchPlan(layers, Xs, Ys)
    plan.run()
    torch.cuda.synchronize()
    return Ys, singles, refs


def test_batch_mixed_layers(gpu):
    """Layers of different shapes and envelope ranks in one plan (served by the general kernel)."""
    specs = [(256, 256, 128, 4), (530, 2100, 1100, 16), (100, 1030, 200, 8), (4096, 4096, 2656, 16)]
    Ys, singles, refs = _batch_case(gpu, specs)
    for Yb, Y1, ref in zip(Ys, singles, refs):
        assert orc.max_rel_error(Yb.cpu().numpy(), ref) <= TOL
        assert orc.max_rel_error(Y1.cpu().numpy(), ref) <= TOL
        # the kernel variants quantise the staged activations differently (fp16 vs three fp6 limbs)
        assert orc.max_rel_error(Yb.cpu().numpy(), Y1.cpu().numpy().astype(np.float64)) <= 5e-4


def test_batch_fast_layers_equal_single_calls(gpu):
    """All layers l = 16 / fp16, one token.  A plan this small runs the fp16-staged kernel, the single calls the
    block-scaled one with the contraction split across workgroups: the two quantise the staged activations
    differently (fp16 against three fp6 limbs)."""
    torch, mb = gpu
    specs = [(530, 2104, 1104, 16), (4096, 4096, 2656, 16), (272, 1032, 4096, 16), (4096, 4096, 2656, 16)]
    Ys, singles, refs = _batch_case(gpu, specs, tokens=lambda i: 1)
    for Yb, Y1, ref in zip(Ys, singles, refs):
        assert orc.max_rel_error(Yb.cpu().numpy(), ref) <= TOL
        assert orc.max_rel_error(Yb.cpu().numpy(), Y1.cpu().numpy().astype(np.float64)) <= 5e-4


def test_plan_of_several_tokens_equals_single_calls(gpu):
    """From a few tokens on, plans and single calls both take the reconstruct-order variant: the same
    fp16-rounded factors and activations; a short single call adds its column blocks in four partial sums
    (split over the waves of a workgroup), a plan in one run, so the fp32 results agree to rounding."""
    torch, mb = gpu
    specs = [(530, 2104, 1104, 16), (272, 1032, 4096, 16), (96, 200, 150, 5), (4096, 4096, 2656, 16)]
    Ys, singles, refs = _batch_case(gpu, specs, tokens=lambda i: 4 + 3 * i)
    for Yb, Y1, ref in zip(Ys, singles, refs):
        assert orc.max_rel_error(Yb.cpu().numpy(), ref) <= TOL
        assert orc.max_rel_error(Yb.cpu().numpy(), Y1.cpu().numpy().astype(np.float64)) <= 2e-5


# ---------------------------------------------------------------- prefill-shaped batch of tokens
@pytest.mark.parametrize("x_dtype", ["f16", "bf16"])
def test_prefill_tokens_sampled_against_oracle(gpu, x_dtype):
    """4096x4096, k=2656, l=16, 2048 tokens, envelopes |N|+0.1 (outputs reach 1e6: fp32 Y).
    All 2048 rows are computed on the GPU; 6 sampled tokens are checked against the oracle."""
    torch, mb = gpu
    L, X = synth.config_prefill(T=2048, x_dtype=x_dtype)
    dl = mb.DeviceLayer.from_host(L)
    Xd = _to_dev(torch, X, x_dtype)
    Y = mb.mdbf_forward(dl, Xd, y_dtype="f32")
    torch.cuda.synchronize()
    Yh = Y.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(Yh))
    rows = [0, 1, 777, 1024, 2046, 2047]
    ref = orc.forward_factored(*_oracle_args(L), X[rows])
    assert orc.max_rel_error(Yh[rows], ref) <= TOL
    # every token is an independent product: rows must not leak into each other
    Ysub = mb.mdbf_forward(dl, Xd[760:800].contiguous(), y_dtype="f32")
    torch.cuda.synchronize()
    assert torch.equal(Ysub, Y[760:800])
    # a single token takes the small-batch kernel variant, which quantises the activations differently
    Y1 = mb.mdbf_forward(dl, Xd[777:778].contiguous(), y_dtype="f32")
    torch.cuda.synchronize()
    assert orc.max_rel_error(Y1[0].cpu().numpy(), Yh[777]) <= 5e-4


# ---------------------------------------------------------------- many tokens: the reconstruct-order variant
MANY = [
    # m, n, k, l, T, env_dtype, x_dtype: every token-slab count, ragged shapes, all envelope ranks and dtypes
    (16, 128, 16, 16, 17, "f16", "f16"),
    (40, 300, 70, 3, 33, "f32", "f32"),
    (130, 129, 257, 8, 65, "bf16", "bf16"),
    (530, 2100, 1100, 16, 100, "f16", "f16"),
    (100, 1030, 200, 1, 130, "f16", "f32"),
    (1100, 520, 2105, 16, 300, "f16", "bf16"),
    (530, 2100, 1100, 8, 100, "f16", "f16"),
    (1100, 520, 2104, 8, 40, "f16", "bf16"),
]


@pytest.mark.parametrize("m,n,k,l,T,env_dtype,x_dtype", MANY)
def test_many_token_variant(gpu, m, n, k, l, T, env_dtype, x_dtype):
    L = synth.make_layer(m, n, k, l, seed=7 * m + n + k, env_dtype=env_dtype, env_kind="unit", signed_env=True)
    X = synth.make_activations(n, T, seed=55 + T, x_dtype=x_dtype)
    ref = orc.forward_factored(*_oracle_args(L), X)
    got = _run(gpu, L, X, x_dtype, "f32")
    assert orc.max_rel_error(got, ref) <= TOL


def test_many_token_exact_integer_inputs(gpu):
    """All-ones envelopes (l = 4) and x in {-1,0,1}, 50 tokens: the rebuilt factor is +-l, every partial sum
    is an integer below 2^11 in stage 1's fp16 operands and below 2^24 in fp32: bit for bit."""
    m, n, k, l, T = 200, 520, 96, 4, 50
    L = synth.make_layer(m, n, k, l, seed=61, env_dtype="f16", env_kind="ones")
    X = synth.make_activations(n, T, seed=62, x_dtype="f16", kind="ternary")
    ref = orc.forward_factored(*_oracle_args(L), X)
    # stage 2 feeds z = l * P1 through fp16: exact while |z| < 2048
    _, Z = orc.forward_factored(*_oracle_args(L), X, return_intermediates=True)
    got = _run(gpu, L, X, "f16", "f32")
    if np.max(np.abs(Z)) < 2048:
        np.testing.assert_array_equal(got, ref)
    else:
        assert orc.max_rel_error(got, ref) <= TOL


def test_many_token_batch(gpu):
    torch, mb = gpu
    specs = [(530, 2104, 1104, 16, 40), (272, 1032, 4096, 16, 17), (96, 200, 150, 5, 64)]
    layers, Xs, Ys, refs = [], [], [], []
    for i, (m, n, k, l, T) in enumerate(specs):
        L = synth.make_layer(m, n, k, l, seed=500 + i, env_dtype="f16", env_kind="llama", signed_env=True)
        X = synth.make_activations(n, T, seed=600 + i, x_dtype="f16")
        layers.append(mb.DeviceLayer.from_host(L))
        Xs.append(_to_dev(torch, X, "f16"))
        Ys.append(torch.zeros((T, m), dtype=torch.float32, device="cuda:0"))
        refs.append(orc.forward_factored(*_oracle_args(L), X))
    plan = mb.BatchPlan(layers, Xs, Ys)
    plan.run()
    torch.cuda.synchronize()
    for Yb, ref in zip(Ys, refs):
        assert orc.max_rel_error(Yb.cpu().numpy(), ref) <= TOL


# ---------------------------------------------------------------- residual stacks: Y += What x
@pytest.mark.parametrize("T,y_dtype,variant", [(1, "f32", "auto"), (1, "f16", "auto"), (1, "f32", "block_scaled"),
                                               (1, "f32", "precise"), (6, "f32", "auto"), (40, "bf16", "auto"),
                                               (1, "f32", "generic")])
def test_residual_stack_accumulates(gpu, T, y_dtype, variant):
    """Two independently factorised terms applied to the same Y, the second with MDBF_FLAG_ACCUMULATE."""
    torch, mb = gpu
    m, n = 530, 2104
    l = 5 if variant == "generic" else 16
    terms = [synth.make_layer(m, n, k, l, seed=900 + i, env_dtype="f16", env_kind="llama", signed_env=True)
             for i, k in enumerate((1104, 520))]
    X = synth.make_activations(n, T, seed=910, x_dtype="f16")
    ref = orc.forward_residual_stack([_oracle_args(L) for L in terms], X)
    Xd = _to_dev(torch, X, "f16")
    kw = dict(precise=(variant == "precise"), block_scaled=(variant == "block_scaled"))
    Y = mb.mdbf_forward(mb.DeviceLayer.from_host(terms[0]), Xd, y_dtype=y_dtype, **kw)
    mb.mdbf_forward(mb.DeviceLayer.from_host(terms[1]), Xd, y_dtype=y_dtype, Y=Y, accumulate=True, **kw)
    torch.cuda.synchronize()
    slack = {"f32": 0.0, "f16": 2.0 ** -10, "bf16": 2.0 ** -7}[y_dtype]   # two roundings to the output type
    assert orc.max_rel_error(Y.float().cpu().numpy(), ref) <= TOL + slack


def test_residual_stack_in_a_plan(gpu):
    torch, mb = gpu
    m, n = 272, 1032
    terms = [synth.make_layer(m, n, k, 16, seed=920 + i, env_dtype="f16", env_kind="llama") for i, k in enumerate((4096, 1104))]
    X = synth.make_activations(n, 1, seed=930, x_dtype="f16")
    ref = orc.forward_residual_stack([_oracle_args(L) for L in terms], X)
    Xd = _to_dev(torch, X, "f16")
    Y = torch.zeros((1, m), dtype=torch.float32, device="cuda:0")
    # the two terms of one output must not share a plan (their order is not defined inside one launch)
    for i, L in enumerate(terms):
        plan = mb.BatchPlan([mb.DeviceLayer.from_host(L)], [Xd], [Y], accumulate=(i > 0))
        plan.run()
    torch.cuda.synchronize()
    assert orc.max_rel_error(Y.cpu().numpy(), ref) <= TOL


# ---------------------------------------------------------------- the synthetic decoder stack
@pytest.mark.parametrize("budget", ["1.0", "1.5", "2.0"])
@pytest.mark.parametrize("T", [1, 8])
def test_decoder_stack_layer_through_batch(gpu, budget, T):
    """One layer of the 32-layer stack (q,k,v,o,gate,up,down: 7 independent products) per budget,
    issued as one plan; each matrix is compared with the oracle."""
    torch, mb = gpu
    layer_idx = {"1.0": 0, "1.5": 15, "2.0": 31}[budget]
    layers, Xs, Ys, refs = [], [], [], []
    for mat in range(7):
        L, X = synth.stack_matrix(budget, layer_idx, mat, T=T)
        layers.append(mb.DeviceLayer.from_host(L))
        Xs.append(_to_dev(torch, X, "f16"))
        Ys.append(torch.zeros((T, L["m"]), dtype=torch.float32, device="cuda:0"))
        refs.append(orc.forward_factored(*_oracle_args(L), X))
        sp = synth.stack_matrix_spec(budget, layer_idx, mat)
        assert abs(mb.mdbf_bpw(sp["m"], sp["n"], sp["k"], sp["l"]) - float(budget)) < 0.01
    plan = mb.BatchPlan(layers, Xs, Ys)
    plan.run()
    torch.cuda.synchronize()
    for Yb, ref in zip(Ys, refs):
        assert orc.max_rel_error(Yb.cpu().numpy(), ref) <= TOL


def test_block_scaled_plan_with_more_items_than_workgroups(gpu):
    """300 small problems of mixed contraction lengths in one block-scaled plan: more work items than the
    device holds workgroups, so that the host's cost-balanced item order and the kernel's walk over several
    items per workgroup are both on the path; every problem is compared with the oracle."""
    torch, mb = gpu
    rng = np.random.default_rng(31)
    layers, Xs, Ys, refs = [], [], [], []
    for i in range(300):
        m = int(rng.integers(17, 80))
        n = int(rng.choice([256, 300, 640, 1280]))
        k = int(rng.choice([130, 256, 640]))
        L = synth.make_layer(m, n, k, 16, seed=7000 + i, env_dtype="f16", env_kind="llama", signed_env=True)
        X = synth.make_activations(n, 1, seed=8000 + i, x_dtype="f16")
        layers.append(mb.DeviceLayer.from_host(L))
        Xs.append(_to_dev(torch, X, "f16"))
        Ys.append(torch.zeros((1, m), dtype=torch.float32, device="cuda:0"))
        refs.append(orc.forward_factored(*_oracle_args(L), X))
    plan = mb.BatchPlan(layers, Xs, Ys, block_scaled=True)
    for _ in range(2):                      # the plan is reusable
        plan.run()
    torch.cuda.synchronize()
    for Yb, ref in zip(Ys, refs):
        assert orc.max_rel_error(Yb.cpu().numpy(), ref) <= TOL


# ---------------------------------------------------------------- factors with the structure of a quantisation run
@pytest.mark.parametrize("rows,cols,R,l,outer", [(320, 288, 96, 4, 1), (272, 400, 160, 16, 0), (272, 400, 160, 16, 2)])
@pytest.mark.parametrize("variant", ["auto", "block_scaled", "tokens", "precise"])
def test_quantized_structured_factors(gpu, rows, cols, R, l, outer, variant):
    """The layer comes from the quantizer oracle run on a dense matrix with a decaying spectrum: sign masks
    correlated with the weights, envelope modes of mixed sign and falling size (the i.i.d. factors of the
    benchmark configurations have neither)."""
    from oracle import mdbf_quantizer as qz
    if variant == "block_scaled" and l != 16:
        pytest.skip("the block-scaled kernel takes rank-16 envelopes")
    W = synth.structured_weight(rows, cols, seed=rows + cols + l)
    L = qz.quantize(W, R, l, outer=outer)
    for key in ("A", "Q", "G", "B"):
        L[key] = synth.round_to_dtype(L[key], "f16")
    L["env_dtype"] = "f16"
    T = 5 if variant == "tokens" else 1
    X = synth.make_activations(cols, T, seed=77 + outer, x_dtype="f16")
    ref = orc.forward_factored(*_oracle_args(L), X)
    got = _run(gpu, L, X, "f16", "f32", precise=(variant == "precise"), block_scaled=(variant == "block_scaled"))
    assert orc.max_rel_error(got, ref) <= (TOL_PRECISE if variant == "precise" else TOL)
    # the layer does stand for W: its product is far closer to W x than W x is to zero
    assert orc.max_rel_error(ref, X.astype(np.float64) @ W.T) < 0.9


# ---------------------------------------------------------------- a tall, ragged projection (vocabulary-sized)
@pytest.mark.parametrize("T,variant", [(1, "auto"), (1, "block_scaled"), (3, "auto"), (70, "auto")])
def test_tall_ragged_projection(gpu, T, variant):
    """m = 32003 rows (2001 row tiles: 31 full groups of the packed layout and a ragged one), k = 1000
    (not a multiple of 128).  Every output is checked: the factored oracle is cheap at this shape."""
    L = synth.make_layer(32003, 1536, 1000, 16, seed=321, env_dtype="f16", env_kind="llama", signed_env=True)
    X = synth.make_activations(1536, T, seed=322, x_dtype="f16")
    ref = orc.forward_factored(*_oracle_args(L), X)
    got = _run(gpu, L, X, "f16", "f32", block_scaled=(variant == "block_scaled"))
    assert got.shape == (T, 32003)
    assert orc.max_rel_error(got, ref) <= TOL


def test_sibling_projections_share_their_input(gpu):
    """q, k, v (and gate, up) of a decoder layer read the same activations: three layers of one plan point
    at one X buffer; each result equals the oracle's for that layer."""
    torch, mb = gpu
    X = synth.make_activations(1024, 1, seed=901, x_dtype="f16")
    Xd = _to_dev(torch, X, "f16")
    layers, Ys, refs = [], [], []
    for i, (m, k) in enumerate([(1024, 640), (1024, 640), (512, 384)]):
        L = synth.make_layer(m, 1024, k, 16, seed=910 + i, env_dtype="f16", env_kind="llama", signed_env=True)
        layers.append(mb.DeviceLayer.from_host(L))
        Ys.append(torch.zeros((1, m), dtype=torch.float32, device="cuda:0"))
        refs.append(orc.forward_factored(*_oracle_args(L), X))
    plan = mb.BatchPlan(layers, [Xd, Xd, Xd], Ys)
    plan.run()
    torch.cuda.synchronize()
    for Yb, ref in zip(Ys, refs):
        assert orc.max_rel_error(Yb.cpu().numpy(), ref) <= TOL


# ---------------------------------------------------------------- small envelope ranks through zero modes
@pytest.mark.parametrize("l,l_to,T", [(1, 8, 1), (3, 8, 1), (2, 16, 1), (3, 8, 5)])
def test_padded_envelopes_denote_the_same_layer(gpu, l, l_to, T):
    """mdbf_pad_envelope appends zero modes: bit-exact copy plus zeros, and the padded layer (which the
    matrix-core kernels take) gives the product of the original one."""
    torch, mb = gpu
    L = synth.make_layer(530, 2100, 1100, l, seed=400 + l, env_dtype="f16", env_kind="llama", signed_env=True)
    dl = mb.DeviceLayer.from_host(L)
    dp = dl.padded(l_to)
    for name in ("A", "Q", "G", "B"):
        src, dst = getattr(dl, name).cpu().numpy(), getattr(dp, name).cpu().numpy()
        assert dst.shape == (src.shape[0], l_to)
        np.testing.assert_array_equal(dst[:, :l].view(np.uint16), src.view(np.uint16))
        assert not dst[:, l:].view(np.uint16).any()
    X = synth.make_activations(2100, T, seed=410, x_dtype="f16")
    ref = orc.forward_factored(*_oracle_args(L), X)
    Xd = _to_dev(torch, X, "f16")
    for layer, bs in ((dl, False), (dp, False), (dp, True)):
        Y = mb.mdbf_forward(layer, Xd, y_dtype="f32", block_scaled=bs)
        torch.cuda.synchronize()
        assert orc.max_rel_error(Y.cpu().numpy().astype(np.float64), ref) <= TOL


# ---------------------------------------------------------------- the matrix itself, through unit vectors
@pytest.mark.parametrize("l,env_dtype", [(16, "f16"), (8, "f16"), (3, "f32")])
def test_forward_on_the_identity_reproduces_the_dense_matrix(gpu, l, env_dtype):
    """The product applied to the n unit vectors is What itself (Eq. "me-dbf-basis"), entry by entry."""
    torch, mb = gpu
    m, n, k = 200, 192, 96
    L = synth.make_layer(m, n, k, l, seed=777 + l, env_dtype=env_dtype, env_kind="unit", signed_env=True)
    W = orc.dense_reconstruct(*_oracle_args(L))
    got = _run(gpu, L, np.eye(n), "f16", "f32")              # (n, m): row j = What e_j
    assert np.abs(got.T - W).max() <= TOL * np.abs(W).max()
    one = _run(gpu, L, np.eye(n)[5:6], "f16", "f32")          # a single unit vector takes the one-token kernels
    assert np.abs(one[0] - W[:, 5]).max() <= TOL * np.abs(W).max()


# ---------------------------------------------------------------- single short calls: the split-K variant
@pytest.mark.parametrize("m,n,k,l,T,x_dtype", [
    (16, 8, 8, 16, 2, "f16"),            # one block, three of the four waves idle
    (300, 1160, 648, 16, 7, "f16"),      # 10 and 6 column blocks: partial last iterations
    (2064, 520, 4104, 16, 16, "bf16"),
    (530, 2104, 1096, 8, 3, "f32"),
    (4096, 4096, 2656, 16, 16, "f16"),
])
def test_short_single_calls(gpu, m, n, k, l, T, x_dtype):
    L = synth.make_layer(m, n, k, l, seed=m + n + k + T, env_dtype="f16", env_kind="unit", signed_env=True)
    X = synth.make_activations(n, T, seed=55 + T, x_dtype=x_dtype)
    ref = orc.forward_factored(*_oracle_args(L), X)
    got = _run(gpu, L, X, x_dtype, "f32")
    assert orc.max_rel_error(got, ref) <= TOL
    again = _run(gpu, L, X, x_dtype, "f32")
    np.testing.assert_array_equal(got, again)     # the partial sums are added in a fixed order


# ---------------------------------------------------------------- HIP graph capture and replay
@pytest.mark.parametrize("T,block_scaled", [(1, False), (1, True), (6, False)])
def test_graph_replay_matches_eager(gpu, T, block_scaled):
    """A plan captured into a HIP graph: every replay, with new activations in the same buffers and eager
    work in between, gives exactly what the eager call gives (the library records kernel launches only)."""
    torch, mb = gpu
    specs = [(530, 2104, 1104, 16), (272, 1032, 4096, 16), (1024, 1024, 640, 8)]
    layers, Xs, Ys = [], [], []
    for i, (m, n, k, l) in enumerate(specs):
        L = synth.make_layer(m, n, k, l, seed=600 + i, env_dtype="f16", env_kind="llama", signed_env=True)
        layers.append(mb.DeviceLayer.from_host(L))
        Xs.append(torch.zeros((T, n), dtype=torch.float16, device="cuda:0"))
        Ys.append(torch.zeros((T, m), dtype=torch.float32, device="cuda:0"))
    plan = mb.BatchPlan(layers, Xs, Ys, block_scaled=block_scaled)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        plan.run(stream=s)                       # warm-up outside the capture (function attributes)
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        plan.run(stream=s)
    for rep in range(3):
        new = [synth.make_activations(X.shape[1], T, seed=700 + 10 * rep + i, x_dtype="f16") for i, X in enumerate(Xs)]
        for X, a in zip(Xs, new):
            X.copy_(_to_dev(torch, a, "f16"))
        for Y in Ys:
            Y.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        replayed = [Y.clone() for Y in Ys]
        for Y in Ys:
            Y.zero_()
        plan.run()
        torch.cuda.synchronize()
        for Yr, Ye in zip(replayed, Ys):
            assert torch.equal(Yr, Ye)
            assert Ye.abs().max().item() > 0


# ---------------------------------------------------------------- a residual stack as one launch
@pytest.mark.parametrize("ranks,T", [((4, 4), 1), ((8, 8), 1), ((1, 1), 1), ((8, 8), 6)])
def test_residual_stack_as_one_concatenated_layer(gpu, ranks, T):
    """P independently factorised terms with sum of ranks <= 16, written as one layer (sign bases
    concatenated along the inner dimension, block-diagonal inner envelope factors): one call instead of P
    accumulating ones; ranks adding up to 8 or 16 take the matrix-core kernels."""
    terms = [synth.make_layer(530, 1032, 520 + 8 * p, l, seed=820 + p, env_dtype="f16", env_kind="llama", signed_env=True)
             for p, l in enumerate(ranks)]
    X = synth.make_activations(1032, T, seed=830, x_dtype="f16")
    ref = orc.forward_residual_stack([_oracle_args(t) for t in terms], X)
    one = concat_terms(terms)
    assert orc.max_rel_error(_run(gpu, one, X, "f16", "f32"), ref) <= TOL
    if sum(ranks) in (8, 16) and T == 1:
        assert orc.max_rel_error(_run(gpu, one, X, "f16", "f32", block_scaled=True), ref) <= TOL


# ---------------------------------------------------------------- magnitudes far from one
@pytest.mark.parametrize("env_scale,x_scale", [(0.5, 1.0), (32.0, 2.0 ** -10), (1.0, 512.0), (4.0, 2.0 ** -4), (0.25, 1.0),
                                               (0.5, 2.0 ** -6)])
@pytest.mark.parametrize("variant", ["auto", "block_scaled", "tokens"])
def test_relative_error_does_not_depend_on_scale(gpu, env_scale, x_scale, variant):
    """Envelopes and activations scaled by powers of two, the scaled activations B o x and Q o z (divided by
    8 in the fp16 variant's staging) staying inside fp16's normal range: the error relative to the largest
    output stays within the gate in every variant."""
    L = synth.make_layer(530, 2104, 1104, 16, seed=941, env_dtype="f16", env_kind="llama", signed_env=True)
    for key in ("A", "Q", "G", "B"):
        L[key] = synth.round_to_dtype(L[key].astype(np.float64) * env_scale, "f16")
    T = 5 if variant == "tokens" else 1
    X = synth.round_to_dtype(synth.make_activations(2104, T, seed=942, x_dtype="f32").astype(np.float64) * x_scale, "f16")
    ref = orc.forward_factored(*_oracle_args(L), X)
    assert np.isfinite(ref).all() and np.abs(ref).max() > 0
    got = _run(gpu, L, X, "f16", "f32", block_scaled=(variant == "block_scaled"))
    assert orc.max_rel_error(got, ref) <= TOL


@pytest.mark.parametrize("env_scale,x_scale", [(2.0 ** -9, 1.0), (2.0 ** -6, 2.0 ** -12), (2.0 ** -3, 2.0 ** -14)])
@pytest.mark.parametrize("block_scaled", [True, False])
def test_one_token_variants_carry_their_own_exponents(gpu, env_scale, x_scale, block_scaled):
    """Far below fp16's normal range (the scaled activations Q o z reach 1e-12 here) both one-token variants
    still meet the gate: the block-scaled records hold an exponent per 32 values, the fp16 variant's
    scale-in kernel one per 1024 columns, and z stays in fp32."""
    L = synth.make_layer(530, 2104, 1104, 16, seed=941, env_dtype="f16", env_kind="llama", signed_env=True)
    for key in ("A", "Q", "G", "B"):
        L[key] = synth.round_to_dtype(L[key].astype(np.float64) * env_scale, "f16")
    X = synth.round_to_dtype(synth.make_activations(2104, 1, seed=942, x_dtype="f32").astype(np.float64) * x_scale, "f16")
    ref = orc.forward_factored(*_oracle_args(L), X)
    assert np.abs(ref).max() > 0
    got = _run(gpu, L, X, "f16", "f32", block_scaled=block_scaled)
    assert orc.max_rel_error(got, ref) <= TOL
