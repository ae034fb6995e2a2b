"""mdbf_forward_static (the entry point that allocates nothing: its scratch is a static device array inside
the library) against mdbf_forward, through the C ABI: same kernels, same arithmetic, so the outputs must be
identical bit for bit; two calls in a row, the second with a smaller input; then every kernel variant."""
import ctypes as C

import numpy as np
import pytest

from oracle import mdbf_oracle as orc
from paper_2512_24545_amd import synth

pytestmark = pytest.mark.gpu

TOL = 2e-3


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2512_24545_amd import binding as mb
    mb.lib()
    return torch, mb


def _case(torch, mb, m, n, k, l, T, seed, **kw):
    L = synth.make_layer(m, n, k, l, seed=seed, env_dtype="f16", env_kind="llama", signed_env=True)
    X = synth.make_activations(n, T, seed=seed + 1, x_dtype="f16")
    dl = mb.DeviceLayer.from_host(L)
    Xd = torch.from_numpy(np.ascontiguousarray(X)).to("cuda:0").half()
    want = mb.mdbf_forward(dl, Xd, y_dtype="f32", **kw)            # the existing entry point
    Y = torch.full((T, m), float("nan"), dtype=torch.float32, device="cuda:0")
    torch.cuda.synchronize()
    mem0 = torch.cuda.memory_allocated()
    mb.mdbf_forward_static(dl, Xd, Y, **kw)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == mem0
    ref = orc.forward_factored(L["SA"], L["SB"], L["A"], L["Q"], L["G"], L["B"], X)
    return Y, want, ref


def test_static_scratch_equals_workspace_call_twice_in_a_row(gpu):
    torch, mb = gpu
    # first a large layer (11008 x 4096, 16 tokens: 7.5 MB of scratch), then a smaller one on the same array,
    # whose results must not see what the first call left behind
    for (m, n, k, l, T, kw) in [(11008, 4096, 4096, 16, 16, dict(block_scaled=True)),
                                (530, 2104, 1104, 16, 1, dict(block_scaled=True)),
                                (4096, 4096, 2656, 16, 1, {}),
                                (300, 1160, 648, 16, 7, {}),
                                (100, 1030, 200, 5, 2, {}),
                                (96, 200, 150, 5, 2, dict(precise=True))]:
        Y, want, ref = _case(torch, mb, m, n, k, l, T, seed=m + n + k + T, **kw)
        assert torch.equal(Y, want), (m, n, k, l, T, kw)
        assert orc.max_rel_error(Y.cpu().numpy(), ref) <= TOL


def test_static_scratch_rejects_what_does_not_fit(gpu):
    torch, mb = gpu
    L = synth.make_layer(64, 4096, 2656, 16, seed=3, env_dtype="f16", env_kind="llama")
    dl = mb.DeviceLayer.from_host(L)
    X = torch.zeros((2048, 4096), dtype=torch.float16, device="cuda:0")
    Y = torch.zeros((2048, 64), dtype=torch.float32, device="cuda:0")
    assert mb.mdbf_workspace_bytes(dl.desc("f16", "f32"), 2048) > (16 << 20)
    with pytest.raises(mb.MdbfError) as ei:
        mb.mdbf_forward_static(dl, X, Y)
    assert ei.value.status == -4      # MDBF_EWORKSPACE, reported before any launch
    torch.cuda.synchronize()
    assert not Y.any().item()
