"""vgg_fc_static, the dense layer for callers that cannot allocate (no workspace argument: the partial sums
live in a buffer inside the library's device image), against vgg_fc: same kernels, so bit-identical output."""
import numpy as np
import pytest
import torch

from paper_1810_09868_amd import binding as B

from gpu_util import TDT, dev, ws_bytes

pytestmark = pytest.mark.gpu


def _both(dtype, N, In, Out, relu, zdt, seed):
    rng = np.random.default_rng(seed)
    a = dev(rng.standard_normal((N, In)).astype(np.float32), TDT[dtype])
    w = dev((rng.standard_normal((Out, In)) * np.sqrt(2.0 / In)).astype(np.float32), TDT[dtype])
    b = dev(rng.standard_normal(Out).astype(np.float32))
    want = torch.full((N, Out), float("nan"), dtype=TDT[zdt], device="cuda")
    got = torch.full((N, Out), float("nan"), dtype=TDT[zdt], device="cuda")
    B.vgg_fc(dtype, N, In, Out, a, w, b, want, zdt, relu, ws_bytes(B.vgg_fc_workspace_bytes(dtype, N, In, Out)))
    B.vgg_fc_static(dtype, N, In, Out, a, w, b, got, zdt, relu)
    torch.cuda.synchronize()
    assert torch.isfinite(want.float()).all()
    assert torch.equal(got, want), (dtype, N, In, Out)


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
def test_fc_static_matches_fc_on_consecutive_calls(dtype):
    # two calls in a row on the same buffer, the second smaller than the first (the buffer still holds the
    # first call's partial sums), then a larger one again and a shape off the 64-byte units
    _both(dtype, 100, 4096, 1000, 0, B.F32, seed=1)
    _both(dtype, 7, 512, 96, 1, dtype, seed=2)
    _both(dtype, 100, 25088, 4096, 1, dtype, seed=3)
    _both(dtype, 10, 10, 10, 0, B.F32, seed=4)


def test_fc_static_rejects_what_does_not_fit_before_touching_the_device():
    N, In, Out = 1100, 8192, 4096
    assert B.vgg_fc_workspace_bytes(B.F32, N, In, Out) > B.FC_STATIC_SCRATCH_BYTES
    a = torch.zeros((16,), device="cuda")
    with pytest.raises(B.VggError) as e:
        B.vgg_fc_static(B.F32, N, In, Out, a, a, None, a, B.F32, 0)     # the tensors are far too small: must not be read
    assert e.value.status == -8
    with pytest.raises(B.VggError):
        B.vgg_fc_static(B.F32, 0, In, Out, a, a, None, a, B.F32, 0)
