"""GPU parity of dybit_maxpool2d_codes against the oracle's pooling on codes (Sec. III-B: activations are
stored as DyBit codes), bit for bit, and the property that makes it useful: pooling the codes equals
encoding the pooled fp32 tensor."""
import numpy as np
import pytest
import torch

from oracle import dybit_ref as R
from paper_2302_12510_amd import binding as B
from gpu_util import dev

pytestmark = pytest.mark.gpu

FMTS = [(2, False), (2, True), (4, False), (4, True), (8, False), (8, True)]


def packed(q, bits):
    return dev(R.pack_rows(q.reshape(-1, q.shape[-1]), bits))


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("geom", [(3, 2, 1), (2, 2, 0), (3, 1, 1), (1, 1, 0), (4, 3, 2)])
def test_maxpool_codes(fmt, geom):
    k, stride, pad = geom
    rng = np.random.default_rng(3 + fmt[0] + k)
    Bn, H, W = 3, 13, 9
    C = (32 // fmt[0]) * 3                       # three words per pixel
    q = rng.integers(0, 1 << fmt[0], (Bn, H, W, C)).astype(np.uint8)
    got = B.dybit_maxpool2d_codes(Bn, H, W, C, k, stride, pad, packed(q, fmt[0]), fmt)
    torch.cuda.synchronize()
    want = R.maxpool2d_codes(q, *fmt, k, stride, pad)
    assert np.array_equal(got.cpu().numpy().reshape(-1), R.pack_rows(want.reshape(-1, C), fmt[0]).reshape(-1))


def test_maxpool_codes_equals_encoding_the_pooled_tensor():
    """The stem of an image network: 112 x 112 x 64 after ReLU, 3 x 3 window, stride 2, 4-bit unsigned."""
    rng = np.random.default_rng(17)
    fmt = (4, False)
    x = np.abs(rng.normal(0, 1, (2, 112, 112, 64))).astype(np.float32)
    xd = dev(x)
    s = B.dybit_absmax_scale(xd.reshape(-1), *fmt)
    q = B.dybit_quantize(xd.reshape(-1), s, *fmt)
    pooled_codes = B.dybit_maxpool2d_codes(2, 112, 112, 64, 3, 2, 1, q, fmt)
    pooled = torch.nn.functional.max_pool2d(xd.permute(0, 3, 1, 2), 3, 2, 1).permute(0, 2, 3, 1).contiguous()
    q2 = B.dybit_quantize(pooled.reshape(-1), s, *fmt)
    torch.cuda.synchronize()
    assert torch.equal(pooled_codes.reshape(-1), q2.reshape(-1))
    want = R.maxpool2d_codes(R.unpack(q.cpu().numpy(), x.size, 4).reshape(x.shape)[:1], *fmt, 3, 2, 1)
    assert np.array_equal(pooled_codes.cpu().numpy().reshape(2, -1)[0], R.pack_rows(want.reshape(-1, 64), 4).reshape(-1))


def test_maxpool_codes_argument_errors():
    a = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    for args, status in [((1, 8, 8, 16, 3, 2, 1, a, (6, False)), B.ERR_UNSUPPORTED_BITS),
                         ((1, 8, 8, 4, 3, 2, 1, a, (4, False)), B.ERR_ALIGNMENT),
                         ((1, 8, 8, 8, 3, 2, 2, a, (4, False)), B.ERR_INVALID_ARG),
                         ((1, 8, 8, 8, 3, 2, 1, None, (4, False)), B.ERR_NULL)]:
        with pytest.raises(B.DybitError) as e:
            B.dybit_maxpool2d_codes(*args, out=a)
        assert e.value.status == status
