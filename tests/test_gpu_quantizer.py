"""The autograd quantizer module (activation forward, error backward) against the oracle."""
import numpy as np
import pytest

from helpers import assert_bit_equal

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import qsim_ref as R                                                          # noqa: E402
from paper_1910_04540_amd import workloads as W                                           # noqa: E402
from paper_1910_04540_amd.quantizer import (BlockFloatingPoint, FixedPoint, FloatingPoint, Quantizer,  # noqa: E402
                                            quantize)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU")


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def test_functional_quantize_matches_the_oracle():
    x = W.lognormal_gradients((6, 10, 7, 8), seed=3, overflow_fraction=0.01)
    d = torch.from_numpy(x).cuda()
    assert_bit_equal(host(quantize(d, FloatingPoint(5, 2, subnormal=True), "stochastic", seed=9, stream_id=4)),
                     R.float_quantize(x, 5, 2, R.STOCHASTIC, R.SATURATE | R.SUBNORMAL, 9, 4), "float")
    assert_bit_equal(host(quantize(d, FixedPoint(8, 6), "nearest_away")),
                     R.fixed_quantize(x, 8, 6, R.RN_AWAY, R.SATURATE), "fixed")
    assert_bit_equal(host(quantize(d, FixedPoint(8, 20, clamp=False, symmetric=True), "nearest_zero")),
                     R.fixed_quantize(x, 8, 20, R.RN_ZERO, R.SYMMETRIC), "fixed, open range")
    for dim, layout in [(None, (1, 1, x.size)), (0, (1, 6, 560)), (1, (6, 10, 56)), (-1, (420, 8, 1))]:
        got = host(quantize(d, BlockFloatingPoint(8, dim), "stochastic", seed=5, stream_id=1))
        assert_bit_equal(got, R.block_quantize(x, *layout, 8, R.STOCHASTIC, 0, 5, 1), f"block dim {dim}")
    assert quantize(d, None) is d
    # a non-contiguous view is quantized in its own (logical) order
    t = d.permute(1, 0, 2, 3)
    want = R.block_quantize(np.ascontiguousarray(x.transpose(1, 0, 2, 3)), 1, 10, 336, 8, R.RN_EVEN)
    assert_bit_equal(host(quantize(t, BlockFloatingPoint(8, 0))), want, "permuted input")


def test_module_quantizes_activation_forward_and_error_backward():
    x = W.normal_tensor(4 * 33 * 17, seed=5).reshape(4, 33, 17)
    up = (W.normal_tensor(4 * 33 * 17, seed=6) * np.float32(1e-3)).reshape(4, 33, 17)
    q = Quantizer(FixedPoint(8, 6), FloatingPoint(5, 2, subnormal=True), "nearest", "stochastic", seed=77).cuda()
    for call in range(3):                                   # every call draws from its own streams
        xd = torch.from_numpy(x).cuda().requires_grad_(True)
        y = q(xd)
        y.backward(torch.from_numpy(up).cuda())
        assert_bit_equal(host(y), R.fixed_quantize(x, 8, 6, R.RN_EVEN, R.SATURATE, 77, 2 * call), f"forward {call}")
        assert_bit_equal(host(xd.grad), R.float_quantize(up, 5, 2, R.STOCHASTIC, R.SATURATE | R.SUBNORMAL, 77, 2 * call + 1),
                         f"backward {call}")
    assert q.calls == 3


def test_module_identity_directions_and_a_training_step():
    x = torch.from_numpy(W.normal_tensor(64 * 32, seed=8).reshape(64, 32)).cuda()
    fwd_only = Quantizer(forward_number=BlockFloatingPoint(8, None), seed=1)
    xin = x.clone().requires_grad_(True)
    g = torch.from_numpy(W.normal_tensor(64 * 32, seed=9).reshape(64, 32)).cuda()
    fwd_only(xin).backward(g)
    assert_bit_equal(host(xin.grad), host(g), "no backward format: the error passes unchanged")
    # a small network with quantizers between its layers takes an optimizer step
    net = torch.nn.Sequential(torch.nn.Linear(32, 48), Quantizer(FloatingPoint(5, 2), FloatingPoint(5, 2), "nearest", "stochastic"),
                              torch.nn.ReLU(), torch.nn.Linear(48, 10),
                              Quantizer(FixedPoint(16, 10), FixedPoint(16, 14), "stochastic", "stochastic", seed=3)).cuda()
    opt = torch.optim.SGD(net.parameters(), lr=0.1)
    before = [p.detach().clone() for p in net.parameters()]
    out = net(x)
    assert torch.equal(out, quantize(out, FixedPoint(16, 10)))          # the output lies on the fixed-point grid
    loss = out.square().mean()
    loss.backward()
    opt.step()
    assert all(torch.isfinite(p).all() for p in net.parameters())
    assert any(not torch.equal(a, b) for a, b in zip(before, net.parameters()))
