"""ReLU with a sign bitmask as its only saved state (Sec. 5.2) through the C ABI against oracle/ops.py: the mask is
integer work and must match bit for bit (both sides decide "x > 0" on the same stored values), y and dx are
selections of input values and must match exactly."""
import numpy as np
import pytest
import torch

from workload import gen, CONFIGS

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2402_18789_amd.binding as B
    from paper_2402_18789_amd import host as HH
    from oracle import ops as OO

C1 = CONFIGS["c1_tiny_f32"]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("n,width", [(1, 1), (3, 31), (5, 32), (4, 33), (7, 40), (9, 64), (6, 200), (300, 1408), (256, 14336),
                                     (2, 14344), (17, 4100)])
def test_relu_bitmask_forward_and_backward(dtype, n, width):
    print(f"relu bitmask {dtype} n={n} width={width}", flush=True)
    cfg = C1.with_(dtype=dtype)
    g = gen.rng(9, "relu_bitmask", dtype, n, width)
    x = gen.storage_round(cfg, g.standard_normal((n, width), dtype=np.float32))
    x[g.random((n, width)) < 0.05] = 0.0                     # exact zeros (and -0.0 below): not positive
    x[g.random((n, width)) < 0.02] = -0.0
    dy = gen.storage_round(cfg, g.standard_normal((n, width), dtype=np.float32))
    y_o, m_o = OO.relu_bitmask_fwd(x.astype(np.float64))
    dx_o = OO.relu_bitmask_bwd(dy.astype(np.float64), m_o)
    dt = HH.TORCH_DTYPE[dtype]
    code = HH.DTYPE_CODE[dtype]
    words = (width + 31) // 32
    x_d, dy_d = torch.from_numpy(x).to("cuda", dt), torch.from_numpy(dy).to("cuda", dt)
    y_d, dx_d = torch.empty_like(x_d), torch.empty_like(dy_d)
    m_d = torch.full((n, words), -1, dtype=torch.int32, device="cuda")       # every bit set: the call must write all of it
    B.flexco_relu_bitmask_fwd(x_d, y_d, m_d, n, width, code)
    B.flexco_relu_bitmask_bwd(dy_d, m_d, dx_d, n, width, code)
    torch.cuda.synchronize()
    m_g = m_d.cpu().numpy().view(np.uint32)
    assert np.array_equal(m_g, m_o), "mask differs"
    assert np.array_equal(y_d.double().cpu().numpy(), y_o)
    assert np.array_equal(dx_d.double().cpu().numpy(), dx_o)
    assert m_g.nbytes * 8 == n * words * 32                   # one bit per element, rows padded to whole words
    # in place: y over x, dx over dy
    B.flexco_relu_bitmask_fwd(x_d, x_d, m_d, n, width, code)
    B.flexco_relu_bitmask_bwd(dy_d, m_d, dy_d, n, width, code)
    torch.cuda.synchronize()
    assert torch.equal(x_d, y_d) and torch.equal(dy_d, dx_d)


def test_relu_bitmask_unaligned_rows_and_errors():
    x = torch.randn(4, 48, device="cuda")
    xs = x.view(-1)[1:1 + 3 * 40].view(3, 40).contiguous()   # fresh tensor: aligned; the unaligned view is below
    flat = torch.randn(3 * 40 + 4, device="cuda")
    un = flat[1:1 + 3 * 40]                                   # starts 4 bytes past a 16-byte boundary
    y = torch.empty(3 * 40 + 4, device="cuda")[1:1 + 3 * 40]
    m = torch.zeros((3, 2), dtype=torch.int32, device="cuda")
    B.flexco_relu_bitmask_fwd(un, y, m, 3, 40, 0)
    torch.cuda.synchronize()
    _, m_o = OO.relu_bitmask_fwd(un.view(3, 40).double().cpu().numpy())
    assert np.array_equal(m.cpu().numpy().view(np.uint32), m_o)
    assert torch.equal(y.view(3, 40), torch.relu(un.view(3, 40)))
    with pytest.raises(B.FlexcoError):
        B.flexco_relu_bitmask_fwd(None, y, m, 3, 40, 0)
    with pytest.raises(B.FlexcoError):
        B.flexco_relu_bitmask_fwd(un, y, m, 70000, 40, 0)
    with pytest.raises(B.FlexcoError):
        B.flexco_relu_bitmask_bwd(un, m, y, 3, 40, 7)
    B.flexco_relu_bitmask_fwd(un, y, m, 0, 40, 0)             # nothing to do
    del xs
