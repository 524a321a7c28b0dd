"""flexco_lora_fwd_static (the entry point that allocates nothing: its rank-r scratch is an array inside
the library's image) against flexco_lora_fwd with a caller-owned scratch buffer, and against the oracle.

Two calls in a row, the second on a smaller input: the array keeps the first call's contents, and the
second result may not depend on them.  Runs last (file name), alone or after the other tests."""
import numpy as np
import pytest
import torch

from workload import gen, CONFIGS

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2402_18789_amd.binding as B
    from paper_2402_18789_amd import host as HH
    from oracle import ops as OO
    from gpu_common import to_np, TOL, assert_close

C1 = CONFIGS["c1_tiny_f32"]


def _case(dtype, T, din, dout, r, seg_off, seg_adapter, seed):
    cfg = C1.with_(dtype=dtype)
    g = gen.rng(seed, "lora_static", din, dout, r, T)
    rnd = lambda shape, s=1.0: gen.storage_round(cfg, (g.standard_normal(shape) * s).astype(np.float32))
    x, y0 = rnd((T, din)), rnd((T, dout))
    As = [rnd((din, r), 0.05) for _ in range(2)]
    Bs = [rnd((r, dout), 0.05) for _ in range(2)]
    ref = y0.astype(np.float64)
    for s, a in enumerate(seg_adapter):
        if a >= 0:
            rows = slice(seg_off[s], seg_off[s + 1])
            ref[rows] += OO.lora_delta(x[rows].astype(np.float64), As[a].astype(np.float64), Bs[a].astype(np.float64), 2.0)
    return x, y0, As, Bs, ref


def _run_both(dtype, T, din, dout, r, seg_off, seg_adapter, seed):
    x, y0, As, Bs, ref = _case(dtype, T, din, dout, r, seg_off, seg_adapter, seed)
    dt = HH.TORCH_DTYPE[dtype]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda", dt)
    x_d, y_ws, y_st = dev(x), dev(y0), dev(y0)
    A_d, B_d = [dev(a.T) for a in As], [dev(b.T) for b in Bs]
    u = torch.zeros(T * r, dtype=torch.float32, device="cuda")
    code = HH.DTYPE_CODE[dtype]
    B.flexco_lora_fwd(x_d, y_ws, T, din, dout, r, 2.0, code, A_d, B_d, seg_off, seg_adapter, u)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.flexco_lora_fwd_static(x_d, y_st, T, din, dout, r, 2.0, code, A_d, B_d, seg_off, seg_adapter)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    got_ws, got_st = to_np(y_ws), to_np(y_st)
    assert np.array_equal(got_st, got_ws), "static-scratch call differs from the workspace call"
    assert_close("lora_fwd_static", got_st, ref, TOL[dtype])
    for s, a in enumerate(seg_adapter):          # rows without adapter are untouched, bit for bit
        if a < 0:
            assert np.array_equal(got_st[seg_off[s]:seg_off[s + 1]], y0[seg_off[s]:seg_off[s + 1]].astype(np.float64))


@pytest.mark.parametrize("dtype,din,dout,r", [("bf16", 512, 1408, 16), ("f32", 256, 688, 8)])
def test_lora_fwd_static_two_calls(dtype, din, dout, r):
    print(f"lora_fwd_static {dtype} in={din} out={dout} r={r}: T=333 then T=77", flush=True)
    _run_both(dtype, 333, din, dout, r, [0, 40, 41, 200, 290, 333], [1, -1, 0, -1, 1], seed=11)
    # second call: fewer rows, other segment boundaries; the array still holds the first call's products
    _run_both(dtype, 77, din, dout, r, [0, 9, 30, 31, 60, 77], [-1, 1, 0, -1, 1], seed=12)


def test_lora_fwd_static_rejects_oversize():
    print("lora_fwd_static: size beyond the built-in scratch is refused, nothing launched", flush=True)
    r, T = 64, 8192 + 1          # T * r = 524352 > 2^19
    x = torch.zeros((T, 64), dtype=torch.float32, device="cuda")
    y = torch.ones((T, 64), dtype=torch.float32, device="cuda")
    A = [torch.zeros((r, 64), dtype=torch.float32, device="cuda")]
    Bm = [torch.zeros((64, r), dtype=torch.float32, device="cuda")]
    with pytest.raises(B.FlexcoError) as ei:
        B.flexco_lora_fwd_static(x, y, T, 64, 64, r, 1.0, HH.DTYPE_CODE["f32"], A, Bm, [0, T], [0])
    assert ei.value.code == B.FLEXCO_EWORKSPACE
    torch.cuda.synchronize()
    assert bool((y == 1).all())
    # the largest size that fits runs
    T = 8192
    B.flexco_lora_fwd_static(x[:T], y[:T], T, 64, 64, r, 1.0, HH.DTYPE_CODE["f32"], A, Bm, [0, T], [0])
    torch.cuda.synchronize()
    assert bool((y == 1).all())      # A = B = 0: y unchanged
