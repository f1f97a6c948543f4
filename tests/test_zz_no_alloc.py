"""tl_linear_step_static: the allocation-free variant of tl_linear_step (for callers that cannot call hipMalloc) must
give what tl_linear_step gives.  Both run the same kernels in the same order, so the outputs are compared bit for bit,
on two calls in a row through the C ABI, the second with a smaller input (the static scratch then still holds the first
call's values), and each against the CPU oracle at the fp32 tolerance.  Sizes beyond the static buffer are refused."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from oracle import templora_oracle as O  # noqa: E402
from paper_2401_11504_amd import synth  # noqa: E402

LR, F32_TOL = 5e-5, 1e-4


def _run(api, H, fn, case, s):
    T, din = case["X"].shape
    dout, r = case["B"].shape
    dev = {k: H.to_dev_f32(v) for k, v in case.items()}
    out = {k: torch.full(shp, float("nan"), device="cuda") for k, shp in
           dict(Y=(T, dout), dX=(T, din), dA=(r, din), dB=(dout, r), A1=(r, din), B1=(dout, r)).items()}
    fn(dev["X"], dev["W"], dev["A"], dev["B"], dev["dY"], s, LR, 0.9, 0.999, 1e-8, 0.01, True,
       out["Y"], out["dX"], out["dA"], out["dB"], out["A1"], out["B1"])
    return {k: v.cpu().numpy() for k, v in out.items()}


def test_static_scratch_variant_matches_the_allocating_one():
    from paper_2401_11504_amd import api, harness as H
    from test_gpu_kernels import check
    s = 16.0 / 8.0
    # first the benchmark's single-layer shape, then a smaller ragged one: the second call finds the first call's
    # H, dH and moments in the shared scratch
    for seed, (T, din, dout, r) in ((1001, (128, 256, 256, 8)), (1002, (77, 200, 136, 5))):
        case = synth.linear_case(seed, T, din, dout, r)
        got = _run(api, H, api.tl_linear_step_static, case, s)
        want = _run(api, H, api.tl_linear_step, case, s)
        ref = O.linear_step(case["X"], case["W"], case["A"], case["B"], case["dY"], s, LR, wd=0.01)
        for k in ("Y", "dX", "dA", "dB", "A1", "B1"):
            assert np.array_equal(got[k], want[k]), k          # same kernels, same order: identical bits
            check(got[k], ref[k], F32_TOL, k)
        check(got["A1"] - case["A"], ref["A1"] - case["A"], 1e-3, "A step")
        check(got["B1"] - case["B"], ref["B1"] - case["B"], 1e-3, "B step")
    # without AdamW the moments are not needed and A_new / B_new may be absent
    case = synth.linear_case(1003, 33, 64, 40, 4)
    dev = {k: H.to_dev_f32(v) for k, v in case.items()}
    outs = []
    for fn in (api.tl_linear_step_static, api.tl_linear_step):
        o = {k: torch.zeros(shp, device="cuda") for k, shp in dict(Y=(33, 40), dX=(33, 64), dA=(4, 64), dB=(40, 4)).items()}
        fn(dev["X"], dev["W"], dev["A"], dev["B"], dev["dY"], s, LR, 0.9, 0.999, 1e-8, 0.0, False,
           o["Y"], o["dX"], o["dA"], o["dB"], None, None)
        outs.append(o)
    for k in outs[0]:
        assert torch.equal(outs[0][k], outs[1][k]), k


def test_static_scratch_variant_refuses_what_does_not_fit():
    from paper_2401_11504_amd import api
    # 2 T r alone exceeds the 2^20-float buffer: refused on the host before anything is launched or read
    T, din, dout, r = 1 << 17, 8, 8, 8
    z = torch.zeros(8, device="cuda")
    X = torch.empty(T, din, device="cuda")
    B = torch.empty(dout, r, device="cuda")
    with pytest.raises(api.TlError) as e:
        api.tl_linear_step_static(X, z, z, B, z, 1.0, LR, 0.9, 0.999, 1e-8, 0.0, False, z, z, z, z, None, None)
    assert e.value.status == -2 and "static" in str(e.value)
