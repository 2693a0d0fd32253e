"""The entry point that allocates nothing: lstm_forward_static_scratch against lstm_forward on the same
inputs (bit for bit: same kernels, same order), two calls in a row with the second on a smaller input,
then lstm_backward from the reserve it filled."""
import numpy as np
import pytest

import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _run(w, static):
    import torch
    import paper_1912_00286_amd as hip
    master0, xs, ys = pu.inputs_for(w)
    ts = pu.make_step(w, master0)
    dx, dy = pu.device_batches(w, xs, ys, ts.lp_dtype, ts.dev)
    L, B, H = w.num_layers, w.batch, w.hidden
    rng = np.random.default_rng(5)
    h0 = torch.from_numpy(rng.uniform(-0.5, 0.5, (L, B, H)).astype(np.float32)).to(ts.lp_dtype).to(ts.dev)
    c0 = torch.from_numpy(rng.uniform(-0.5, 0.5, (L, B, H)).astype(np.float32)).to(ts.dev)
    hT, cT = torch.zeros_like(h0), torch.zeros_like(c0)
    ts.reserve.fill_(0x5a)                         # regions nobody writes compare equal
    ts.scratch.fill_(0xff)
    if static:
        hip.lstm_forward_static_scratch(ts.cfg, ts.params_lp, dx[0], dy[0], h0, c0, ts.reserve, ts.losses[0:1], hT, cT)
    else:
        hip.lstm_forward(ts.cfg, ts.params_lp, dx[0], dy[0], h0, c0, ts.reserve, ts.scratch, ts.losses[0:1], hT, cT)
    hip.lstm_backward(ts.cfg, ts.params_lp, dx[0], dy[0], ts.reserve, ts.scratch, ts.loss_scale, ts.grads[0])
    torch.cuda.synchronize()
    return dict(loss=ts.losses.cpu().numpy().copy(), hT=hT.float().cpu().numpy(), cT=cT.cpu().numpy(),
                reserve=ts.reserve.cpu().numpy().copy(), grads=ts.grads.float().cpu().numpy())


def test_static_scratch_forward_matches_the_workspace_form():
    import paper_1912_00286_amd as hip
    first = wl.Workload("na_first", 2, 24, 200, 12, 64, "fp16", wl.HEAD_STEP_BCE, loss_scale=256.0, target_p=0.4, data_seed=31, weight_seed=32)
    second = wl.Workload("na_second", 1, 5, 72, 3, 17, "bf16", wl.HEAD_STEP_MSE, target_kind="normal", data_seed=33, weight_seed=34)
    for w in (first, second):                      # the second call finds the first one's leftovers in the array
        _, sb = hip.lstm_workspace_bytes(pu.make_cfg(w))
        assert 0 < sb <= hip.STATIC_SCRATCH_BYTES
        print(f"[case] {w.name}: scratch {sb} bytes, static", flush=True)
        got = _run(w, True)
        print(f"[case] {w.name}: workspace form", flush=True)
        want = _run(w, False)
        assert np.isfinite(got["loss"]).all() and got["loss"][0] > 0
        for k in ("loss", "hT", "cT", "reserve", "grads"):
            np.testing.assert_array_equal(got[k], want[k], err_msg=f"{w.name}: {k}")


def test_static_scratch_refuses_what_does_not_fit():
    import torch
    import paper_1912_00286_amd as hip
    w = wl.CONFIGS["jet"]                          # 212 MB of scratch
    cfg = pu.make_cfg(w)
    rb, sb = hip.lstm_workspace_bytes(cfg)
    assert sb > hip.STATIC_SCRATCH_BYTES
    buf = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(hip.LstmError) as e:
        hip.lstm_forward_static_scratch(cfg, buf, buf, buf, None, None, buf, buf, reserve_bytes=rb)
    assert e.value.status == -3 and "scratch" in str(e.value)
