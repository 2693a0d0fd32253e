"""The one-launch-per-layer recurrences (a workgroup walks its 32 rows through all time steps): shapes around
their limits against the oracle — 256 units (eight unit blocks), widths whose last block and last K chunk are
partly padding, a batch that is not a multiple of 64 (a half-empty last tile, no blocked copies), input widths
that are not multiples of 32, a single time step, bf16, a chunk that starts from a non-zero state — and a check
that these shapes really take that path (two launches of the step class per layer)."""
import numpy as np
import pytest

import workloads as wl
from oracle import lstm_oracle as orc
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

CASES = [
    # name, L, I, H, T, B, dtype, head
    ("h256", 2, 24, 256, 3, 8192, "fp16", wl.HEAD_STEP_BCE),
    ("h136_ragged_batch", 1, 9, 136, 2, 8200, "fp16", wl.HEAD_STEP_MSE),
    ("h200_one_step_bf16", 2, 64, 200, 1, 8192, "bf16", wl.HEAD_STEP_BCE),
    ("h104_rows16384", 1, 200, 104, 3, 16384, "fp16", wl.HEAD_LAST_BCE),
    ("h200_three_layers_in40", 3, 40, 200, 4, 8192, "fp16", wl.HEAD_STEP_BCE),
    ("h232_bf16", 1, 130, 232, 3, 8192, "bf16", wl.HEAD_STEP_BCE),
    ("h96_two_layers", 2, 8, 96, 3, 4096, "fp16", wl.HEAD_STEP_BCE),          # 4H too narrow for the blocked dU product
    ("h136_three_layers_bf16", 3, 33, 136, 3, 6144, "bf16", wl.HEAD_STEP_BCE),
    ("rows3072_smallest_batch", 2, 64, 200, 3, 3072, "fp16", wl.HEAD_STEP_BCE),
    ("rows4100_ragged", 2, 8, 200, 2, 4100, "fp16", wl.HEAD_LAST_BCE),
]


@pytest.fixture(scope="module")
def hip():
    import paper_1912_00286_amd as pkg
    pkg.load_library()
    return pkg


@pytest.mark.parametrize("spec", CASES, ids=[c[0] for c in CASES])
def test_row_ownership_shapes(hip, spec):
    import torch
    name, L, I, H, T, B, dtype, head = spec
    kw = dict(target_kind="normal") if head == wl.HEAD_STEP_MSE else dict(target_p=0.4)
    w = wl.Workload(name, L, I, H, T, B, dtype, head, loss_scale=1024.0 if dtype == "fp16" else 1.0, data_seed=81, weight_seed=82, **kw)
    print(f"[case] {name}: L={L} I={I} H={H} T={T} B={B} {dtype}", flush=True)
    master0, xs, ys = pu.inputs_for(w)
    ts = pu.make_step(w, master0)
    for buf in list(ts.reserves) + list(ts.scratches):
        buf.fill_(255)
    dx, dy = pu.device_batches(w, xs, ys, ts.lp_dtype, ts.dev)
    hip.lstm_timing_enable(True)
    ts.step(dx, dy, pu.lr_for(w, 0))
    torch.cuda.synchronize()
    launches = hip.lstm_timing_read(hip.KERNEL_CLASSES.index("gemm_step"))["launches"]
    hip.lstm_timing_enable(False)
    assert launches == 2 * L, f"{launches} launches of the step class: this shape did not take the one-launch-per-layer path"
    assert int(ts.found_inf.item()) == 0
    want = pu.run_oracle_step(w)
    loss = ts.losses.double().cpu().numpy()
    assert np.all(np.abs(loss - want["losses"]) <= pu.LOSS_RTOL * np.abs(want["losses"]))
    got = ts.grads.double().cpu().numpy() / w.loss_scale
    assert np.all(np.isfinite(got))
    pu.assert_grads_close(got[0], want["grads"][0], want["shapes"], pu.GRAD_RTOL[dtype], name)


def test_row_ownership_from_a_given_state(hip):
    import torch
    L, I, H, T, B = 2, 64, 200, 3, 8192
    w = wl.Workload("rows_state", L, I, H, T, B, "fp16", wl.HEAD_STEP_BCE, loss_scale=512.0, target_p=0.4, data_seed=83, weight_seed=84)
    master0, xs, ys = pu.inputs_for(w)
    dev = torch.device("cuda:0")
    ts = pu.make_step(w, master0, dev)
    for buf in list(ts.reserves) + list(ts.scratches):
        buf.fill_(255)
    rng = np.random.default_rng(85)
    h0 = torch.from_numpy(rng.uniform(-0.9, 0.9, (L, B, H)).astype(np.float32)).to(ts.lp_dtype).to(dev)
    c0 = torch.from_numpy(rng.normal(0.0, 1.0, (L, B, H)).astype(np.float32)).to(dev)
    hT = torch.full((L, B, H), float("nan"), dtype=ts.lp_dtype, device=dev)
    cT = torch.full((L, B, H), float("nan"), device=dev)
    x = torch.from_numpy(xs[0]).to(ts.lp_dtype).to(dev)
    y = torch.from_numpy(ys[0]).to(dev)
    hip.lstm_forward(ts.cfg, ts.params_lp, x, y, h0, c0, ts.reserve, ts.scratch, ts.losses[0:1], hT, cT)
    hip.lstm_backward(ts.cfg, ts.params_lp, x, y, ts.reserve, ts.scratch, ts.loss_scale, ts.grads[0])
    torch.cuda.synchronize()
    shapes = pu.oracle_shapes(w)
    params = orc.unflatten(ts.params_lp.double().cpu().numpy(), shapes)
    loss, cache = orc.forward(params, L, x.double().cpu().numpy(), ys[0], w.head, h0.double().cpu().numpy(), c0.double().cpu().numpy())
    g = orc.flatten(orc.backward(params, L, cache, 1.0), shapes)
    assert abs(float(ts.losses[0].item()) - loss) <= pu.LOSS_RTOL * abs(loss)
    pu.assert_grads_close(ts.grads[0].double().cpu().numpy() / w.loss_scale, g, shapes, pu.GRAD_RTOL["fp16"], "rows, given state")
    h_ref = np.stack([cache["layers"][l]["h"][-1] for l in range(L)])
    c_ref = np.stack([cache["layers"][l]["c"][-1] for l in range(L)])
    np.testing.assert_allclose(hT.double().cpu().numpy(), h_ref, atol=6e-3)
    np.testing.assert_allclose(cT.double().cpu().numpy(), c_ref, atol=2.4e-2)
