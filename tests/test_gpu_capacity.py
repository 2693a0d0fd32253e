"""Capacity on the device (the experiment of Table 1: how many 200-unit layers fit at 128 time steps): a stack deep
enough to occupy a real share of the 288 GB runs forward and backward once.  No oracle finishes this size; what
is checked is that every gradient is finite, that the workspaces the plan reports are what the run needs (they
are allocated at exactly that size), and, on the layers whose gradients have not vanished, that batch rows do not
interact: the whole batch against the mean of its two halves.  The measured time and memory are printed; the
figures quoted in the design notes come from this test."""
import time

import numpy as np
import pytest

import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _run(w, master0, x, y):
    import torch
    import paper_1912_00286_amd as hip
    torch.cuda.reset_peak_memory_stats()
    ts = pu.make_step(w, master0)
    dx = torch.from_numpy(np.ascontiguousarray(x)).to(ts.lp_dtype).to(ts.dev)
    dy = torch.from_numpy(np.ascontiguousarray(y)).to(ts.dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    hip.lstm_forward(ts.cfg, ts.params_lp, dx, dy, None, None, ts.reserve, ts.scratch, ts.losses[0:1])
    hip.lstm_backward(ts.cfg, ts.params_lp, dx, dy, ts.reserve, ts.scratch, ts.loss_scale, ts.grads[0])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    out = dict(loss=float(ts.losses[0].item()), grads=ts.grads[0].double().cpu().numpy() / w.loss_scale, seconds=dt,
               reserve=ts.reserve.numel(), scratch=ts.scratch.numel(), peak=torch.cuda.max_memory_allocated())
    del ts, dx, dy
    torch.cuda.empty_cache()
    return out


@pytest.mark.parametrize("L,batch,dtype", [(512, 256, "bf16"), (2304, 256, "fp16")], ids=["512_layers_bf16", "2304_layers_fp16"])
def test_deep_stack_on_the_device(L, batch, dtype):
    w = wl.Workload(f"capacity_{L}", L, 9, 200, 128, batch, dtype, wl.HEAD_STEP_BCE, loss_scale=1.0 if dtype == "bf16" else 1024.0,
                    target_p=0.4, data_seed=91, weight_seed=92)
    master0, xs, ys = pu.inputs_for(w)
    print(f"[case] {L} layers x 200 units, T=128, B={batch}, {dtype}: {wl.param_count(w) / 1e6:.0f} M parameters", flush=True)
    whole = _run(w, master0, xs[0], ys[0])
    print(f"  forward + backward {whole['seconds'] * 1e3:.0f} ms; reserve {whole['reserve'] / 2**30:.1f} GiB, scratch "
          f"{whole['scratch'] / 2**30:.1f} GiB, peak device memory {whole['peak'] / 2**30:.1f} GiB", flush=True)
    assert np.isfinite(whole["loss"]) and np.all(np.isfinite(whole["grads"]))
    assert whole["peak"] > (40 << 30)
    if L > 512:
        return
    half = w.with_(batch=batch // 2)
    h1 = _run(half, master0, xs[0][:, :batch // 2], ys[0][:, :batch // 2])
    h2 = _run(half, master0, xs[0][:, batch // 2:], ys[0][:, batch // 2:])
    assert abs(whole["loss"] - 0.5 * (h1["loss"] + h2["loss"])) <= 1e-4 * abs(whole["loss"])
    # the layers near the top, whose gradients are far from the underflow threshold, and the head
    shapes = pu.oracle_shapes(w)
    off, top = 0, {}
    for name, shape in shapes:
        n = int(np.prod(shape))
        if name in ("w_head", "b_head") or (name[1:].isdigit() and int(name[1:]) >= L - 4):
            top[name] = (off, n)
        off += n
    mean = 0.5 * (h1["grads"] + h2["grads"])
    for name, (o, n) in top.items():
        a, b = whole["grads"][o:o + n], mean[o:o + n]
        assert np.linalg.norm(b) > 0, name
        assert np.linalg.norm(a - b) <= pu.GRAD_RTOL[dtype] * np.linalg.norm(b), name
