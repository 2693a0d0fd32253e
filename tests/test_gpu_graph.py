"""The captured-graph form of the training step must reproduce the eager form bit for bit.

Replays are interleaved with eager work and synchronisations, and every replay is
checked: a graph node that misbehaves on later replays would show up here."""
import numpy as np
import pytest

import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _snapshot(ts):
    import torch
    torch.cuda.synchronize()
    return dict(losses=ts.losses.clone(), grads=ts.grads.clone(), avg=ts.avg.clone(), master=ts.master.clone(),
                params_lp=ts.params_lp.clone(), state1=ts.state1.clone(), scale=ts.loss_scale.clone(),
                found_inf=ts.found_inf.clone(), good=ts.good_steps.clone())


def _assert_same(a, b, what):
    import torch
    for k in a:
        assert torch.equal(a[k], b[k]), f"{what}: {k} differs between eager and graph replay"


@pytest.mark.parametrize("name", ["jet", "text", "rows2048", "rows4096", "wide1024", "tile1024", "tile2048", "stacked"])
def test_graph_replay_matches_eager(name):
    import torch
    batched = False
    if name == "jet":
        w = wl.CONFIGS[name].with_(seq_len=24, n_workers=2, dynamic_scale=True, loss_scale=4096.0)
    elif name == "text":
        w = wl.CONFIGS[name].with_(seq_len=40)
    elif name == "rows2048":        # two thousand rows per step: one launch per cell on 32x32 tiles
        w = wl.Workload(name, 2, 64, 200, 6, 2048, "fp16", wl.HEAD_STEP_BCE, loss_scale=1024.0, target_p=0.4, data_seed=51, weight_seed=52)
    elif name == "rows4096":        # a layer's whole recurrence in one launch per direction
        w = wl.Workload(name, 2, 64, 200, 6, 4096, "fp16", wl.HEAD_STEP_BCE, loss_scale=1024.0, target_p=0.4, data_seed=57, weight_seed=58)
    elif name == "wide1024":        # wide layers: two launches per BPTT step
        w = wl.Workload(name, 2, 40, 1024, 5, 128, "bf16", wl.HEAD_STEP_MSE, target_kind="normal", data_seed=53, weight_seed=54)
    elif name == "tile1024":        # the benchmark's path: tile kernels on the lagged diagonals, chunked projection GEMMs
        w = wl.Workload(name, 3, 64, 1024, 40, 192, "fp16", wl.HEAD_STEP_MSE, target_kind="normal", loss_scale=256.0,
                        data_seed=59, weight_seed=60)
    elif name == "tile2048":        # the same with every tensor in packed form only and layer 0 on the packed-operand GEMMs
        w = wl.Workload(name, 2, 256, 2048, 34, 256, "fp16", wl.HEAD_STEP_MSE, target_kind="normal", loss_scale=256.0,
                        data_seed=61, weight_seed=62)
    else:                           # several workers stacked into one call per direction
        w = wl.Workload(name, 2, 64, 200, 6, 128, "fp16", wl.HEAD_STEP_BCE, n_workers=4, loss_scale=1024.0, target_p=0.4,
                        data_seed=55, weight_seed=56)
        batched = True
    master0, xs, ys = pu.inputs_for(w)
    n_steps = 4

    eager = pu.make_step(w, master0, batched=batched)
    dx, dy = pu.device_batches(w, xs, ys, eager.lp_dtype, eager.dev)
    if batched:
        dx, dy = eager.stack_workers(dx, dy)
    ref = []
    for k in range(n_steps):
        eager.step(dx, dy, pu.lr_for(w, k))
        ref.append(_snapshot(eager))

    graph = pu.make_step(w, master0, batched=batched)
    gx = dx.clone() if batched else [t.clone() for t in dx]
    gy = dy.clone() if batched else [t.clone() for t in dy]
    graph.capture(gx, gy)
    # capture runs nothing: the state is still the initial one
    assert torch.equal(graph.master, torch.as_tensor(master0, dtype=torch.float32, device=graph.dev))
    scratch_noise = torch.empty(1 << 20, device=graph.dev)
    for k in range(n_steps):
        graph.step_captured(pu.lr_for(w, k))
        _assert_same(ref[k], _snapshot(graph), f"step {k}")
        # eager work of the program between replays
        scratch_noise.normal_()
        torch.cuda.synchronize()
    assert graph.step_index == n_steps


@pytest.mark.parametrize("captured", [False, True])
def test_workers_on_several_streams_match_one_stream(captured):
    """Five simulated workers spread over three streams (each with its own workspace) give
    bit for bit what one stream gives, eagerly and as a captured fork-join graph."""
    import torch
    w = wl.CONFIGS["jet"].with_(seq_len=12, n_workers=5, dynamic_scale=True, loss_scale=2048.0)
    master0, xs, ys = pu.inputs_for(w)
    one = pu.make_step(w, master0)
    dx, dy = pu.device_batches(w, xs, ys, one.lp_dtype, one.dev)
    many = pu.make_step(w, master0, n_streams=3)
    assert many.n_streams == 3 and len(many.side_streams) == 2
    if captured:
        many.capture(dx, dy)
    for k in range(3):
        lr = pu.lr_for(w, k)
        one.step(dx, dy, lr)
        if captured:
            many.step_captured(lr)
        else:
            many.step(dx, dy, lr)
        _assert_same(_snapshot(one), _snapshot(many), f"step {k}")


def test_step_captured_requires_capture():
    w = wl.CONFIGS["tiny"]
    master0, xs, ys = pu.inputs_for(w)
    ts = pu.make_step(w, master0)
    with pytest.raises(RuntimeError):
        ts.step_captured(1e-3)
