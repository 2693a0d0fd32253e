"""The wide-layer recurrence (recurrent_tile.hip and the lagged diagonal schedule that feeds it) against the
oracle at its limits: the completely unrolled K loops (widths 1024 and 2048) and the run-time one, several
chunks of the 32-step lag with a ragged last one, one layer and several, batches of 192 to 384 rows, both
16-bit types, all heads; with a check that the shapes really take that path."""
import numpy as np
import pytest

import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

CASES = [
    # name, L, I, H, T, B, dtype, head
    ("three_layers_unrolled16_three_chunks", 3, 40, 1024, 70, 256, "fp16", wl.HEAD_STEP_MSE),
    ("two_layers_runtime_loop_two_chunks", 2, 24, 1152, 37, 192, "bf16", wl.HEAD_STEP_BCE),
    ("one_layer_unrolled32", 1, 8, 2048, 3, 320, "fp16", wl.HEAD_LAST_BCE),
    ("four_layers_short_sequence", 4, 130, 1024, 5, 384, "bf16", wl.HEAD_STEP_BCE),
    ("two_layers_one_step", 2, 16, 1280, 1, 256, "fp16", wl.HEAD_STEP_MSE),
    ("width_2048_two_layers", 2, 64, 2048, 33, 256, "fp16", wl.HEAD_STEP_MSE),
    # every tensor in packed form only, layer 0 included (input width a multiple of 256)
    ("width_2048_packed_input", 2, 256, 2048, 8, 256, "bf16", wl.HEAD_STEP_BCE),
]


def _workload(spec):
    name, L, I, H, T, B, dtype, head = spec
    kw = dict(target_kind="normal") if head == wl.HEAD_STEP_MSE else dict(target_p=0.4)
    return wl.Workload(f"tile_{name}", L, I, H, T, B, dtype, head, loss_scale=1024.0 if dtype == "fp16" else 1.0,
                       data_seed=71, weight_seed=72, **kw)


@pytest.mark.parametrize("spec", CASES, ids=[c[0] for c in CASES])
def test_wide_layers_against_the_oracle(spec):
    import paper_1912_00286_amd as hip
    w = _workload(spec)
    print(f"[case] {w.name}: L={w.num_layers} I={w.input_dim} H={w.hidden} T={w.seq_len} B={w.batch} {w.dtype} head={w.head}", flush=True)
    # the plan of this shape holds the per-layer chunk buffers of the lagged schedule: one more scratch region
    # per layer above the first than a shape just outside its range (a batch that is no multiple of 64)
    n_in = len([r for r in hip.lstm_debug_plan_regions(pu.make_cfg(w)) if r[0] == 1])
    n_out = len([r for r in hip.lstm_debug_plan_regions(pu.make_cfg(w.with_(batch=w.batch + 8))) if r[0] == 1])
    assert n_in != n_out, "this shape is meant to run on the wide-layer tile kernels"
    got = pu.run_gpu_step(w)
    want = pu.run_oracle_step(w, with_terms=True)
    used = []
    pu.assert_step_close(w, got, want, used)
    assert not used, used


def test_wide_layers_run_to_run_identical():
    import torch
    w = _workload(CASES[0])
    a = pu.run_gpu_step(w)
    b = pu.run_gpu_step(w)
    np.testing.assert_array_equal(a["grads"], b["grads"])
    np.testing.assert_array_equal(a["losses"], b["losses"])


def test_wide_layers_identical_over_many_runs_with_refilled_workspaces():
    """One 2048-wide layer, two time steps, thirty forward + backward passes on the same inputs with the scratch
    buffer refilled before each (0xFF bytes and zeros in turn): every pass must give the first pass's gradients bit
    for bit.  (The step kernels count their outstanding loads from the youngest backwards; a load issued out of its
    chunk's turn before the first barrier once left a workgroup, now and then, multiplying LDS bytes that had not
    arrived yet, and only back-to-back passes on refilled buffers showed it.)"""
    import torch
    import paper_1912_00286_amd as hip
    w = wl.Workload("tile_repeat", 1, 256, 2048, 2, 256, "fp16", wl.HEAD_LAST_BCE, loss_scale=1024.0, target_p=0.4,
                    data_seed=11, weight_seed=12)
    master0, xs, ys = pu.inputs_for(w)
    ts = pu.make_step(w, master0)
    dx, dy = pu.device_batches(w, xs, ys, ts.lp_dtype, ts.dev)
    x, y = dx[0], dy[0]
    first = None
    for i in range(30):
        ts.scratch.fill_(255 if i % 2 == 0 else 0)
        ts.grads.view(torch.uint8).fill_(255)
        hip.lstm_forward(ts.cfg, ts.params_lp, x, y, None, None, ts.reserve, ts.scratch, ts.losses[0:1])
        hip.lstm_backward(ts.cfg, ts.params_lp, x, y, ts.reserve, ts.scratch, ts.loss_scale, ts.grads[0])
        torch.cuda.synchronize()
        g = ts.grads[0].cpu().view(torch.int16).numpy()
        if first is None:
            first = g
            assert np.isfinite(ts.grads[0].float().cpu().numpy()).all()
        else:
            assert np.array_equal(g, first), f"pass {i} differs from the first pass in {int((g != first).sum())} elements"
