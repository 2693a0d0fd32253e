"""No result may depend on what the caller's workspaces held before the call.  The reserve and scratch
buffers are caller-owned and arrive uninitialised; here they (and the gradient output) are filled with
0xFF bytes, a NaN in every storage type, before the step, on one shape per kernel family (narrow layers,
wide layers, thousands of rows per step with the step kernels projecting their own input, embeddings,
the fp32 mode, stacked workers), widths whose padding to whole tiles is owned by no workgroup included.
A kernel that reads a padding element it never wrote turns the loss or a gradient into NaN.  Each shape runs
twice, first on zero-filled workspaces: the two passes must agree bit for bit."""
import numpy as np
import pytest

import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _w(name, L, I, H, T, B, dtype, head=wl.HEAD_STEP_BCE, **kw):
    scale = 1024.0 if dtype == "fp16" else 1.0
    return wl.Workload(name, L, I, H, T, B, dtype, head, loss_scale=scale, data_seed=11, weight_seed=12, target_p=0.4, **kw)


CASES = [
    (_w("rows8192_3layers", 3, 64, 200, 3, 8192, "fp16"), False),
    (_w("rows8192_1layer", 1, 64, 200, 3, 8192, "fp16"), False),
    (_w("rows2048_h40", 2, 24, 40, 3, 2048, "fp16"), False),
    (_w("rows4100_h520", 2, 3, 520, 3, 4100, "fp16", wl.HEAD_LAST_BCE), False),
    (_w("narrow_h200", 2, 64, 200, 4, 128, "fp16"), False),
    (_w("narrow_3layers_bf16", 3, 9, 200, 4, 256, "bf16"), False),
    (_w("embedding", 1, 0, 256, 4, 128, "fp16", wl.HEAD_LAST_BCE, vocab=300, embed_dim=128), False),
    (_w("wide_h1024", 2, 130, 1024, 3, 256, "fp16", wl.HEAD_STEP_MSE, target_kind="normal"), False),
    (_w("wide_h1032_ragged", 1, 8, 1032, 3, 100, "fp16"), False),
    (_w("wide_tiles_3layers", 3, 24, 1024, 36, 256, "fp16"), False),
    (_w("wide_tiles_h1280_b192", 2, 8, 1280, 5, 192, "bf16", wl.HEAD_LAST_BCE), False),
    (_w("wide_tiles_h2048_packed_copies_only", 2, 256, 2048, 3, 256, "fp16"), False),
    (_w("wide_tiles_h2048_embedding", 1, 0, 2048, 2, 256, "fp16", wl.HEAD_LAST_BCE, vocab=300, embed_dim=256), False),
    (_w("rows1024_h520", 2, 24, 520, 3, 1024, "fp16"), False),
    (_w("odd_sizes", 2, 5, 33, 4, 17, "fp16"), False),
    (_w("fp32_odd_sizes", 2, 5, 33, 4, 17, "fp32"), False),
    (_w("fp32_rows1000", 2, 64, 200, 3, 1000, "fp32"), False),
    (_w("stacked_workers", 2, 64, 200, 3, 128, "fp16", n_workers=4), True),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0].name for c in CASES])
def test_results_do_not_depend_on_workspace_contents(case):
    import torch
    w, batched = case
    print(f"[case] {w.name}: L={w.num_layers} I={w.input_dim} H={w.hidden} T={w.seq_len} B={w.batch} N={w.n_workers} {w.dtype}", flush=True)
    master0, xs, ys = pu.inputs_for(w)
    ts = pu.make_step(w, master0, batched=batched)
    dx, dy = pu.device_batches(w, xs, ys, ts.lp_dtype, ts.dev)
    # a first pass on zeroed workspaces, then the checked one on workspaces full of 0xFF bytes: the same bits
    for buf in list(ts.reserves) + list(ts.scratches):
        buf.fill_(0)
    ts.grads.view(torch.uint8).fill_(255)
    ts.forward_backward(dx, dy)
    torch.cuda.synchronize()
    on_zeros = ts.grads.clone()
    for buf in list(ts.reserves) + list(ts.scratches):
        buf.fill_(255)
    ts.grads.view(torch.uint8).fill_(255)
    ts.step(dx, dy, pu.lr_for(w, 0))
    torch.cuda.synchronize()
    assert int(ts.found_inf.item()) == 0, "a non-finite gradient came out of finite inputs"
    assert torch.equal(ts.grads.view(torch.uint8), on_zeros.view(torch.uint8)), "the gradients depend on what the workspaces held"
    want = pu.run_oracle_step(w)
    losses = ts.losses.double().cpu().numpy()
    assert np.all(np.abs(losses - want["losses"]) <= pu.LOSS_RTOL * np.abs(want["losses"])), (losses, want["losses"])
    grads = ts.grads.double().cpu().numpy() / w.loss_scale
    assert np.all(np.isfinite(grads))
    for k in range(w.n_workers):
        pu.assert_grads_close(grads[k], want["grads"][k], want["shapes"], pu.GRAD_RTOL[w.dtype], f"worker {k}")
