"""All simulated workers' micro-batches through one forward and one backward call
(lstm_config.workers > 1): per-worker losses and per-worker raw gradients must come out as
if every worker had run alone (the workers only meet in the gradient average: Section
"Distributed computing framework", steps 3-4)."""
import numpy as np
import pytest

import workloads as wl
from oracle import lstm_oracle as orc
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hip():
    import paper_1912_00286_amd as pkg
    pkg.load_library()
    return pkg


CASES = [
    # name, L, I, H, T, B, dtype, head, workers
    ("bw_fp16_step", 2, 16, 48, 5, 64, "fp16", wl.HEAD_STEP_BCE, 3),
    ("bw_bf16_last", 1, 24, 64, 4, 128, "bf16", wl.HEAD_LAST_BCE, 2),
    ("bw_fp16_mse_ragged_h", 2, 20, 72, 3, 64, "fp16", wl.HEAD_STEP_MSE, 5),
    ("bw_fp16_jet_width", 2, 64, 200, 4, 128, "fp16", wl.HEAD_STEP_BCE, 4),
]


@pytest.mark.parametrize("spec", CASES, ids=[c[0] for c in CASES])
def test_batched_workers_match_oracle_worker_by_worker(hip, spec):
    name, L, I, H, T, B, dtype, head, N = spec
    print(f"[case] {name}", flush=True)
    w = wl.Workload(name, L, I, H, T, B, dtype, head, n_workers=N, loss_scale=1.0 if dtype == "bf16" else 1024.0,
                    dynamic_scale=True, n_half=4.0, warmup_steps=2, gamma=0.9,
                    target_kind="normal" if head == wl.HEAD_STEP_MSE else "bernoulli", target_p=0.3,
                    data_seed=500 + N, weight_seed=51)
    got = pu.run_gpu_step(w, batched=True)
    want = pu.run_oracle_step(w)
    pu.assert_step_close(w, got, want)           # losses and raw gradients of every worker, average, update


def test_batched_equals_one_by_one(hip):
    """Same library, two ways of calling it: forward values are bit-identical (a row's
    arithmetic does not depend on the rows next to it), weight gradients agree to rounding
    (their sums over T*B run in a different order)."""
    import torch
    w = wl.Workload("bw_cmp", 2, 16, 64, 6, 64, "fp16", wl.HEAD_STEP_BCE, n_workers=3, loss_scale=512.0, data_seed=71, weight_seed=72)
    master0, xs, ys = pu.inputs_for(w)
    one = pu.make_step(w, master0)
    dx, dy = pu.device_batches(w, xs, ys, one.lp_dtype, one.dev)
    both = pu.make_step(w, master0, batched=True)
    one.forward_backward(dx, dy)
    both.forward_backward(dx, dy)
    torch.cuda.synchronize()
    assert torch.equal(one.losses, both.losses)
    a, b = one.grads.float(), both.grads.float()
    assert torch.allclose(a, b, rtol=2e-2, atol=2e-3 * float(a.abs().max()))


def test_batched_form_refuses_what_it_cannot_do(hip):
    for w in (wl.Workload("bw_fp32", 1, 8, 64, 4, 64, "fp32", wl.HEAD_STEP_BCE, n_workers=2),
              wl.Workload("bw_b8", 1, 8, 64, 4, 8, "fp16", wl.HEAD_STEP_BCE, n_workers=2),
              wl.Workload("bw_text", 1, 0, 64, 4, 64, "fp16", wl.HEAD_LAST_BCE, vocab=50, embed_dim=16, n_workers=2)):
        cfg = pu.make_cfg(w)
        cfg.workers = w.n_workers
        with pytest.raises(hip.LstmError) as e:
            hip.lstm_workspace_bytes(cfg)
        assert e.value.status == -2


def test_config5_sixty_four_workers_batched(hip):
    """Config 5 at full size in the batched form: 64 x 128 samples per time step.  Averaged
    gradient against the oracle on the concatenated batch (the identity the oracle is pinned
    with), workers 0, 31 and 63 one by one."""
    w = wl.CONFIGS["workers64"]
    print("[case] workers64 batched: HIP step", flush=True)
    gpu = pu.run_gpu_step(w, batched=True)
    master0, xs, ys = pu.inputs_for(w)
    shapes = pu.oracle_shapes(w)
    params = orc.unflatten(master0, shapes)
    tol = pu.GRAD_RTOL[w.dtype]
    print("[case] workers64 batched: oracle on the concatenated batch", flush=True)
    xcat = np.concatenate(xs, axis=1).astype(np.float64); ycat = np.concatenate(ys, axis=1)
    loss_cat, cache = orc.forward(params, w.num_layers, xcat, ycat, w.head)
    avg_ref = orc.flatten(orc.backward(params, w.num_layers, cache, 1.0), shapes)
    del cache
    assert gpu["found_inf"][-1] == 0
    assert abs(gpu["losses"].mean() - loss_cat) <= pu.LOSS_RTOL * abs(loss_cat)
    pu.assert_grads_close(gpu["avg"], avg_ref, shapes, tol, "averaged over 64 workers")
    for k in (0, 31, w.n_workers - 1):
        loss, cache = orc.forward(params, w.num_layers, xs[k].astype(np.float64), ys[k], w.head)
        g = orc.flatten(orc.backward(params, w.num_layers, cache, 1.0), shapes)
        assert abs(gpu["losses"][k] - loss) <= pu.LOSS_RTOL * abs(loss)
        pu.assert_grads_close(gpu["grads"][k], g, shapes, tol, f"worker {k}")
