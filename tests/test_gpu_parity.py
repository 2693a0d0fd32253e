"""Parity of the HIP path with the CPU oracle, through the C ABI, on the same
seeded inputs.  Run with -m gpu on an MI355X."""
import numpy as np
import pytest

import workloads as wl
from oracle import lstm_oracle as orc
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hip():
    import paper_1912_00286_amd as pkg
    pkg.load_library()          # fails loudly if the HIP library is not built
    return pkg


def _check(w):
    print(f"[case] {w.name} L={w.num_layers} I={w.input_dim} H={w.hidden} T={w.seq_len} B={w.batch} "
          f"{w.dtype} head={w.head} N={w.n_workers}", flush=True)
    gpu = pu.run_gpu_step(w)
    ref = pu.run_oracle_step(w)
    pu.assert_step_close(w, gpu, ref)
    return gpu, ref


# ------------------------------------------------------------------ config 1
def test_config1_tiny_fp32(hip):
    gpu, ref = _check(wl.CONFIGS["tiny"])
    # plain SGD, lr 1e-3: W' = W - lr * g
    np.testing.assert_allclose(gpu["master"], gpu["master0"] - 1e-3 * gpu["avg"], rtol=0, atol=2e-7)


# ------------------------------------------------------------------ small shapes: several tiles + ragged tails
SMALL = [
    # name, L, I, H, T, B, dtype, head
    ("s_fp32_ragged", 2, 13, 36, 5, 6, "fp32", wl.HEAD_STEP_BCE),
    ("s_fp32_mse", 3, 20, 70, 7, 9, "fp32", wl.HEAD_STEP_MSE),
    ("s_fp32_last", 1, 8, 130, 6, 70, "fp32", wl.HEAD_LAST_BCE),
    ("s_fp16_aligned", 2, 64, 200, 6, 40, "fp16", wl.HEAD_STEP_BCE),
    ("s_fp16_ragged", 2, 13, 36, 5, 6, "fp16", wl.HEAD_STEP_BCE),      # K % 8 != 0: scalar-load path
    ("s_fp16_tiles", 1, 72, 264, 4, 150, "fp16", wl.HEAD_STEP_MSE),    # > 1 tile in every dimension, ragged
    ("s_fp16_last", 2, 24, 48, 9, 10, "fp16", wl.HEAD_LAST_BCE),
    ("s_bf16", 2, 64, 200, 6, 40, "bf16", wl.HEAD_STEP_BCE),
    ("s_bf16_mse", 1, 40, 136, 5, 130, "bf16", wl.HEAD_STEP_MSE),
    ("s_T1_B1", 1, 16, 32, 1, 1, "fp16", wl.HEAD_STEP_BCE),            # degenerate: one step, one sample
    ("s_H1", 1, 3, 1, 4, 3, "fp32", wl.HEAD_STEP_BCE),                 # one hidden unit
    ("s_fp16_L3_T1", 3, 8, 40, 1, 5, "fp16", wl.HEAD_STEP_BCE),        # anti-diagonal schedule, a single time step
    ("s_bf16_L9_T3", 9, 8, 24, 3, 4, "bf16", wl.HEAD_STEP_MSE),        # more layers than cells per launch, L > T
    ("s_fp16_L4_last", 4, 10, 72, 7, 9, "fp16", wl.HEAD_LAST_BCE),     # four layers, last-step head, ragged sizes
    ("s_fp16_tile32", 2, 24, 264, 3, 600, "fp16", wl.HEAD_STEP_MSE),   # narrow-layer kernels on 32x32 tiles, ragged both ways
    ("s_bf16_tile32", 1, 40, 264, 2, 600, "bf16", wl.HEAD_STEP_BCE),
]


@pytest.mark.parametrize("spec", SMALL, ids=[s[0] for s in SMALL])
def test_small_shapes(hip, spec):
    name, L, I, H, T, B, dtype, head = spec
    w = wl.Workload(name, L, I, H, T, B, dtype, head, loss_scale=1.0 if dtype == "fp32" else 256.0,
                    target_kind="normal" if head == wl.HEAD_STEP_MSE else "bernoulli", target_p=0.3,
                    data_seed=50 + len(name), weight_seed=60 + len(name))
    _check(w)


def test_small_embedding_text_model(hip):
    w = wl.Workload("s_text", 1, 0, 48, 12, 20, "fp16", wl.HEAD_LAST_BCE, vocab=50, embed_dim=24,
                    loss_scale=1024.0, target_p=0.5, data_seed=77, weight_seed=78)
    _check(w)
    _check(w.with_(dtype="fp32", loss_scale=1.0, name="s_text32"))


def test_small_embedding_two_layers(hip):
    """Embedding front-end under the anti-diagonal schedule: the data gradient of layer 0 (for the
    embedding rows) is still a whole-sequence product, the one of layer 1 arrives step by step."""
    w = wl.Workload("s_text2", 2, 0, 40, 9, 12, "fp16", wl.HEAD_LAST_BCE, vocab=37, embed_dim=16,
                    loss_scale=1024.0, target_p=0.5, data_seed=79, weight_seed=80)
    _check(w)
    _check(w.with_(dtype="bf16", loss_scale=1.0, head=wl.HEAD_STEP_BCE, target_p=0.3, name="s_text2_bf16"))


def test_small_many_workers(hip):
    w = wl.Workload("s_workers", 2, 16, 40, 6, 8, "fp16", wl.HEAD_STEP_BCE, n_workers=5, loss_scale=4096.0,
                    dynamic_scale=True, n_half=4.0, warmup_steps=3, gamma=0.9, data_seed=300, weight_seed=31)
    gpu, ref = _check(w)
    assert gpu["good_steps"] == 1 and gpu["final_scale"] == 4096.0


# ------------------------------------------------------------------ configs 2, 3 at full size
def test_config2_jet_fp16(hip):
    _check(wl.CONFIGS["jet"])


def test_config3_text_fp16(hip):
    _check(wl.CONFIGS["text"])


def test_config2_bf16_variant(hip):
    _check(wl.CONFIGS["jet"].with_(dtype="bf16", loss_scale=1.0, name="jet_bf16"))


# ------------------------------------------------------------------ overflow handling
def test_dynamic_loss_scale_overflow_and_retry(hip):
    """A scale far too large for half precision: the step must be skipped with
    every buffer bit-unchanged and the scale halved until gradients are finite."""
    import torch
    w = wl.Workload("s_overflow", 1, 16, 32, 6, 8, "fp16", wl.HEAD_STEP_BCE, loss_scale=2.0 ** 22,
                    dynamic_scale=True, data_seed=5, weight_seed=6)
    master0, xs, ys = pu.inputs_for(w)
    ts = pu.make_step(w, master0)
    dx, dy = pu.device_batches(w, xs, ys, ts.lp_dtype, ts.dev)
    before = (ts.master.clone(), ts.state1.clone(), ts.params_lp.clone())
    ts.step(dx, dy, 0.01)
    torch.cuda.synchronize()
    assert int(ts.found_inf.item()) == 1
    assert float(ts.loss_scale.item()) == 2.0 ** 21 and int(ts.good_steps.item()) == 0
    assert torch.equal(before[0], ts.master) and torch.equal(before[1], ts.state1) and torch.equal(before[2], ts.params_lp)
    gpu, ref = _check(w)
    assert len(gpu["scales"]) > 1 and gpu["final_scale"] == gpu["scales"][-1]
    # static scale: overflow is reported, the step skipped, the scale kept
    ws = w.with_(dynamic_scale=False)
    ts = pu.make_step(ws, master0)
    ts.step(dx, dy, 0.01)
    torch.cuda.synchronize()
    assert int(ts.found_inf.item()) == 1 and float(ts.loss_scale.item()) == 2.0 ** 22
    assert torch.equal(before[0], ts.master)


# ------------------------------------------------------------------ states in / out
def test_chunked_sequence_with_carried_state(hip):
    import torch
    w = wl.Workload("s_chunk", 2, 24, 40, 8, 12, "fp16", wl.HEAD_STEP_MSE, target_kind="normal", data_seed=9, weight_seed=10)
    master0, xs, ys = pu.inputs_for(w)
    dev = torch.device("cuda:0")
    cfg = pu.make_cfg(w)
    half = pu.make_cfg(w.with_(seq_len=4))
    P = hip.lstm_param_count(cfg)
    par = torch.from_numpy(master0).to(torch.float16).to(dev)
    x = torch.from_numpy(xs[0]).to(torch.float16).to(dev); y = torch.from_numpy(ys[0]).to(dev)
    rb, sb = hip.lstm_workspace_bytes(cfg)
    res = torch.empty(rb, dtype=torch.uint8, device=dev); scr = torch.empty(sb, dtype=torch.uint8, device=dev)
    L, B, H = w.num_layers, w.batch, w.hidden
    loss = torch.zeros(3, device=dev)
    hT = torch.zeros(L, B, H, dtype=torch.float16, device=dev); cT = torch.zeros(L, B, H, device=dev)
    hA = torch.zeros_like(hT); cA = torch.zeros_like(cT); hB = torch.zeros_like(hT); cB = torch.zeros_like(cT)
    hip.lstm_forward(cfg, par, x, y, None, None, res, scr, loss[0:1], hT, cT)
    hip.lstm_forward(half, par, x[:4].contiguous(), y[:4].contiguous(), None, None, res, scr, loss[1:2], hA, cA)
    hip.lstm_forward(half, par, x[4:].contiguous(), y[4:].contiguous(), hA, cA, res, scr, loss[2:3], hB, cB)
    torch.cuda.synchronize()
    assert torch.equal(hT, hB)
    assert torch.allclose(cT, cB, rtol=0, atol=0)
    l = loss.cpu().numpy()
    assert abs(l[0] - 0.5 * (l[1] + l[2])) <= 1e-6 * abs(l[0])
    # against the oracle, including the final states
    params = orc.unflatten(master0, pu.oracle_shapes(w))
    lo, cache = orc.forward(params, L, xs[0].astype(np.float64), ys[0], w.head)
    assert abs(l[0] - lo) <= pu.LOSS_RTOL * abs(lo)
    for k in range(L):
        np.testing.assert_allclose(hT[k].double().cpu().numpy(), cache["layers"][k]["h"][-1], atol=4e-3)
        np.testing.assert_allclose(cT[k].double().cpu().numpy(), cache["layers"][k]["c"][-1], atol=4e-3)
