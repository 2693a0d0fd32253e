"""Stateful truncated BPTT over a long shot and deep stacks (the paper trains on
shots of thousands of steps cut into chunks of 128 with the recurrent state
carried over, and grows capacity by stacking layers: Section "Neural Network
architecture", Table 1)."""
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


def test_long_shot_in_chunks_with_updates(hip):
    """Three chunks of one shot: chunk k starts from the state chunk k-1 ended in, gets
    its own forward + BPTT + SGD-momentum update (gradients do not cross the cut).  The
    oracle does the same with its own carried state; losses, every chunk's gradient and
    the weights after the last update are compared."""
    import torch
    chunk, n_chunks = 16, 3
    w = wl.Workload("shot", 2, 12, 48, chunk * n_chunks, 16, "fp16", wl.HEAD_STEP_BCE, loss_scale=256.0,
                    momentum=0.9, lr0=0.05, data_seed=21, weight_seed=22)
    master0, xs, ys = pu.inputs_for(w)
    wc = w.with_(seq_len=chunk)
    dev = torch.device("cuda:0")
    ts = pu.make_step(wc, master0, dev)
    L, B, H = w.num_layers, w.batch, w.hidden
    x = torch.from_numpy(xs[0]).to(ts.lp_dtype).to(dev)
    y = torch.from_numpy(ys[0]).to(dev)
    h_in = torch.zeros(L, B, H, dtype=ts.lp_dtype, device=dev); c_in = torch.zeros(L, B, H, device=dev)
    h_out = torch.zeros_like(h_in); c_out = torch.zeros_like(c_in)

    shapes = pu.oracle_shapes(wc)
    W_ref = master0.astype(np.float64)
    V_ref = np.zeros_like(W_ref)
    h_ref = np.zeros((L, B, H)); c_ref = np.zeros((L, B, H))
    lr = w.lr0
    for k in range(n_chunks):
        print(f"[case] shot chunk {k}", flush=True)
        xk = x[k * chunk:(k + 1) * chunk].contiguous(); yk = y[k * chunk:(k + 1) * chunk].contiguous()
        hip.lstm_forward(ts.cfg, ts.params_lp, xk, yk, h_in, c_in, ts.reserve, ts.scratch, ts.losses[0:1], h_out, c_out)
        hip.lstm_backward(ts.cfg, ts.params_lp, xk, yk, ts.reserve, ts.scratch, ts.loss_scale, ts.grads[0])
        ts.update(lr)
        torch.cuda.synchronize()
        assert int(ts.found_inf.item()) == 0
        # oracle: same chunk, its own carried state, weights rounded to storage like the working copy
        params = orc.unflatten(orc.round_storage(W_ref, "fp16"), shapes)
        xo = xs[0][k * chunk:(k + 1) * chunk].astype(np.float64); yo = ys[0][k * chunk:(k + 1) * chunk]
        loss, cache = orc.forward(params, L, xo, yo, w.head, h_ref, c_ref)
        g = orc.flatten(orc.backward(params, L, cache, 1.0), shapes)
        assert abs(float(ts.losses[0].item()) - loss) <= pu.LOSS_RTOL * abs(loss)
        got = ts.grads[0].double().cpu().numpy() / w.loss_scale
        pu.assert_grads_close(got, g, shapes, pu.GRAD_RTOL["fp16"], f"chunk {k}")
        W_ref, V_ref = orc.sgd_momentum_update(W_ref, V_ref, g, lr, w.momentum)
        h_ref = np.stack([cache["layers"][l]["h"][-1] for l in range(L)])
        c_ref = np.stack([cache["layers"][l]["c"][-1] for l in range(L)])
        np.testing.assert_allclose(h_out.double().cpu().numpy(), h_ref, atol=6e-3)
        np.testing.assert_allclose(c_out.double().cpu().numpy(), c_ref, atol=6e-3)
        h_in, h_out = h_out, h_in
        c_in, c_out = c_out, c_in
    dW = np.abs(W_ref - master0).max()
    np.testing.assert_allclose(ts.master.double().cpu().numpy(), W_ref, atol=pu.GRAD_RTOL["fp16"] * dW + 2e-7)


@pytest.mark.parametrize("dtype,L", [("fp16", 4), ("bf16", 12), ("fp32", 6)])
def test_deep_stack(hip, dtype, L):
    """Capacity grows by stacking layers of 200 units (Table 1): a deep stack at the
    paper's width, short sequence so that the fp64 oracle stays within seconds.
    With freshly initialised weights the gradient shrinks by about a factor of ten per
    layer; at twelve layers the bottom gradients (1e-12) and the top ones (0.4) no longer
    fit the half-precision range under any single loss scale, so the fp16 case stops at
    four layers with the scale at 2^15, and the twelve-layer case runs in bf16."""
    w = wl.Workload(f"deep_{dtype}", L, 9, 200, 12, 64, dtype, wl.HEAD_STEP_BCE,
                    loss_scale=1.0 if dtype != "fp16" else 32768.0, data_seed=31, weight_seed=32)
    print(f"[case] deep stack {dtype} L={L}", flush=True)
    got = pu.run_gpu_step(w)
    want = pu.run_oracle_step(w)
    pu.assert_step_close(w, got, want)


STATE_CASES = [
    ("narrow", 2, 24, 200, 4, 128, "fp16"),
    ("narrow_ragged_bf16", 3, 9, 104, 4, 100, "bf16"),
    ("wide", 1, 40, 1024, 3, 128, "fp16"),
    ("wide_tiles_two_chunks", 2, 40, 1024, 40, 256, "fp16"),
    ("wide_tiles_64_rows_bf16", 2, 24, 1152, 3, 192, "bf16"),
    ("wide_tiles_2048_packed_copies_only", 2, 256, 2048, 4, 256, "fp16"),
    ("rows2048", 2, 64, 200, 3, 2048, "fp16"),
    ("rows1024_h520", 1, 8, 520, 3, 1024, "fp16"),
    ("odd_sizes", 2, 5, 33, 4, 17, "fp16"),
    ("fp32", 2, 5, 72, 4, 70, "fp32"),
]


@pytest.mark.parametrize("spec", STATE_CASES, ids=[c[0] for c in STATE_CASES])
def test_nonzero_initial_state(hip, spec):
    """A chunk that starts from a given (h_0, c_0) on every kernel family: loss, gradients and the state handed
    on, (h_T, c_T), against the oracle started from the same state.  The workspaces hold NaN bytes before the call."""
    import torch
    name, L, I, H, T, B, dtype = spec
    w = wl.Workload(f"state_{name}", L, I, H, T, B, dtype, wl.HEAD_STEP_BCE, loss_scale=1.0 if dtype != "fp16" else 512.0,
                    target_p=0.4, data_seed=41, weight_seed=42)
    print(f"[case] {w.name}: L={L} I={I} H={H} T={T} B={B} {dtype}", flush=True)
    master0, xs, ys = pu.inputs_for(w)
    dev = torch.device("cuda:0")
    ts = pu.make_step(w, master0, dev)
    for buf in list(ts.reserves) + list(ts.scratches):
        buf.fill_(255)
    rng = np.random.default_rng(43)
    h0 = torch.from_numpy(rng.uniform(-0.9, 0.9, (L, B, H)).astype(np.float32)).to(ts.lp_dtype).to(dev)   # storage-rounded
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
    got = ts.grads[0].double().cpu().numpy() / w.loss_scale
    assert np.all(np.isfinite(got))
    pu.assert_grads_close(got, g, shapes, pu.GRAD_RTOL[dtype], "chunk with initial state")
    h_ref = np.stack([cache["layers"][l]["h"][-1] for l in range(L)])
    c_ref = np.stack([cache["layers"][l]["c"][-1] for l in range(L)])
    atol = {"fp16": 6e-3, "bf16": 4e-2, "fp32": 1e-5}[dtype]
    np.testing.assert_allclose(hT.double().cpu().numpy(), h_ref, atol=atol)
    np.testing.assert_allclose(cT.double().cpu().numpy(), c_ref, atol=atol * 4)
