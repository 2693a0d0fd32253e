"""Shared helpers of the parity tests, the smoke check and the benchmark's
CPU-baseline leg: run one training step on the HIP path and on the CPU oracle
from the same seeded inputs, and compare.

Tolerances (stated by the task for this method): loss 1e-3 relative;
gradients 1e-4 relative for an fp32 run and 2e-2 relative for an fp16/bf16
run, measured per parameter tensor as ||g_hip - g_ref||_2 / ||g_ref||_2 and
element-wise as max|g_hip - g_ref| <= tol * max|g_ref|.
"""
from __future__ import annotations

import numpy as np

import workloads as wl


class _LazyOracle:
    """The CPU oracle, imported on first use: code that only drives the HIP path through the
    helpers below (bench.py's timed region) never loads it."""
    _mod = None

    def __getattr__(self, name):
        if _LazyOracle._mod is None:
            from oracle import lstm_oracle
            _LazyOracle._mod = lstm_oracle
        return getattr(_LazyOracle._mod, name)


orc = _LazyOracle()

LOSS_RTOL = 1e-3
GRAD_RTOL = {"fp32": 1e-4, "fp16": 2e-2, "bf16": 2e-2}
LP_MAX = {"fp16": 65504.0, "bf16": 3.3895313892515355e38, "fp32": 3.4028234663852886e38}
EFF_LR_MAX = 0.1


def oracle_shapes(w: wl.Workload):
    return orc.param_shapes(w.num_layers, w.input_dim, w.hidden, w.vocab, w.embed_dim, w.fc_units)


def inputs_for(w: wl.Workload):
    """Seeded inputs, rounded once to the storage type (returned as fp32/ints)."""
    master0 = wl.round_to_storage(wl.make_params(w), w.dtype)
    xs, ys = [], []
    for k in range(w.n_workers):
        x, y = wl.make_batch(w, k)
        if w.vocab == 0:
            x = wl.round_to_storage(x, w.dtype)
        xs.append(x)
        ys.append(y)
    return master0, xs, ys


# ------------------------------------------------------------------ HIP path
def make_cfg(w: wl.Workload):
    import paper_1912_00286_amd as hip
    return hip.LstmConfig(num_layers=w.num_layers, input_dim=max(w.input_dim, 0), hidden=w.hidden, seq_len=w.seq_len,
                          batch=w.batch, dtype=wl.DTYPE_CODE[w.dtype], head=w.head, out_dim=1, vocab=w.vocab,
                          embed_dim=w.embed_dim, head_hidden=w.fc_units)


def make_opt(w: wl.Workload, kind=0):
    import paper_1912_00286_amd as hip
    return hip.OptimizerConfig(kind=kind, momentum=w.momentum, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0,
                               dynamic_scale=1 if w.dynamic_scale else 0, scale_backoff=0.5, scale_growth=2.0,
                               growth_interval=2000)


def lr_for(w: wl.Workload, index: int) -> float:
    import paper_1912_00286_amd as hip
    return hip.lr_schedule(w.lr0, w.n_workers, w.n_half, EFF_LR_MAX, w.warmup_steps, w.gamma, index)


def device_batches(w: wl.Workload, xs, ys, lp_dtype, dev):
    import torch
    dx, dy = [], []
    for x, y in zip(xs, ys):
        if w.vocab > 0:
            dx.append(torch.from_numpy(x.astype(np.int32)).to(dev))
        else:
            dx.append(torch.from_numpy(x).to(lp_dtype).to(dev).contiguous())
        dy.append(torch.from_numpy(y).to(dev).contiguous())
    return dx, dy


def make_step(w: wl.Workload, master0, dev="cuda:0", n_streams=1, batched=False):
    import paper_1912_00286_amd as hip
    return hip.TrainingStep(make_cfg(w), make_opt(w), w.n_workers, master0, w.loss_scale, dev, n_streams=n_streams,
                            batched=batched)


def run_gpu_step(w: wl.Workload, max_retries: int = 20, batched: bool = False):
    """One training iteration on the HIP path (retrying after overflow when the
    loss scale is dynamic).  Returns host copies of everything comparable."""
    import torch
    master0, xs, ys = inputs_for(w)
    ts = make_step(w, master0, batched=batched)
    dx, dy = device_batches(w, xs, ys, ts.lp_dtype, ts.dev)
    lr = lr_for(w, 0)
    scales, flags = [], []
    for attempt in range(max_retries):
        scales.append(float(ts.loss_scale.item()))
        ts.step(dx, dy, lr)
        torch.cuda.synchronize()
        flags.append(int(ts.found_inf.item()))
        if not flags[-1] or not w.dynamic_scale:
            break
    S = scales[-1]
    return dict(losses=ts.losses.double().cpu().numpy(),
                grads=ts.grads.double().cpu().numpy() / S,
                avg=ts.avg.double().cpu().numpy(), found_inf=flags, scales=scales,
                master=ts.master.double().cpu().numpy(), params_lp=ts.params_lp.double().cpu().numpy(),
                state1=ts.state1.double().cpu().numpy(), final_scale=float(ts.loss_scale.item()),
                good_steps=int(ts.good_steps.item()), lr=lr, master0=master0.astype(np.float64))


# ------------------------------------------------------------------ oracle
def run_oracle_step(w: wl.Workload):
    master0, xs, ys = inputs_for(w)
    shapes = oracle_shapes(w)
    params = orc.unflatten(master0, shapes)
    losses, grads = [], []
    for x, y in zip(xs, ys):
        loss, cache = orc.forward(params, w.num_layers, x if w.vocab else x.astype(np.float64), y, w.head)
        g = orc.backward(params, w.num_layers, cache, 1.0)
        losses.append(loss)
        grads.append(orc.flatten(g, shapes))
    grads = np.stack(grads)
    avg, _ = orc.grad_average(grads, 1.0)
    lr = orc.lr_schedule(w.lr0, w.n_workers, w.n_half, EFF_LR_MAX, w.warmup_steps, w.gamma, 0)
    W, Hb = orc.sgd_momentum_update(master0.astype(np.float64), np.zeros_like(avg), avg, lr, w.momentum)
    return dict(losses=np.array(losses), grads=grads, avg=avg, master=W, state1=Hb, lr=lr,
                max_abs_grad=float(np.max(np.abs(grads))), shapes=shapes)


# ------------------------------------------------------------------ comparison
def tensor_errors(got, ref, shapes):
    out, off = {}, 0
    for name, shape in shapes:
        n = int(np.prod(shape))
        a, b = got[off:off + n], ref[off:off + n]
        nb = np.linalg.norm(b)
        l2 = np.linalg.norm(a - b) / nb if nb > 0 else np.linalg.norm(a - b)
        mx = np.max(np.abs(b))
        el = np.max(np.abs(a - b)) / mx if mx > 0 else np.max(np.abs(a - b))
        out[name] = (float(l2), float(el))
        off += n
    return out


def assert_grads_close(got, ref, shapes, tol, what=""):
    errs = tensor_errors(got, ref, shapes)
    bad = {k: v for k, v in errs.items() if not (v[0] <= tol and v[1] <= tol)}
    assert not bad, f"{what} gradient mismatch (l2 rel, max rel) > {tol}: {bad}"
    return errs


def assert_step_close(w: wl.Workload, gpu, ref):
    tol = GRAD_RTOL[w.dtype]
    shapes = ref["shapes"]
    # overflow decisions: every attempt but the last must have overflowed
    lpmax = LP_MAX[w.dtype]
    for S, flag in zip(gpu["scales"], gpu["found_inf"]):
        peak = S * ref["max_abs_grad"]
        if peak > 1.02 * lpmax:
            assert flag == 1, f"scale {S}: scaled gradient peak {peak} must overflow"
        elif peak < 0.98 * lpmax:
            assert flag == 0, f"scale {S}: scaled gradient peak {peak} must not overflow"
    assert gpu["found_inf"][-1] == 0, "step never produced finite gradients"
    assert np.all(np.isfinite(gpu["grads"]))
    # loss
    rel = np.abs(gpu["losses"] - ref["losses"]) / np.abs(ref["losses"])
    assert np.all(rel <= LOSS_RTOL), f"loss mismatch: {gpu['losses']} vs {ref['losses']}"
    # per-worker gradients and their average
    for k in range(w.n_workers):
        assert_grads_close(gpu["grads"][k], ref["grads"][k], shapes, tol, f"worker {k}")
    assert_grads_close(gpu["avg"], ref["avg"], shapes, tol, "averaged")
    # learning rate, master weights after Eq. 1-2, working copy
    assert abs(gpu["lr"] - ref["lr"]) <= 1e-6 * abs(ref["lr"])
    dW = ref["master"] - gpu["master0"]
    bound = tol * np.max(np.abs(dW)) + 1.2e-7 * np.abs(ref["master"]) + 1e-12
    assert np.all(np.abs(gpu["master"] - ref["master"]) <= bound), "master weights after update differ"
    np.testing.assert_array_equal(gpu["params_lp"], orc.round_storage(gpu["master"], w.dtype),
                                  err_msg="working copy is not the round-to-nearest-even cast of the master weights")
