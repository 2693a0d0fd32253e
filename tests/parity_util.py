"""Shared helpers of the parity tests, the smoke check and the benchmark's
CPU-baseline leg: run one training step on the HIP path and on the CPU oracle
from the same seeded inputs, and compare.

Tolerances (stated by the task for this method): loss 1e-3 relative;
gradients 1e-4 relative for an fp32 run and 2e-2 relative for an fp16/bf16
run, measured per parameter tensor as ||g_hip - g_ref||_2 / ||g_ref||_2 and
as max|g_hip - g_ref| <= tol * max|g_ref| (both per tensor).  A 16-bit run may
exceed that on a tensor whose elements are sums of cancelling terms; such a
tensor must then stay, element by element, inside a bound derived from the
terms of its sums (rounding_bound), and the same shape must pass in fp32.
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
def term_magnitudes(w: wl.Workload, params, cache, trace):
    """For every gradient element, what its sum is made of.  A weight gradient is a sum over all
    (t, b) rows of products (dW[j,k] = sum_r da[r,j] x[r,k], db[j] = sum_r da[r,j], ...).  Returned per
    tensor, flat in parameter order, from the oracle's own fp64 intermediates:
      A[j] = sum_r |term_r|            (what one relative rounding error per term can add up to)
      X[j] = sum_r |other factor_r|    (what one absolute error in every stored da can add up to)."""
    T, B = cache["T"], cache["B"]
    A, X = {}, {}
    for l in range(w.num_layers):
        lay = cache["layers"][l]
        da = np.abs(trace[f"da{l}"]).reshape(T * B, -1)
        inp = np.abs(lay["inp"]).reshape(T * B, -1)
        hp = np.abs(lay["h"][:-1]).reshape(T * B, -1)
        A[f"W{l}"], X[f"W{l}"] = da.T @ inp, np.broadcast_to(inp.sum(axis=0), (da.shape[1], inp.shape[1]))
        A[f"U{l}"], X[f"U{l}"] = da.T @ hp, np.broadcast_to(hp.sum(axis=0), (da.shape[1], hp.shape[1]))
        A[f"b{l}"], X[f"b{l}"] = da.sum(axis=0), np.full(da.shape[1], float(T * B))
    top = np.abs(cache["layers"][-1]["h"][1:])
    dz = np.abs(trace["dz"])
    if cache["head"] == orc.HEAD_FC_HINGE:
        act, dpre = np.abs(cache["fc_act"]).reshape(T * B, -1), np.abs(trace["d_pre"]).reshape(T * B, -1)
        A["w_head"] = dz.reshape(-1) @ act
        A["W_fc"], X["W_fc"] = dpre.T @ top.reshape(T * B, -1), np.broadcast_to(top.reshape(T * B, -1).sum(axis=0), (dpre.shape[1], top.shape[2]))
        A["b_fc"], X["b_fc"] = dpre.sum(axis=0), np.full(dpre.shape[1], float(T * B))
    elif cache["head"] == orc.HEAD_LAST_BCE:
        A["w_head"] = dz @ top[T - 1]
    else:
        A["w_head"] = np.einsum("tb,tbh->h", dz, top)
    A["b_head"] = np.array([dz.sum()])
    if cache["ids"] is not None:
        dE = np.zeros_like(params["E"])
        np.add.at(dE, cache["ids"].reshape(-1), np.abs(trace["d_input"]).reshape(T * B, -1))
        A["E"] = dE
        cnt = np.zeros(params["E"].shape[0])
        np.add.at(cnt, cache["ids"].reshape(-1), 1.0)
        X["E"] = np.broadcast_to(cnt[:, None], dE.shape)
    return A, X


def run_oracle_step(w: wl.Workload, with_terms: bool = False):
    master0, xs, ys = inputs_for(w)
    shapes = oracle_shapes(w)
    params = orc.unflatten(master0, shapes)
    losses, grads, terms_a, terms_x = [], [], [], []
    for x, y in zip(xs, ys):
        loss, cache = orc.forward(params, w.num_layers, x if w.vocab else x.astype(np.float64), y, w.head)
        trace = {} if with_terms else None
        g = orc.backward(params, w.num_layers, cache, 1.0, trace)
        losses.append(loss)
        grads.append(orc.flatten(g, shapes))
        if with_terms:
            A, X = term_magnitudes(w, params, cache, trace)
            terms_a.append(orc.flatten(A, shapes))
            terms_x.append(orc.flatten({n: X.get(n, np.zeros(sh)) for n, sh in shapes}, shapes))
    grads = np.stack(grads)
    avg, _ = orc.grad_average(grads, 1.0)
    lr = orc.lr_schedule(w.lr0, w.n_workers, w.n_half, EFF_LR_MAX, w.warmup_steps, w.gamma, 0)
    W, Hb = orc.sgd_momentum_update(master0.astype(np.float64), np.zeros_like(avg), avg, lr, w.momentum)
    out = dict(losses=np.array(losses), grads=grads, avg=avg, master=W, state1=Hb, lr=lr,
               max_abs_grad=float(np.max(np.abs(grads))), shapes=shapes)
    if with_terms:
        out["terms_a"], out["terms_x"] = np.stack(terms_a), np.stack(terms_x)
    return out


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


# Storage rounding, for the bound derived from the terms of a gradient's sum (below).
UNIT_ROUNDOFF = {"fp16": 2.0 ** -11, "bf16": 2.0 ** -8, "fp32": 2.0 ** -24}     # largest relative error of one rounding
SUBNORMAL_HALF_QUANTUM = {"fp16": 2.0 ** -25, "bf16": 0.0, "fp32": 0.0}         # largest absolute error below the normal range
ROUNDINGS_PER_TERM = 4.0     # see rounding_bound()


def _roundings(w: wl.Workload, shapes):
    """Per element: how many roundings a term of that tensor's sums has been through.  Four inside its own
    layer (the stored da, the gate and cell values in its product, the incoming dh, the other factor); the
    gradient entering layer l has also crossed the L-1-l layers above it, each of which stored its own da
    and the dX it handed down (twice four more per layer crossed: measured on 4-layer stacks, a layer-1
    bias gradient needs 12 where 20 is allowed); the embedding table sits one more product below layer 0."""
    out = []
    for name, shape in shapes:
        crossed = 0
        if name[0] in "WUb" and name[1:].isdigit():
            crossed = w.num_layers - 1 - int(name[1:])
        elif name == "E":
            crossed = w.num_layers
        out.append(np.full(int(np.prod(shape)), ROUNDINGS_PER_TERM * (1 + 2 * crossed)))
    return np.concatenate(out)


def rounding_bound(w: wl.Workload, terms_a, terms_x, scale, shapes=None):
    """Element-wise bound on what storage rounding alone can do to a gradient.

    Element j is a sum over the T*B rows, g_j = sum_r da[r,j] * x[r,k].  The 16-bit modes store da (times
    the loss scale S), the gates and c_t it is computed from, the hidden states and the gradient handed
    down from the layer above in the storage type, each rounded to nearest: every term carries a few
    relative errors of at most u (unit round-off), and, in half precision, an absolute error of at most
    2^-25 on the stored S*da once it falls below the normal range (what the loss multiplier of Section
    "Performance evaluation" is there to prevent).  To first order
        |error_j| <= c * (u * sum_r |term_r|  +  2^-25 / S * sum_r |x[r,k]|)
    with c the number of roundings a term goes through (_roundings: 4 in the top layer, 8 more per layer
    the gradient has crossed on its way down; the measured cases need at most 60 % of it).
    The sums come from the oracle's fp64 intermediates.  Where |g_j| << sum_r |term_r| (cancellation:
    bias gradients under a zero-mean loss derivative, the weights of a single input feature) the bound
    exceeds the plain relative tolerance; elsewhere it is far below it."""
    u = UNIT_ROUNDOFF[w.dtype]
    eta = SUBNORMAL_HALF_QUANTUM[w.dtype] / float(scale)
    c = _roundings(w, shapes if shapes is not None else oracle_shapes(w))
    return c * (u * np.asarray(terms_a) + eta * np.asarray(terms_x))


def assert_grads_close(got, ref, shapes, tol, what="", bound=None, used=None):
    """Per tensor: l2-relative and largest-element-relative error within tol.  With `bound` (element-wise,
    from rounding_bound) a tensor over tol still passes if EVERY element's error is within
    max(tol * max|ref|, bound_j) and the l2 norm of the error within max(tol * ||ref||, ||bound||);
    `used` collects the tensors that needed it."""
    errs = tensor_errors(got, ref, shapes)
    bad = {k: v for k, v in errs.items() if not (v[0] <= tol and v[1] <= tol)}
    if bad and bound is not None:
        off = 0
        for name, shape in shapes:
            n = int(np.prod(shape))
            if name in bad:
                d = np.abs(got[off:off + n] - ref[off:off + n])
                lim = np.maximum(tol * np.max(np.abs(ref[off:off + n])), bound[off:off + n])
                l2_lim = max(tol * np.linalg.norm(ref[off:off + n]), np.linalg.norm(bound[off:off + n]))
                if np.all(d <= lim) and np.linalg.norm(d) <= l2_lim:
                    kappa = float(np.max(bound[off:off + n]) / max(np.max(np.abs(ref[off:off + n])), 1e-300))
                    if used is not None:
                        used.append((what, name, bad[name], kappa))
                    del bad[name]
            off += n
    assert not bad, f"{what} gradient mismatch (l2 rel, max rel) > {tol}: {bad}"
    return errs


def assert_step_close(w: wl.Workload, gpu, ref, used=None):
    """ref from run_oracle_step(w, with_terms=True) switches the derived rounding bound on for tensors
    whose sums cancel (see rounding_bound); `used` then lists the tensors that needed it."""
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
    S = gpu["scales"][-1]
    bounds = None
    if "terms_a" in ref and w.dtype != "fp32":
        bounds = [rounding_bound(w, ref["terms_a"][k], ref["terms_x"][k], S) for k in range(w.n_workers)]
    for k in range(w.n_workers):
        assert_grads_close(gpu["grads"][k], ref["grads"][k], shapes, tol, f"worker {k}", bounds[k] if bounds else None, used)
    # the average of N gradients: its error is at most the mean of theirs
    avg_bound = np.mean(bounds, axis=0) if bounds else None
    assert_grads_close(gpu["avg"], ref["avg"], shapes, tol, "averaged", avg_bound, used)
    # learning rate, master weights after Eq. 1-2, working copy
    assert abs(gpu["lr"] - ref["lr"]) <= 1e-6 * abs(ref["lr"])
    dW = ref["master"] - gpu["master0"]
    allow = tol * np.max(np.abs(dW))
    if avg_bound is not None:
        allow = np.maximum(allow, gpu["lr"] * avg_bound)      # first step from zero momentum: dW = -lr * g
    bound = allow + 1.2e-7 * np.abs(ref["master"]) + 1e-12
    assert np.all(np.abs(gpu["master"] - ref["master"]) <= bound), "master weights after update differ"
    np.testing.assert_array_equal(gpu["params_lp"], orc.round_storage(gpu["master"], w.dtype),
                                  err_msg="working copy is not the round-to-nearest-even cast of the master weights")
