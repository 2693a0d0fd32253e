"""CPU fp64 oracle for one data-parallel worker's stacked-LSTM training step.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
HIP path is checked against.  It shares no code with the HIP path and must
never be imported by the product package; only tests, the smoke check and the
benchmark's cpu_baseline leg call it.

What it follows (paper: "Training distributed deep recurrent neural networks
with mixed precision on GPU clusters"):
  * Section "Neural Network architecture": a stack of LSTM layers (forget-gate
    LSTM of Gers et al., logistic gates) followed by a per-time-slice output
    layer; one iteration = fprop, loss, bprop (BPTT), weight update.
  * Section "Distributed computing framework", steps 3-5 and Eq. 1-2: each
    worker computes raw gradients on its mini-batch, the gradients are summed
    and averaged, and SGD with momentum  H_k = m H_{k-1} - lambda dW,
    W_k = W_{k-1} + H_k  is applied to the global weights.
  * Section "Learning rate schedule", Eq. 3-4 and the clipping rule.
  * Section "Half-precision training modes" / "Performance evaluation": the
    loss is multiplied by a scalar alpha before bprop (Eq. 6); half precision
    has largest finite value 65504; gradients are exchanged in half precision.

The paper prints no LSTM equations; the readings taken here (gate order
i,f,g,o; one bias vector per layer; zero initial state; mean-reduced loss;
sum-then-divide averaging) are listed in the design document.

Every array is float64.  The time loop and the layer loop are written out in
the order the algorithm states them; numpy's matmul is the only library
primitive used as a step.

Pins (tests/test_oracle_*.py): central finite differences, torch.nn.LSTM +
autograd as a library special case, zero-weight closed forms, a hand-computed
scalar cell, tanh odd symmetry, loss-scale invariance, the big-batch
equivalence of worker averaging, batch permutation, chunked-sequence
consistency, closed forms of Eq. 1-4, and IEEE half facts.
Full-size results of the five benchmark configurations have no printed values
to compare with: parity unpinned beyond the pins above.
"""
from __future__ import annotations

import numpy as np

HEAD_STEP_BCE = 1
HEAD_LAST_BCE = 2
HEAD_STEP_MSE = 3
HEAD_FC_HINGE = 4           # the paper's own head: see forward()

FP16_MAX = 65504.0          # Section "Half-precision training modes"


# --------------------------------------------------------------------------
# parameter bookkeeping
# --------------------------------------------------------------------------
def param_shapes(num_layers, input_dim, hidden, vocab=0, embed_dim=0, fc_units=0):
    """Ordered (name, shape) list of the flat parameter vector:
    [E[V,D]] then per layer W[4H,I_l], U[4H,H], b[4H], then w_head[H], b_head[1].
    Rows of W, U, b are grouped by gate in the order i, f, g, o.
    With fc_units = F > 0 (the head of Fig. 2) the tail is W_fc[F,H], b_fc[F],
    w_head[F], b_head[1]."""
    shapes = []
    first = input_dim
    if vocab > 0:
        shapes.append(("E", (vocab, embed_dim)))
        first = embed_dim
    G = 4 * hidden
    for l in range(num_layers):
        shapes.append((f"W{l}", (G, first if l == 0 else hidden)))
        shapes.append((f"U{l}", (G, hidden)))
        shapes.append((f"b{l}", (G,)))
    if fc_units > 0:
        shapes.append(("W_fc", (fc_units, hidden)))
        shapes.append(("b_fc", (fc_units,)))
        shapes.append(("w_head", (fc_units,)))
    else:
        shapes.append(("w_head", (hidden,)))
    shapes.append(("b_head", (1,)))
    return shapes


def param_count(num_layers, input_dim, hidden, vocab=0, embed_dim=0, fc_units=0):
    return sum(int(np.prod(s)) for _, s in param_shapes(num_layers, input_dim, hidden, vocab, embed_dim, fc_units))


def unflatten(flat, shapes):
    out, off = {}, 0
    flat = np.asarray(flat, dtype=np.float64)
    for name, shape in shapes:
        n = int(np.prod(shape))
        out[name] = flat[off:off + n].reshape(shape).copy()
        off += n
    assert off == flat.size, (off, flat.size)
    return out


def flatten(tensors, shapes):
    return np.concatenate([np.asarray(tensors[name], dtype=np.float64).reshape(-1) for name, _ in shapes])


# --------------------------------------------------------------------------
# elementary functions
# --------------------------------------------------------------------------
def sigmoid(a):
    """Logistic function 1/(1+e^-a), evaluated without overflow."""
    a = np.asarray(a, dtype=np.float64)
    e = np.exp(-np.abs(a))
    return np.where(a >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


# --------------------------------------------------------------------------
# forward pass (fprop + loss)
# --------------------------------------------------------------------------
def forward(params, num_layers, x, targets, head, h0=None, c0=None):
    """Forward through time for all layers, then the head and the mean loss.

    params : dict name -> float64 array (see param_shapes)
    x      : float64 [T,B,I], or integer token ids [T,B] when params has "E"
    targets: float64 [T,B,1] (per-step heads) or [B,1] (last-step head)
    h0, c0 : optional [L,B,H] initial states (zero when None)
    returns (loss, cache); loss is the unscaled mean over all head outputs.
    """
    ids = None
    if "E" in params:
        ids = np.asarray(x)
        x = params["E"][ids]                      # x_t,b = E[id_t,b]
    x = np.asarray(x, dtype=np.float64)
    T, B, _ = x.shape
    layers = []
    inp = x
    for l in range(num_layers):
        W, U, b = params[f"W{l}"], params[f"U{l}"], params[f"b{l}"]
        H = U.shape[1]
        h_prev = np.zeros((B, H)) if h0 is None else np.asarray(h0[l], dtype=np.float64)
        c_prev = np.zeros((B, H)) if c0 is None else np.asarray(c0[l], dtype=np.float64)
        gi = np.empty((T, B, H)); gf = np.empty((T, B, H))
        gg = np.empty((T, B, H)); go = np.empty((T, B, H))
        cs = np.empty((T + 1, B, H)); hs = np.empty((T + 1, B, H))
        cs[0], hs[0] = c_prev, h_prev
        for t in range(T):
            a = inp[t] @ W.T + hs[t] @ U.T + b    # [B,4H]
            i = sigmoid(a[:, 0 * H:1 * H])
            f = sigmoid(a[:, 1 * H:2 * H])
            g = np.tanh(a[:, 2 * H:3 * H])
            o = sigmoid(a[:, 3 * H:4 * H])
            c = f * cs[t] + i * g
            h = o * np.tanh(c)
            gi[t], gf[t], gg[t], go[t] = i, f, g, o
            cs[t + 1], hs[t + 1] = c, h
        layers.append(dict(inp=inp, i=gi, f=gf, g=gg, o=go, c=cs, h=hs))
        inp = hs[1:]
    top = inp                                      # [T,B,H]
    w_head, b_head = params["w_head"], params["b_head"]
    y = np.asarray(targets, dtype=np.float64)
    fc_pre = fc_act = None
    if head == HEAD_FC_HINGE:
        # Fig. 2: a fully connected ReLU layer applied to every temporal slice, then one
        # output per slice; hinge loss max(0, 1 - t*y) with labels t = +-1 (Eq. 6 without
        # its multiplier, which backward() applies).  Subgradient 0 at the kink.
        fc_pre = top @ params["W_fc"].T + params["b_fc"]      # [T,B,F]
        fc_act = np.maximum(fc_pre, 0.0)
        z = fc_act @ w_head + b_head[0]                        # [T,B]
        yy = y.reshape(T, B)
        margin = 1.0 - yy * z
        ell = np.maximum(margin, 0.0)
        dldz = np.where(margin > 0.0, -yy, 0.0)
    elif head == HEAD_LAST_BCE:
        z = top[T - 1] @ w_head + b_head[0]        # [B]
        yy = y.reshape(B)
    else:
        z = top @ w_head + b_head[0]               # [T,B]
        yy = y.reshape(T, B)
    M = z.size
    if head in (HEAD_STEP_BCE, HEAD_LAST_BCE):
        # -y log s(z) - (1-y) log(1-s(z)), written without overflow
        ell = np.maximum(z, 0.0) - z * yy + np.log1p(np.exp(-np.abs(z)))
        dldz = sigmoid(z) - yy
    elif head == HEAD_STEP_MSE:
        ell = (z - yy) ** 2
        dldz = 2.0 * (z - yy)
    elif head != HEAD_FC_HINGE:
        raise ValueError(f"unknown head {head}")
    loss = float(ell.sum() / M)
    cache = dict(layers=layers, ids=ids, z=z, dldz=dldz / M, head=head, T=T, B=B, fc_pre=fc_pre, fc_act=fc_act)
    return loss, cache


# --------------------------------------------------------------------------
# backward pass (bprop = BPTT), loss multiplied by the scale first
# --------------------------------------------------------------------------
def backward(params, num_layers, cache, loss_scale=1.0, trace=None):
    """Gradients of (loss_scale * loss) w.r.t. every parameter tensor.

    Returns dict name -> float64 array holding S * dloss/dtheta (the *scaled*
    raw gradient a worker would hand to the exchange step).

    trace: optional dict that receives intermediates of the pass (no effect on
    the result): "dz" [T,B] or [B], "d_top" [T,B,H] (gradient entering the top
    layer), and per layer "da{l}" [T,B,4H], the gradient of the gate
    pre-activations whose sums over (t, b) are the weight gradients.
    """
    T, B = cache["T"], cache["B"]
    S = float(loss_scale)
    grads = {k: np.zeros_like(v) for k, v in params.items()}
    w_head = params["w_head"]
    top = cache["layers"][-1]["h"][1:]             # [T,B,H]
    H = top.shape[2]
    dz = S * cache["dldz"]                         # seed: d(S*loss)/dz
    d_above = np.zeros((T, B, H))
    if cache["head"] == HEAD_FC_HINGE:
        a = cache["fc_act"]                                     # [T,B,F]
        grads["w_head"] = np.einsum("tb,tbf->f", dz, a)
        grads["b_head"] = np.array([dz.sum()])
        d_pre = dz[:, :, None] * w_head[None, None, :] * (cache["fc_pre"] > 0.0)   # through the ReLU
        grads["W_fc"] = np.einsum("tbf,tbh->fh", d_pre, top)
        grads["b_fc"] = d_pre.sum(axis=(0, 1))
        H = top.shape[2]
        d_above = d_pre @ params["W_fc"]                         # [T,B,H]
    elif cache["head"] == HEAD_LAST_BCE:
        grads["w_head"] = dz @ top[T - 1]
        grads["b_head"] = np.array([dz.sum()])
        d_above[T - 1] = np.outer(dz, w_head)
    else:
        grads["w_head"] = np.einsum("tb,tbh->h", dz, top)
        grads["b_head"] = np.array([dz.sum()])
        d_above = dz[:, :, None] * w_head[None, None, :]
    if trace is not None:
        trace["dz"] = dz
        trace["d_top"] = d_above
        if cache["head"] == HEAD_FC_HINGE:
            trace["d_pre"] = d_pre
    for l in range(num_layers - 1, -1, -1):
        lay = cache["layers"][l]
        W, U = params[f"W{l}"], params[f"U{l}"]
        Hl = U.shape[1]
        inp = lay["inp"]
        d_inp = np.zeros_like(inp)
        dh_rec = np.zeros((B, Hl))
        dc_rec = np.zeros((B, Hl))
        dW = np.zeros_like(W); dU = np.zeros_like(U); db = np.zeros(4 * Hl)
        for t in range(T - 1, -1, -1):
            i, f, g, o = lay["i"][t], lay["f"][t], lay["g"][t], lay["o"][t]
            c_t, c_prev, h_prev = lay["c"][t + 1], lay["c"][t], lay["h"][t]
            tc = np.tanh(c_t)
            dh = d_above[t] + dh_rec
            do = dh * tc
            dc = dc_rec + dh * o * (1.0 - tc * tc)
            di = dc * g
            dg = dc * i
            df = dc * c_prev
            dc_rec = dc * f
            da = np.concatenate([di * i * (1.0 - i),
                                 df * f * (1.0 - f),
                                 dg * (1.0 - g * g),
                                 do * o * (1.0 - o)], axis=1)   # [B,4H]
            if trace is not None:
                trace.setdefault(f"da{l}", np.empty((T, B, 4 * Hl)))[t] = da
            d_inp[t] = da @ W
            dh_rec = da @ U
            dW += da.T @ inp[t]
            dU += da.T @ h_prev
            db += da.sum(axis=0)
        grads[f"W{l}"], grads[f"U{l}"], grads[f"b{l}"] = dW, dU, db
        d_above = d_inp
    if trace is not None:
        trace["d_input"] = d_above
    if cache["ids"] is not None:
        dE = np.zeros_like(params["E"])
        np.add.at(dE, cache["ids"].reshape(-1), d_above.reshape(T * B, -1))
        grads["E"] = dE
    return grads


# --------------------------------------------------------------------------
# gradient exchange arithmetic, schedule, update
# --------------------------------------------------------------------------
def grad_average(worker_grads, loss_scale):
    """Sum the workers' scaled gradients, divide by N (step 4 of the framework
    list) and undo the loss scale.  worker_grads: [N,P].  Returns (avg[P],
    found_inf) where found_inf says any worker value was Inf or NaN."""
    g = np.asarray(worker_grads, dtype=np.float64)
    N = g.shape[0]
    found_inf = bool(not np.all(np.isfinite(g)))
    with np.errstate(invalid="ignore"):
        total = g.sum(axis=0)
    return total / N / float(loss_scale), found_inf


def grad_average_partial(worker_grads, loss_scale, participating):
    """Fault-tolerant variant of step 4 (Section "Distributed computing
    framework", closing paragraph): the master averages once a fraction of the
    workers has delivered, so only the gradients that arrived are summed and
    the divisor is their number.  worker_grads: [N,P]; participating: N flags.
    Rows of absent workers are never looked at.  Returns (avg[P], found_inf,
    n_present); with nobody present the average is zero."""
    g = np.asarray(worker_grads, dtype=np.float64)
    N, P = g.shape
    total = np.zeros(P, dtype=np.float64)
    n_present = 0
    found_inf = False
    for w in range(N):
        if not participating[w]:
            continue
        n_present += 1
        if not np.all(np.isfinite(g[w])):
            found_inf = True
        with np.errstate(invalid="ignore"):
            total = total + g[w]
    if n_present == 0:
        return total, False, 0
    return total / n_present / float(loss_scale), found_inf, n_present


def lr_schedule(lr0, n_workers, n_half, eff_lr_max, warmup_steps, gamma, index):
    """Learning rate for iteration/epoch `index` with N workers.

    Eq. 4: base rate lr0 / (1 + N/n).  Clipping rule: the product N * base is
    held at eff_lr_max at most.  Eq. 3: exponential decay gamma^i.  A linear
    warm-up over the first `warmup_steps` indices (benchmark config 5) ramps
    (k+1)/W; decay then counts from the end of the warm-up.
    """
    base = lr0 / (1.0 + n_workers / n_half)
    if base * n_workers > eff_lr_max:
        base = eff_lr_max / n_workers
    k = int(index)
    if k < warmup_steps:
        return base * (k + 1) / warmup_steps
    return base * gamma ** (k - warmup_steps + 1 if warmup_steps > 0 else k)


def sgd_momentum_update(W, Hbuf, grad, lr, momentum, weight_decay=0.0):
    """Eq. 1-2: H <- m H - lr * dW ;  W <- W + H.  Returns new (W, H)."""
    g = grad + weight_decay * W
    H_new = momentum * Hbuf - lr * g
    return W + H_new, H_new


def adam_update(W, m, v, grad, lr, step, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """Adam (Kingma & Ba) with bias correction; `step` counts from 1."""
    g = grad + weight_decay * W
    m_new = beta1 * m + (1.0 - beta1) * g
    v_new = beta2 * v + (1.0 - beta2) * g * g
    mhat = m_new / (1.0 - beta1 ** step)
    vhat = v_new / (1.0 - beta2 ** step)
    return W - lr * mhat / (np.sqrt(vhat) + eps), m_new, v_new


def loss_scale_policy(scale, good_steps, found_inf, dynamic, backoff=0.5, growth=2.0, growth_interval=2000):
    """Static: scale never changes.  Dynamic: halve after an overflowed step,
    multiply by `growth` after `growth_interval` clean steps in a row."""
    if not dynamic:
        return scale, good_steps
    if found_inf:
        return scale * backoff, 0
    good_steps += 1
    if good_steps >= growth_interval:
        return scale * growth, 0
    return scale, good_steps


# --------------------------------------------------------------------------
# storage rounding (round to nearest even), own implementation
# --------------------------------------------------------------------------
def round_fp16(x):
    """IEEE binary16 round-to-nearest-even of float64 values, returned as
    float64; magnitudes that round above 65504 become +-inf."""
    with np.errstate(over="ignore"):
        return np.asarray(x, dtype=np.float64).astype(np.float16).astype(np.float64)


def round_bf16(x):
    """bfloat16 (8-bit exponent, 7-bit mantissa) round-to-nearest-even of the
    float32 value of x, by integer arithmetic on the bit pattern."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    out = (rounded & 0xFFFFFFFF).astype(np.uint32).view(np.float32).astype(np.float64)
    return np.where(np.isnan(f), np.nan, out)


def round_storage(x, dtype):
    if dtype == "fp16":
        return round_fp16(x)
    if dtype == "bf16":
        return round_bf16(x)
    return np.asarray(x, dtype=np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# one whole training step (used by tests, smoke and the CPU baseline timing)
# --------------------------------------------------------------------------
def training_step(flat_params, shapes, num_layers, batches, head, loss_scale, lr, momentum,
                  Hbuf=None, weight_decay=0.0):
    """fprop + bprop for every worker's batch, average, SGD-momentum update.

    batches: list of (x, targets), one per simulated worker.
    Returns dict(losses, worker_grads[N,P] scaled, avg_grad, found_inf, W, H).
    """
    params = unflatten(flat_params, shapes)
    losses, wg = [], []
    for x, y in batches:
        loss, cache = forward(params, num_layers, x, y, head)
        g = backward(params, num_layers, cache, loss_scale)
        losses.append(loss)
        wg.append(flatten(g, shapes))
    wg = np.stack(wg)
    avg, found_inf = grad_average(wg, loss_scale)
    W = np.asarray(flat_params, dtype=np.float64)
    Hb = np.zeros_like(W) if Hbuf is None else np.asarray(Hbuf, dtype=np.float64)
    if not found_inf:
        W, Hb = sgd_momentum_update(W, Hb, avg, lr, momentum, weight_decay)
    return dict(losses=losses, worker_grads=wg, avg_grad=avg, found_inf=found_inf, W=W, H=Hb)
