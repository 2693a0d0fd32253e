"""Shapes on which a 16-bit run exceeds the 2e-2 per-tensor tolerance through storage rounding alone,
kept as tests instead of being drawn around.  Each is run in all three storage types on the same seed:
  * fp32 must meet 1e-4 (the arithmetic of the kernels is right on this shape);
  * fp16 / bf16 must meet 2e-2 except on tensors whose elements are sums of cancelling terms, and there
    every element must stay inside the bound derived from the terms of its sum (parity_util.rounding_bound:
    unit round-off times the sum of the absolute terms, plus, in half precision, the absolute error of
    stored values below the normal range);
  * the errors of the flagged tensors must scale with the unit round-off (bf16 : fp16 = 8 : 1 nominally),
    so that an error that does not come from rounding would stand out.
"""
import numpy as np
import pytest

import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

CASES = {
    # thousands of rows per step, three layers, half precision at a low loss multiplier: the bottom layer's
    # scaled dA falls below the normal range of binary16
    "rows_three_layers_low_scale": (wl.Workload("rb_rows", 3, 64, 232, 3, 5000, "fp16", wl.HEAD_STEP_BCE, loss_scale=64.0,
                                                target_p=0.4, data_seed=6825, weight_seed=6925), False, ("W0", "U0", "b0")),
    # stacked workers, squared-error head: bias gradients are sums of a few hundred cancelling terms
    "stacked_workers_bias": (wl.Workload("rb_stk", 2, 64, 520, 4, 128, "bf16", wl.HEAD_STEP_MSE, n_workers=16, target_kind="normal",
                                         data_seed=5804, weight_seed=5904), True, ("b0", "b1")),
    # four narrow layers in bfloat16, 33 samples
    "four_narrow_layers": (wl.Workload("rb_deep", 4, 3, 104, 4, 33, "bf16", wl.HEAD_STEP_BCE, target_p=0.4, data_seed=3, weight_seed=4),
                           False, ("W3", "U3", "b3")),
}


def _errors(w, batched):
    got = pu.run_gpu_step(w, batched=batched)
    ref = pu.run_oracle_step(w, with_terms=w.dtype != "fp32")
    used = []
    pu.assert_step_close(w, got, ref, used)
    errs = [pu.tensor_errors(got["grads"][k], ref["grads"][k], ref["shapes"]) for k in range(w.n_workers)]
    return errs, used


@pytest.mark.parametrize("name", list(CASES))
def test_error_beyond_tolerance_is_rounding(name):
    w, batched, watch = CASES[name]
    print(f"[case] {name}: fp32", flush=True)
    e32, _ = _errors(w.with_(dtype="fp32", loss_scale=1.0), False if w.n_workers > 1 else batched)
    print(f"[case] {name}: fp16", flush=True)
    e16, used16 = _errors(w.with_(dtype="fp16", loss_scale=w.loss_scale if w.dtype == "fp16" else 1024.0), batched)
    print(f"[case] {name}: bf16", flush=True)
    eb, usedb = _errors(w.with_(dtype="bf16", loss_scale=1.0), batched)
    print(f"  tensors that needed the derived bound: fp16 {[(a, b) for a, b, _, _ in used16]}, bf16 {[(a, b) for a, b, _, _ in usedb]}", flush=True)
    # the shape is in this file because its native storage type goes past 2e-2 somewhere
    native = used16 if w.dtype == "fp16" else usedb
    assert native, "this shape no longer exceeds the plain tolerance: move it to the ordinary parity cases"
    # errors scale with the unit round-off: worst l2 error over workers per watched tensor
    for t in watch:
        r32 = max(e[t][0] for e in e32); r16 = max(e[t][0] for e in e16); rb = max(e[t][0] for e in eb)
        print(f"  {t}: l2 rel error fp32 {r32:.2e}, fp16 {r16:.2e}, bf16 {rb:.2e}", flush=True)
        assert r32 <= 1e-4
        if w.dtype == "bf16":
            assert 2.0 <= rb / r16 <= 32.0, (t, rb, r16)


def test_loss_multiplier_lifts_the_bottom_layer_out_of_the_subnormal_range():
    """Section "Performance evaluation": the loss is multiplied by a scalar so that small gradients survive
    half precision.  The three-layer case above at multiplier 64 has a bottom-layer weight gradient off by
    more than 2e-2; at 16384 the same step meets the plain tolerance with no help from the derived bound."""
    w, batched, _ = CASES["rows_three_layers_low_scale"]
    lo, used_lo = _errors(w, batched)
    hi, used_hi = _errors(w.with_(loss_scale=16384.0), batched)
    print(f"  W0 l2 rel error: S=64 {lo[0]['W0'][0]:.3e}, S=16384 {hi[0]['W0'][0]:.3e}", flush=True)
    assert used_lo and not used_hi
    assert hi[0]["W0"][0] < 0.25 * lo[0]["W0"][0]
