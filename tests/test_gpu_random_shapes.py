"""Seeded random small configurations against the oracle: layer counts, widths, batch sizes
(ragged and multiples of 64), sequence lengths, storage types and heads drawn at random, so that
combinations nobody wrote down by hand (which schedule, which GEMM path, which vector path) are
exercised too."""
import numpy as np
import pytest

import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _check(w):
    """2e-2 (1e-4 in fp32) per tensor; a 16-bit tensor beyond that must stay inside the rounding bound
    derived from the terms of its sums, and the same shape must then pass in fp32 at 1e-4."""
    got = pu.run_gpu_step(w)
    want = pu.run_oracle_step(w, with_terms=True)
    used = []
    pu.assert_step_close(w, got, want, used)
    if used:
        print("  rounding bound needed for:", [(what, name, tuple(round(e, 4) for e in err), round(kappa / pu.GRAD_RTOL[w.dtype], 1))
                                                for what, name, err, kappa in used[:6]], flush=True)
        w32 = w.with_(dtype="fp32", loss_scale=1.0)
        pu.assert_step_close(w32, pu.run_gpu_step(w32), pu.run_oracle_step(w32))


def _draw(seed):
    rng = np.random.default_rng(9000 + seed)
    dtype = ["fp16", "bf16", "fp32"][int(rng.integers(0, 3))]
    L = int(rng.integers(1, 5))
    H = int(rng.choice([1, 7, 8, 24, 33, 48, 64, 72, 130]))
    B = int(rng.choice([1, 3, 8, 17, 64, 70, 128]))
    T = int(rng.integers(1, 7))
    I = int(rng.choice([1, 5, 8, 16, 40]))
    head = int(rng.choice([wl.HEAD_STEP_BCE, wl.HEAD_LAST_BCE, wl.HEAD_STEP_MSE, wl.HEAD_FC_HINGE]))
    kw = {}
    if head == wl.HEAD_FC_HINGE:
        kw = dict(fc_units=int(rng.choice([3, 16, 50])), target_kind="sign", target_p=0.4)
    elif head == wl.HEAD_STEP_MSE:
        kw = dict(target_kind="normal")
    else:
        kw = dict(target_p=0.4)
    if head == wl.HEAD_FC_HINGE:
        # Hinge and ReLU are decisions: a sample that 16-bit rounding moves across a kink changes a whole
        # term of every gradient below it, which no rounding bound covers.  The 16-bit runs of this head
        # are the fixed cases of test_gpu_paper_head.py; the random draws keep it in fp32.
        dtype = "fp32"
    scale = 1.0 if dtype != "fp16" else float(rng.choice([64.0, 1024.0]))
    return wl.Workload(f"rnd{seed}", L, I, H, T, B, dtype, head, loss_scale=scale, data_seed=700 + seed, weight_seed=800 + seed, **kw)


@pytest.mark.parametrize("seed", range(24))
def test_random_configuration(seed):
    w = _draw(seed)
    print(f"[case] rnd{seed}: L={w.num_layers} I={w.input_dim} H={w.hidden} T={w.seq_len} B={w.batch} {w.dtype} head={w.head} "
          f"F={w.fc_units}", flush=True)
    _check(w)


def _draw_narrow(seed):
    """Shapes the one-launch-per-cell kernels take (16-bit storage, H a multiple of 8): tile edges that do
    and do not divide the batch and the width, more layers than cells per launch, single steps."""
    rng = np.random.default_rng(9500 + seed)
    dtype = ["fp16", "bf16"][int(rng.integers(0, 2))]
    L = int(rng.integers(1, 4))
    H = int(rng.choice([8, 16, 40, 56, 104, 136, 200, 264]))
    B = int(rng.choice([1, 15, 16, 33, 64, 100, 192, 256]))
    T = int(rng.integers(1, 6))
    I = int(rng.choice([3, 8, 24, 64]))
    head = int(rng.choice([wl.HEAD_STEP_BCE, wl.HEAD_LAST_BCE, wl.HEAD_STEP_MSE]))
    kw = dict(target_kind="normal") if head == wl.HEAD_STEP_MSE else dict(target_p=0.4)
    scale = 1.0 if dtype != "fp16" else float(rng.choice([64.0, 1024.0]))
    return wl.Workload(f"nar{seed}", L, I, H, T, B, dtype, head, loss_scale=scale, data_seed=1700 + seed, weight_seed=1800 + seed, **kw)


@pytest.mark.parametrize("seed", range(24))
def test_random_narrow_configuration(seed):
    w = _draw_narrow(seed)
    print(f"[case] nar{seed}: L={w.num_layers} I={w.input_dim} H={w.hidden} T={w.seq_len} B={w.batch} {w.dtype} head={w.head}", flush=True)
    _check(w)


def _draw_wide(seed):
    """Layers too wide for the one-launch cells (H > 768): the per-step kernels with the contraction split by
    gate over workgroups, ragged widths and batches."""
    rng = np.random.default_rng(31000 + seed)
    dtype = ["fp16", "bf16"][int(rng.integers(0, 2))]
    L = int(rng.integers(1, 3))
    H = int(rng.choice([776, 800, 1024, 1032, 904]))
    B = int(rng.choice([1, 17, 64, 100, 128, 200, 256]))
    T = int(rng.integers(1, 4))
    I = int(rng.choice([3, 8, 24, 64, 130]))
    head = int(rng.choice([wl.HEAD_STEP_BCE, wl.HEAD_LAST_BCE, wl.HEAD_STEP_MSE]))
    kw = dict(target_kind="normal") if head == wl.HEAD_STEP_MSE else dict(target_p=0.4)
    scale = 1.0 if dtype != "fp16" else float(rng.choice([64.0, 1024.0]))
    return wl.Workload(f"wide{seed}", L, I, H, T, B, dtype, head, loss_scale=scale, data_seed=2700 + seed, weight_seed=2800 + seed, **kw)


@pytest.mark.parametrize("seed", range(12))
def test_random_wide_configuration(seed):
    w = _draw_wide(seed)
    print(f"[case] wide{seed}: L={w.num_layers} I={w.input_dim} H={w.hidden} T={w.seq_len} B={w.batch} {w.dtype} head={w.head}", flush=True)
    _check(w)


def _draw_many_rows(seed):
    """A thousand to eight thousand rows per time step (what stacked workers look like to the kernels): the
    single-wavefront forward cells, cells that project their own input, the one-launch BPTT step, widths whose
    padding to whole tiles nobody owns, and the fp32 mode at such batches."""
    rng = np.random.default_rng(32000 + seed)
    dtype = ["fp16", "bf16", "fp32"][int(rng.integers(0, 3))]
    L = int(rng.integers(1, 4))
    H = int(rng.choice([8, 40, 100, 200, 264, 520]))
    B = int(rng.choice([960, 1000, 1024, 2048, 4100, 8192]))
    T = int(rng.integers(1, 4))
    I = int(rng.choice([3, 8, 24, 64, 200]))
    head = int(rng.choice([wl.HEAD_STEP_BCE, wl.HEAD_LAST_BCE, wl.HEAD_STEP_MSE]))
    kw = dict(target_kind="normal") if head == wl.HEAD_STEP_MSE else dict(target_p=0.4)
    scale = 1.0 if dtype != "fp16" else float(rng.choice([64.0, 1024.0]))
    return wl.Workload(f"rows{seed}", L, I, H, T, B, dtype, head, loss_scale=scale, data_seed=3700 + seed, weight_seed=3800 + seed, **kw)


@pytest.mark.parametrize("seed", range(12))
def test_random_many_rows_configuration(seed):
    w = _draw_many_rows(seed)
    print(f"[case] rows{seed}: L={w.num_layers} I={w.input_dim} H={w.hidden} T={w.seq_len} B={w.batch} {w.dtype} head={w.head}", flush=True)
    _check(w)
