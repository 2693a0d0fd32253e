"""The paper's own head (Fig. 2: fully connected ReLU layer per temporal slice, one
output; Eq. 6: hinge loss times a scalar multiplier) against the CPU oracle."""
import numpy as np
import pytest

import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hip():
    import paper_1912_00286_amd as pkg
    pkg.load_library()
    return pkg


CASES = [
    # name, L, I, H, T, B, dtype, F, loss scale
    ("fc_fp32_small", 1, 5, 12, 6, 4, "fp32", 7, 1.0),
    ("fc_fp32_ragged", 2, 9, 33, 5, 7, "fp32", 50, 10.0),
    ("fc_fp16_ragged", 2, 9, 40, 9, 12, "fp16", 36, 10.0),          # the paper's static multiplier 10
    ("fc_bf16", 1, 9, 64, 8, 64, "bf16", 48, 1.0),
    ("fc_fp16_blocked", 2, 16, 192, 6, 64, "fp16", 200, 1024.0),    # large-tile GEMM paths below the head
]


@pytest.mark.parametrize("spec", CASES, ids=[c[0] for c in CASES])
def test_fc_hinge_head_step(hip, spec):
    name, L, I, H, T, B, dtype, F, S = spec
    print(f"[case] {name}", flush=True)
    w = wl.Workload(name, L, I, H, T, B, dtype, wl.HEAD_FC_HINGE, fc_units=F, target_kind="sign", target_p=0.3,
                    loss_scale=S, data_seed=41, weight_seed=42)
    got = pu.run_gpu_step(w)
    want = pu.run_oracle_step(w)
    pu.assert_step_close(w, got, want)
    # both sides of the hinge and of the ReLU are exercised
    assert 0.0 < want["losses"][0] < 2.0


def test_fig2_model_at_paper_shape(hip):
    """Fig. 2 at its printed shape: 2 x LSTM(200) on 9 features, FC(200) + ReLU, 1 output;
    batch 256, hinge multiplier 10; sequence shortened to 16 of the 128 steps so that the
    fp64 oracle stays within seconds."""
    w = wl.Workload("fig2", 2, 9, 200, 16, 256, "fp16", wl.HEAD_FC_HINGE, fc_units=200, target_kind="sign", target_p=0.1,
                    loss_scale=10.0, data_seed=43, weight_seed=44)
    print("[case] fig2", flush=True)
    got = pu.run_gpu_step(w)
    want = pu.run_oracle_step(w)
    pu.assert_step_close(w, got, want)


def test_fc_head_rejects_missing_width(hip):
    w = wl.Workload("bad", 1, 4, 8, 2, 2, "fp32", wl.HEAD_FC_HINGE, fc_units=0)
    with pytest.raises(hip.LstmError):
        hip.lstm_param_count(pu.make_cfg(w))
