"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and its pure-host entry points (layout,
workspace plan, schedule, argument validation) behave as documented."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import workloads as wl
from oracle import lstm_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", "lstm_mi355.h"), os.path.join(ROOT, "include", "lstm_mi355_debug.h")]


@pytest.fixture(scope="module")
def hip():
    import paper_1912_00286_amd as pkg
    if not os.path.exists(pkg.library_path()):
        import __graft_entry__ as g
        g.build()
    pkg.load_library()
    return pkg


def _declared_functions():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?(?:int|float|char)\s*\*?\s*(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_header_symbols_are_exported(hip):
    names = _declared_functions()
    for expected in ("lstm_forward", "lstm_backward", "grad_average", "master_update", "lr_schedule",
                     "lstm_param_count", "lstm_param_offset", "lstm_workspace_bytes", "lstm_abi_version",
                     "lstm_last_error", "lstm_cast_params", "grad_average_masked", "lstm_debug_plan_regions", "lstm_timing_read"):
        assert expected in names
    lib = hip.load_library()
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"
    assert hip.lstm_abi_version() == 4
    # the product header declares no diagnostic
    assert "lstm_debug" not in open(HEADERS[0]).read() and "lstm_timing" not in open(HEADERS[0]).read()


def _cfg(hip, w):
    from tests.parity_util import make_cfg
    return make_cfg(w)


PAPER_HEAD = wl.Workload("paper_head", 2, 9, 200, 128, 256, "fp16", wl.HEAD_FC_HINGE, fc_units=200, target_kind="sign")


@pytest.mark.parametrize("name", list(wl.CONFIGS) + ["paper_head"])
def test_param_layout_agrees_with_oracle_and_generator(hip, name):
    w = PAPER_HEAD if name == "paper_head" else wl.CONFIGS[name]
    cfg = _cfg(hip, w)
    P = hip.lstm_param_count(cfg)
    assert P == wl.param_count(w) == orc.param_count(w.num_layers, w.input_dim, w.hidden, w.vocab, w.embed_dim, w.fc_units)
    kinds = {"E": 0, "W": 1, "U": 2, "b": 3, "w_head": 4, "b_head": 5, "W_fc": 6, "b_fc": 7}
    off = 0
    for nm, shape in orc.param_shapes(w.num_layers, w.input_dim, w.hidden, w.vocab, w.embed_dim, w.fc_units):
        if nm in ("E", "w_head", "b_head", "W_fc", "b_fc"):
            o, c = hip.lstm_param_offset(cfg, kinds[nm], 0)
        else:
            o, c = hip.lstm_param_offset(cfg, kinds[nm[0]], int(nm[1:]))
        assert (o, c) == (off, int(np.prod(shape))), nm
        off += c
    assert off == P
    assert [n for n, _ in wl.param_segments(w)] == [n for n, _ in orc.param_shapes(w.num_layers, w.input_dim, w.hidden, w.vocab,
                                                                                   w.embed_dim, w.fc_units)]


def test_param_counts_of_the_benchmark_configs(hip):
    want = {"tiny": 6049, "jet": 533001, "text": 2954497, "large": 88107009, "workers64": 533001}
    for name, n in want.items():
        assert hip.lstm_param_count(_cfg(hip, wl.CONFIGS[name])) == n


def test_workspace_plan(hip):
    w = wl.CONFIGS["large"]
    r, s = hip.lstm_workspace_bytes(_cfg(hip, w))
    saved = 6 * w.hidden * 2 * w.seq_len * w.batch * w.num_layers     # 4 gates + c + h in fp16
    assert saved <= r <= 1.25 * saved + (1 << 20)                     # + a blocked copy of h and of the input
    assert 0 < s < 8 << 30
    r1, s1 = hip.lstm_workspace_bytes(_cfg(hip, wl.CONFIGS["tiny"]))
    assert r1 % 256 == 0 and s1 % 256 == 0 and r1 < r and s1 < s


def test_capacity_trends_of_table1(hip):
    """Table 1: at 200 units and 128 steps, halving the element size or quartering the batch
    lets a deeper stack fit the device memory.  The workspace plan must show the same trends
    (bytes per added layer: fp16 well below fp32, batch 64 well below batch 256)."""
    def per_layer(dtype, batch):
        def total(L):
            w = wl.Workload("cap", L, 9, 200, 128, batch, dtype, wl.HEAD_STEP_BCE)
            cfg = _cfg(hip, w)
            r, s = hip.lstm_workspace_bytes(cfg)
            es = 4 if dtype == "fp32" else 2
            return r + s + hip.lstm_param_count(cfg) * (2 * es + 12)     # + weights, gradient, master, momentum, average
        # deep enough that the stack is memory-bound (the faster diagonal backward schedule, which
        # keeps one dA per layer, is only used while that extra stays small)
        return (total(1600) - total(1200)) / 400.0
    f32, f16 = per_layer("fp32", 256), per_layer("fp16", 256)
    f32s, f16s = per_layer("fp32", 64), per_layer("fp16", 64)
    assert 1.5 < f32 / f16 <= 2.0 and 1.5 < f32s / f16s <= 2.0
    assert 3.0 < f32 / f32s <= 4.0 and 3.0 < f16 / f16s <= 4.0
    # the paper's P100 held 58 fp16 layers at batch 256 in 16 GB; this plan needs less per layer
    assert 16e9 / f16 > 58


def test_invalid_arguments_are_rejected_on_the_host(hip):
    w = wl.CONFIGS["tiny"]
    for field, val, status in (("batch", 0, -1), ("seq_len", 0, -1), ("hidden", 0, -1), ("num_layers", 0, -1),
                               ("dtype", 7, -1), ("head", 0, -1), ("head", 5, -1), ("out_dim", 2, -2), ("input_dim", 0, -1)):
        cfg = _cfg(hip, w)
        setattr(cfg, field, val)
        with pytest.raises(hip.LstmError) as e:
            hip.lstm_param_count(cfg)
        assert e.value.status == status and hip.lstm_last_error()
    cfg = _cfg(hip, w)
    with pytest.raises(hip.LstmError):
        hip.lstm_param_offset(cfg, 1, 5)
    with pytest.raises(hip.LstmError):
        hip.lstm_param_offset(cfg, 0, 0)         # no embedding in this config
    # null / misaligned device pointers are refused before anything is enqueued
    big = dict(reserve_bytes=1 << 30, scratch_bytes=1 << 30)
    with pytest.raises(hip.LstmError):
        hip.lstm_forward(cfg, 0, 0, 0, None, None, 0, 0, 0, stream=0, **big)
    with pytest.raises(hip.LstmError) as e:
        hip.lstm_forward(cfg, 4096 + 2, 4096, 4096, None, None, 4096, 4096, 4096, stream=0, **big)
    assert "aligned" in str(e.value)
    # a workspace one byte short of the plan is refused with its own status, in both directions
    r, s = hip.lstm_workspace_bytes(cfg)
    for rb, sb in ((r - 1, s), (r, s - 1), (0, 0)):
        with pytest.raises(hip.LstmError) as e:
            hip.lstm_forward(cfg, 4096, 4096, 4096, None, None, 4096, 4096, 4096, stream=0, reserve_bytes=rb, scratch_bytes=sb)
        assert e.value.status == -3 and "workspace too small" in str(e.value)
        with pytest.raises(hip.LstmError) as e:
            hip.lstm_backward(cfg, 4096, 4096, 4096, 4096, 4096, 4096, 4096, stream=0, reserve_bytes=rb, scratch_bytes=sb)
        assert e.value.status == -3
    # buffers sized for one config do not serve an edited one that plans a larger workspace
    bigger = _cfg(hip, w)
    bigger.batch = 64
    with pytest.raises(hip.LstmError) as e:
        hip.lstm_forward(bigger, 4096, 4096, 4096, None, None, 4096, 4096, 4096, stream=0, reserve_bytes=r, scratch_bytes=s)
    assert e.value.status == -3
    with pytest.raises(hip.LstmError):
        hip.grad_average(10, 0, 4096, 1, 4096, 4096, 4096, stream=0)
    opt = hip.OptimizerConfig(kind=9)
    with pytest.raises(hip.LstmError):
        hip.master_update(10, opt, 0.1, 1, 4096, 4096, None, 4096, 4096, 4096, 4096, 4096, 1, stream=0)
    opt = hip.OptimizerConfig(kind=1)
    with pytest.raises(hip.LstmError):          # Adam without its second state
        hip.master_update(10, opt, 0.1, 1, 4096, 4096, None, 4096, 4096, 4096, 4096, 4096, 1, stream=0)


def test_lr_schedule_matches_oracle_and_paper(hip):
    rng = np.random.default_rng(0)
    for _ in range(200):
        lr0 = float(10 ** rng.uniform(-4, -1)); N = int(rng.integers(1, 200)); n = float(rng.integers(1, 128))
        W = int(rng.integers(0, 8)); gamma = float(rng.uniform(0.8, 1.0)); k = int(rng.integers(0, 30))
        got = hip.lr_schedule(lr0, N, n, 0.1, W, gamma, k)
        want = orc.lr_schedule(np.float32(lr0), N, np.float32(n), np.float32(0.1), W, np.float32(gamma), k)
        assert got == pytest.approx(want, rel=2e-7)
    assert hip.lr_schedule(0.001, 8, 8.0, 1e9, 0, 1.0, 0) == pytest.approx(0.0005, rel=1e-7)   # halved at N = n
    assert hip.lr_schedule(0.05, 8, 8.0, 0.1, 0, 1.0, 0) == pytest.approx(0.0125, rel=1e-7)     # clipped
    assert hip.lr_schedule(0.001, 0, 8.0, 0.1, 0, 1.0, 0) == 0.0                                 # invalid
    w = wl.CONFIGS["workers64"]
    vals = [hip.lr_schedule(w.lr0, 64, 64.0, 0.1, 5, 0.97, k) for k in range(8)]
    assert vals[4] == pytest.approx(5e-4, rel=1e-6) and vals[0] == pytest.approx(1e-4, rel=1e-6)
    assert vals[7] == pytest.approx(5e-4 * 0.97 ** 3, rel=1e-6)


def test_product_package_does_not_import_the_oracle():
    pkg_dir = os.path.join(ROOT, "paper_1912_00286_amd")
    for dirpath, _, files in os.walk(pkg_dir):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
    otext = open(os.path.join(ROOT, "oracle", "lstm_oracle.py")).read()
    assert "paper_1912_00286_amd" not in otext and "import workloads" not in otext


def test_bench_helpers_do_not_load_the_oracle():
    """bench.py drives the HIP path through tests/parity_util.py; only its CPU-baseline leg may
    touch the oracle.  Importing the helpers and building a config must not load it."""
    import subprocess
    import sys
    code = ("import sys; sys.path.insert(0, %r); import workloads as wl; from tests import parity_util as pu; "
            "pu.make_cfg(wl.CONFIGS['jet']); pu.make_opt(wl.CONFIGS['jet']); pu.inputs_for(wl.CONFIGS['tiny']); "
            "print(any(m == 'oracle' or m.startswith('oracle.') for m in sys.modules))" % ROOT)
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    assert out.stdout.strip().splitlines()[-1] == "False"
    bench = open(os.path.join(ROOT, "bench.py")).read()
    _, _, tail = bench.partition("def cpu_baseline")
    # the only import of the oracle in bench.py sits inside cpu_baseline()
    assert bench.count("from oracle import") == 1 and "from oracle import" in tail.split("\ndef ")[0]


def _plan_grid():
    """One or more shapes per kernel family and layout the plan chooses between."""
    out = []
    for dtype in ("fp32", "fp16", "bf16"):
        for L in (1, 2, 3, 5):
            for H in (8, 33, 200, 256, 264, 776, 1032, 2048):
                for T, B in ((1, 1), (3, 17), (4, 64), (5, 128), (2, 1024), (3, 3072), (2, 8192)):
                    if H >= 1032 and B > 1024:
                        continue
                    for head, I, V in ((wl.HEAD_STEP_BCE, 24, 0), (wl.HEAD_LAST_BCE, 0, 50), (wl.HEAD_FC_HINGE, 9, 0)):
                        out.append(wl.Workload("grid", L, I, H, T, B, dtype, head, vocab=V, embed_dim=16 if V else 0,
                                               fc_units=20 if head == wl.HEAD_FC_HINGE else 0))
    return out


def test_workspace_regions_are_disjoint_and_inside_the_reported_sizes(hip):
    """Every region the plan hands out (saved activations, packed operands, partial sums, per-layer
    buffers of the diagonal schedules, ...) lies inside the size lstm_workspace_bytes reports and
    overlaps no other region of the same buffer, over a grid of shapes that reaches every kernel
    family; with several workers stacked into one call too."""
    checked = 0
    cases = [(w, 1) for w in _plan_grid()]
    cases += [(wl.Workload("stk", L, 24, H, 4, B, "fp16", wl.HEAD_STEP_BCE), W) for L in (1, 2) for H in (56, 200, 520)
              for B in (64, 128) for W in (2, 16, 64)]
    cases += [(w, 1) for w in wl.CONFIGS.values()] + [(wl.CONFIGS["workers64"], 64)]
    for w, workers in cases:
        cfg = _cfg(hip, w)
        cfg.workers = workers
        r, s = hip.lstm_workspace_bytes(cfg)
        regions = hip.lstm_debug_plan_regions(cfg)
        assert regions, w
        for which, total in ((0, r), (1, s)):
            spans = sorted((off, off + size) for k, off, size in regions if k == which)
            assert all(a % 256 == 0 for a, _ in spans)
            assert all(b <= total for _, b in spans), (w, workers, which)
            assert all(spans[i][1] <= spans[i + 1][0] for i in range(len(spans) - 1)), (w, workers, which)
        checked += 1
    assert checked > 1000
