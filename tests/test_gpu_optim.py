"""grad_average and master_update against the CPU oracle at the benchmark's
parameter counts (88 107 009 with one worker, 533 001 with 64 workers: odd
sizes, unaligned worker rows) and at edge sizes."""
import numpy as np
import pytest

from oracle import lstm_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hip():
    import paper_1912_00286_amd as pkg
    pkg.load_library()
    return pkg


def _tdtype(torch, name):
    return {"fp32": torch.float32, "fp16": torch.float16, "bf16": torch.bfloat16}[name]


CODE = {"fp32": 0, "fp16": 1, "bf16": 2}


@pytest.mark.parametrize("P,N,dtype", [(1, 1, "fp16"), (7, 3, "fp16"), (8, 2, "bf16"), (4099, 5, "fp16"), (4096, 4, "fp32"),
                                       (533001, 64, "fp16"), (533001, 64, "bf16"), (88107009, 1, "fp16"), (1000003, 3, "fp32")])
def test_grad_average_matches_oracle(hip, P, N, dtype):
    import torch
    print(f"[case] grad_average P={P} N={N} {dtype}", flush=True)
    gen = torch.Generator(device="cuda").manual_seed(P % 1000 + N)
    S = 1024.0
    g = (torch.randn((N, P), device="cuda", generator=gen) * 3.0).to(_tdtype(torch, dtype))
    scale = torch.tensor([S], device="cuda"); avg = torch.empty(P, device="cuda"); flag = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    hip.grad_average(P, N, g, CODE[dtype], scale, avg, flag)
    torch.cuda.synchronize()
    want, inf = orc.grad_average(g.double().cpu().numpy(), S)
    assert int(flag.item()) == 0 and not inf
    np.testing.assert_allclose(avg.double().cpu().numpy(), want, rtol=2e-6, atol=1e-9)
    # a single Inf / NaN anywhere (first element, last element of the last worker, middle) raises the flag
    for pos, val in (((0, 0), float("inf")), ((N - 1, P - 1), float("nan")), ((N // 2, P // 2), float("-inf"))):
        g2 = g.clone(); g2[pos] = val
        hip.grad_average(P, N, g2, CODE[dtype], scale, avg, flag)
        torch.cuda.synchronize()
        assert int(flag.item()) == 1, (pos, val)
        assert orc.grad_average(g2.double().cpu().numpy(), S)[1]
    hip.grad_average(P, N, g, CODE[dtype], scale, avg, flag)    # flag is reset by every call
    torch.cuda.synchronize()
    assert int(flag.item()) == 0


def test_grad_average_fp16_largest_finite_is_not_overflow(hip):
    import torch
    g = torch.full((2, 16), 65504.0, dtype=torch.float16, device="cuda")
    scale = torch.tensor([2.0], device="cuda"); avg = torch.empty(16, device="cuda"); flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    hip.grad_average(16, 2, g, 1, scale, avg, flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0 and torch.all(avg == 32752.0)


def _opt(hip, kind, dynamic=0, m=0.9, wd=0.0, interval=2000):
    return hip.OptimizerConfig(kind=kind, momentum=m, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=wd,
                               dynamic_scale=dynamic, scale_backoff=0.5, scale_growth=2.0, growth_interval=interval)


@pytest.mark.parametrize("P,dtype", [(1, "fp16"), (5, "bf16"), (4099, "fp16"), (533001, "fp16"), (88107009, "fp16"), (10007, "fp32")])
def test_sgd_momentum_update_matches_oracle(hip, P, dtype):
    import torch
    print(f"[case] master_update sgd P={P} {dtype}", flush=True)
    gen = torch.Generator(device="cuda").manual_seed(P % 977)
    W = torch.randn(P, device="cuda", generator=gen) * 0.1
    Hb = torch.randn(P, device="cuda", generator=gen) * 1e-3
    g = torch.randn(P, device="cuda", generator=gen) * 1e-2
    W0, H0 = W.double().cpu().numpy(), Hb.double().cpu().numpy()
    flag = torch.zeros(1, dtype=torch.int32, device="cuda"); scale = torch.tensor([32768.0], device="cuda")
    good = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = torch.zeros(P, dtype=_tdtype(torch, dtype), device="cuda")
    hip.master_update(P, _opt(hip, 0, dynamic=1, wd=1e-4), 0.01, 1, W, Hb, None, g, flag, scale, good, out, CODE[dtype])
    torch.cuda.synchronize()
    Wr, Hr = orc.sgd_momentum_update(W0, H0, g.double().cpu().numpy(), np.float32(0.01), np.float32(0.9), np.float32(1e-4))
    np.testing.assert_allclose(Hb.double().cpu().numpy(), Hr, rtol=3e-6, atol=1e-10)
    np.testing.assert_allclose(W.double().cpu().numpy(), Wr, rtol=3e-7, atol=1e-9)
    # the working copy is the round-to-nearest-even cast of the fp32 master (decided in fp32 on both sides)
    np.testing.assert_array_equal(out.double().cpu().numpy(), orc.round_storage(W.double().cpu().numpy(), dtype))
    assert float(scale.item()) == 32768.0 and int(good.item()) == 1


def test_update_skipped_on_overflow_and_scale_policy(hip):
    import torch
    P = 1000
    W = torch.randn(P, device="cuda"); Hb = torch.randn(P, device="cuda"); g = torch.randn(P, device="cuda")
    out = torch.full((P,), 3.0, dtype=torch.float16, device="cuda")
    W0, H0, out0 = W.clone(), Hb.clone(), out.clone()
    flag = torch.ones(1, dtype=torch.int32, device="cuda"); scale = torch.tensor([32768.0], device="cuda")
    good = torch.full((1,), 5, dtype=torch.int32, device="cuda")
    hip.master_update(P, _opt(hip, 0, dynamic=1), 0.1, 1, W, Hb, None, g, flag, scale, good, out, 1)
    torch.cuda.synchronize()
    assert torch.equal(W, W0) and torch.equal(Hb, H0) and torch.equal(out, out0)
    assert (float(scale.item()), int(good.item())) == orc.loss_scale_policy(32768.0, 5, True, True) == (16384.0, 0)
    # static policy: skipped, scale untouched
    hip.master_update(P, _opt(hip, 0, dynamic=0), 0.1, 1, W, Hb, None, g, flag, scale, good, out, 1)
    torch.cuda.synchronize()
    assert torch.equal(W, W0) and float(scale.item()) == 16384.0 and int(good.item()) == 0
    # growth after `interval` clean steps
    flag.zero_()
    for k in range(3):
        hip.master_update(P, _opt(hip, 0, dynamic=1, interval=3), 0.0, 1, W, Hb, None, g, flag, scale, good, out, 1)
    torch.cuda.synchronize()
    assert (float(scale.item()), int(good.item())) == (32768.0, 0)


def test_two_steps_closed_form_of_eq_1_2(hip):
    import torch
    P = 64
    W = torch.zeros(P, device="cuda"); Hb = torch.zeros(P, device="cuda")
    g1 = torch.full((P,), 2.0, device="cuda"); g2 = torch.full((P,), -1.0, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda"); out = torch.zeros(P, device="cuda")
    opt = _opt(hip, 0, m=0.5)
    hip.master_update(P, opt, 0.25, 1, W, Hb, None, g1, flag, None, None, out, 0)
    hip.master_update(P, opt, 0.125, 2, W, Hb, None, g2, flag, None, None, out, 0)
    torch.cuda.synchronize()
    # H2 = -m l1 g1 - l2 g2 = -0.25 + 0.125 ; W2 = -l1 g1 + H2
    assert torch.all(Hb == -0.125) and torch.all(W == -0.625) and torch.equal(W, out)


@pytest.mark.parametrize("P,dtype", [(4099, "fp16"), (533001, "bf16")])
def test_adam_update_matches_oracle(hip, P, dtype):
    import torch
    gen = torch.Generator(device="cuda").manual_seed(3)
    W = torch.randn(P, device="cuda", generator=gen) * 0.1
    m = torch.zeros(P, device="cuda"); v = torch.zeros(P, device="cuda")
    Wr, mr, vr = W.double().cpu().numpy(), np.zeros(P), np.zeros(P)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = torch.zeros(P, dtype=_tdtype(torch, dtype), device="cuda")
    for step in (1, 2, 3):
        g = torch.randn(P, device="cuda", generator=gen) * 1e-2
        hip.master_update(P, _opt(hip, 1), 1e-3, step, W, m, v, g, flag, None, None, out, CODE[dtype])
        torch.cuda.synchronize()
        Wr, mr, vr = orc.adam_update(Wr, mr, vr, g.double().cpu().numpy(), np.float32(1e-3), step,
                                     np.float32(0.9), np.float32(0.999), np.float32(1e-8))
    np.testing.assert_allclose(W.double().cpu().numpy(), Wr, rtol=2e-5, atol=2e-8)
    np.testing.assert_allclose(m.double().cpu().numpy(), mr, rtol=1e-5, atol=2e-9)   # |g| ~ 1e-2: a few fp32 ulps of the addends
    np.testing.assert_allclose(v.double().cpu().numpy(), vr, rtol=1e-5, atol=1e-12)
    np.testing.assert_array_equal(out.double().cpu().numpy(), orc.round_storage(W.double().cpu().numpy(), dtype))


@pytest.mark.parametrize("P,N,dtype,present", [(7, 3, "fp16", [1, 0, 1]), (4099, 5, "bf16", [0, 1, 1, 1, 0]), (4096, 4, "fp32", [1, 1, 1, 1]),
                                               (533001, 64, "fp16", None), (64, 4, "fp16", [0, 0, 0, 0]), (1, 2, "fp16", [0, 1])])
def test_grad_average_masked_matches_oracle(hip, P, N, dtype, present):
    """Fault-tolerant average: only the workers that reported count; what the absent rows
    hold (Inf and NaN included) is never read."""
    import torch
    print(f"[case] grad_average_masked P={P} N={N} {dtype}", flush=True)
    gen = torch.Generator(device="cuda").manual_seed(P % 1000 + 7 * N)
    S = 512.0
    if present is None:                                    # 60 of 64 workers: a 94 % quorum
        rng = np.random.default_rng(5)
        present = np.ones(N, dtype=np.int32)
        present[rng.choice(N, 4, replace=False)] = 0
    present = np.asarray(present, dtype=np.int32)
    g = (torch.randn((N, P), device="cuda", generator=gen) * 3.0).to(_tdtype(torch, dtype))
    for w in range(N):                                     # poison the absent rows
        if not present[w]:
            g[w] = float("nan") if w % 2 else float("inf")
    mask = torch.tensor(present, dtype=torch.int32, device="cuda") * 5     # any non-zero value means present
    scale = torch.tensor([S], device="cuda"); avg = torch.full((P,), -7.0, device="cuda")
    flag = torch.full((1,), 7, dtype=torch.int32, device="cuda"); cnt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    hip.grad_average_masked(P, N, g, CODE[dtype], scale, mask, avg, flag, cnt)
    torch.cuda.synchronize()
    want, inf, n = orc.grad_average_partial(g.double().cpu().numpy(), S, present)
    assert int(cnt.item()) == n == int(present.sum())
    assert int(flag.item()) == 0 and not inf
    np.testing.assert_allclose(avg.double().cpu().numpy(), want, rtol=2e-6, atol=1e-9)
    if n:
        w = int(np.flatnonzero(present)[-1])
        g[w, P - 1] = float("inf")                          # an overflow in a present worker is reported
        hip.grad_average_masked(P, N, g, CODE[dtype], scale, mask, avg, flag, None)
        torch.cuda.synchronize()
        assert int(flag.item()) == 1
        assert orc.grad_average_partial(g.double().cpu().numpy(), S, present)[1]


def test_grad_average_masked_all_present_equals_lockstep(hip):
    import torch
    P, N = 20011, 6
    g = (torch.randn((N, P), device="cuda") * 2.0).half()
    scale = torch.tensor([64.0], device="cuda")
    a0 = torch.empty(P, device="cuda"); a1 = torch.empty(P, device="cuda"); flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    hip.grad_average(P, N, g, 1, scale, a0, flag)
    hip.grad_average_masked(P, N, g, 1, scale, torch.ones(N, dtype=torch.int32, device="cuda"), a1, flag)
    torch.cuda.synchronize()
    assert torch.equal(a0, a1)
    with pytest.raises(hip.LstmError):
        hip.grad_average_masked(P, N, g, 1, scale, None, a1, flag)
