"""The whole-sequence GEMM kernels on their own, through the C ABI's diagnostic entry point,
against a float64 matmul on the same fp16/bf16-rounded operands: every operand layout the
training step uses (row-major K-contiguous, row-major transposed, 64x64-blocked in three role
combinations), shapes with several tiles and ragged edges, and split-K; the fp32
mode's kernel against the same matmul."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hip():
    import paper_1912_00286_amd as pkg
    pkg.load_library()
    return pkg


def _blocked(hip, torch, t, code):
    R, C = t.shape
    out = torch.full((((R + 63) // 64) * ((C + 63) // 64) * 4096,), float("nan"), dtype=t.dtype, device=t.device)
    hip.lstm_debug_pack_blocked(code, t.contiguous(), R, C, out)
    return out


SHAPES = [(256, 256, 64), (520, 264, 136), (1024, 512, 448), (192, 200, 72), (777 // 8 * 8, 328, 1000)]


@pytest.mark.parametrize("layout", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_gemm_layouts_match_matmul(hip, layout, dtype):
    import torch
    code = {"fp16": 1, "bf16": 2}[dtype]
    tdt = {"fp16": torch.float16, "bf16": torch.bfloat16}[dtype]
    dev = torch.device("cuda:0")
    for (M, N, K) in SHAPES:
        for splits in (1, 3):
            print(f"[case] gemm layout {layout} {dtype} M={M} N={N} K={K} splits={splits}", flush=True)
            gen = torch.Generator(device="cuda").manual_seed(M + N + K + layout)
            a_t = layout in (1, 4)          # A stored [K, M]
            b_t = layout in (1, 3, 4)       # B stored [K, N]
            A0 = torch.randn((K, M) if a_t else (M, K), device=dev, generator=gen).to(tdt)
            B0 = torch.randn((K, N) if b_t else (N, K), device=dev, generator=gen).to(tdt)
            A64 = A0.double().cpu().numpy(); B64 = B0.double().cpu().numpy()
            ref = (A64.T if a_t else A64) @ (B64 if b_t else B64.T)
            A, B = (A0, B0) if layout <= 1 else (_blocked(hip, torch, A0, code), _blocked(hip, torch, B0, code))
            C = torch.full((M, N), float("nan"), dtype=tdt, device=dev)
            ws = torch.empty(splits * M * N, device=dev) if splits > 1 else None
            hip.lstm_debug_gemm(code, layout, M, N, K, A, B, C, ws, splits)
            torch.cuda.synchronize()
            got = C.double().cpu().numpy()
            # fp32 accumulation, one rounding to the 16-bit type at the end
            tol = (2.0 ** -8 if dtype == "bf16" else 2.0 ** -11) * np.abs(ref) + 1e-3 * np.sqrt(K) * 2.0 ** -9
            assert np.all(np.isfinite(got))
            assert np.all(np.abs(got - ref) <= tol + 1e-6), float(np.max(np.abs(got - ref) - tol))


F32_SHAPES = [(128, 800, 200), (100, 37, 9), (1100, 1030, 77), (320, 200, 4096), (2048, 1024, 64), (64, 64, 3), (33, 65, 132)]


def test_gemm_fp32_matches_matmul(hip):
    """The all-fp32 baseline mode's GEMM (fp32 MFMA): both tile sizes, 16-byte and element-wise loads
    (K % 4 != 0), ragged edges, split-K; error within the fp32 summation bound K u sum|a||b|."""
    import torch
    dev = torch.device("cuda:0")
    for (M, N, K) in F32_SHAPES:
        for splits in (1, 3):
            print(f"[case] gemm fp32 M={M} N={N} K={K} splits={splits}", flush=True)
            gen = torch.Generator(device="cuda").manual_seed(M + N + K)
            A = torch.randn((M, K), device=dev, generator=gen)
            B = torch.randn((N, K), device=dev, generator=gen)
            A64 = A.double().cpu().numpy(); B64 = B.double().cpu().numpy()
            ref = A64 @ B64.T
            C = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
            ws = torch.empty(splits * M * N, device=dev) if splits > 1 else None
            hip.lstm_debug_gemm(0, 0, M, N, K, A, B, C, ws, splits)
            torch.cuda.synchronize()
            got = C.double().cpu().numpy()
            tol = 2.0 * (K + 4) * 2.0 ** -24 * (np.abs(A64) @ np.abs(B64).T)
            assert np.all(np.isfinite(got))
            assert np.all(np.abs(got - ref) <= tol), float(np.max(np.abs(got - ref) - tol))


@pytest.mark.parametrize("shape", [(130, 70), (130, 72), (64, 200), (1, 8)], ids=["element_wise", "vector_ragged_rows", "vector_one_row_block", "vector_tiny"])
def test_blocked_packing_layout(hip, shape):
    import torch
    dev = torch.device("cuda:0")
    R, C = shape
    nrb, ncb = (R + 63) // 64, (C + 63) // 64
    src = (torch.arange(R * C, device=dev, dtype=torch.float32).reshape(R, C) % 2039).to(torch.float16)
    dst = _blocked(hip, torch, src, 1).cpu().numpy().astype(np.float64).reshape(nrb, ncb, 64, 64)
    s = src.cpu().numpy().astype(np.float64)
    want = np.zeros((nrb * 64, ncb * 64)); want[:R, :C] = s
    want = want.reshape(nrb, 64, ncb, 64).transpose(0, 2, 1, 3)
    assert np.array_equal(dst, want)


def test_unsupported_shapes_are_rejected(hip):
    import torch
    dev = torch.device("cuda:0")
    A = torch.zeros(64 * 64, dtype=torch.float16, device=dev)
    with pytest.raises(hip.LstmError):
        hip.lstm_debug_gemm(1, 1, 64, 64, 64, A, A, A)          # transposed form needs M, N >= 192
    with pytest.raises(hip.LstmError):
        hip.lstm_debug_gemm(0, 2, 256, 256, 64, A, A, A)        # blocked form has no fp32 kernel
