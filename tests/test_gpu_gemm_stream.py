"""The whole-sequence GEMM on packed (MFMA-fragment order) operands against torch's fp32 matmul.

The operands are packed here, on the host, from the layout formula the header states, so the test also pins the
layout itself; the products the training step sends through this kernel are covered by the parity tests of the
wide-layer schedule."""
import numpy as np
import pytest
import torch

import paper_1912_00286_amd as hip

pytestmark = pytest.mark.gpu

DT = {"fp16": (hip.DTYPE_FP16, torch.float16, 2e-3), "bf16": (hip.DTYPE_BF16, torch.bfloat16, 1.6e-2)}


def pack_tiles(x: torch.Tensor, tile_rows: int) -> torch.Tensor:
    """[R, K] -> [R / tile_rows][K / 64][chunk], element (row, k) of a chunk at
    ((k/16 * nblk + row/32) * 64 + 32 * (k/8 % 2) + row % 32) * 8 + k % 8."""
    R, K = x.shape
    assert R % tile_rows == 0 and K % 64 == 0
    nblk = tile_rows // 32
    row = torch.arange(tile_rows).view(-1, 1).expand(tile_rows, 64)
    k = torch.arange(64).view(1, -1).expand(tile_rows, 64)
    off = ((k // 16 * nblk + row // 32) * 64 + 32 * (k // 8 % 2) + row % 32) * 8 + k % 8
    chunks = x.view(R // tile_rows, tile_rows, K // 64, 64).permute(0, 2, 1, 3).reshape(-1, tile_rows * 64)
    out = torch.empty_like(chunks)
    out[:, off.reshape(-1)] = chunks
    return out.reshape(-1)


CASES = [
    # M, N, K, rows_per_step, gated, bias
    (512, 512, 256, 256, False, False),
    (768, 384, 512, 192, False, True),      # steps of three row tiles, N not a multiple of the 256-column tile
    (448, 1024, 256, 64, True, True),       # M not a multiple of the 256-row tile, gate-interleaved columns
    (2048, 2560, 1024, 256, True, True),    # H = 640: the last column tile is half empty
    (1024, 2048, 2048, 512, False, False),
    (320, 328, 256, 64, False, True),       # N a multiple of 8 only: a lane pair of the result stores straddles the edge
    (256, 384, 512, 128, True, True),       # H = 96: the second B tile of the last column tile is empty
]


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("M,N,K,rps,gated,with_bias", CASES)
def test_gemm_stream_matches_fp32_matmul(dtype, M, N, K, rps, gated, with_bias):
    code, tdt, tol = DT[dtype]
    g = torch.Generator().manual_seed(M * 7 + N * 3 + K)
    A = (torch.randn(M, K, generator=g) * 0.5).to(tdt)
    B = (torch.randn(N, K, generator=g) * 0.5).to(tdt)
    bias = torch.randn(N, generator=g).to(tdt) if with_bias else None
    ref = A.float() @ B.float().T + (bias.float() if with_bias else 0.0)
    # A: every time step's rows packed on their own, steps a padded stride apart
    steps = M // rps
    per_step = rps * K
    stride = per_step + 4096
    Apk = torch.zeros(steps * stride, dtype=tdt)
    for s in range(steps):
        Apk[s * stride: s * stride + per_step] = pack_tiles(A[s * rps:(s + 1) * rps], 64)
    if gated:
        H = N // 4
        assert H % 32 == 0
        # B tile j holds, for each gate g, the rows g H + 32 j .. g H + 32 j + 31
        idx = torch.arange(N).view(4, H // 32, 32).permute(1, 0, 2).reshape(-1)
        Bt = B[idx]
        gate_h = H
    else:
        pad = (-N) % 128
        Bt = torch.cat([B, torch.zeros(pad, K, dtype=tdt)]) if pad else B
        gate_h = 0
    Bpk = pack_tiles(Bt, 128)
    dev = torch.device("cuda:0")
    C = torch.full((M, N), float("nan"), dtype=tdt, device=dev)
    hip.lstm_debug_gemm_stream(code, M, N, K, rps, stride, gate_h, Apk.to(dev), Bpk.to(dev),
                               bias.to(dev) if with_bias else None, C)
    torch.cuda.synchronize()
    got = C.float().cpu()
    assert torch.isfinite(got).all()
    err = (got - ref).abs().max().item()
    scale = ref.abs().max().item()
    assert err <= tol * scale, f"max error {err:.3e} against scale {scale:.3e}"


TN_CASES = [
    # M, N, K
    (512, 512, 256),
    (768, 320, 384),        # N not a multiple of the 256-column tile, nor of 64
    (264, 1024, 1152),      # M not a multiple of 64
    (2048, 2048, 4096),
]


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("M,N,K", TN_CASES)
def test_gemm_stream_tn_matches_fp32_matmul(dtype, M, N, K):
    """C = A^T B with both operands 64x64-blocked and the contraction index as their rows (the weight-gradient
    products), on the second kernel (layout 5 of the diagnostic GEMM call)."""
    code, tdt, tol = DT[dtype]
    g = torch.Generator().manual_seed(M + 3 * N + 7 * K)
    A = (torch.randn(K, M, generator=g) * 0.5).to(tdt)
    B = (torch.randn(K, N, generator=g) * 0.5).to(tdt)
    ref = A.float().T @ B.float()
    dev = torch.device("cuda:0")

    def blocked(x):
        r, c = x.shape
        out = torch.empty(((r + 63) // 64) * ((c + 63) // 64) * 4096, dtype=tdt, device=dev)
        hip.lstm_debug_pack_blocked(code, x.to(dev).contiguous(), r, c, out)
        return out

    C = torch.full((M, N), float("nan"), dtype=tdt, device=dev)
    hip.lstm_debug_gemm(code, 5, M, N, K, blocked(A), blocked(B), C)
    torch.cuda.synchronize()
    got = C.float().cpu()
    assert torch.isfinite(got).all()
    err = (got - ref).abs().max().item()
    scale = ref.abs().max().item()
    assert err <= tol * scale, f"max error {err:.3e} against scale {scale:.3e}"


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("M,N,K", [(512, 512, 256), (768, 320 + 64, 384), (2048, 2048, 4096)])
def test_gemm_stream_tn_on_fragment_order_blocks(dtype, M, N, K):
    """The same product with every 64x64 block of both operands in fragment order (layout 6): the packed h_t / dA_t
    copies of the recurrence, one time step after the other, serve as the weight-gradient operands as they are."""
    code, tdt, tol = DT[dtype]
    g = torch.Generator().manual_seed(5 * M + N + K)
    A = (torch.randn(K, M, generator=g) * 0.5).to(tdt)
    B = (torch.randn(K, N, generator=g) * 0.5).to(tdt)
    ref = A.float().T @ B.float()
    dev = torch.device("cuda:0")
    C = torch.full((M, N), float("nan"), dtype=tdt, device=dev)
    hip.lstm_debug_gemm(code, 6, M, N, K, pack_tiles(A, 64).to(dev), pack_tiles(B, 64).to(dev), C)
    torch.cuda.synchronize()
    got = C.float().cpu()
    assert torch.isfinite(got).all()
    err = (got - ref).abs().max().item()
    scale = ref.abs().max().item()
    assert err <= tol * scale, f"max error {err:.3e} against scale {scale:.3e}"


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("layout", [5, 6])
@pytest.mark.parametrize("M,N,K,splits", [(512, 256, 1024, 4), (768, 320, 768, 2), (2048, 512, 8192, 4)])
def test_gemm_stream_tn_split_k(dtype, layout, M, N, K, splits):
    """A narrow result (few tiles) with the contraction cut into equal splits: fp32 partial tiles in the caller's
    workspace, added up in split order."""
    code, tdt, tol = DT[dtype]
    g = torch.Generator().manual_seed(7 * M + N + K + splits)
    A = (torch.randn(K, M, generator=g) * 0.5).to(tdt)
    B = (torch.randn(K, N, generator=g) * 0.5).to(tdt)
    ref = A.float().T @ B.float()
    dev = torch.device("cuda:0")
    C = torch.full((M, N), float("nan"), dtype=tdt, device=dev)
    ws = torch.full((splits, M, N), float("nan"), dtype=torch.float32, device=dev)

    def blocked(x):
        r, c = x.shape
        out = torch.empty(((r + 63) // 64) * ((c + 63) // 64) * 4096, dtype=tdt, device=dev)
        hip.lstm_debug_pack_blocked(code, x.to(dev).contiguous(), r, c, out)
        return out

    form = blocked if layout == 5 else (lambda x: pack_tiles(x, 64).to(dev))
    hip.lstm_debug_gemm(code, layout, M, N, K, form(A), form(B), C, ws, splits)
    torch.cuda.synchronize()
    got = C.float().cpu()
    assert torch.isfinite(got).all()
    err = (got - ref).abs().max().item()
    scale = ref.abs().max().item()
    assert err <= tol * scale, f"max error {err:.3e} against scale {scale:.3e}"
