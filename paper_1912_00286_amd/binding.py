"""ctypes binding of liblstm_mi355.so: argument marshalling only.

Every function mirrors the C entry point of the same name in
include/lstm_mi355.h.  Tensors are passed as raw device addresses
(`tensor.data_ptr()`), the stream as torch's current HIP stream handle.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "liblstm_mi355.so"

DTYPE_FP32, DTYPE_FP16, DTYPE_BF16 = 0, 1, 2
HEAD_STEP_BCE, HEAD_LAST_BCE, HEAD_STEP_MSE, HEAD_FC_HINGE = 1, 2, 3, 4
OPT_SGD_MOMENTUM, OPT_ADAM = 0, 1
P_EMBED, P_W, P_U, P_B, P_HEAD_W, P_HEAD_B, P_FC_W, P_FC_B = 0, 1, 2, 3, 4, 5, 6, 7


class LstmError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"lstm_mi355 status {status}: {text}")
        self.status = status


class LstmConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("num_layers", "input_dim", "hidden", "seq_len", "batch", "dtype", "head",
                                         "out_dim", "vocab", "embed_dim", "head_hidden", "workers")]


class OptimizerConfig(C.Structure):
    _fields_ = [("kind", C.c_int32), ("momentum", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float), ("dynamic_scale", C.c_int32),
                ("scale_backoff", C.c_float), ("scale_growth", C.c_float), ("growth_interval", C.c_int32)]


def library_path() -> str:
    return os.path.join(HERE, _LIB_NAME)


_lib = None


def load_library():
    """Load the HIP library built in-tree.  No fallback: raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback for the HIP path)")
    lib = C.CDLL(path)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    cfgp, optp = C.POINTER(LstmConfig), C.POINTER(OptimizerConfig)
    lib.lstm_abi_version.restype = C.c_int
    lib.lstm_last_error.restype = C.c_char_p
    lib.lstm_param_count.argtypes = [cfgp, C.POINTER(i64)]
    lib.lstm_param_offset.argtypes = [cfgp, i32, i32, C.POINTER(i64), C.POINTER(i64)]
    lib.lstm_workspace_bytes.argtypes = [cfgp, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    sz = C.c_size_t
    lib.lstm_forward.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, sz, vp, sz, vp, vp, vp, vp]
    lib.lstm_backward.argtypes = [cfgp, vp, vp, vp, vp, sz, vp, sz, vp, vp, vp]
    lib.lstm_forward_static_scratch.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, sz, vp, vp, vp, vp]
    lib.lstm_forward_static_scratch.restype = C.c_int
    lib.lstm_cast_params.argtypes = [i64, vp, vp, i32, vp]
    lib.lstm_debug_plan_regions.argtypes = [cfgp, i32, C.POINTER(i32), C.POINTER(sz), C.POINTER(sz), C.POINTER(i32)]
    lib.grad_average.argtypes = [i64, i32, vp, i32, vp, vp, vp, vp]
    lib.grad_average_masked.argtypes = [i64, i32, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.master_update.argtypes = [i64, optp, f32, i64, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp]
    lib.lr_schedule.argtypes = [f32, i32, f32, f32, i32, f32, i64]
    lib.lr_schedule.restype = f32
    lib.lstm_debug_gemm.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, i32, vp]
    lib.lstm_debug_pack_blocked.argtypes = [i32, vp, i32, i32, vp, vp]
    lib.lstm_debug_gemm_stream.argtypes = [i32, i32, i32, i32, i32, i64, i32, vp, vp, vp, vp, vp]
    lib.lstm_debug_mfma_rate.argtypes = [i32, vp, i32, vp, C.POINTER(C.c_double), vp]
    lib.lstm_timing_enable.argtypes = [i32]
    lib.lstm_timing_read.argtypes = [i32, C.POINTER(i64), C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double)]
    for name in ("lstm_param_count", "lstm_param_offset", "lstm_workspace_bytes", "lstm_forward", "lstm_backward",
                 "grad_average", "grad_average_masked", "master_update", "lstm_cast_params", "lstm_timing_enable", "lstm_timing_read",
                 "lstm_debug_gemm", "lstm_debug_gemm_stream", "lstm_debug_pack_blocked", "lstm_debug_mfma_rate", "lstm_debug_plan_regions"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        raise LstmError(status, lstm_last_error())


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (None passes NULL); ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def lstm_abi_version() -> int:
    return load_library().lstm_abi_version()


def lstm_last_error() -> str:
    return load_library().lstm_last_error().decode()


def lstm_param_count(cfg: LstmConfig) -> int:
    n = C.c_int64()
    _check(load_library().lstm_param_count(C.byref(cfg), C.byref(n)))
    return n.value


def lstm_param_offset(cfg: LstmConfig, kind: int, layer: int = 0):
    off, cnt = C.c_int64(), C.c_int64()
    _check(load_library().lstm_param_offset(C.byref(cfg), kind, layer, C.byref(off), C.byref(cnt)))
    return off.value, cnt.value


def lstm_workspace_bytes(cfg: LstmConfig):
    r, s = C.c_size_t(), C.c_size_t()
    _check(load_library().lstm_workspace_bytes(C.byref(cfg), C.byref(r), C.byref(s)))
    return r.value, s.value


def _nbytes(t, given) -> int:
    """Size in bytes of a workspace tensor; a raw address needs the size spelled out."""
    if given is not None:
        return int(given)
    if t is None or isinstance(t, int):
        return 0
    return t.numel() * t.element_size()


def lstm_forward(cfg, params_lp, x, targets, h0, c0, reserve, scratch, loss, hT=None, cT=None, stream=None,
                 reserve_bytes=None, scratch_bytes=None):
    _check(load_library().lstm_forward(C.byref(cfg), _ptr(params_lp), _ptr(x), _ptr(targets), _ptr(h0), _ptr(c0),
                                       _ptr(reserve), _nbytes(reserve, reserve_bytes), _ptr(scratch),
                                       _nbytes(scratch, scratch_bytes), _ptr(loss), _ptr(hT), _ptr(cT), _stream(stream)))


STATIC_SCRATCH_BYTES = 32 << 20


def lstm_forward_static_scratch(cfg, params_lp, x, targets, h0, c0, reserve, loss, hT=None, cT=None, stream=None,
                                reserve_bytes=None):
    _check(load_library().lstm_forward_static_scratch(C.byref(cfg), _ptr(params_lp), _ptr(x), _ptr(targets), _ptr(h0),
                                                      _ptr(c0), _ptr(reserve), _nbytes(reserve, reserve_bytes), _ptr(loss),
                                                      _ptr(hT), _ptr(cT), _stream(stream)))


def lstm_backward(cfg, params_lp, x, targets, reserve, scratch, loss_scale, grads_lp, stream=None, reserve_bytes=None,
                  scratch_bytes=None):
    _check(load_library().lstm_backward(C.byref(cfg), _ptr(params_lp), _ptr(x), _ptr(targets), _ptr(reserve),
                                        _nbytes(reserve, reserve_bytes), _ptr(scratch), _nbytes(scratch, scratch_bytes),
                                        _ptr(loss_scale), _ptr(grads_lp), _stream(stream)))


def lstm_cast_params(n_params, master, params_lp_out, dtype, stream=None):
    _check(load_library().lstm_cast_params(n_params, _ptr(master), _ptr(params_lp_out), dtype, _stream(stream)))


def grad_average(n_params, n_workers, grads_lp, dtype, loss_scale, avg_grad, found_inf, stream=None):
    _check(load_library().grad_average(n_params, n_workers, _ptr(grads_lp), dtype, _ptr(loss_scale), _ptr(avg_grad),
                                       _ptr(found_inf), _stream(stream)))


def grad_average_masked(n_params, n_workers, grads_lp, dtype, loss_scale, participating, avg_grad, found_inf,
                        n_participating=None, stream=None):
    _check(load_library().grad_average_masked(n_params, n_workers, _ptr(grads_lp), dtype, _ptr(loss_scale),
                                              _ptr(participating), _ptr(avg_grad), _ptr(found_inf),
                                              _ptr(n_participating), _stream(stream)))


def master_update(n_params, opt, lr, step, master, state1, state2, avg_grad, found_inf, loss_scale, good_steps,
                  params_lp_out, dtype, stream=None):
    _check(load_library().master_update(n_params, C.byref(opt), lr, step, _ptr(master), _ptr(state1), _ptr(state2),
                                        _ptr(avg_grad), _ptr(found_inf), _ptr(loss_scale), _ptr(good_steps),
                                        _ptr(params_lp_out), dtype, _stream(stream)))


def lr_schedule(lr0, n_workers, n_half, eff_lr_max, warmup_steps, gamma, index) -> float:
    return float(load_library().lr_schedule(lr0, n_workers, n_half, eff_lr_max, warmup_steps, gamma, index))


KERNEL_CLASSES = ("gemm_batched", "gemm_step", "pointwise", "aux", "grad_average", "master_update")


def lstm_timing_enable(on: bool) -> None:
    _check(load_library().lstm_timing_enable(1 if on else 0))


def lstm_timing_read(kernel_class: int):
    n, ms, fl, by = C.c_int64(), C.c_double(), C.c_double(), C.c_double()
    _check(load_library().lstm_timing_read(kernel_class, C.byref(n), C.byref(ms), C.byref(fl), C.byref(by)))
    return dict(launches=n.value, total_ms=ms.value, flops=fl.value, bytes=by.value)


def lstm_debug_gemm(dtype, layout, M, N, K, A, B, Cout, splitk_ws=None, splits=1, stream=None):
    _check(load_library().lstm_debug_gemm(dtype, layout, M, N, K, _ptr(A), _ptr(B), _ptr(Cout), _ptr(splitk_ws), splits,
                                          _stream(stream)))


def lstm_debug_gemm_stream(dtype, M, N, K, rows_per_step, a_step_stride, gate_h, A, B, bias, Cout, stream=None):
    _check(load_library().lstm_debug_gemm_stream(dtype, M, N, K, rows_per_step, a_step_stride, gate_h, _ptr(A), _ptr(B),
                                                 _ptr(bias), _ptr(Cout), _stream(stream)))


def lstm_debug_mfma_rate(dtype, operands, iters, sink, stream=None) -> float:
    """Enqueue the register-resident MFMA loop; returns the flops it performs."""
    fl = C.c_double()
    _check(load_library().lstm_debug_mfma_rate(dtype, _ptr(operands), iters, _ptr(sink), C.byref(fl), _stream(stream)))
    return fl.value


def lstm_debug_pack_blocked(dtype, src, rows, cols, dst, stream=None):
    _check(load_library().lstm_debug_pack_blocked(dtype, _ptr(src), rows, cols, _ptr(dst), _stream(stream)))


def lstm_debug_plan_regions(cfg):
    """[(which, offset, bytes)] of the workspace plan: which = 0 reserve, 1 scratch."""
    lib = load_library()
    n = C.c_int32()
    _check(lib.lstm_debug_plan_regions(C.byref(cfg), 0, None, None, None, C.byref(n)))
    which, off, size = (C.c_int32 * n.value)(), (C.c_size_t * n.value)(), (C.c_size_t * n.value)()
    _check(lib.lstm_debug_plan_regions(C.byref(cfg), n.value, which, off, size, C.byref(n)))
    return [(which[i], off[i], size[i]) for i in range(n.value)]


# --------------------------------------------------------------------------
# buffer plumbing for a whole training step (no arithmetic here)
# --------------------------------------------------------------------------
class TrainingStep:
    """Owns the device buffers of one model and enqueues the entry points in
    the order of the paper's iteration: per worker fprop + bprop, then the
    gradient average, the schedule and the master update."""

    def __init__(self, cfg: LstmConfig, opt: OptimizerConfig, n_workers: int, master_fp32, loss_scale: float,
                 device="cuda:0", n_streams: int = 1, batched: bool = False):
        import copy
        import torch
        self.torch = torch
        self.cfg, self.opt, self.N = cfg, opt, int(n_workers)
        self.dev = torch.device(device)
        self.lp_dtype = {DTYPE_FP32: torch.float32, DTYPE_FP16: torch.float16, DTYPE_BF16: torch.bfloat16}[cfg.dtype]
        self.P = lstm_param_count(cfg)
        # batched: all workers' micro-batches go through one forward and one backward call
        # (lstm_config.workers); the per-worker losses and gradients come out as if each worker
        # had run alone.  Raises LstmError where the library has no such path for the shape.
        self.batched = bool(batched) and self.N > 1
        self.call_cfg = cfg
        if self.batched:
            self.call_cfg = copy.copy(cfg)
            self.call_cfg.workers = self.N
            n_streams = 1
        rb, sb = lstm_workspace_bytes(self.call_cfg)
        self.master = torch.as_tensor(master_fp32, dtype=torch.float32).to(self.dev).contiguous()
        assert self.master.numel() == self.P
        self.params_lp = torch.empty(self.P, dtype=self.lp_dtype, device=self.dev)
        lstm_cast_params(self.P, self.master, self.params_lp, cfg.dtype)      # the library's own rounding
        self.state1 = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        self.state2 = torch.zeros(self.P, dtype=torch.float32, device=self.dev) if opt.kind == OPT_ADAM else None
        self.grads = torch.zeros((self.N, self.P), dtype=self.lp_dtype, device=self.dev)
        self.avg = torch.zeros(self.P, dtype=torch.float32, device=self.dev)
        # The simulated workers are independent until their gradients are averaged.  With
        # n_streams > 1 they are spread over that many streams (default priority), each with a
        # workspace of its own, so that the short dependent kernel chains of small models overlap.
        self.n_streams = max(1, min(int(n_streams), self.N))
        self.reserves = [torch.empty(rb, dtype=torch.uint8, device=self.dev) for _ in range(self.n_streams)]
        self.scratches = [torch.empty(sb, dtype=torch.uint8, device=self.dev) for _ in range(self.n_streams)]
        self.reserve, self.scratch = self.reserves[0], self.scratches[0]
        self.side_streams = [torch.cuda.Stream(device=self.dev) for _ in range(self.n_streams - 1)]
        self.losses = torch.zeros(self.N, dtype=torch.float32, device=self.dev)
        self.loss_scale = torch.tensor([loss_scale], dtype=torch.float32, device=self.dev)
        self.found_inf = torch.zeros(1, dtype=torch.int32, device=self.dev)
        self.good_steps = torch.zeros(1, dtype=torch.int32, device=self.dev)
        self.step_index = 0

    def _worker(self, w, xs, ys, k, stream=None):
        lstm_forward(self.cfg, self.params_lp, xs[w], ys[w], None, None, self.reserves[k], self.scratches[k],
                     self.losses[w:w + 1], stream=stream)
        lstm_backward(self.cfg, self.params_lp, xs[w], ys[w], self.reserves[k], self.scratches[k], self.loss_scale,
                      self.grads[w], stream=stream)

    def stack_workers(self, xs, ys):
        """Per-worker tensors -> the [T, W, B, ...] layout of the batched form (copies)."""
        torch = self.torch
        x_all = torch.stack(list(xs), dim=1).contiguous()
        y_all = torch.stack(list(ys), dim=1 if ys[0].dim() == 3 else 0).contiguous()
        return x_all, y_all

    def forward_backward(self, xs, ys):
        """xs, ys: per-worker device tensors (x lp [T,B,I] or int32 ids; targets fp32).  In
        the batched form also accepted already stacked (see stack_workers)."""
        torch = self.torch
        if self.batched:
            if isinstance(xs, (list, tuple)):
                xs, ys = self.stack_workers(xs, ys)
            lstm_forward(self.call_cfg, self.params_lp, xs, ys, None, None, self.reserve, self.scratch, self.losses)
            lstm_backward(self.call_cfg, self.params_lp, xs, ys, self.reserve, self.scratch, self.loss_scale, self.grads)
            return
        if self.n_streams == 1:
            for w in range(self.N):
                self._worker(w, xs, ys, 0)
            return
        main = torch.cuda.current_stream(self.dev)
        for st in self.side_streams:                       # fork: the side streams see the current weights
            st.wait_stream(main)
        for w in range(self.N):
            k = w % self.n_streams
            self._worker(w, xs, ys, k, None if k == 0 else self.side_streams[k - 1])
        for st in self.side_streams:                       # join before the gradients are averaged
            main.wait_stream(st)

    def update(self, lr: float):
        grad_average(self.P, self.N, self.grads, self.cfg.dtype, self.loss_scale, self.avg, self.found_inf)
        self.step_index += 1
        master_update(self.P, self.opt, lr, self.step_index, self.master, self.state1, self.state2, self.avg,
                      self.found_inf, self.loss_scale, self.good_steps, self.params_lp, self.cfg.dtype)

    def step(self, xs, ys, lr: float):
        self.forward_backward(xs, ys)
        self.update(lr)

    # ---- the same step as one HIP graph launch plus the master update -----------------
    # Small models are bound by the host's launch rate (three launches per layer and time
    # step); replaying a recorded graph removes the per-launch host work.  The library
    # allocates nothing, never synchronises and records no memset, so its launches can be
    # captured as they are.  The graph holds the addresses of xs / ys: later batches are
    # copied into those same tensors.  The learning rate and the step count change from step
    # to step and are passed by value, so master_update stays outside the graph.
    def capture(self, xs, ys):
        torch = self.torch
        if self.batched and isinstance(xs, (list, tuple)):
            xs, ys = self.stack_workers(xs, ys)
        self._captured_inputs = (xs, ys)             # the graph reads these buffers on every replay
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.forward_backward(xs, ys)
            grad_average(self.P, self.N, self.grads, self.cfg.dtype, self.loss_scale, self.avg, self.found_inf)
        self.graph = graph

    def step_captured(self, lr: float):
        if getattr(self, "graph", None) is None:
            raise RuntimeError("step_captured: call capture(xs, ys) first")
        self.graph.replay()
        self.step_index += 1
        master_update(self.P, self.opt, lr, self.step_index, self.master, self.state1, self.state2, self.avg,
                      self.found_inf, self.loss_scale, self.good_steps, self.params_lp, self.cfg.dtype)
