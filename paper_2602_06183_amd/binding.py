"""ctypes binding of libsparseffn.so: argument marshalling only.

bf16 tensors are torch.bfloat16 (or int16/uint16 bit-pattern) CUDA tensors; outputs are allocated
here with torch.empty and returned.  Kernels are enqueued on torch's current stream.
"""
import ctypes
import os

import torch

MODE_HARD, MODE_SOFT = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class SffnError(RuntimeError):
    pass


class _Buffers(ctypes.Structure):
    _fields_ = [("scratch", ctypes.c_void_p), ("scratch_bytes", ctypes.c_size_t), ("saved", ctypes.c_void_p), ("saved_bytes", ctypes.c_size_t),
                ("weights", ctypes.c_void_p), ("weights_bytes", ctypes.c_size_t)]


class _Cfg(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int64), ("D", ctypes.c_int64), ("F", ctypes.c_int64), ("V", ctypes.c_int32),
                ("M", ctypes.c_int32), ("mode", ctypes.c_int32), ("flags", ctypes.c_int32)]


class _Layout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in ("w1_vals", "w1_meta", "w2t_vals", "w2t_meta", "y1", "y2_vals", "y2_meta",
                                               "colidx", "dy2", "dy1_vals", "y1_kept", "y1_kept_bytes", "total")]


class _Fp8Layout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in ("w1_codes", "w1_meta", "w2t_codes", "w2t_meta", "y1", "y2_codes", "y2_meta", "colidx",
                                               "dy2", "dy1_vals", "y1_kept", "total")]


class _Fp8Scales(ctypes.Structure):
    _fields_ = [(n, ctypes.c_float) for n in ("x", "w1", "w2", "y2", "dy", "dy1")]


class _RouterLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in ("y1c", "vals", "meta", "colidx", "dy2c", "dvals", "total")]


def lib_path():
    return os.path.join(_HERE, "libsparseffn.so")


def load():
    """Loads the HIP library; raises if it has not been built (there is no fallback path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise SffnError("libsparseffn.so is not built: run `python -m paper_2602_06183_amd.build` "
                        "(or __graft_entry__.build()); there is no CPU fallback")
    lib = ctypes.CDLL(path)
    p, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    lib.sffn_version.restype = ctypes.c_int
    lib.sffn_last_error.restype = ctypes.c_char_p
    lib.sffn_workspace_bytes.restype = sz
    lib.sffn_workspace_bytes.argtypes = [ctypes.POINTER(_Cfg)]
    lib.sffn_workspace_layout.argtypes = [ctypes.POINTER(_Cfg), ctypes.POINTER(_Layout)]
    lib.sffn_vnm_spmm_workspace_bytes.restype = sz
    lib.sffn_vnm_spmm_workspace_bytes.argtypes = [i64, i64, i64, i32]
    lib.sffn_vnm_wgrad_workspace_bytes.restype = sz
    lib.sffn_vnm_wgrad_workspace_bytes.argtypes = [i64, i64, i64]
    lib.prune24_compress.argtypes = [p, i64, i64, i64, i32, i32, p, p, p]
    lib.sqrelu_vnm_compress.argtypes = [p, i64, i64, i32, i32, p, p, p, p]
    lib.spmm24_fwd.argtypes = [p, p, p, p, i64, i64, i64, p, p]
    lib.spmm24_dgrad.argtypes = [p, p, p, i64, i64, i64, p, p]
    lib.sffn_prepared24_bytes.restype = sz
    lib.sffn_prepared24_bytes.argtypes = [i64, i64]
    lib.prune24_compress_prepared.argtypes = [p, i64, i64, i64, i32, p, p, p, p]
    lib.sffn_spmm24_prepared_workspace_bytes.restype = sz
    lib.sffn_spmm24_prepared_workspace_bytes.argtypes = [i64, i64]
    lib.spmm24_prepared.argtypes = [p, p, p, i64, i64, i64, p, p, sz, p]
    lib.vnm_spmm.argtypes = [p, p, p, p, i64, i32, i64, i64, i64, i32, i32, p, p, sz, p]
    lib.dsqrelu_vnm.argtypes = [p, p, p, p, i64, i64, i32, i32, p, p]
    lib.vnm_wgrad.argtypes = [p, p, p, p, i64, i64, i64, i32, i32, i32, p, p, sz, p]
    lib.ffn_sparse_step.argtypes = [ctypes.POINTER(_Cfg)] + [p] * 9 + [p, sz, p]
    lib.ffn_sparse_step_noalloc.argtypes = [ctypes.POINTER(_Cfg)] + [p] * 9 + [p]
    lib.sffn_grouped_workspace_bytes.restype = sz
    lib.sffn_grouped_workspace_bytes.argtypes = [ctypes.POINTER(_Cfg), i32]
    lib.sffn_grouped_workspace_layout.argtypes = [ctypes.POINTER(_Cfg), i32, ctypes.POINTER(_Layout)]
    lib.ffn_sparse_step_grouped.argtypes = [ctypes.POINTER(_Cfg), i32, ctypes.POINTER(ctypes.c_int64)] + [p] * 9 + [p, sz, p]
    lib.sffn_venom_rows.restype = i64
    lib.sffn_venom_rows.argtypes = [i64, i32]
    lib.sffn_venom_route_workspace_bytes.restype = sz
    lib.sffn_venom_route_workspace_bytes.argtypes = [i64, i32]
    lib.venom_route.argtypes = [p, p, i64, i64, i32, p, p, p, p, p, p, sz, p]
    lib.sffn_venom_matmul_workspace_bytes.restype = sz
    lib.sffn_venom_matmul_workspace_bytes.argtypes = [i64, i64, i64, i32]
    lib.venom_expert_matmul.argtypes = [ctypes.POINTER(_Cfg), ctypes.POINTER(ctypes.c_int64)] + [p] * 8 + [p, sz, p]
    lib.sffn_router_workspace_bytes.restype = sz
    lib.sffn_router_workspace_bytes.argtypes = [ctypes.POINTER(_Cfg)]
    lib.sffn_router_workspace_layout.argtypes = [ctypes.POINTER(_Cfg), ctypes.POINTER(_RouterLayout)]
    lib.ffn_router_step.argtypes = [ctypes.POINTER(_Cfg), ctypes.POINTER(ctypes.c_int64)] + [p] * 10 + [p, sz, p]
    lib.sffn_router_full_workspace_bytes.restype = sz
    lib.sffn_router_full_workspace_bytes.argtypes = [ctypes.POINTER(_Cfg)]
    lib.ffn_router_full_step.argtypes = [ctypes.POINTER(_Cfg)] + [p] * 10 + [p, sz, p]
    f32 = ctypes.c_float
    lib.quantize_fp8.argtypes = [p, i64, f32, p, p, p]
    lib.prune24_compress_fp8.argtypes = [p, i64, i64, i64, i32, i32, f32, p, p, p, p]
    lib.sqrelu_vnm_compress_fp8.argtypes = [p, i64, i64, i32, i32, f32, p, p, p, p, p]
    lib.spmm24_fp8.argtypes = [p, f32, p, p, f32, p, i64, i64, i64, p, p]
    lib.sffn_vnm_spmm_fp8_workspace_bytes.restype = sz
    lib.sffn_vnm_spmm_fp8_workspace_bytes.argtypes = [i64, i64, i64]
    lib.vnm_spmm_fp8.argtypes = [p, p, p, f32, p, f32, i32, i64, i64, i64, i32, i32, p, p, sz, p]
    lib.sffn_fp8_workspace_bytes.restype = sz
    lib.sffn_fp8_workspace_bytes.argtypes = [ctypes.POINTER(_Cfg)]
    lib.sffn_fp8_workspace_layout.argtypes = [ctypes.POINTER(_Cfg), ctypes.POINTER(_Fp8Layout)]
    lib.ffn_sparse_step_fp8.argtypes = [ctypes.POINTER(_Cfg), ctypes.POINTER(_Fp8Scales), p, p, p, p, p, p, p, p, p, p, sz, p, p]
    lib.sffn_fp8_grouped_workspace_layout.argtypes = [ctypes.POINTER(_Cfg), i32, ctypes.POINTER(_Fp8Layout)]
    lib.ffn_sparse_step_fp8_grouped.argtypes = [ctypes.POINTER(_Cfg), ctypes.POINTER(_Fp8Scales), i32, p, p, p, p, p, p, p, p, p, p, p, sz, p, p]
    cfgp, scp, segp, bufp = ctypes.POINTER(_Cfg), ctypes.POINTER(_Fp8Scales), ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(_Buffers)
    lib.sffn_buffer_sizes.argtypes = [cfgp, i32, bufp]
    lib.sffn_fp8_buffer_sizes.argtypes = [cfgp, i32, bufp]
    lib.ffn_sparse_forward.argtypes = [cfgp] + [p] * 5 + [bufp, p]
    lib.ffn_sparse_backward.argtypes = [cfgp] + [p] * 5 + [bufp, p]
    lib.ffn_sparse_forward_grouped.argtypes = [cfgp, i32, segp] + [p] * 5 + [bufp, p]
    lib.ffn_sparse_backward_grouped.argtypes = [cfgp, i32, segp] + [p] * 5 + [bufp, p]
    lib.ffn_sparse_forward_fp8.argtypes = [cfgp, scp] + [p] * 5 + [bufp, p, p]
    lib.ffn_sparse_backward_fp8.argtypes = [cfgp, scp] + [p] * 4 + [bufp, p, p]
    lib.ffn_sparse_forward_fp8_grouped.argtypes = [cfgp, scp, i32, segp] + [p] * 5 + [bufp, p, p]
    lib.ffn_sparse_backward_fp8_grouped.argtypes = [cfgp, scp, i32, segp] + [p] * 4 + [bufp, p, p]
    lib.ffn_router_forward.argtypes = [cfgp, segp] + [p] * 6 + [p, sz, p]
    lib.ffn_router_backward.argtypes = [cfgp, segp] + [p] * 5 + [p, sz, p]
    lib.ffn_router_full_forward.argtypes = [cfgp] + [p] * 6 + [p, sz, p]
    lib.ffn_router_full_backward.argtypes = [cfgp] + [p] * 4 + [p, sz, p]
    lib.sffn_dense_sqrelu.argtypes = [p, p, i64, p]
    lib.sffn_dense_dsqrelu.argtypes = [p, p, p, i64, p]
    lib.sffn_profile_enable.argtypes = [i32]
    lib.sffn_profile_read.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_char_p), i32]
    _LIB = lib
    return lib


def _check(rc):
    if rc != 0:
        raise SffnError("libsparseffn error %d: %s" % (rc, load().sffn_last_error().decode()))


def _ptr(t, rows_strided=False):
    if t is None:
        return None
    ok = t.is_contiguous() or (rows_strided and t.dim() == 2 and t.stride(1) == 1)
    if not t.is_cuda or not ok:
        raise SffnError("expected a contiguous device tensor")
    return ctypes.c_void_p(t.data_ptr())


_BF16 = (torch.bfloat16, torch.int16, torch.uint16)      # bf16 values or their bit patterns
_U8 = (torch.uint8,)
_F32 = (torch.float32,)
_I32 = (torch.int32,)


def _want(name, t, shape, kinds, optional=False):
    """The C ABI sees raw pointers only, so sizes and element types are checked here, before any call: a short or
    mistyped tensor would otherwise become an out-of-bounds device access inside a kernel."""
    if t is None:
        if optional:
            return
        raise SffnError("%s: missing tensor" % name)
    if tuple(t.shape) != tuple(int(v) for v in shape):
        raise SffnError("%s: expected shape %s, got %s" % (name, tuple(int(v) for v in shape), tuple(t.shape)))
    if t.dtype not in kinds:
        raise SffnError("%s: expected dtype %s, got %s" % (name, " / ".join(str(k) for k in kinds), t.dtype))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _bf16(shape, dev):
    return torch.empty(shape, dtype=torch.bfloat16, device=dev)


def _u8(shape, dev):
    return torch.empty(shape, dtype=torch.uint8, device=dev)


def version():
    return load().sffn_version()


def profile_enable(on=True):
    _check(load().sffn_profile_enable(int(on)))


def profile_read():
    """[(stage name, milliseconds)] for every kernel launch of the most recent ffn_sparse_step."""
    ms = (ctypes.c_float * 32)()
    names = (ctypes.c_char_p * 32)()
    n = load().sffn_profile_read(ms, names, 32)
    if n < 0:
        _check(n)
    return [(names[i].decode(), float(ms[i])) for i in range(n)]


FLAG_KEEP_DENSE = 1
FLAG_UNFUSED = 2
FLAG_FP8_WGRAD = 4
FLAG_LEAN = 8
FLAG_WEIGHTS_PACKED = 16
FLAG_DW_FP32_ACCUMULATE = 32


def dense_sqrelu(y1, out):
    """Measurement aid: eq. (2) on a whole tensor in one pass (the dense baseline's element-wise kernel)."""
    _want("dense_sqrelu: out", out, y1.shape, _BF16)
    _check(load().sffn_dense_sqrelu(_ptr(y1), _ptr(out), y1.numel(), _stream()))
    return out


def dense_dsqrelu(dy2, y1, out):
    """Measurement aid: eq. (6) on whole tensors in one pass."""
    _want("dense_dsqrelu: y1", y1, dy2.shape, _BF16)
    _want("dense_dsqrelu: out", out, dy2.shape, _BF16)
    _check(load().sffn_dense_dsqrelu(_ptr(dy2), _ptr(y1), _ptr(out), dy2.numel(), _stream()))
    return out


def _cfg(T, D, F, mode=MODE_HARD, V=64, M=8, flags=0):
    return _Cfg(T, D, F, V, M, mode, flags)


def _dw(shape, device, fp32):
    """A weight-gradient output: bf16, overwritten by every call, or a float32 accumulator (zero) that every call adds to."""
    return torch.zeros(shape, dtype=torch.float32, device=device) if fp32 else _bf16(shape, device)


class _StepBuffers:
    """The three regions of a step's workspace (scratch | saved | weights, in the order of the layout's offsets).  Without `scratch` they are
    one allocation (`ws`), which is also what the one-call entry points take; with `scratch` (a uint8 CUDA tensor that several step objects may
    share: nothing in it outlives a call) the saved and weights regions are this object's own and only forward() / backward() can run."""

    def _alloc_regions(self, sizes_fn, n_experts, device, scratch, weights_of=None):
        b = _Buffers()
        _check(sizes_fn(ctypes.byref(self.cfg), n_experts, ctypes.byref(b)))
        self._b1, self._b2 = b.scratch_bytes, b.scratch_bytes + b.saved_bytes
        total = self._b2 + b.weights_bytes
        if scratch is None and weights_of is None:
            self.ws = _u8((total,), device)
            self._scratch, self._saved, self._weights = self.ws[:self._b1], self.ws[self._b1:self._b2], self.ws[self._b2:]
        else:
            if scratch is None:
                scratch = _u8((b.scratch_bytes,), device)
            if scratch.dtype != torch.uint8 or not scratch.is_cuda or scratch.numel() < b.scratch_bytes or scratch.data_ptr() % 256:
                raise SffnError("scratch must be a 256-byte aligned uint8 CUDA tensor of at least %d bytes" % b.scratch_bytes)
            if weights_of is not None and weights_of._weights.numel() != b.weights_bytes:
                raise SffnError("weights_of: that step object has another shape")
            self.ws = None
            self._scratch, self._saved = scratch, _u8((b.saved_bytes,), device)
            # weights_of: another micro-batch of the same layer; the packed weights are that object's (it calls forward() first, this one
            # then runs forward(..., weights_packed=True))
            self._weights = weights_of._weights if weights_of is not None else _u8((b.weights_bytes,), device)
        b.scratch, b.saved, b.weights = self._scratch.data_ptr(), self._saved.data_ptr(), self._weights.data_ptr()
        b.scratch_bytes = self._scratch.numel()
        self._buf = b
        return total

    def _one_buffer(self):
        if self.ws is None:
            raise SffnError("this step object was built on a shared scratch buffer: use forward() / backward()")
        return _ptr(self.ws)

    def _drop_unwritten(self, out, M, weight_keys, activation_keys):
        """SFFN_FLAG_LEAN: the canonical copies that are not written have no room in the layout either."""
        if getattr(self, "lean", False):
            for k in weight_keys + (activation_keys if M == 8 else ()):
                out.pop(k, None)
        return out

    def _region_bytes(self, off, nbytes):
        """nbytes at layout offset `off`, wherever its region lives."""
        if off < self._b1:
            return self._scratch[off:off + nbytes]
        if off < self._b2:
            return self._saved[off - self._b1:off - self._b1 + nbytes]
        return self._weights[off - self._b2:off - self._b2 + nbytes]


def buffer_sizes(T, D, F, mode=MODE_HARD, M=8, keep_dense=False, lean=False, n_experts=1, fp8=False, wgrad_fp8=False):
    """Bytes of the three buffers of the split forward / backward calls: dict(scratch, saved, weights)."""
    flags = (FLAG_KEEP_DENSE if keep_dense else 0) | (FLAG_LEAN if lean else 0) | (FLAG_FP8_WGRAD if (fp8 and wgrad_fp8) else 0)
    c, b = _cfg(T, D, F, mode, M=M, flags=flags), _Buffers()
    _check((load().sffn_fp8_buffer_sizes if fp8 else load().sffn_buffer_sizes)(ctypes.byref(c), n_experts, ctypes.byref(b)))
    return dict(scratch=b.scratch_bytes, saved=b.saved_bytes, weights=b.weights_bytes)


def _cfg_with(cfg, weights_packed):
    """The step's configuration, with SFFN_FLAG_WEIGHTS_PACKED added when the caller says that the previous call on this object ran on
    the same W1 / W2 (micro-batches between two optimizer steps, Section 3.4): the pruning passes are then skipped."""
    if not weights_packed:
        return cfg
    return _Cfg(cfg.T, cfg.D, cfg.F, cfg.V, cfg.M, cfg.mode, cfg.flags | FLAG_WEIGHTS_PACKED)


def _flags(keep_dense, unfused=False, lean=False):
    return (FLAG_KEEP_DENSE if keep_dense else 0) | (FLAG_UNFUSED if unfused else 0) | (FLAG_LEAN if lean else 0)


def workspace_bytes(T, D, F, mode=MODE_HARD, M=8, keep_dense=False, unfused=False, lean=False):
    c = _cfg(T, D, F, mode, M=M, flags=_flags(keep_dense, unfused, lean))
    return load().sffn_workspace_bytes(ctypes.byref(c))


def workspace_layout(T, D, F, mode=MODE_HARD, M=8, keep_dense=False, unfused=False, lean=False):
    c, lay = _cfg(T, D, F, mode, M=M, flags=_flags(keep_dense, unfused, lean)), _Layout()
    _check(load().sffn_workspace_layout(ctypes.byref(c), ctypes.byref(lay)))
    return {n: getattr(lay, n) for n, _ in _Layout._fields_}


def prune24_compress(src, trans=False, mode=MODE_HARD):
    """src [R, K] (trans=False) or [K, R] (trans=True: groups run down the rows).  -> vals [R, K/2], meta [R, K/8]."""
    if src is None or src.dim() != 2 or src.dtype not in _BF16:
        raise SffnError("prune24_compress: src must be a 2-D bf16 tensor")
    rows, cols = src.shape
    R, K = (cols, rows) if trans else (rows, cols)
    vals, meta = _bf16((R, K // 2), src.device), _u8((R, K // 8), src.device)
    _check(load().prune24_compress(_ptr(src, True), R, K, src.stride(0), int(trans), mode, _ptr(vals), _ptr(meta), _stream()))
    return vals, meta


def sqrelu_vnm_compress(y1, V=64, M=8):
    if y1 is None or y1.dim() != 2 or y1.dtype not in _BF16:
        raise SffnError("sqrelu_vnm_compress: y1 must be a 2-D bf16 tensor")
    T, F = y1.shape
    vals, meta = _bf16((T, 2 * F // M), y1.device), _u8((T, F // (2 * M)), y1.device)
    colidx = _u8((T // V, F // M, 4), y1.device)
    _check(load().sqrelu_vnm_compress(_ptr(y1), T, F, V, M, _ptr(vals), _ptr(meta), _ptr(colidx), _stream()))
    return vals, meta, colidx


def spmm24_fwd(X, w_vals, w_meta, bias=None):
    if X is None or X.dim() != 2 or w_vals is None or w_vals.dim() != 2:
        raise SffnError("spmm24_fwd: X and w_vals must be 2-D tensors")
    T, K = X.shape
    N = w_vals.shape[0]
    _want("spmm24_fwd: X", X, (T, K), _BF16)
    _want("spmm24_fwd: w_vals", w_vals, (N, K // 2), _BF16)
    _want("spmm24_fwd: w_meta", w_meta, (N, K // 8), _U8)
    _want("spmm24_fwd: bias", bias, (N,), _F32, optional=True)
    out = _bf16((T, N), X.device)
    _check(load().spmm24_fwd(_ptr(X), _ptr(w_vals), _ptr(w_meta), _ptr(bias), T, N, K, _ptr(out), _stream()))
    return out


def prune24_compress_prepared(src, mode=MODE_HARD):
    """src [R, K] -> (vals [R, K/2], meta [R, K/8], prepared): the canonical packing plus the same matrix in the layout the
    matrix-core kernel streams fastest (an opaque byte tensor for spmm24_prepared)."""
    if src is None or src.dim() != 2 or src.dtype not in _BF16:
        raise SffnError("prune24_compress_prepared: src must be a 2-D bf16 tensor")
    R, K = src.shape
    vals, meta = _bf16((R, K // 2), src.device), _u8((R, K // 8), src.device)
    prepared = _u8((max(load().sffn_prepared24_bytes(R, K), 16),), src.device)
    _check(load().prune24_compress_prepared(_ptr(src, True), R, K, src.stride(0), mode, _ptr(vals), _ptr(meta), _ptr(prepared), _stream()))
    return vals, meta, prepared


def spmm24_prepared(X, w_prepared, N, bias=None, workspace=None):
    """eq. (1) / eq. (4) on a prepared weight operand of N rows: out [T, N]."""
    if X is None or X.dim() != 2:
        raise SffnError("spmm24_prepared: X must be a 2-D tensor")
    T, K = X.shape
    _want("spmm24_prepared: X", X, (T, K), _BF16)
    _want("spmm24_prepared: w_prepared", w_prepared, (max(load().sffn_prepared24_bytes(N, K), 16),), _U8)
    _want("spmm24_prepared: bias", bias, (N,), _F32, optional=True)
    nbytes = load().sffn_spmm24_prepared_workspace_bytes(T, K)
    ws = workspace if workspace is not None else _u8((max(nbytes, 16),), X.device)
    out = _bf16((T, N), X.device)
    _check(load().spmm24_prepared(_ptr(X), _ptr(w_prepared), _ptr(bias), T, N, K, _ptr(out), _ptr(ws), nbytes, _stream()))
    return out


def spmm24_dgrad(dY, wt_vals, wt_meta):
    if dY is None or dY.dim() != 2 or wt_vals is None or wt_vals.dim() != 2:
        raise SffnError("spmm24_dgrad: dY and wt_vals must be 2-D tensors")
    T, K = dY.shape
    N = wt_vals.shape[0]
    _want("spmm24_dgrad: dY", dY, (T, K), _BF16)
    _want("spmm24_dgrad: wt_vals", wt_vals, (N, K // 2), _BF16)
    _want("spmm24_dgrad: wt_meta", wt_meta, (N, K // 8), _U8)
    out = _bf16((T, N), dY.device)
    _check(load().spmm24_dgrad(_ptr(dY), _ptr(wt_vals), _ptr(wt_meta), T, N, K, _ptr(out), _stream()))
    return out


def vnm_spmm(a_vals, a_meta, a_colidx, Wd, w_kmajor, V=64, M=8):
    if a_vals is None or a_vals.dim() != 2 or Wd is None or Wd.dim() != 2:
        raise SffnError("vnm_spmm: a_vals and Wd must be 2-D tensors")
    T = a_vals.shape[0]
    Kfull = a_vals.shape[1] * M // 2
    N = Wd.shape[1] if w_kmajor else Wd.shape[0]
    _want("vnm_spmm: a_vals", a_vals, (T, 2 * Kfull // M), _BF16)
    _want("vnm_spmm: a_meta", a_meta, (T, Kfull // (2 * M)), _U8)
    _want("vnm_spmm: a_colidx", a_colidx, (T // V, Kfull // M, 4), _U8)
    _want("vnm_spmm: Wd", Wd, (Kfull, N) if w_kmajor else (N, Kfull), _BF16)
    out = _bf16((T, N), a_vals.device)
    nbytes = load().sffn_vnm_spmm_workspace_bytes(T, N, Kfull, int(w_kmajor))
    ws = _u8((max(nbytes, 16),), a_vals.device)
    _check(load().vnm_spmm(_ptr(a_vals), _ptr(a_meta), _ptr(a_colidx), _ptr(Wd, True), Wd.stride(0), int(w_kmajor), T, N, Kfull,
                           V, M, _ptr(out), _ptr(ws), nbytes, _stream()))
    return out


def dsqrelu_vnm(dy2, y1, meta, colidx, V=64, M=8):
    if y1 is None or y1.dim() != 2:
        raise SffnError("dsqrelu_vnm: y1 must be a 2-D tensor")
    T, F = y1.shape
    _want("dsqrelu_vnm: y1", y1, (T, F), _BF16)
    _want("dsqrelu_vnm: dy2", dy2, (T, F), _BF16)
    _want("dsqrelu_vnm: meta", meta, (T, F // (2 * M)), _U8)
    _want("dsqrelu_vnm: colidx", colidx, (T // V, F // M, 4), _U8)
    dvals = _bf16((T, 2 * F // M), y1.device)
    _check(load().dsqrelu_vnm(_ptr(dy2), _ptr(y1), _ptr(meta), _ptr(colidx), T, F, V, M, _ptr(dvals), _stream()))
    return dvals


def vnm_wgrad(a_vals, a_meta, a_colidx, G, out_f_major, V=64, M=8):
    if G is None or G.dim() != 2 or a_vals is None or a_vals.dim() != 2:
        raise SffnError("vnm_wgrad: G and a_vals must be 2-D tensors")
    T, N = G.shape
    F = a_vals.shape[1] * M // 2
    _want("vnm_wgrad: G", G, (T, N), _BF16)
    _want("vnm_wgrad: a_vals", a_vals, (T, 2 * F // M), _BF16)
    _want("vnm_wgrad: a_meta", a_meta, (T, F // (2 * M)), _U8)
    _want("vnm_wgrad: a_colidx", a_colidx, (T // V, F // M, 4), _U8)
    out = _bf16((F, N) if out_f_major else (N, F), G.device)
    nbytes = load().sffn_vnm_wgrad_workspace_bytes(T, F, N)
    ws = _u8((max(nbytes, 16),), G.device)
    _check(load().vnm_wgrad(_ptr(a_vals), _ptr(a_meta), _ptr(a_colidx), _ptr(G), T, F, N, V, M, int(out_f_major), _ptr(out),
                            _ptr(ws), nbytes, _stream()))
    return out


class FfnStep(_StepBuffers):
    """Pre-allocated outputs and workspace for repeated ffn_sparse_step calls on one shape."""

    def __init__(self, T, D, F, mode=MODE_HARD, device="cuda", keep_dense=False, M=8, unfused=False, lean=False, scratch=None, weights_of=None,
                 dw_fp32=False):
        """keep_dense: also store the dense y1 and dy2 (SFFN_FLAG_KEEP_DENSE); otherwise only y1 at y2's kept
        slots is saved for the backward pass.  M: V:N:M block width, 8, 16, 32 or 64.  unfused (M >= 16): the path
        with separate eq. (2) / eq. (6) kernels that always stores y1 and dy2 and produces no y1_kept.  lean:
        the canonical copies of the packed weights (and, at M = 8, of the packed activations) are not written (SFFN_FLAG_LEAN);
        saved() then holds stale data for them.  scratch: a uint8 CUDA tensor to use as the scratch region (see _StepBuffers); layers whose
        calls are ordered on one stream can share it, each keeping only its saved and weights regions.  weights_of: another FfnStep of the same
        configuration whose weights region this object shares (a second micro-batch of one layer)."""
        self.T, self.D, self.F, self.mode, self.keep_dense, self.M = T, D, F, mode, keep_dense, M
        self.cfg = _cfg(T, D, F, mode, M=M, flags=_flags(keep_dense, unfused, lean) | (FLAG_DW_FP32_ACCUMULATE if dw_fp32 else 0))
        self.layout = workspace_layout(T, D, F, mode, M, keep_dense, unfused, lean)
        self.lean = lean and self.layout["w1_meta"] == self.layout["w1_vals"]       # (the unfused path ignores the flag)
        assert self._alloc_regions(load().sffn_buffer_sizes, 1, device, scratch, weights_of) == self.layout["total"]
        self.Y3, self.dX = _bf16((T, D), device), _bf16((T, D), device)
        # dw_fp32 (SFFN_FLAG_DW_FP32_ACCUMULATE): dW1 / dW2 are float32 buffers, zero here, that every call adds its weight gradients to
        self.dW1, self.dW2 = _dw((F, D), device, dw_fp32), _dw((D, F), device, dw_fp32)

    def __call__(self, X, W1, W2, b1, dY, weights_packed=False):
        T, D, F = self.T, self.D, self.F
        _want("ffn_sparse_step: X", X, (T, D), _BF16)
        _want("ffn_sparse_step: W1", W1, (F, D), _BF16)
        _want("ffn_sparse_step: W2", W2, (D, F), _BF16)
        _want("ffn_sparse_step: b1", b1, (F,), _F32, optional=True)
        _want("ffn_sparse_step: dY", dY, (T, D), _BF16)
        _check(load().ffn_sparse_step(ctypes.byref(_cfg_with(self.cfg, weights_packed)), _ptr(X), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(dY), _ptr(self.Y3),
                                      _ptr(self.dX), _ptr(self.dW1), _ptr(self.dW2), self._one_buffer(), self.layout["total"], _stream()))
        return self.Y3, self.dX, self.dW1, self.dW2

    def forward(self, X, W1, W2, b1, weights_packed=False):
        """Alg. 1 alone (ffn_sparse_forward): Y3; what the backward pass needs stays in this object's workspace."""
        T, D, F = self.T, self.D, self.F
        _want("ffn_sparse_forward: X", X, (T, D), _BF16)
        _want("ffn_sparse_forward: W1", W1, (F, D), _BF16)
        _want("ffn_sparse_forward: W2", W2, (D, F), _BF16)
        _want("ffn_sparse_forward: b1", b1, (F,), _F32, optional=True)
        _check(load().ffn_sparse_forward(ctypes.byref(_cfg_with(self.cfg, weights_packed)), _ptr(X), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(self.Y3),
                                         ctypes.byref(self._buf), _stream()))
        return self.Y3

    def backward(self, W1, dY):
        """Alg. 2 alone (ffn_sparse_backward) on what the last forward() of this object left: dX, dW1, dW2."""
        T, D, F = self.T, self.D, self.F
        _want("ffn_sparse_backward: W1", W1, (F, D), _BF16)
        _want("ffn_sparse_backward: dY", dY, (T, D), _BF16)
        _check(load().ffn_sparse_backward(ctypes.byref(self.cfg), _ptr(W1), _ptr(dY), _ptr(self.dX), _ptr(self.dW1), _ptr(self.dW2),
                                          ctypes.byref(self._buf), _stream()))
        return self.dX, self.dW1, self.dW2

    def saved(self):
        """Views of the intermediates the step leaves in its workspace (Alg. 2 line 1 and friends)."""
        T, D, F, M, L = self.T, self.D, self.F, self.M, self.layout

        def view(off, shape, dtype):
            n = 1
            for s in shape:
                n *= s
            nbytes = n * (2 if dtype == torch.bfloat16 else 1)
            return self._region_bytes(off, nbytes).view(dtype).view(shape)

        out = dict(w1_vals=view(L["w1_vals"], (F, D // 2), torch.bfloat16), w1_meta=view(L["w1_meta"], (F, D // 8), torch.uint8),
                   w2t_vals=view(L["w2t_vals"], (F, D // 2), torch.bfloat16), w2t_meta=view(L["w2t_meta"], (F, D // 8), torch.uint8),
                   y2_vals=view(L["y2_vals"], (T, 2 * F // M), torch.bfloat16),
                   y2_meta=view(L["y2_meta"], (T, F // (2 * M)), torch.uint8), colidx=view(L["colidx"], (T // 64, F // M, 4), torch.uint8),
                   dy1_vals=view(L["dy1_vals"], (T, 2 * F // M), torch.bfloat16))
        if L["y2_vals"] > L["y1"]:          # the dense y1 / dy2 have room in the workspace only when they are stored
            out["y1"], out["dy2"] = view(L["y1"], (T, F), torch.bfloat16), view(L["dy2"], (T, F), torch.bfloat16)
        if L["y1_kept_bytes"]:
            out["y1_kept"] = view(L["y1_kept"], (T, 2 * F // M), torch.bfloat16)
        return self._drop_unwritten(out, self.M, ('w1_vals', 'w1_meta', 'w2t_vals', 'w2t_meta'), ('y2_vals', 'dy1_vals'))


class FfnStepGrouped(_StepBuffers):
    """Pre-allocated outputs and workspace for ffn_sparse_step_grouped: n_experts FFNs, expert e on token rows
    seg[e]..seg[e+1] (host integers, multiples of 64; T = seg[-1])."""

    def __init__(self, seg, D, F, mode=MODE_HARD, device="cuda", keep_dense=False, M=8, lean=False, scratch=None, dw_fp32=False):
        self.seg = [int(v) for v in seg]
        self.E, self.T, self.D, self.F, self.mode, self.keep_dense, self.M = len(self.seg) - 1, self.seg[-1], D, F, mode, keep_dense, M
        self.seg_c = (ctypes.c_int64 * len(self.seg))(*self.seg)
        self.cfg = _cfg(self.T, D, F, mode, M=M, flags=_flags(keep_dense, False, lean) | (FLAG_DW_FP32_ACCUMULATE if dw_fp32 else 0))
        lay = _Layout()
        _check(load().sffn_grouped_workspace_layout(ctypes.byref(self.cfg), self.E, ctypes.byref(lay)))
        self.layout = {n: getattr(lay, n) for n, _ in _Layout._fields_}
        self.lean = lean and self.layout["w1_meta"] == self.layout["w1_vals"]
        assert self._alloc_regions(load().sffn_buffer_sizes, self.E, device, scratch) == self.layout["total"]
        self.Y3, self.dX = _bf16((self.T, D), device), _bf16((self.T, D), device)
        self.dW1, self.dW2 = _dw((self.E, F, D), device, dw_fp32), _dw((self.E, D, F), device, dw_fp32)

    def __call__(self, X, W1, W2, b1, dY, weights_packed=False):
        T, D, F, E = self.T, self.D, self.F, self.E
        _want("ffn_sparse_step_grouped: X", X, (T, D), _BF16)
        _want("ffn_sparse_step_grouped: W1", W1, (E, F, D), _BF16)
        _want("ffn_sparse_step_grouped: W2", W2, (E, D, F), _BF16)
        _want("ffn_sparse_step_grouped: b1", b1, (E, F), _F32, optional=True)
        _want("ffn_sparse_step_grouped: dY", dY, (T, D), _BF16)
        _check(load().ffn_sparse_step_grouped(ctypes.byref(_cfg_with(self.cfg, weights_packed)), self.E, self.seg_c, _ptr(X), _ptr(W1), _ptr(W2), _ptr(b1),
                                              _ptr(dY), _ptr(self.Y3), _ptr(self.dX), _ptr(self.dW1), _ptr(self.dW2), self._one_buffer(), self.layout["total"], _stream()))
        return self.Y3, self.dX, self.dW1, self.dW2

    def forward(self, X, W1, W2, b1, weights_packed=False):
        """Alg. 1 alone for every expert (ffn_sparse_forward_grouped)."""
        T, D, F, E = self.T, self.D, self.F, self.E
        _want("ffn_sparse_forward_grouped: X", X, (T, D), _BF16)
        _want("ffn_sparse_forward_grouped: W1", W1, (E, F, D), _BF16)
        _want("ffn_sparse_forward_grouped: W2", W2, (E, D, F), _BF16)
        _want("ffn_sparse_forward_grouped: b1", b1, (E, F), _F32, optional=True)
        _check(load().ffn_sparse_forward_grouped(ctypes.byref(_cfg_with(self.cfg, weights_packed)), self.E, self.seg_c, _ptr(X), _ptr(W1), _ptr(W2),
                                                 _ptr(b1), _ptr(self.Y3), ctypes.byref(self._buf), _stream()))
        return self.Y3

    def backward(self, W1, dY):
        """Alg. 2 alone for every expert (ffn_sparse_backward_grouped) on what the last forward() left."""
        T, D, F, E = self.T, self.D, self.F, self.E
        _want("ffn_sparse_backward_grouped: W1", W1, (E, F, D), _BF16)
        _want("ffn_sparse_backward_grouped: dY", dY, (T, D), _BF16)
        _check(load().ffn_sparse_backward_grouped(ctypes.byref(self.cfg), self.E, self.seg_c, _ptr(W1), _ptr(dY), _ptr(self.dX), _ptr(self.dW1),
                                                  _ptr(self.dW2), ctypes.byref(self._buf), _stream()))
        return self.dX, self.dW1, self.dW2

    def saved(self):
        """As FfnStep.saved(); weight-shaped tensors carry a leading expert axis."""
        T, D, F, E, L, M = self.T, self.D, self.F, self.E, self.layout, self.M

        def view(off, shape, dtype):
            n = 1
            for s in shape:
                n *= s
            nbytes = n * (2 if dtype == torch.bfloat16 else 1)
            return self._region_bytes(off, nbytes).view(dtype).view(shape)

        out = dict(w1_vals=view(L["w1_vals"], (E, F, D // 2), torch.bfloat16), w1_meta=view(L["w1_meta"], (E, F, D // 8), torch.uint8),
                   w2t_vals=view(L["w2t_vals"], (E, F, D // 2), torch.bfloat16), w2t_meta=view(L["w2t_meta"], (E, F, D // 8), torch.uint8),
                   y2_vals=view(L["y2_vals"], (T, 2 * F // M), torch.bfloat16),
                   y2_meta=view(L["y2_meta"], (T, F // (2 * M)), torch.uint8), colidx=view(L["colidx"], (T // 64, F // M, 4), torch.uint8),
                   dy1_vals=view(L["dy1_vals"], (T, 2 * F // M), torch.bfloat16),
                   y1_kept=view(L["y1_kept"], (T, 2 * F // M), torch.bfloat16))
        if self.keep_dense:
            out["y1"], out["dy2"] = view(L["y1"], (T, F), torch.bfloat16), view(L["dy2"], (T, F), torch.bfloat16)
        return self._drop_unwritten(out, self.M, ('w1_vals', 'w1_meta', 'w2t_vals', 'w2t_meta'), ('y2_vals', 'dy1_vals'))


def ffn_sparse_step(X, W1, W2, b1, dY, mode=MODE_HARD, keep_dense=True, M=8, unfused=False):
    T, D = X.shape
    F = W1.shape[0]
    step = FfnStep(T, D, F, mode, X.device, keep_dense, M, unfused)
    out = step(X, W1, W2, b1, dY)
    return out, step


# ---- fp8 (E4M3) operands: Section 3.4's closing paragraph ---------------------------------------------------------------------
def _amax_buf(want, dev):
    return torch.zeros((1,), dtype=torch.float32, device=dev) if want else None


def quantize_fp8(x, scale, want_amax=False):
    """bf16 tensor -> E4M3 codes (uint8, same shape) with the caller's per-tensor scale; optionally also amax (device float [1])."""
    if x is None or x.dtype not in _BF16 or x.numel() % 8:
        raise SffnError("quantize_fp8: x must be a bf16 tensor with a multiple of 8 elements")
    codes, amax = _u8(tuple(x.shape), x.device), _amax_buf(want_amax, x.device)
    _check(load().quantize_fp8(_ptr(x), x.numel(), float(scale), _ptr(codes), _ptr(amax), _stream()))
    return (codes, amax) if want_amax else codes


def prune24_compress_fp8(src, scale, trans=False, mode=MODE_HARD, want_amax=False):
    """As prune24_compress with the survivors stored as E4M3 codes: -> codes [R, K/2] u8, meta [R, K/8] (, amax)."""
    if src is None or src.dim() != 2 or src.dtype not in _BF16:
        raise SffnError("prune24_compress_fp8: src must be a 2-D bf16 tensor")
    rows, cols = src.shape
    R, K = (cols, rows) if trans else (rows, cols)
    codes, meta, amax = _u8((R, K // 2), src.device), _u8((R, K // 8), src.device), _amax_buf(want_amax, src.device)
    _check(load().prune24_compress_fp8(_ptr(src, True), R, K, src.stride(0), int(trans), mode, float(scale), _ptr(codes), _ptr(meta), _ptr(amax), _stream()))
    return (codes, meta, amax) if want_amax else (codes, meta)


def sqrelu_vnm_compress_fp8(y1, scale, V=64, M=8, want_amax=False):
    if y1 is None or y1.dim() != 2 or y1.dtype not in _BF16:
        raise SffnError("sqrelu_vnm_compress_fp8: y1 must be a 2-D bf16 tensor")
    T, F = y1.shape
    codes, meta = _u8((T, 2 * F // M), y1.device), _u8((T, F // (2 * M)), y1.device)
    colidx, amax = _u8((T // V, F // M, 4), y1.device), _amax_buf(want_amax, y1.device)
    _check(load().sqrelu_vnm_compress_fp8(_ptr(y1), T, F, V, M, float(scale), _ptr(codes), _ptr(meta), _ptr(colidx), _ptr(amax), _stream()))
    return (codes, meta, colidx, amax) if want_amax else (codes, meta, colidx)


def spmm24_fp8(Xq, scale_x, w_codes, w_meta, scale_w, bias=None):
    if Xq is None or Xq.dim() != 2 or w_codes is None or w_codes.dim() != 2:
        raise SffnError("spmm24_fp8: Xq and w_codes must be 2-D tensors")
    T, K = Xq.shape
    N = w_codes.shape[0]
    _want("spmm24_fp8: Xq", Xq, (T, K), _U8)
    _want("spmm24_fp8: w_codes", w_codes, (N, K // 2), _U8)
    _want("spmm24_fp8: w_meta", w_meta, (N, K // 8), _U8)
    _want("spmm24_fp8: bias", bias, (N,), _F32, optional=True)
    out = _bf16((T, N), Xq.device)
    _check(load().spmm24_fp8(_ptr(Xq), float(scale_x), _ptr(w_codes), _ptr(w_meta), float(scale_w), _ptr(bias), T, N, K, _ptr(out), _stream()))
    return out


def vnm_spmm_fp8(a_codes, a_meta, a_colidx, scale_a, Wq, scale_w, w_kmajor, V=64, M=8):
    if a_codes is None or a_codes.dim() != 2 or Wq is None or Wq.dim() != 2:
        raise SffnError("vnm_spmm_fp8: a_codes and Wq must be 2-D tensors")
    T = a_codes.shape[0]
    Kfull = a_codes.shape[1] * M // 2
    N = Wq.shape[1] if w_kmajor else Wq.shape[0]
    _want("vnm_spmm_fp8: a_codes", a_codes, (T, 2 * Kfull // M), _U8)
    _want("vnm_spmm_fp8: a_meta", a_meta, (T, Kfull // (2 * M)), _U8)
    _want("vnm_spmm_fp8: a_colidx", a_colidx, (T // V, Kfull // M, 4), _U8)
    _want("vnm_spmm_fp8: Wq", Wq, (Kfull, N) if w_kmajor else (N, Kfull), _U8)
    out = _bf16((T, N), a_codes.device)
    nbytes = load().sffn_vnm_spmm_fp8_workspace_bytes(T, N, Kfull)
    ws = _u8((max(nbytes, 16),), a_codes.device)
    _check(load().vnm_spmm_fp8(_ptr(a_codes), _ptr(a_meta), _ptr(a_colidx), float(scale_a), _ptr(Wq), float(scale_w), int(w_kmajor), T, N, Kfull,
                               V, M, _ptr(out), _ptr(ws), nbytes, _stream()))
    return out


class FfnStepFp8(_StepBuffers):
    """ffn_sparse_step_fp8 with outputs and workspace allocated once.  scales: dict with the six per-tensor scales
    x, w1, w2, y2, dy, dy1 (positive floats; delayed scaling: the caller derives them from earlier steps)."""

    def __init__(self, T, D, F, scales, mode=MODE_HARD, device="cuda", keep_dense=False, wgrad_fp8=False, lean=False, M=8, scratch=None, dw_fp32=False):
        """wgrad_fp8: eqs. (5), (8) contract codes as well (SFFN_FLAG_FP8_WGRAD); otherwise they are the bf16 contractions.
        lean: the canonical copies of the packed tensors are not written (SFFN_FLAG_LEAN).  M: columns per V:N:M block (8, 16, 32, 64)."""
        self.T, self.D, self.F, self.mode, self.M = T, D, F, mode, M
        self.cfg = _cfg(T, D, F, mode, M=M, flags=(FLAG_KEEP_DENSE if keep_dense else 0) | (FLAG_FP8_WGRAD if wgrad_fp8 else 0) | (FLAG_LEAN if lean else 0) | (FLAG_DW_FP32_ACCUMULATE if dw_fp32 else 0))
        self.scales = _Fp8Scales(*[float(scales[k]) for k in ("x", "w1", "w2", "y2", "dy", "dy1")])
        lay = _Fp8Layout()
        _check(load().sffn_fp8_workspace_layout(ctypes.byref(self.cfg), ctypes.byref(lay)))
        self.layout = {n: getattr(lay, n) for n, _ in _Fp8Layout._fields_}
        self.keep_dense = keep_dense
        self.lean = lean
        assert self._alloc_regions(load().sffn_fp8_buffer_sizes, 1, device, scratch) == self.layout["total"]
        self.Y3, self.dX = _bf16((T, D), device), _bf16((T, D), device)
        self.dW1, self.dW2 = _dw((F, D), device, dw_fp32), _dw((D, F), device, dw_fp32)
        self.amax = torch.zeros((8,), dtype=torch.float32, device=device)        # [0:6]: x, w1, w2, y2, dy, dy1 after every call

    def set_scales(self, scales):
        """New per-tensor scales for the following calls (e.g. amax / 448 of the step before)."""
        self.scales = _Fp8Scales(*[float(scales[k]) for k in ("x", "w1", "w2", "y2", "dy", "dy1")])

    def amax_dict(self):
        """The six maxima the last call left on the device (synchronises)."""
        a = self.amax[:6].tolist()
        return dict(zip(("x", "w1", "w2", "y2", "dy", "dy1"), a))

    def __call__(self, X, W1, W2, b1, dY, weights_packed=False):
        T, D, F = self.T, self.D, self.F
        _want("ffn_sparse_step_fp8: X", X, (T, D), _BF16)
        _want("ffn_sparse_step_fp8: W1", W1, (F, D), _BF16)
        _want("ffn_sparse_step_fp8: W2", W2, (D, F), _BF16)
        _want("ffn_sparse_step_fp8: b1", b1, (F,), _F32, optional=True)
        _want("ffn_sparse_step_fp8: dY", dY, (T, D), _BF16)
        _check(load().ffn_sparse_step_fp8(ctypes.byref(_cfg_with(self.cfg, weights_packed)), ctypes.byref(self.scales), _ptr(X), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(dY),
                                          _ptr(self.Y3), _ptr(self.dX), _ptr(self.dW1), _ptr(self.dW2), self._one_buffer(), self.layout["total"], _ptr(self.amax), _stream()))
        return self.Y3, self.dX, self.dW1, self.dW2

    def forward(self, X, W1, W2, b1, weights_packed=False):
        """Alg. 1 alone (ffn_sparse_forward_fp8): Y3; amax[0:4] (x, w1, w2, y2) are written, what the backward pass needs stays in the workspace."""
        T, D, F = self.T, self.D, self.F
        _want("ffn_sparse_forward_fp8: X", X, (T, D), _BF16)
        _want("ffn_sparse_forward_fp8: W1", W1, (F, D), _BF16)
        _want("ffn_sparse_forward_fp8: W2", W2, (D, F), _BF16)
        _want("ffn_sparse_forward_fp8: b1", b1, (F,), _F32, optional=True)
        _check(load().ffn_sparse_forward_fp8(ctypes.byref(_cfg_with(self.cfg, weights_packed)), ctypes.byref(self.scales), _ptr(X), _ptr(W1), _ptr(W2),
                                             _ptr(b1), _ptr(self.Y3), ctypes.byref(self._buf), _ptr(self.amax), _stream()))
        return self.Y3

    def backward(self, dY):
        """Alg. 2 alone (ffn_sparse_backward_fp8) on what the last forward() left (W1 is read as the codes that call wrote); amax[4:6] are written."""
        _want("ffn_sparse_backward_fp8: dY", dY, (self.T, self.D), _BF16)
        _check(load().ffn_sparse_backward_fp8(ctypes.byref(self.cfg), ctypes.byref(self.scales), _ptr(dY), _ptr(self.dX), _ptr(self.dW1), _ptr(self.dW2),
                                              ctypes.byref(self._buf), _ptr(self.amax), _stream()))
        return self.dX, self.dW1, self.dW2

    def saved(self):
        """Views of what the step leaves in its workspace."""
        T, D, F, L, M = self.T, self.D, self.F, self.layout, self.M

        def view(off, shape, dtype):
            n = 1
            for d in shape:
                n *= d
            nbytes = n * (2 if dtype == torch.bfloat16 else 1)
            return self._region_bytes(off, nbytes).view(dtype).view(shape)

        u8 = torch.uint8
        out = dict(w1_codes=view(L["w1_codes"], (F, D // 2), u8), w1_meta=view(L["w1_meta"], (F, D // 8), u8),
                   w2t_codes=view(L["w2t_codes"], (F, D // 2), u8), w2t_meta=view(L["w2t_meta"], (F, D // 8), u8),
                   y2_codes=view(L["y2_codes"], (T, 2 * F // M), u8), y2_meta=view(L["y2_meta"], (T, F // (2 * M)), u8),
                   colidx=view(L["colidx"], (T // 64, F // M, 4), u8), y1_kept=view(L["y1_kept"], (T, 2 * F // M), torch.bfloat16))
        # dy1's survivors: bf16 at M = 8, codes (the operand of eq. (7) on gathered rows) at M >= 16
        if M == 8:
            out["dy1_vals"] = view(L["dy1_vals"], (T, F // 4), torch.bfloat16)
        else:
            out["dy1_codes"] = view(L["dy1_vals"], (T, 2 * F // M), u8)
        if self.keep_dense:
            out["y1"], out["dy2"] = view(L["y1"], (T, F), torch.bfloat16), view(L["dy2"], (T, F), torch.bfloat16)
        return self._drop_unwritten(out, self.M, ('w1_codes', 'w1_meta', 'w2t_codes', 'w2t_meta'), ('y2_codes',))


class FfnStepFp8Grouped(FfnStepFp8):
    """ffn_sparse_step_fp8_grouped: n_experts FFNs, expert e on token rows seg[e]..seg[e+1] (host integers, multiples of 64; T = seg[-1])."""

    def __init__(self, seg, D, F, scales, mode=MODE_HARD, device="cuda", keep_dense=False, wgrad_fp8=False, lean=False, M=8, scratch=None, dw_fp32=False):
        self.seg = [int(v) for v in seg]
        self.E, self.T, self.D, self.F, self.mode, self.keep_dense, self.M = len(self.seg) - 1, self.seg[-1], D, F, mode, keep_dense, M
        self.seg_c = (ctypes.c_int64 * len(self.seg))(*self.seg)
        self.cfg = _cfg(self.T, D, F, mode, M=M, flags=(FLAG_KEEP_DENSE if keep_dense else 0) | (FLAG_FP8_WGRAD if wgrad_fp8 else 0) | (FLAG_LEAN if lean else 0) | (FLAG_DW_FP32_ACCUMULATE if dw_fp32 else 0))
        self.set_scales(scales)
        lay = _Fp8Layout()
        _check(load().sffn_fp8_grouped_workspace_layout(ctypes.byref(self.cfg), self.E, ctypes.byref(lay)))
        self.layout = {n: getattr(lay, n) for n, _ in _Fp8Layout._fields_}
        self.lean = lean
        assert self._alloc_regions(load().sffn_fp8_buffer_sizes, self.E, device, scratch) == self.layout["total"]
        self.Y3, self.dX = _bf16((self.T, D), device), _bf16((self.T, D), device)
        self.dW1, self.dW2 = _dw((self.E, F, D), device, dw_fp32), _dw((self.E, D, F), device, dw_fp32)
        self.amax = torch.zeros((8,), dtype=torch.float32, device=device)

    def __call__(self, X, W1, W2, b1, dY, weights_packed=False):
        T, D, F, E = self.T, self.D, self.F, self.E
        _want("ffn_sparse_step_fp8_grouped: X", X, (T, D), _BF16)
        _want("ffn_sparse_step_fp8_grouped: W1", W1, (E, F, D), _BF16)
        _want("ffn_sparse_step_fp8_grouped: W2", W2, (E, D, F), _BF16)
        _want("ffn_sparse_step_fp8_grouped: b1", b1, (E, F), _F32, optional=True)
        _want("ffn_sparse_step_fp8_grouped: dY", dY, (T, D), _BF16)
        _check(load().ffn_sparse_step_fp8_grouped(ctypes.byref(_cfg_with(self.cfg, weights_packed)), ctypes.byref(self.scales), self.E, self.seg_c, _ptr(X), _ptr(W1), _ptr(W2),
                                                  _ptr(b1), _ptr(dY), _ptr(self.Y3), _ptr(self.dX), _ptr(self.dW1), _ptr(self.dW2), self._one_buffer(), self.layout["total"], _ptr(self.amax), _stream()))
        return self.Y3, self.dX, self.dW1, self.dW2

    def forward(self, X, W1, W2, b1, weights_packed=False):
        """Alg. 1 alone for every expert (ffn_sparse_forward_fp8_grouped); amax[0:4] are written."""
        T, D, F, E = self.T, self.D, self.F, self.E
        _want("ffn_sparse_forward_fp8_grouped: X", X, (T, D), _BF16)
        _want("ffn_sparse_forward_fp8_grouped: W1", W1, (E, F, D), _BF16)
        _want("ffn_sparse_forward_fp8_grouped: W2", W2, (E, D, F), _BF16)
        _want("ffn_sparse_forward_fp8_grouped: b1", b1, (E, F), _F32, optional=True)
        _check(load().ffn_sparse_forward_fp8_grouped(ctypes.byref(_cfg_with(self.cfg, weights_packed)), ctypes.byref(self.scales), self.E, self.seg_c,
                                                     _ptr(X), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(self.Y3), ctypes.byref(self._buf),
                                                     _ptr(self.amax), _stream()))
        return self.Y3

    def backward(self, dY):
        """Alg. 2 alone for every expert (ffn_sparse_backward_fp8_grouped) on what the last forward() left; amax[4:6] are written."""
        _want("ffn_sparse_backward_fp8_grouped: dY", dY, (self.T, self.D), _BF16)
        _check(load().ffn_sparse_backward_fp8_grouped(ctypes.byref(self.cfg), ctypes.byref(self.scales), self.E, self.seg_c, _ptr(dY), _ptr(self.dX),
                                                      _ptr(self.dW1), _ptr(self.dW2), ctypes.byref(self._buf), _ptr(self.amax), _stream()))
        return self.dX, self.dW1, self.dW2

    def saved(self):
        """As FfnStepFp8.saved(); weight-shaped tensors carry a leading expert axis."""
        T, D, F, E, L, M = self.T, self.D, self.F, self.E, self.layout, self.M

        def view(off, shape, dtype):
            n = 1
            for d in shape:
                n *= d
            nbytes = n * (2 if dtype == torch.bfloat16 else 1)
            return self._region_bytes(off, nbytes).view(dtype).view(shape)

        u8 = torch.uint8
        out = dict(w1_codes=view(L["w1_codes"], (E, F, D // 2), u8), w1_meta=view(L["w1_meta"], (E, F, D // 8), u8),
                   w2t_codes=view(L["w2t_codes"], (E, F, D // 2), u8), w2t_meta=view(L["w2t_meta"], (E, F, D // 8), u8),
                   y2_codes=view(L["y2_codes"], (T, 2 * F // M), u8), y2_meta=view(L["y2_meta"], (T, F // (2 * M)), u8),
                   colidx=view(L["colidx"], (T // 64, F // M, 4), u8), y1_kept=view(L["y1_kept"], (T, 2 * F // M), torch.bfloat16))
        # dy1's survivors: bf16 at M = 8, codes (the operand of eq. (7) on gathered rows) at M >= 16
        if M == 8:
            out["dy1_vals"] = view(L["dy1_vals"], (T, F // 4), torch.bfloat16)
        else:
            out["dy1_codes"] = view(L["dy1_vals"], (T, 2 * F // M), u8)
        if self.keep_dense:
            out["y1"], out["dy2"] = view(L["y1"], (T, F), torch.bfloat16), view(L["dy2"], (T, F), torch.bfloat16)
        return self._drop_unwritten(out, self.M, ('w1_codes', 'w1_meta', 'w2t_codes', 'w2t_meta'), ('y2_codes',))


NOALLOC_WORKSPACE_MAX = 32 << 20


def ffn_sparse_step_noalloc(X, W1, W2, b1, dY, out, mode=MODE_HARD, M=8):
    """ffn_sparse_step_noalloc: the library's built-in workspace, nothing allocated by the call.  out = (Y3, dX, dW1, dW2),
    allocated by the caller beforehand (this wrapper allocates nothing either)."""
    if X is None or X.dim() != 2 or W1 is None or W1.dim() != 2:
        raise SffnError("ffn_sparse_step_noalloc: X and W1 must be 2-D tensors")
    T, D = X.shape
    F = W1.shape[0]
    Y3, dX, dW1, dW2 = out
    for name, t, shape, kinds, opt in (("X", X, (T, D), _BF16, False), ("W1", W1, (F, D), _BF16, False), ("W2", W2, (D, F), _BF16, False),
                                       ("b1", b1, (F,), _F32, True), ("dY", dY, (T, D), _BF16, False), ("Y3", Y3, (T, D), _BF16, False),
                                       ("dX", dX, (T, D), _BF16, False), ("dW1", dW1, (F, D), _BF16, False), ("dW2", dW2, (D, F), _BF16, False)):
        _want("ffn_sparse_step_noalloc: " + name, t, shape, kinds, optional=opt)
    c = _cfg(T, D, F, mode, M=M)
    _check(load().ffn_sparse_step_noalloc(ctypes.byref(c), _ptr(X), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(dY), _ptr(Y3), _ptr(dX),
                                          _ptr(dW1), _ptr(dW2), _stream()))
    return out


def venom_route_launch(X, means, M, want_scores=False):
    """venom_route without the read-back: seg stays a device tensor (int32, first M/4 + 1 entries)."""
    if X is None or X.dim() != 2:
        raise SffnError("venom_route: X must be a 2-D tensor")
    T, D = X.shape
    E = M // 4
    _want("venom_route: X", X, (T, D), _BF16)
    _want("venom_route: means", means, (E, D), _BF16)
    rows = load().sffn_venom_rows(T, M)
    dev = X.device
    i32t = lambda n: torch.empty((n,), dtype=torch.int32, device=dev)
    expert, perm, row_of_token, seg = i32t(T), i32t(rows), i32t(T), i32t(E + 4)
    scores = torch.empty((T, E), dtype=torch.float32, device=dev) if want_scores else None
    nbytes = load().sffn_venom_route_workspace_bytes(T, M)
    ws = _u8((max(nbytes, 16),), dev)
    _check(load().venom_route(_ptr(X), _ptr(means), T, D, M, _ptr(expert), _ptr(perm), _ptr(row_of_token), _ptr(seg), _ptr(scores),
                              _ptr(ws), nbytes, _stream()))
    return dict(expert=expert, perm=perm, row_of_token=row_of_token, seg=seg[:E + 1], scores=scores)


def venom_route(X, means, M, want_scores=False):
    """Steps 1-2 of Section 3.3: top-1 expert per token and the stable, 64-row padded grouping.
    -> dict(expert [T] i32, perm [rows] i32, row_of_token [T] i32, seg (host list, M/4 + 1), scores [T, M/4] f32 or None).
    Reading seg back synchronises with the stream (the next call sizes its launch from it)."""
    r = venom_route_launch(X, means, M, want_scores)
    r["seg"] = [int(v) for v in r["seg"].cpu()]
    return r


def venom_expert_matmul(X, perm, seg, W1, b1, M, mode=MODE_HARD, keep_y1c=True, workspace=None):
    """Step 3 of Section 3.3: the grouped matmul that emits V:N:M.  -> (vals, meta, colidx, y1c or None) over
    sffn_venom_rows(T, M) rows."""
    if X is None or X.dim() != 2 or W1 is None or W1.dim() != 2:
        raise SffnError("venom_expert_matmul: X and W1 must be 2-D tensors")
    T, D = X.shape
    F = W1.shape[0]
    E = M // 4
    rows = load().sffn_venom_rows(T, M)
    _want("venom_expert_matmul: X", X, (T, D), _BF16)
    _want("venom_expert_matmul: W1", W1, (F, D), _BF16)
    _want("venom_expert_matmul: b1", b1, (F,), _F32, optional=True)
    _want("venom_expert_matmul: perm", perm, (rows,), _I32)
    if len(seg) != E + 1:
        raise SffnError("venom_expert_matmul: seg must hold M / 4 + 1 run offsets")
    dev = X.device
    vals, meta = _bf16((rows, 2 * F // M), dev), _u8((rows, F // (2 * M)), dev)
    colidx = _u8((rows // 64, F // M, 4), dev)
    y1c = _bf16((rows, 4 * F // M), dev) if keep_y1c else None
    nbytes = load().sffn_venom_matmul_workspace_bytes(T, D, F, M)
    ws = workspace if workspace is not None else _u8((max(nbytes, 16),), dev)
    c = _cfg(T, D, F, mode, M=M)
    seg_arr = (ctypes.c_int64 * (E + 1))(*[int(v) for v in seg])
    _check(load().venom_expert_matmul(ctypes.byref(c), seg_arr, _ptr(X), _ptr(perm), _ptr(W1), _ptr(b1), _ptr(y1c), _ptr(vals), _ptr(meta),
                                      _ptr(colidx), _ptr(ws), nbytes, _stream()))
    return vals, meta, colidx, y1c


def moe_to_venom(X, W1, b1, means, M, mode=MODE_HARD):
    """Alg. 3: route, permute, grouped matmul.  -> dict(expert, perm, row_of_token, seg, vals, meta, colidx, y1c)."""
    r = venom_route(X, means, M)
    vals, meta, colidx, y1c = venom_expert_matmul(X, r["perm"], r["seg"], W1, b1, M, mode)
    r.update(vals=vals, meta=meta, colidx=colidx, y1c=y1c)
    return r


class FfnRouterStep:
    """ffn_router_step with a workspace allocated once (shapes and the routing's row capacity are fixed by T, D, F, M)."""

    def __init__(self, T, D, F, M, mode=MODE_HARD, device="cuda", keep_dense=False):
        """keep_dense: also store dy2c (SFFN_FLAG_KEEP_DENSE); eq. (6) is evaluated in the epilogue of eq. (4) either way."""
        self.T, self.D, self.F, self.M, self.mode = T, D, F, M, mode
        self.cfg = _cfg(T, D, F, mode, M=M, flags=FLAG_KEEP_DENSE if keep_dense else 0)
        lay = _RouterLayout()
        _check(load().sffn_router_workspace_layout(ctypes.byref(self.cfg), ctypes.byref(lay)))
        self.layout = {n: getattr(lay, n) for n, _ in _RouterLayout._fields_}
        self.rows = load().sffn_venom_rows(T, M)
        self.ws_bytes = load().sffn_router_full_workspace_bytes(ctypes.byref(self.cfg))    # step workspace + routing buffers
        self.ws = _u8((self.ws_bytes,), device)
        self.Y3, self.dX = _bf16((T, D), device), _bf16((T, D), device)
        self.dW1, self.dW2 = _bf16((F, D), device), _bf16((D, F), device)

    def _want_inputs(self, who, X, W1, W2, b1, dY):
        T, D, F = self.T, self.D, self.F
        _want(who + ": X", X, (T, D), _BF16)
        _want(who + ": W1", W1, (F, D), _BF16)
        _want(who + ": W2", W2, (D, F), _BF16)
        _want(who + ": b1", b1, (F,), _F32, optional=True)
        _want(who + ": dY", dY, (T, D), _BF16)

    def __call__(self, route, X, W1, W2, b1, dY, weights_packed=False):
        """route: the dict venom_route returned for X."""
        E = self.M // 4
        self._want_inputs("ffn_router_step", X, W1, W2, b1, dY)
        _want("ffn_router_step: perm", route["perm"], (self.rows,), _I32)
        if len(route["seg"]) != E + 1:
            raise SffnError("ffn_router_step: seg must hold M / 4 + 1 run offsets")
        seg_arr = (ctypes.c_int64 * (E + 1))(*[int(v) for v in route["seg"]])
        _check(load().ffn_router_step(ctypes.byref(_cfg_with(self.cfg, weights_packed)), seg_arr, _ptr(route["perm"]), _ptr(X), _ptr(W1),
                                      _ptr(W2), _ptr(b1), _ptr(dY), _ptr(self.Y3), _ptr(self.dX), _ptr(self.dW1), _ptr(self.dW2),
                                      _ptr(self.ws), self.layout["total"], _stream()))
        return self.Y3, self.dX, self.dW1, self.dW2

    def full(self, means, X, W1, W2, b1, dY, weights_packed=False):
        """Routing included (ffn_router_full_step): no read-back of the run offsets, nothing but launches on the stream."""
        self._want_inputs("ffn_router_full_step", X, W1, W2, b1, dY)
        _want("ffn_router_full_step: means", means, (self.M // 4, self.D), _BF16)
        _check(load().ffn_router_full_step(ctypes.byref(_cfg_with(self.cfg, weights_packed)), _ptr(means), _ptr(X), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(dY),
                                           _ptr(self.Y3), _ptr(self.dX), _ptr(self.dW1), _ptr(self.dW2), _ptr(self.ws), self.ws_bytes, _stream()))
        return self.Y3, self.dX, self.dW1, self.dW2

    def forward(self, route, X, W1, W2, b1, weights_packed=False):
        """Alg. 1 with Alg. 3 as the sparsifier (ffn_router_forward); route: the dict venom_route returned for X."""
        T, D, F, E = self.T, self.D, self.F, self.M // 4
        _want("ffn_router_forward: X", X, (T, D), _BF16)
        _want("ffn_router_forward: W1", W1, (F, D), _BF16)
        _want("ffn_router_forward: W2", W2, (D, F), _BF16)
        _want("ffn_router_forward: b1", b1, (F,), _F32, optional=True)
        _want("ffn_router_forward: perm", route["perm"], (self.rows,), _I32)
        if len(route["seg"]) != E + 1:
            raise SffnError("ffn_router_forward: seg must hold M / 4 + 1 run offsets")
        seg_arr = (ctypes.c_int64 * (E + 1))(*[int(v) for v in route["seg"]])
        _check(load().ffn_router_forward(ctypes.byref(_cfg_with(self.cfg, weights_packed)), seg_arr, _ptr(route["perm"]), _ptr(X), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(self.Y3),
                                         _ptr(self.ws), self.layout["total"], _stream()))
        return self.Y3

    def backward(self, route, dY):
        """Alg. 2 (ffn_router_backward) on what the last forward() left, with the same route."""
        E = self.M // 4
        _want("ffn_router_backward: dY", dY, (self.T, self.D), _BF16)
        _want("ffn_router_backward: perm", route["perm"], (self.rows,), _I32)
        seg_arr = (ctypes.c_int64 * (E + 1))(*[int(v) for v in route["seg"]])
        _check(load().ffn_router_backward(ctypes.byref(self.cfg), seg_arr, _ptr(route["perm"]), _ptr(dY), _ptr(self.dX), _ptr(self.dW1),
                                          _ptr(self.dW2), _ptr(self.ws), self.layout["total"], _stream()))
        return self.dX, self.dW1, self.dW2

    def full_forward(self, means, X, W1, W2, b1, weights_packed=False):
        """Routing + Alg. 1 (ffn_router_full_forward); the routing stays in the workspace for full_backward()."""
        T, D, F = self.T, self.D, self.F
        _want("ffn_router_full_forward: X", X, (T, D), _BF16)
        _want("ffn_router_full_forward: W1", W1, (F, D), _BF16)
        _want("ffn_router_full_forward: W2", W2, (D, F), _BF16)
        _want("ffn_router_full_forward: b1", b1, (F,), _F32, optional=True)
        _want("ffn_router_full_forward: means", means, (self.M // 4, D), _BF16)
        _check(load().ffn_router_full_forward(ctypes.byref(_cfg_with(self.cfg, weights_packed)), _ptr(means), _ptr(X), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(self.Y3),
                                              _ptr(self.ws), self.ws_bytes, _stream()))
        return self.Y3

    def full_backward(self, dY):
        """Alg. 2 (ffn_router_full_backward) on the routing and the intermediates the last full_forward() left."""
        _want("ffn_router_full_backward: dY", dY, (self.T, self.D), _BF16)
        _check(load().ffn_router_full_backward(ctypes.byref(self.cfg), _ptr(dY), _ptr(self.dX), _ptr(self.dW1), _ptr(self.dW2),
                                               _ptr(self.ws), self.ws_bytes, _stream()))
        return self.dX, self.dW1, self.dW2

    def saved(self):
        rows, Kc, L = self.rows, 4 * self.F // self.M, self.layout

        def view(off, shape, dtype):
            n = 1
            for d in shape:
                n *= d
            nbytes = n * (2 if dtype == torch.bfloat16 else 1)
            return self.ws[off:off + nbytes].view(dtype).view(shape)

        return dict(y1c=view(L["y1c"], (rows, Kc), torch.bfloat16), vals=view(L["vals"], (rows, Kc // 2), torch.bfloat16),
                    meta=view(L["meta"], (rows, Kc // 8), torch.uint8), colidx=view(L["colidx"], (rows // 64, self.F // self.M, 4), torch.uint8),
                    dy2c=view(L["dy2c"], (rows, Kc), torch.bfloat16), dvals=view(L["dvals"], (rows, Kc // 2), torch.bfloat16))
