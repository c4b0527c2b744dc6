"""Host-side checks that need no GPU: the shared library loads, exports every symbol the header
declares, and rejects bad arguments before enqueuing anything."""
import ctypes
import os
import re

import pytest

import paper_2602_06183_amd as sffn
from paper_2602_06183_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sparseffn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined", "sizeof"})


def test_library_exports_every_declared_symbol():
    lib = sffn.load()
    names = declared_symbols()
    for must in ("prune24_compress", "sqrelu_vnm_compress", "spmm24_fwd", "spmm24_dgrad", "vnm_wgrad", "ffn_sparse_step",
                 "vnm_spmm", "dsqrelu_vnm", "sffn_workspace_bytes", "sffn_workspace_layout"):
        assert must in names
    for n in names:
        assert hasattr(lib, n), n
    assert sffn.version() >= 100


def test_workspace_queries():
    assert sffn.workspace_bytes(512, 256, 1024) > 0
    assert sffn.workspace_bytes(500, 256, 1024) == 0          # T not a multiple of 64
    lay = sffn.workspace_layout(512, 256, 1024)
    # the workspace is [scratch | saved | weights]: what outlives nothing, what the backward pass reads of the forward pass, what the pruning passes write
    offs = [lay[k] for k in ("y1", "dy2", "y2_vals", "dy1_vals", "y2_meta", "colidx", "y1_kept", "w1_vals", "w1_meta", "w2t_vals", "w2t_meta")]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs) and lay["total"] == sffn.workspace_bytes(512, 256, 1024)
    lib = sffn.load()
    assert lib.sffn_vnm_spmm_workspace_bytes(64, 64, 64, 1) == lib.sffn_vnm_spmm_workspace_bytes(64, 64, 64, 0) == 4096 + 512 + 8192
    assert lib.sffn_vnm_wgrad_workspace_bytes(64, 64, 63) == 0


def test_bad_arguments_are_rejected_without_touching_the_gpu():
    lib = sffn.load()
    fake = ctypes.c_void_p(0x1000)        # 16-byte aligned, never dereferenced: every call below fails validation first
    odd = ctypes.c_void_p(0x1008)
    assert lib.prune24_compress(None, 64, 64, 64, 0, 0, fake, fake, None) == -1
    assert lib.prune24_compress(fake, 64, 60, 64, 0, 0, fake, fake, None) == -1
    assert lib.prune24_compress(fake, 64, 64, 32, 0, 0, fake, fake, None) == -1
    assert lib.prune24_compress(fake, 64, 64, 64, 0, 7, fake, fake, None) == -1
    assert lib.prune24_compress(odd, 64, 64, 64, 0, 0, fake, fake, None) == -1
    assert b"aligned" in lib.sffn_last_error()
    assert lib.sqrelu_vnm_compress(fake, 64, 64, 64, 12, fake, fake, fake, None) == -2      # M = 12 is not a built block width
    assert lib.sqrelu_vnm_compress(fake, 64, 64, 32, 8, fake, fake, fake, None) == -2       # V = 32 neither
    assert lib.sqrelu_vnm_compress(fake, 64, 64, 64, 64, fake, fake, fake, None) == -1      # F must be a multiple of 2 M
    assert lib.sqrelu_vnm_compress(fake, 63, 64, 64, 8, fake, fake, fake, None) == -1
    assert lib.spmm24_fwd(fake, fake, fake, None, 64, 64, 65, fake, None) == -1
    assert lib.sffn_prepared24_bytes(64, 64) == 64 * 64 + 512 and lib.sffn_prepared24_bytes(64, 65) == 0
    assert lib.prune24_compress_prepared(fake, 64, 64, 32, 0, fake, fake, fake, None) == -1        # ld < K
    assert lib.spmm24_prepared(fake, fake, None, 64, 64, 64, fake, None, 0, None) == -3            # no workspace
    assert lib.spmm24_dgrad(fake, fake, None, 64, 64, 64, fake, None) == -1
    assert lib.vnm_spmm(fake, fake, fake, fake, 64, 0, 64, 64, 64, 64, 8, fake, None, 0, None) == -3
    assert lib.vnm_spmm(fake, fake, fake, fake, 64, 0, 64, 64, 64, 32, 8, fake, fake, 1 << 20, None) == -2
    assert lib.dsqrelu_vnm(fake, fake, fake, fake, 64, 100, 64, 8, fake, None) == -1
    assert lib.vnm_wgrad(fake, fake, fake, fake, 64, 64, 64, 64, 8, 0, fake, fake, 16, None) == -3
    cfg = binding._Cfg(512, 256, 1024, 64, 8, 0, 0)
    args = [fake] * 9
    assert lib.ffn_sparse_step(ctypes.byref(cfg), *args, fake, 16, None) == -3
    bad = binding._Cfg(512, 250, 1024, 64, 8, 0, 0)
    assert lib.ffn_sparse_step(ctypes.byref(bad), *args, fake, 1 << 30, None) == -1
    assert len(lib.sffn_last_error()) > 0
    huge = binding._Cfg(64, 16384, 65536, 64, 8, 0, 0)                    # a 2 GiB weight matrix: beyond the 31-bit offsets of the V:2:8 kernel's loads
    assert lib.ffn_sparse_step(ctypes.byref(huge), *args, fake, 1 << 50, None) == -2
    assert lib.ffn_sparse_step(ctypes.byref(binding._Cfg(512, 256, 1024, 64, 8, 0, 64)), *args, fake, 1 << 40, None) == -1        # unknown flag
    # Alg. 1 / Alg. 2 as separate calls on three buffers (scratch | saved | weights): sizes add up to the one-call workspace, and each half
    # checks its own pointers, the buffers and the path before any launch
    sizes = binding._Buffers()
    assert lib.sffn_buffer_sizes(ctypes.byref(cfg), 1, ctypes.byref(sizes)) == 0
    assert sizes.scratch_bytes + sizes.saved_bytes + sizes.weights_bytes == lib.sffn_workspace_bytes(ctypes.byref(cfg))
    assert min(sizes.scratch_bytes, sizes.saved_bytes, sizes.weights_bytes) > 0 and sizes.scratch is None
    assert lib.sffn_buffer_sizes(ctypes.byref(bad), 1, ctypes.byref(sizes)) == -1
    assert lib.sffn_buffer_sizes(ctypes.byref(cfg), 1, ctypes.byref(sizes)) == 0
    far = 1 << 40               # (fake device addresses, far enough apart for any of these sizes)
    good = binding._Buffers(far, sizes.scratch_bytes, 2 * far, sizes.saved_bytes, 3 * far, sizes.weights_bytes)
    short = binding._Buffers(far, sizes.scratch_bytes, 2 * far, sizes.saved_bytes - 256, 3 * far, sizes.weights_bytes)
    skew = binding._Buffers(far, sizes.scratch_bytes, 2 * far + 16, sizes.saved_bytes, 3 * far, sizes.weights_bytes)
    assert lib.ffn_sparse_forward(ctypes.byref(cfg), fake, fake, fake, fake, fake, None, None) == -1
    assert lib.ffn_sparse_forward(ctypes.byref(cfg), fake, fake, fake, fake, fake, ctypes.byref(short), None) == -3
    assert lib.ffn_sparse_forward(ctypes.byref(cfg), fake, fake, fake, fake, fake, ctypes.byref(skew), None) == -1
    overlap = binding._Buffers(far, sizes.scratch_bytes, far + sizes.scratch_bytes - 256, sizes.saved_bytes, 3 * far, sizes.weights_bytes)
    carved = binding._Buffers(far, sizes.scratch_bytes, far + sizes.scratch_bytes, sizes.saved_bytes, far + sizes.scratch_bytes + sizes.saved_bytes, sizes.weights_bytes)
    assert lib.ffn_sparse_forward(ctypes.byref(cfg), fake, fake, fake, fake, fake, ctypes.byref(overlap), None) == -1
    assert lib.ffn_sparse_forward(ctypes.byref(cfg), None, fake, fake, fake, fake, ctypes.byref(carved), None) == -1        # (buffers accepted: the null X is what fails)
    assert "null pointer" in lib.sffn_last_error().decode()
    assert lib.ffn_sparse_forward(ctypes.byref(cfg), None, fake, fake, fake, fake, ctypes.byref(good), None) == -1
    assert lib.ffn_sparse_backward(ctypes.byref(cfg), fake, fake, fake, fake, fake, ctypes.byref(short), None) == -3
    assert lib.ffn_sparse_backward(ctypes.byref(cfg), fake, None, fake, fake, fake, ctypes.byref(good), None) == -1
    wide_unfused = binding._Cfg(512, 256, 1024, 64, 16, 0, 2)
    assert lib.sffn_buffer_sizes(ctypes.byref(wide_unfused), 1, ctypes.byref(sizes)) == 0
    big = binding._Buffers(far, far, 2 * far, far, 3 * far, far)
    assert lib.ffn_sparse_backward(ctypes.byref(wide_unfused), fake, fake, fake, fake, fake, ctypes.byref(big), None) == -2   # unfused path
    assert lib.ffn_sparse_forward_grouped(ctypes.byref(cfg), 2, None, fake, fake, fake, fake, fake, ctypes.byref(big), None) == -1
    assert lib.ffn_sparse_backward_grouped(ctypes.byref(cfg), 2, None, fake, fake, fake, fake, fake, ctypes.byref(big), None) == -1
    assert lib.ffn_sparse_step(ctypes.byref(binding._Cfg(512, 256, 1024, 64, 16, 0, 2 | 32)), *args, fake, 1 << 40, None) == -2   # float32 accumulation: fused paths only
    # SFFN_FLAG_WEIGHTS_PACKED (16) exists for the fused paths only: the unfused wide-block path (flag 2) refuses it before any launch
    assert lib.ffn_sparse_step(ctypes.byref(binding._Cfg(512, 256, 1024, 64, 16, 0, 2 | 16)), *args, fake, 1 << 40, None) == -2
    # the fp8 step: scales are a host struct; shapes, flags, scales and the workspace are checked before anything is enqueued
    sc = binding._Fp8Scales(1.0, 1.0, 1.0, 1.0, 1.0, 1.0)
    assert lib.ffn_sparse_step_fp8(ctypes.byref(cfg), None, *args, fake, 1 << 40, None, None) == -1                 # no scales
    assert lib.ffn_sparse_step_fp8(ctypes.byref(cfg), ctypes.byref(sc), *args, fake, 16, None, None) == -3          # workspace too small
    assert lib.ffn_sparse_step_fp8(ctypes.byref(binding._Cfg(512, 192, 1024, 64, 8, 0, 0)), ctypes.byref(sc), *args, fake, 1 << 40, None, None) == -1   # D % 128
    assert lib.ffn_sparse_step_fp8(ctypes.byref(binding._Cfg(512, 256, 1024, 64, 12, 0, 0)), ctypes.byref(sc), *args, fake, 1 << 40, None, None) == -2  # M = 12
    assert lib.ffn_sparse_step_fp8(ctypes.byref(binding._Cfg(512, 256, 1280, 64, 64, 0, 0)), ctypes.byref(sc), *args, fake, 1 << 40, None, None) == -1  # 4 F / M = 80
    assert lib.ffn_sparse_step_fp8(ctypes.byref(binding._Cfg(512, 256, 1024, 64, 16, 0, 0)), ctypes.byref(sc), *args, fake, 16, None, None) == -3       # M = 16: workspace
    assert lib.ffn_sparse_step_fp8(ctypes.byref(binding._Cfg(512, 256, 1024, 64, 8, 0, 2)), ctypes.byref(sc), *args, fake, 1 << 40, None, None) == -1   # unknown flag
    f8sizes = binding._Buffers()
    assert lib.sffn_fp8_buffer_sizes(ctypes.byref(cfg), 1, ctypes.byref(f8sizes)) == 0
    assert f8sizes.scratch_bytes + f8sizes.saved_bytes + f8sizes.weights_bytes == lib.sffn_fp8_workspace_bytes(ctypes.byref(cfg))
    f8good = binding._Buffers(far, f8sizes.scratch_bytes, 2 * far, f8sizes.saved_bytes, 3 * far, f8sizes.weights_bytes)
    f8short = binding._Buffers(far, f8sizes.scratch_bytes, 2 * far, f8sizes.saved_bytes, 3 * far, f8sizes.weights_bytes - 256)
    assert lib.ffn_sparse_forward_fp8(ctypes.byref(cfg), ctypes.byref(sc), None, fake, fake, fake, fake, ctypes.byref(f8good), None, None) == -1
    assert lib.ffn_sparse_forward_fp8(ctypes.byref(cfg), ctypes.byref(sc), fake, fake, fake, fake, fake, ctypes.byref(f8short), None, None) == -3
    assert lib.ffn_sparse_backward_fp8(ctypes.byref(cfg), ctypes.byref(sc), fake, fake, fake, None, ctypes.byref(f8good), None, None) == -1
    assert lib.ffn_sparse_backward_fp8(ctypes.byref(cfg), ctypes.byref(sc), fake, fake, fake, fake, ctypes.byref(f8short), None, None) == -3
    assert lib.ffn_sparse_forward_fp8_grouped(ctypes.byref(cfg), ctypes.byref(sc), 2, None, fake, fake, fake, fake, fake, ctypes.byref(f8good), None, None) == -1
    assert lib.ffn_sparse_backward_fp8_grouped(ctypes.byref(cfg), ctypes.byref(sc), 2, None, fake, fake, fake, fake, ctypes.byref(f8good), None, None) == -1
    zero = binding._Fp8Scales(1.0, 1.0, 0.0, 1.0, 1.0, 1.0)
    assert lib.ffn_sparse_step_fp8(ctypes.byref(cfg), ctypes.byref(zero), *args, fake, 1 << 40, None, None) == -1 and b"scales" in lib.sffn_last_error()
    assert lib.sffn_fp8_workspace_bytes(ctypes.byref(cfg)) > 0 and lib.sffn_fp8_workspace_bytes(ctypes.byref(binding._Cfg(512, 192, 1024, 64, 8, 0, 0))) == 0
    # grouped step: the segment table is a host array and is validated before anything is enqueued
    big = 1 << 40
    seg = lambda *v: (ctypes.c_int64 * len(v))(*v)
    assert lib.ffn_sparse_step_grouped(ctypes.byref(cfg), 2, None, *args, fake, big, None) == -1
    assert lib.ffn_sparse_step_grouped(ctypes.byref(cfg), 0, seg(0), *args, fake, big, None) == -1
    assert lib.ffn_sparse_step_grouped(ctypes.byref(cfg), 65, seg(*([0] * 66)), *args, fake, big, None) == -1
    assert lib.ffn_sparse_step_grouped(ctypes.byref(cfg), 2, seg(0, 100, 512), *args, fake, big, None) == -1     # not a multiple of 64
    assert lib.ffn_sparse_step_grouped(ctypes.byref(cfg), 2, seg(0, 320, 448), *args, fake, big, None) == -1     # does not end at T
    assert lib.ffn_sparse_step_grouped(ctypes.byref(cfg), 2, seg(64, 320, 512), *args, fake, big, None) == -1    # does not start at 0
    assert lib.ffn_sparse_step_grouped(ctypes.byref(cfg), 3, seg(0, 320, 256, 512), *args, fake, big, None) == -1  # descending
    assert lib.ffn_sparse_step_grouped(ctypes.byref(cfg), 2, seg(0, 320, 512), *args, fake, 16, None) == -3
    assert lib.sffn_grouped_workspace_bytes(ctypes.byref(cfg), 1) == lib.sffn_workspace_bytes(ctypes.byref(cfg))
    assert lib.sffn_grouped_workspace_bytes(ctypes.byref(cfg), 4) > lib.sffn_workspace_bytes(ctypes.byref(cfg))
    assert lib.sffn_grouped_workspace_bytes(ctypes.byref(cfg), 0) == 0


def test_router_entry_points_validate_on_the_host():
    lib = sffn.load()
    fake = ctypes.c_void_p(0x1000)
    assert lib.sffn_venom_rows(100, 16) == 128 + 64 * 4 and lib.sffn_venom_rows(8192, 8) == 8192 + 128
    assert lib.sffn_venom_rows(100, 12) == 0
    assert lib.sffn_venom_route_workspace_bytes(100, 16) >= 4 * 4
    assert lib.venom_route(fake, fake, 100, 64, 12, fake, fake, fake, fake, None, fake, 1 << 20, None) == -2     # M / 4 experts
    assert lib.venom_route(fake, fake, 100, 60, 16, fake, fake, fake, fake, None, fake, 1 << 20, None) == -1     # D not a multiple of 8
    assert lib.venom_route(fake, fake, 100, 64, 16, fake, fake, fake, fake, None, fake, 0, None) == -3
    assert lib.venom_route(fake, None, 100, 64, 16, fake, fake, fake, fake, None, fake, 1 << 20, None) == -1
    cfg = binding._Cfg(100, 64, 1024, 64, 16, 0, 0)
    seg = lambda *v: (ctypes.c_int64 * len(v))(*v)
    big = 1 << 40
    ok = seg(0, 64, 128, 128, 192)
    tail = [fake] * 8
    assert lib.sffn_venom_matmul_workspace_bytes(100, 64, 1024, 16) > 0
    assert lib.sffn_venom_matmul_workspace_bytes(100, 64, 640, 16) == 0                                          # 4 F / M not a multiple of 64
    assert lib.venom_expert_matmul(ctypes.byref(cfg), ok, *tail, fake, 16, None) == -3
    assert lib.venom_expert_matmul(ctypes.byref(cfg), None, *tail, fake, big, None) == -1
    assert lib.venom_expert_matmul(ctypes.byref(cfg), seg(0, 64, 100, 128, 192), *tail, fake, big, None) == -1   # not a multiple of 64
    assert lib.venom_expert_matmul(ctypes.byref(cfg), seg(0, 64, 128, 64, 192), *tail, fake, big, None) == -1    # descending
    assert lib.venom_expert_matmul(ctypes.byref(cfg), seg(64, 64, 128, 128, 192), *tail, fake, big, None) == -1  # does not start at 0
    assert lib.venom_expert_matmul(ctypes.byref(cfg), seg(0, 64, 128, 256, 448), *tail, fake, big, None) == -1   # beyond the row capacity (384)
    bad = binding._Cfg(100, 64, 640, 64, 16, 0, 0)
    assert lib.venom_expert_matmul(ctypes.byref(bad), ok, *tail, fake, big, None) == -1
    # the router's whole step: same host-side checks, plus its workspace layout
    args = [fake] * 10
    assert lib.sffn_router_workspace_bytes(ctypes.byref(cfg)) > 0 and lib.sffn_router_workspace_bytes(ctypes.byref(bad)) == 0
    lay = binding._RouterLayout()
    assert lib.sffn_router_workspace_layout(ctypes.byref(cfg), ctypes.byref(lay)) == 0
    offs = [getattr(lay, n) for n in ("y1c", "vals", "meta", "colidx", "dy2c", "dvals")]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs) and lay.total == lib.sffn_router_workspace_bytes(ctypes.byref(cfg))
    assert lib.ffn_router_step(ctypes.byref(cfg), ok, *args, fake, 16, None) == -3
    assert lib.ffn_router_step(ctypes.byref(cfg), None, *args, fake, big, None) == -1
    assert lib.ffn_router_step(ctypes.byref(cfg), seg(0, 64, 100, 128, 192), *args, fake, big, None) == -1
    assert lib.ffn_router_step(ctypes.byref(cfg), seg(0, 64, 128, 256, 448), *args, fake, big, None) == -1
    assert lib.ffn_router_step(ctypes.byref(bad), ok, *args, fake, big, None) == -1
    m12 = binding._Cfg(100, 64, 1024, 64, 12, 0, 0)
    assert lib.ffn_router_step(ctypes.byref(m12), ok, *args, fake, big, None) == -2
    assert lib.ffn_router_step(ctypes.byref(binding._Cfg(cfg.T, cfg.D, cfg.F, 64, cfg.M, 0, 16)), ok, *args, fake, 16, None) == -3      # packed weights: accepted, the workspace is what fails
    assert lib.ffn_router_step(ctypes.byref(binding._Cfg(cfg.T, cfg.D, cfg.F, 64, cfg.M, 0, 32)), ok, *args, fake, big, None) == -2     # no float32 accumulation
    assert lib.sffn_router_full_workspace_bytes(ctypes.byref(cfg)) > lib.sffn_router_workspace_bytes(ctypes.byref(cfg))
    assert lib.sffn_router_full_workspace_bytes(ctypes.byref(bad)) == 0
    assert lib.ffn_router_full_step(ctypes.byref(cfg), *args, fake, 16, None) == -3
    assert lib.ffn_router_full_step(ctypes.byref(cfg), None, *args[1:], fake, big, None) == -1
    assert lib.ffn_router_full_step(ctypes.byref(m12), *args, fake, big, None) == -2
    # the router's step as two calls: each half checks what it reads
    assert lib.ffn_router_forward(ctypes.byref(cfg), ok, fake, fake, fake, fake, fake, fake, fake, 16, None) == -3
    assert lib.ffn_router_forward(ctypes.byref(cfg), ok, fake, None, fake, fake, fake, fake, fake, big, None) == -1
    assert lib.ffn_router_backward(ctypes.byref(cfg), ok, fake, None, fake, fake, fake, fake, big, None) == -1
    assert lib.ffn_router_backward(ctypes.byref(cfg), None, fake, fake, fake, fake, fake, fake, big, None) == -1
    assert lib.ffn_router_backward(ctypes.byref(m12), ok, fake, fake, fake, fake, fake, fake, big, None) == -2
    assert lib.ffn_router_full_forward(ctypes.byref(cfg), None, fake, fake, fake, fake, fake, fake, big, None) == -1
    assert lib.ffn_router_full_forward(ctypes.byref(cfg), fake, fake, fake, fake, fake, fake, fake, 16, None) == -3
    assert lib.ffn_router_full_backward(ctypes.byref(cfg), None, fake, fake, fake, fake, big, None) == -1
    assert lib.ffn_router_full_backward(ctypes.byref(cfg), fake, fake, fake, fake, fake, 16, None) == -3


def test_lean_workspace_has_no_room_for_the_copies_it_does_not_write():
    T, D, F = 512, 256, 1024
    assert sffn.workspace_bytes(T, D, F) - sffn.workspace_bytes(T, D, F, lean=True) == 2 * F * D + 2 * (F * D // 8) + 2 * (T * F // 2)
    assert sffn.workspace_bytes(T, D, F, M=16) - sffn.workspace_bytes(T, D, F, M=16, lean=True) == 2 * F * D + 2 * (F * D // 8)    # eqs. (3), (7) read the packed activations
    assert sffn.workspace_bytes(T, D, F, M=16, unfused=True) == sffn.workspace_bytes(T, D, F, M=16, unfused=True, lean=True)        # the unfused path ignores the flag
    lay = sffn.workspace_layout(T, D, F, lean=True)
    assert lay["w1_vals"] == lay["w1_meta"] == lay["w2t_vals"] == lay["w2t_meta"]                                                   # empty regions


def test_workspace_has_no_dense_activation_unless_it_is_stored():
    """Without SFFN_FLAG_KEEP_DENSE the fused M = 8 step never writes the dense y1 / dy2, and its workspace has no room for
    them: exactly 2 x 2 T F bytes smaller.  The unfused wide-block path always stores them.  Unknown M: no layout."""
    T, D, F = 512, 256, 1024
    small, big = sffn.workspace_bytes(T, D, F), sffn.workspace_bytes(T, D, F, keep_dense=True)
    assert big - small == 2 * 2 * T * F
    lay = sffn.workspace_layout(T, D, F)
    assert lay["dy2"] == lay["y1"] == lay["y2_vals"]                                # empty regions
    layk = sffn.workspace_layout(T, D, F, keep_dense=True)
    assert layk["dy2"] - layk["y1"] == 2 * T * F and layk["y2_vals"] - layk["dy2"] == 2 * T * F
    # blocks of 16 columns: fused like M = 8 when the gathered-row kernel covers the shape (4 F / M a multiple of 64), else / on request unfused
    assert sffn.workspace_bytes(T, D, F, M=16, keep_dense=True) - sffn.workspace_bytes(T, D, F, M=16) == 2 * 2 * T * F
    assert sffn.workspace_bytes(T, D, F, M=16, unfused=True) == sffn.workspace_bytes(T, D, F, M=16, keep_dense=True, unfused=True) > 0
    assert sffn.workspace_bytes(T, D, 640, M=16) == sffn.workspace_bytes(T, D, 640, M=16, keep_dense=True) > 0
    assert sffn.workspace_layout(T, D, F, M=16)["y1_kept_bytes"] == T * 2 * F // 16 * 2 and sffn.workspace_layout(T, D, F, M=16, unfused=True)["y1_kept_bytes"] == 0
    assert sffn.workspace_layout(T, D, F)["y1_kept_bytes"] == T * F // 4 * 2
    lib = sffn.load()
    for M in (0, 4, 12, 128):
        c = binding._Cfg(T, D, F, 64, M, 0, 0)
        assert lib.sffn_workspace_bytes(ctypes.byref(c)) == 0
        assert lib.sffn_workspace_layout(ctypes.byref(c), ctypes.byref(binding._Layout())) == -1
        assert lib.ffn_sparse_step(ctypes.byref(c), *([ctypes.c_void_p(0x1000)] * 9), ctypes.c_void_p(0x1000), 1 << 40, None) == -2
    c = binding._Cfg(T, D, F, 32, 8, 0, 0)
    assert lib.sffn_workspace_bytes(ctypes.byref(c)) == 0


def test_binding_rejects_mismatched_tensors_before_any_call(monkeypatch):
    """The binding is the only layer that knows tensor sizes: a wrong shape or element type must raise before the C
    entry point is reached (checked here by making every entry point unreachable), for every wrapper that takes tensors."""
    import torch

    class Unreachable:
        def __getattr__(self, name):
            if name.startswith("sffn_") and ("bytes" in name or "rows" in name or "layout" in name):
                return getattr(real, name)

            def reached(*a):
                raise AssertionError("C entry point %s reached" % name)
            return reached
    real = sffn.load()
    bf, u8, f32, i32 = torch.bfloat16, torch.uint8, torch.float32, torch.int32
    z = lambda shape, dt=bf: torch.zeros(shape, dtype=dt)
    T, D, F, M = 128, 64, 256, 8
    step = sffn.FfnStep.__new__(sffn.FfnStep)
    step.T, step.D, step.F, step.M, step.mode, step.keep_dense = T, D, F, M, 0, False
    step.cfg = binding._cfg(T, D, F)
    grouped = sffn.FfnStepGrouped.__new__(sffn.FfnStepGrouped)
    grouped.T, grouped.D, grouped.F, grouped.E = T, D, F, 2
    router = sffn.FfnRouterStep.__new__(sffn.FfnRouterStep)
    router.T, router.D, router.F, router.M, router.rows = T, D, F, 16, real.sffn_venom_rows(T, 16)
    monkeypatch.setattr(binding, "_LIB", Unreachable())
    good = dict(X=z((T, D)), W1=z((F, D)), W2=z((D, F)), b1=z((F,), f32), dY=z((T, D)))
    cases = [
        lambda: step(z((T - 64, D)), good["W1"], good["W2"], good["b1"], good["dY"]),              # short X
        lambda: step(good["X"], good["W1"], good["W2"], z((F,), bf), good["dY"]),                   # bf16 bias where fp32 is read
        lambda: step(good["X"], z((F, D), f32), good["W2"], good["b1"], good["dY"]),                # fp32 weights
        lambda: step(good["X"], good["W1"], z((F, D)), good["b1"], good["dY"]),                     # W2 transposed
        lambda: step(good["X"], good["W1"], good["W2"], good["b1"], z((T, D + 64))),
        lambda: grouped(good["X"], z((1, F, D)), z((2, D, F)), None, good["dY"]),
        lambda: grouped(good["X"], z((2, F, D)), z((2, D, F)), z((F,), f32), good["dY"]),
        lambda: router.full(z((3, D)), good["X"], good["W1"], good["W2"], good["b1"], good["dY"]),   # M / 4 = 4 means wanted
        lambda: router(dict(perm=z((router.rows - 1,), i32), seg=[0] * 5), good["X"], good["W1"], good["W2"], good["b1"], good["dY"]),
        lambda: router(dict(perm=z((router.rows,), i32), seg=[0] * 4), good["X"], good["W1"], good["W2"], good["b1"], good["dY"]),
        lambda: sffn.spmm24_fwd(good["X"], z((F, D // 2 - 8)), z((F, D // 8), u8)),                # w_vals narrower than K / 2
        lambda: sffn.spmm24_fwd(good["X"], z((F, D // 2)), z((F, D // 8), u8), z((F,), bf)),
        lambda: sffn.spmm24_dgrad(good["dY"], z((F, D // 2)), z((F, D // 8), i32)),
        lambda: sffn.vnm_spmm(z((T, F // 4)), z((T, F // 16), u8), z((T // 64, F // 8, 3), u8), good["W1"], 1),
        lambda: sffn.vnm_spmm(z((T, F // 4)), z((T, F // 16), u8), z((T // 64, F // 8, 4), u8), good["W1"], 0),   # W given in the other orientation
        lambda: sffn.dsqrelu_vnm(z((T, F)), z((T + 64, F)), z((T, F // 16), u8), z((T // 64, F // 8, 4), u8)),
        lambda: sffn.vnm_wgrad(z((T, F // 4)), z((T, F // 16), u8), z((T // 64, F // 8, 4), u8), z((T // 2, D)), 1),
        lambda: sffn.venom_route_launch(good["X"], z((2, D)), 16),
        lambda: sffn.venom_expert_matmul(good["X"], z((router.rows,), torch.int64), [0] * 5, good["W1"], good["b1"], 16),
        lambda: sffn.prune24_compress(z((F, D), f32)),
        lambda: sffn.sqrelu_vnm_compress(z((T, F), u8)),
    ]
    for n, case in enumerate(cases):
        with pytest.raises(sffn.SffnError):
            case()
    # and matching host tensors get as far as the device check, still without a call
    with pytest.raises(sffn.SffnError, match="device"):
        step(**good)


def test_host_validation_under_sanitizers(tmp_path):
    """The argument checks of every entry-point family, run from a C++ driver with the library's host code built under
    AddressSanitizer + UndefinedBehaviorSanitizer: every bad call must come back with its error code and no sanitizer report."""
    import subprocess
    from paper_2602_06183_amd import build
    exe = build.build_host_sanitized(os.path.join(ROOT, "tests", "abi_host_check.cpp"), str(tmp_path / "abi_host_check"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout
    assert "all argument checks behave" in r.stdout and "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout, r.stdout


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "_HERE", str(tmp_path))
    with pytest.raises(sffn.SffnError):
        binding.load()


def test_workspace_layout_properties_over_random_configurations():
    """Host logic of the layouts, for shapes and flags drawn at random: the public regions are 256-byte aligned, disjoint, large enough for
    what the header says they hold and inside the workspace; the three buffers of the split calls add up to it; SFFN_FLAG_KEEP_DENSE only
    adds the two dense activations and SFFN_FLAG_LEAN only removes the copies it does not write; the grouped layout scales the
    weight-shaped regions by the number of experts and nothing else."""
    from hypothesis import given, settings, strategies as st
    lib = sffn.load()

    def regions(T, D, F, M, flags, E=1):
        c, lay, buf = binding._Cfg(T, D, F, 64, M, 0, flags), binding._Layout(), binding._Buffers()
        assert lib.sffn_grouped_workspace_layout(ctypes.byref(c), E, ctypes.byref(lay)) == 0
        assert lib.sffn_buffer_sizes(ctypes.byref(c), E, ctypes.byref(buf)) == 0
        return {n: getattr(lay, n) for n, _ in binding._Layout._fields_}, buf

    @settings(max_examples=150, deadline=None)
    @given(st.integers(1, 40), st.integers(1, 12), st.integers(1, 24), st.sampled_from([8, 16, 32, 64]), st.sampled_from([0, 1, 2, 8, 9, 10]),
           st.integers(1, 5))
    def check(t, d, f, M, flags, E):
        T, D, F = 64 * t, 64 * d, 2 * M * f
        if F % 64:
            return
        lay, buf = regions(T, D, F, M, flags, E)
        assert buf.scratch_bytes + buf.saved_bytes + buf.weights_bytes == lay["total"]
        fused = M == 8 or (not (flags & 2) and (4 * F // M) % 64 == 0 and 4 * F // M <= 7168)
        dense, lean = bool(flags & 1) or not fused, bool(flags & 8) and fused
        need = dict(w1_vals=0 if lean else E * F * D, w1_meta=0 if lean else E * F * D // 8, w2t_vals=0 if lean else E * F * D,
                    w2t_meta=0 if lean else E * F * D // 8, y1=2 * T * F if dense else 0, dy2=2 * T * F if dense else 0,
                    y2_vals=0 if (lean and M == 8) else 4 * T * F // M, dy1_vals=0 if (lean and M == 8) else 4 * T * F // M,
                    y2_meta=T * F // (2 * M), colidx=T // 64 * (F // M) * 4, y1_kept=4 * T * F // M if fused else 0)
        assert lay["y1_kept_bytes"] == need["y1_kept"]
        spans = sorted((lay[k], lay[k] + need[k]) for k in need)
        for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
            assert a1 <= b0                                            # disjoint
        assert all(lay[k] % 256 == 0 for k in need) and spans[-1][1] <= lay["total"]
        # which buffer a region lands in: scratch, saved, weights, in this order of offsets
        b1_, b2_ = buf.scratch_bytes, buf.scratch_bytes + buf.saved_bytes
        for k in ("y1", "dy2", "y2_vals", "dy1_vals"):
            assert lay[k] + need[k] <= b1_
        for k in ("y2_meta", "colidx", "y1_kept"):
            assert b1_ <= lay[k] and lay[k] + need[k] <= b2_
        for k in ("w1_vals", "w1_meta", "w2t_vals", "w2t_meta"):
            assert b2_ <= lay[k]
        if fused:
            more, _ = regions(T, D, F, M, flags | 1, E)
            less, _ = regions(T, D, F, M, flags | 8, E)
            assert more["total"] - lay["total"] == (0 if dense else 2 * 2 * T * F)
            assert lay["total"] - less["total"] == (0 if lean else 2 * E * F * D + 2 * (E * F * D // 8) + (2 * (4 * T * F // M) if M == 8 else 0))

    check()
