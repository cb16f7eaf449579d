"""ctypes binding of libtm_w4.so.  Same names as the C ABI; tensors are torch CUDA(=HIP) tensors.

The library is loaded from this directory and nowhere else; if it is missing the import of any entry point fails
loudly (there is no fallback path of any kind)."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtm_w4.so")
_lib = None

TM_OK = 0


class TmError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"tm_w4 error {code}: {message}")
        self.code = code


def lib_path() -> str:
    return _LIB_PATH


class TmEpilogue(ctypes.Structure):
    _fields_ = [("bias", ctypes.c_void_p), ("residual", ctypes.c_void_p), ("act", ctypes.c_int)]


def load_library():
    """dlopen libtm_w4.so (built by paper_2508_15601_amd/build.py) and declare every entry point."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch-ROCm ships its own HIP runtime (same soname as the system one).  Import torch first so that the
    # library binds to the runtime torch's allocator and streams live in; two runtimes in one process see no device.
    import torch  # noqa: F401
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
    lib = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    vp, sz, i = c.c_void_p, c.c_size_t, c.c_int
    lib.tm_pack_w4.restype = vp
    lib.tm_pack_w4.argtypes = [vp, vp, vp, i, i, i]
    lib.tm_pack_w4_on.restype = vp
    lib.tm_pack_w4_on.argtypes = [vp, vp, vp, i, i, i, vp]
    lib.tm_kv_create.restype = vp
    lib.tm_kv_create.argtypes = [i, i, i, i]
    lib.tm_kv_free.restype = None
    lib.tm_kv_free.argtypes = [vp]
    lib.tm_kv_append.restype = i
    lib.tm_kv_append.argtypes = [vp, vp, vp, vp, i, vp]
    lib.tm_attn_decode.restype = i
    lib.tm_attn_decode.argtypes = [vp, vp, vp, vp, i, ctypes.c_float, i, vp]
    lib.tm_attn_prefill.restype = i
    lib.tm_attn_prefill.argtypes = [vp, vp, vp, vp, i, vp, i, ctypes.c_float, vp]
    lib.tm_kv_raw.restype = i
    lib.tm_kv_raw.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.tm_pack_w4_actorder.restype = vp
    lib.tm_pack_w4_actorder.argtypes = [vp, vp, vp, vp, i, i, i, i, vp]
    lib.tm_pack_w8.restype = vp
    lib.tm_pack_w8.argtypes = [vp, vp, vp, i, i, i, vp]
    lib.tm_pack_w8_fp8.restype = vp
    lib.tm_pack_w8_fp8.argtypes = [vp, vp, i, i, i, vp]
    lib.tm_packed_bits.restype = i
    lib.tm_packed_bits.argtypes = [vp]
    lib.tm_group_experts.restype = vp
    lib.tm_group_experts.argtypes = [vp, i]
    lib.tm_free_expert_group.restype = None
    lib.tm_free_expert_group.argtypes = [vp]
    lib.tm_gemm_w4a16_grouped.restype = i
    lib.tm_gemm_w4a16_grouped.argtypes = [vp, vp, vp, vp, i, vp]
    lib.tm_gemm_w4a16_grouped_act.restype = i
    lib.tm_gemm_w4a16_grouped_act.argtypes = [vp, vp, vp, vp, i, i, vp]
    lib.tm_get_grouped_plan.restype = i
    lib.tm_get_grouped_plan.argtypes = [vp, i, vp, vp]
    lib.tm_pack_w4_layout.restype = vp
    lib.tm_pack_w4_layout.argtypes = [vp, vp, vp, i, i, i, i, vp]
    lib.tm_gemm_w4a16.restype = i
    lib.tm_gemm_w4a16.argtypes = [vp, vp, vp, i, vp]
    lib.tm_gemm_w4a16_static.restype = i
    lib.tm_gemm_w4a16_static.argtypes = [vp, vp, vp, i, vp]
    lib.tm_gemm_w4a16_ex.restype = i
    lib.tm_gemm_w4a16_ex.argtypes = [vp, vp, vp, i, c.POINTER(TmEpilogue), vp]
    lib.tm_pack_w4_gate_up.restype = vp
    lib.tm_pack_w4_gate_up.argtypes = [vp, vp, vp, i, i, i, vp]
    lib.tm_gemm_w4a16_ws.restype = i
    lib.tm_gemm_w4a16_ws.argtypes = [vp, vp, vp, i, vp, sz, vp]
    lib.tm_reset_workspace.restype = i
    lib.tm_reset_workspace.argtypes = [vp, vp]
    lib.tm_gemm_workspace_bytes.restype = sz
    lib.tm_gemm_workspace_bytes.argtypes = [vp, i]
    lib.tm_free_packed.restype = None
    lib.tm_free_packed.argtypes = [vp]
    lib.tm_packed_info.restype = i
    lib.tm_packed_info.argtypes = [vp, c.POINTER(i), c.POINTER(i), c.POINTER(i), c.POINTER(sz)]
    lib.tm_unpack_w4.restype = i
    lib.tm_unpack_w4.argtypes = [vp, vp, vp, vp, vp]
    lib.tm_packed_raw.restype = i
    lib.tm_packed_raw.argtypes = [vp, c.POINTER(vp), c.POINTER(sz), c.POINTER(vp), c.POINTER(sz)]
    lib.tm_get_plan.restype = i
    lib.tm_get_plan.argtypes = [vp, i, c.POINTER(i), c.POINTER(i), c.POINTER(i), c.POINTER(i)]
    lib.tm_get_plan_units_per_wave.restype = i
    lib.tm_get_plan_units_per_wave.argtypes = [vp, i]
    lib.tm_set_variant.restype = i
    lib.tm_set_variant.argtypes = [i, i]
    lib.tm_set_mfma_shape.restype = i
    lib.tm_set_mfma_shape.argtypes = [i]
    lib.tm_get_plan_mfma_shape.restype = i
    lib.tm_get_plan_mfma_shape.argtypes = [vp, i]
    lib.tm_set_launch.restype = i
    lib.tm_set_launch.argtypes = [i, i]
    lib.tm_variant_name.restype = c.c_char_p
    lib.tm_variant_name.argtypes = [i]
    lib.tm_bench_copy.restype = i
    lib.tm_bench_copy.argtypes = [vp, vp, sz, vp]
    lib.tm_bench_read.restype = i
    lib.tm_bench_read.argtypes = [vp, sz, vp, vp]
    lib.tm_bench_clock.restype = i
    lib.tm_bench_clock.argtypes = [vp, i, i, vp]
    lib.tm_bench_mfma.restype = i
    lib.tm_bench_mfma.argtypes = [vp, i, i, i, i, vp]
    lib.tm_bench_read_shape.restype = i
    lib.tm_bench_read_shape.argtypes = [vp, sz, vp, i, i, i, i, vp]
    lib.tm_last_error.restype = c.c_char_p
    lib.tm_last_error.argtypes = []
    lib.tm_version.restype = c.c_char_p
    lib.tm_version.argtypes = []
    _lib = lib
    return lib


def tm_last_error() -> str:
    return load_library().tm_last_error().decode()


def tm_version() -> str:
    return load_library().tm_version().decode()


def _check(rc: int):
    if rc != TM_OK:
        raise TmError(rc, tm_last_error())


def _stream_ptr(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_ptr(t, dtype, what):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what} must be a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{what} must have dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


class PackedW4:
    """Owner of a tm_packed_w4 handle; freed when garbage-collected or on ``close()``."""

    def __init__(self, handle: int, K: int, N: int, group: int):
        self._h = handle
        self.K, self.N, self.group = K, N, group
        self.bits = 4

    @property
    def handle(self):
        if not self._h:
            raise ValueError("packed handle already freed")
        return ctypes.c_void_p(self._h)

    def close(self):
        if self._h:
            import torch
            torch.cuda.synchronize()
            load_library().tm_free_packed(ctypes.c_void_p(self._h))
            self._h = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def tm_pack_w4(qweight, scales, zeros, K: int, N: int, group: int, stream=None) -> PackedW4:
    """qweight int32 [K, N/8] (interchange nibble order), scales/zeros float16 [K/group, N] -> PackedW4.
    zeros=None packs symmetric weights (zero-point 8); group may be 32, 64 or a multiple of 128 dividing K."""
    return tm_pack_w4_layout(qweight, scales, zeros, K, N, group, TM_LAYOUT_N8, stream)


def tm_pack_w4_actorder(qweight, scales, zeros, g_idx, K: int, N: int, group: int, layout: int = 2, stream=None) -> PackedW4:
    """Activation-order checkpoint: as tm_pack_w4_layout plus g_idx int32 [K] (device), the K-group of every row."""
    import torch
    lib = load_library()
    qshape = (K // 8, N) if layout == TM_LAYOUT_K8 else (K, N // 8)
    zshape, zdtype = ((K // group, N), torch.float16) if layout == TM_LAYOUT_N8 else ((K // group, N // 8), torch.int32)
    if tuple(qweight.shape) != qshape or tuple(scales.shape) != (K // group, N) or g_idx.numel() != K or \
            (zeros is not None and tuple(zeros.shape) != zshape):
        raise ValueError("tensor shapes do not match K, N, group, layout")
    zptr = None if zeros is None else _dev_ptr(zeros, zdtype, "zeros")
    h = lib.tm_pack_w4_actorder(_dev_ptr(qweight, torch.int32, "qweight"), _dev_ptr(scales, torch.float16, "scales"), zptr,
                                _dev_ptr(g_idx, torch.int32, "g_idx"), K, N, group, layout, _stream_ptr(stream))
    if not h:
        raise TmError(-1, tm_last_error())
    return PackedW4(h, K, N, min(group, 128))


def tm_pack_w8(qweight, scales, zeros, K: int, N: int, group: int, stream=None) -> PackedW4:
    """8-bit codes: qweight int32 [K, N/4] (byte t = column 4j+t), scales float16 [K/group, N], zeros float16 of the
    same shape or None (symmetric, zero-point 128) -> PackedW4 usable with tm_gemm_w4a16."""
    import torch
    lib = load_library()
    if tuple(qweight.shape) != (K, N // 4) or tuple(scales.shape) != (K // group, N) or \
            (zeros is not None and tuple(zeros.shape) != (K // group, N)):
        raise ValueError("tensor shapes do not match K, N, group")
    zptr = None if zeros is None else _dev_ptr(zeros, torch.float16, "zeros")
    h = lib.tm_pack_w8(_dev_ptr(qweight, torch.int32, "qweight"), _dev_ptr(scales, torch.float16, "scales"), zptr,
                       K, N, group, _stream_ptr(stream))
    if not h:
        raise TmError(-1, tm_last_error())
    p = PackedW4(h, K, N, min(group, 128))
    p.bits = 8
    return p


def tm_pack_w8_fp8(qweight, scales, K: int, N: int, group: int, stream=None) -> PackedW4:
    """FP8 E4M3 codes: qweight int32 [K, N/4] (byte t = column 4j+t), scales float16 [K/group, N] -> PackedW4."""
    import torch
    lib = load_library()
    if tuple(qweight.shape) != (K, N // 4) or tuple(scales.shape) != (K // group, N):
        raise ValueError("tensor shapes do not match K, N, group")
    h = lib.tm_pack_w8_fp8(_dev_ptr(qweight, torch.int32, "qweight"), _dev_ptr(scales, torch.float16, "scales"),
                           K, N, group, _stream_ptr(stream))
    if not h:
        raise TmError(-1, tm_last_error())
    p = PackedW4(h, K, N, min(group, 128))
    p.bits = 8
    return p


TM_LAYOUT_N8, TM_LAYOUT_N8_INTERLEAVED, TM_LAYOUT_K8 = 0, 1, 2
TM_READ_NONTEMPORAL, TM_READ_CHUNKED, TM_READ_SHARED = 1, 2, 4        # flags of tm_bench_read_shape


def tm_pack_w4_layout(qweight, scales, zeros, K: int, N: int, group: int, layout: int, stream=None) -> PackedW4:
    """Pack from one of the interchange layouts of tm_layout: qweight int32 [K, N/8] (layouts 0, 1) or [K/8, N]
    (layout 2); zeros float16 [K/group, N] (layout 0) or int32 [K/group, N/8] (layouts 1, 2)."""
    import torch
    lib = load_library()
    qshape = (K // 8, N) if layout == TM_LAYOUT_K8 else (K, N // 8)
    zshape, zdtype = ((K // group, N), torch.float16) if layout == TM_LAYOUT_N8 else ((K // group, N // 8), torch.int32)
    if tuple(qweight.shape) != qshape or tuple(scales.shape) != (K // group, N) or \
            (zeros is not None and tuple(zeros.shape) != zshape):
        raise ValueError("tensor shapes do not match K, N, group, layout")
    zptr = None if zeros is None else _dev_ptr(zeros, zdtype, "zeros")
    h = lib.tm_pack_w4_layout(_dev_ptr(qweight, torch.int32, "qweight"), _dev_ptr(scales, torch.float16, "scales"),
                              zptr, K, N, group, layout, _stream_ptr(stream))
    if not h:
        raise TmError(-1, tm_last_error())
    return PackedW4(h, K, N, min(group, 128))


class ExpertGroup:
    """Owner of a tm_expert_group handle; keeps its PackedW4 experts alive."""

    def __init__(self, handle: int, experts):
        self._h = handle
        self.experts = list(experts)
        self.K, self.N, self.group = experts[0].K, experts[0].N, experts[0].group

    @property
    def handle(self):
        if not self._h:
            raise ValueError("expert group already freed")
        return ctypes.c_void_p(self._h)

    def close(self):
        if self._h:
            import torch
            torch.cuda.synchronize()
            load_library().tm_free_expert_group(ctypes.c_void_p(self._h))
            self._h = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def tm_group_experts(experts) -> ExpertGroup:
    """experts: sequence of PackedW4 with equal K, N, group -> ExpertGroup."""
    lib = load_library()
    arr = (ctypes.c_void_p * len(experts))(*[p.handle for p in experts])
    h = lib.tm_group_experts(arr, len(experts))
    if not h:
        raise TmError(-1, tm_last_error())
    return ExpertGroup(h, experts)


def tm_gemm_w4a16_grouped(X, group: ExpertGroup, offsets, Y, stream=None):
    """Rows offsets[e]..offsets[e+1] of X [R,K] times expert e -> the same rows of Y [R,N]; offsets int32 on the device."""
    import torch
    R = X.shape[0]
    if X.dim() != 2 or X.shape[1] != group.K or tuple(Y.shape) != (R, group.N) or offsets.numel() != len(group.experts) + 1:
        raise ValueError("X/Y/offsets shapes do not match the expert group")
    if R == 0:
        return Y
    _check(load_library().tm_gemm_w4a16_grouped(_dev_ptr(X, torch.float16, "X"), group.handle,
                                                _dev_ptr(offsets, torch.int32, "offsets"),
                                                _dev_ptr(Y, torch.float16, "Y"), R, _stream_ptr(stream)))
    return Y


def tm_gemm_w4a16_grouped_act(X, group: ExpertGroup, offsets, Y, act: int = 1, stream=None):
    """The grouped call with silu(gate)*up fused: experts packed by tm_pack_w4_gate_up, Y [R, N/2]."""
    import torch
    R = X.shape[0]
    n_out = group.N // 2 if act == 1 else group.N
    if X.dim() != 2 or X.shape[1] != group.K or tuple(Y.shape) != (R, n_out) or offsets.numel() != len(group.experts) + 1:
        raise ValueError("X/Y/offsets shapes do not match the expert group")
    if R == 0:
        return Y
    _check(load_library().tm_gemm_w4a16_grouped_act(_dev_ptr(X, torch.float16, "X"), group.handle,
                                                    _dev_ptr(offsets, torch.int32, "offsets"),
                                                    _dev_ptr(Y, torch.float16, "Y"), R, int(act), _stream_ptr(stream)))
    return Y


def tm_get_grouped_plan(group: ExpertGroup, total_rows: int):
    v, st = ctypes.c_int(), ctypes.c_int()
    _check(load_library().tm_get_grouped_plan(group.handle, total_rows, ctypes.byref(v), ctypes.byref(st)))
    return v.value, st.value


def tm_gemm_w4a16(X, packed: PackedW4, Y, stream=None):
    """Y[M,N] = X[M,K] * dequant(packed); X, Y float16 device tensors; enqueued on the current stream."""
    import torch
    M = X.shape[0]
    if X.dim() != 2 or X.shape[1] != packed.K or tuple(Y.shape) != (M, packed.N):
        raise ValueError("X/Y shapes do not match the packed weight")
    if M == 0:
        return Y
    _check(load_library().tm_gemm_w4a16(_dev_ptr(X, torch.float16, "X"), packed.handle,
                                        _dev_ptr(Y, torch.float16, "Y"), M, _stream_ptr(stream)))
    return Y


def tm_gemm_w4a16_static(X, packed: PackedW4, Y, stream=None):
    """tm_gemm_w4a16 through the library's fixed scratch array: the call allocates nothing (see include/tm_w4.h)."""
    import torch
    M = X.shape[0]
    if X.dim() != 2 or X.shape[1] != packed.K or tuple(Y.shape) != (M, packed.N):
        raise ValueError("X/Y shapes do not match the packed weight")
    if M == 0:
        return Y
    _check(load_library().tm_gemm_w4a16_static(_dev_ptr(X, torch.float16, "X"), packed.handle,
                                               _dev_ptr(Y, torch.float16, "Y"), M, _stream_ptr(stream)))
    return Y


TM_ACT_NONE, TM_ACT_SILU_MUL = 0, 1


def tm_gemm_w4a16_ex(X, packed: PackedW4, Y, bias=None, residual=None, act: int = TM_ACT_NONE, stream=None):
    """Y = fp16(act(X * dequant(packed) + bias) + residual); with TM_ACT_SILU_MUL (handles of tm_pack_w4_gate_up) Y and
    residual are [M, N/2].  All float16 device tensors."""
    import torch
    M = X.shape[0]
    n_out = packed.N // 2 if act == TM_ACT_SILU_MUL else packed.N
    if X.dim() != 2 or X.shape[1] != packed.K or tuple(Y.shape) != (M, n_out) or \
            (bias is not None and tuple(bias.shape) != (packed.N,)) or (residual is not None and tuple(residual.shape) != (M, n_out)):
        raise ValueError("X / Y / bias / residual shapes do not match the packed weight")
    if M == 0:
        return Y
    epi = TmEpilogue(None if bias is None else _dev_ptr(bias, torch.float16, "bias"),
                     None if residual is None else _dev_ptr(residual, torch.float16, "residual"), int(act))
    _check(load_library().tm_gemm_w4a16_ex(_dev_ptr(X, torch.float16, "X"), packed.handle, _dev_ptr(Y, torch.float16, "Y"), M,
                                           ctypes.byref(epi), _stream_ptr(stream)))
    return Y


def tm_pack_w4_gate_up(qweight, scales, zeros, K: int, N: int, group: int, stream=None) -> PackedW4:
    """Fused [gate | up] weight in the layout of tm_pack_w4 -> handle for tm_gemm_w4a16_ex(..., act=TM_ACT_SILU_MUL)."""
    import torch
    if tuple(qweight.shape) != (K, N // 8) or tuple(scales.shape) != (K // group, N) or \
            (zeros is not None and tuple(zeros.shape) != (K // group, N)):
        raise ValueError("tensor shapes do not match K, N, group")
    h = load_library().tm_pack_w4_gate_up(_dev_ptr(qweight, torch.int32, "qweight"), _dev_ptr(scales, torch.float16, "scales"),
                                          None if zeros is None else _dev_ptr(zeros, torch.float16, "zeros"), K, N, group,
                                          _stream_ptr(stream))
    if not h:
        raise TmError(-1, tm_last_error())
    return PackedW4(h, K, N, min(group, 128))


def tm_gemm_w4a16_ws(X, packed: PackedW4, Y, workspace, stream=None):
    import torch
    M = X.shape[0]
    if X.dim() != 2 or X.shape[1] != packed.K or tuple(Y.shape) != (M, packed.N):
        raise ValueError("X/Y shapes do not match the packed weight")
    if M == 0:
        return Y
    _check(load_library().tm_gemm_w4a16_ws(_dev_ptr(X, torch.float16, "X"), packed.handle,
                                           _dev_ptr(Y, torch.float16, "Y"), M,
                                           _dev_ptr(workspace, torch.uint8, "workspace"), workspace.numel(),
                                           _stream_ptr(stream)))
    return Y


def tm_reset_workspace(workspace=None, stream=None):
    """Zero the split-K arrival counters of `workspace` (None: of the library's own workspaces); see include/tm_w4.h."""
    ptr = None if workspace is None else ctypes.c_void_p(workspace.data_ptr())
    _check(load_library().tm_reset_workspace(ptr, _stream_ptr(stream)))


def tm_gemm_workspace_bytes(packed: PackedW4, M: int) -> int:
    return int(load_library().tm_gemm_workspace_bytes(packed.handle, M))


def tm_unpack_w4(packed: PackedW4, stream=None):
    """Device-side inverse permutation -> (qweight int32 [K,N/8], scales f16, zeros f16)."""
    import torch
    K, N, g = packed.K, packed.N, packed.group
    q = torch.empty((K, N // 8), dtype=torch.int32, device="cuda")
    s = torch.empty((K // g, N), dtype=torch.float16, device="cuda")
    z = torch.empty((K // g, N), dtype=torch.float16, device="cuda")
    _check(load_library().tm_unpack_w4(packed.handle, ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(s.data_ptr()),
                                       ctypes.c_void_p(z.data_ptr()), _stream_ptr(stream)))
    return q, s, z


def tm_packed_raw(packed: PackedW4):
    """Copies of the handle's raw device buffers as host numpy uint32 arrays (weights words, scale|zero words)."""
    import numpy as np
    import torch
    lib = load_library()
    w, sz = ctypes.c_void_p(), ctypes.c_void_p()
    wb, szb = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib.tm_packed_raw(packed.handle, ctypes.byref(w), ctypes.byref(wb), ctypes.byref(sz), ctypes.byref(szb)))
    torch.cuda.synchronize()
    outs = []
    for ptr, nbytes in ((w, wb.value), (sz, szb.value)):
        tmp = torch.empty(nbytes // 4, dtype=torch.int32, device="cuda")
        _check(lib.tm_bench_copy(ctypes.c_void_p(tmp.data_ptr()), ptr, nbytes, _stream_ptr(None)))
        outs.append(tmp.cpu().numpy().view(np.uint32))
    return outs[0], outs[1]


def tm_get_plan(packed: PackedW4, M: int) -> dict:
    lib = load_library()
    v, s, g, b = ctypes.c_int(), ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib.tm_get_plan(packed.handle, M, ctypes.byref(v), ctypes.byref(s), ctypes.byref(g), ctypes.byref(b)))
    upw = lib.tm_get_plan_units_per_wave(packed.handle, M)
    if upw < 0:
        raise TmError(upw, tm_last_error())
    shape = lib.tm_get_plan_mfma_shape(packed.handle, M)
    if shape < 0:
        raise TmError(shape, tm_last_error())
    return {"variant": v.value, "name": lib.tm_variant_name(v.value).decode(), "split_k": s.value,
            "grid": g.value, "block": b.value, "one_shot_units_per_wave": upw, "mfma_shape": shape}


def tm_set_variant(variant: int = -1, split_k: int = 0):
    _check(load_library().tm_set_variant(variant, split_k))


def tm_set_mfma_shape(shape: int = 0):
    _check(load_library().tm_set_mfma_shape(shape))


def tm_set_launch(waves: int = 0, stage_steps: int = 0):
    _check(load_library().tm_set_launch(waves, stage_steps))


def tm_variant_name(variant: int) -> str:
    return load_library().tm_variant_name(variant).decode()


def tm_bench_copy(dst, src, stream=None):
    nbytes = src.numel() * src.element_size()
    _check(load_library().tm_bench_copy(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()), nbytes,
                                        _stream_ptr(stream)))


def tm_bench_read(src, sink, stream=None):
    nbytes = src.numel() * src.element_size()
    _check(load_library().tm_bench_read(ctypes.c_void_p(src.data_ptr()), nbytes, ctypes.c_void_p(sink.data_ptr()),
                                        _stream_ptr(stream)))


def tm_bench_clock(out, micros: int, delay_micros: int = 0, stream=None) -> int:
    """A one-wave launch that waits `delay_micros`, then watches the shader clock for `micros` microseconds
    (include/tm_w4.h); `out` is an int32 device tensor of at least 4 elements.  Returns the constant-rate counter's
    frequency in kHz."""
    khz = load_library().tm_bench_clock(ctypes.c_void_p(out.data_ptr()), delay_micros, micros, _stream_ptr(stream))
    _check(min(khz, 0))
    return khz


def tm_bench_mfma(out, grid: int, block: int, iters: int, pattern: int = 1, stream=None):
    """A launch of matrix instructions only (include/tm_w4.h); `out` is an int32 device tensor of at least 4 elements."""
    _check(load_library().tm_bench_mfma(ctypes.c_void_p(out.data_ptr()), grid, block, iters, pattern, _stream_ptr(stream)))


def tm_bench_read_shape(src_ptr: int, nbytes: int, sink, grid: int, block: int, unroll: int, flags: int = 0, stream=None):
    """Read-only stream over nbytes at the raw device address src_ptr in the given launch shape (see include/tm_w4.h)."""
    _check(load_library().tm_bench_read_shape(ctypes.c_void_p(src_ptr), nbytes, ctypes.c_void_p(sink.data_ptr()), grid, block,
                                              unroll, flags, _stream_ptr(stream)))


# ------------------------------------------------------------------ attention over a quantised KV cache (tm_attn.h)

class KvCache:
    """Owner of a tm_kv_cache handle (8-bit codes, head dimension 128)."""

    def __init__(self, batch: int, kv_heads: int, capacity: int, bits: int = 8):
        h = load_library().tm_kv_create(batch, kv_heads, capacity, bits)
        if not h:
            raise TmError(-1, tm_last_error())
        self._h = h
        tok = 256 // bits                           # the library rounds the capacity up to whole 4 KiB blocks of codes
        self.batch, self.kv_heads, self.capacity, self.bits = batch, kv_heads, (capacity + tok - 1) // tok * tok, bits

    @property
    def handle(self):
        if not self._h:
            raise ValueError("cache already freed")
        return ctypes.c_void_p(self._h)

    def close(self):
        if self._h:
            import torch
            torch.cuda.synchronize()
            load_library().tm_kv_free(ctypes.c_void_p(self._h))
            self._h = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def tm_kv_create(batch: int, kv_heads: int, capacity: int, bits: int = 8) -> KvCache:
    return KvCache(batch, kv_heads, capacity, bits)


def tm_kv_append(cache: KvCache, K_new, V_new, positions, stream=None):
    """K_new, V_new float16 [batch, count, kv_heads, 128]; positions int32 [batch] (device)."""
    import torch
    if K_new.dim() != 4 or tuple(K_new.shape) != tuple(V_new.shape) or K_new.shape[0] != cache.batch or \
            K_new.shape[2] != cache.kv_heads or K_new.shape[3] != 128 or positions.numel() != cache.batch:
        raise ValueError("K_new / V_new / positions shapes do not match the cache")
    _check(load_library().tm_kv_append(cache.handle, _dev_ptr(K_new, torch.float16, "K_new"),
                                       _dev_ptr(V_new, torch.float16, "V_new"), _dev_ptr(positions, torch.int32, "positions"),
                                       K_new.shape[1], _stream_ptr(stream)))


def tm_attn_decode(Q, cache: KvCache, lens, O, scale: float, max_len: int = 0, stream=None):
    """Q, O float16 [batch, q_heads, 128]; lens int32 [batch] (device)."""
    import torch
    if Q.dim() != 3 or Q.shape[0] != cache.batch or Q.shape[2] != 128 or tuple(O.shape) != tuple(Q.shape) or \
            lens.numel() != cache.batch:
        raise ValueError("Q / O / lens shapes do not match the cache")
    _check(load_library().tm_attn_decode(_dev_ptr(Q, torch.float16, "Q"), cache.handle, _dev_ptr(lens, torch.int32, "lens"),
                                         _dev_ptr(O, torch.float16, "O"), Q.shape[1], float(scale), int(max_len),
                                         _stream_ptr(stream)))
    return O


def tm_attn_prefill(Q, cache: KvCache, positions, O, scale: float, counts=None, stream=None):
    """Causal attention of a chunk of prompt tokens over the cache: Q, O fp16 [batch][count][q_heads][128] device tensors,
    positions int32 [batch], counts int32 [batch] or None (see include/tm_attn.h)."""
    import torch
    if Q.dim() != 4 or Q.shape[3] != 128 or tuple(O.shape) != tuple(Q.shape):
        raise ValueError("Q and O must be [batch][count][q_heads][128]")
    cp = None if counts is None else _dev_ptr(counts, torch.int32, "counts")
    _check(load_library().tm_attn_prefill(_dev_ptr(Q, torch.float16, "Q"), cache.handle, _dev_ptr(positions, torch.int32, "positions"),
                                          cp, Q.shape[1], _dev_ptr(O, torch.float16, "O"), Q.shape[2], scale, _stream_ptr(stream)))
    return O


def tm_kv_raw(cache: KvCache):
    """Device pointers and sizes of the cache's buffers: (k_ptr, v_ptr, pair_ptr, code_bytes, pair_bytes)."""
    k, v, p = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
    cb, pb = ctypes.c_size_t(), ctypes.c_size_t()
    _check(load_library().tm_kv_raw(cache.handle, ctypes.byref(k), ctypes.byref(v), ctypes.byref(p), ctypes.byref(cb),
                                    ctypes.byref(pb)))
    return k.value, v.value, p.value, cb.value, pb.value


def tm_bench_copy_raw(dst_ptr: int, src_ptr: int, nbytes: int, stream=None):
    """Plain device copy between raw device addresses (multiples of 16 bytes)."""
    _check(load_library().tm_bench_copy(ctypes.c_void_p(dst_ptr), ctypes.c_void_p(src_ptr), nbytes, _stream_ptr(stream)))


def tm_kv_download(cache: KvCache):
    """Host copies of the cache's buffers: (K codes uint8, V codes uint8, pairs uint32), flat."""
    import numpy as np
    import torch
    lib = load_library()
    k, v, p, cb, pb = tm_kv_raw(cache)
    torch.cuda.synchronize()
    outs = []
    for ptr, nbytes in ((k, cb), (v, cb), (p, pb)):
        tmp = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        _check(lib.tm_bench_copy(ctypes.c_void_p(tmp.data_ptr()), ctypes.c_void_p(ptr), nbytes, _stream_ptr(None)))
        outs.append(tmp.cpu().numpy())
    return outs[0], outs[1], outs[2].view(np.uint32)


def tm_kv_upload(cache: KvCache, kbuf, vbuf, szbuf):
    """Overwrite the cache's buffers with host arrays in the cache layout (tests and benchmarks)."""
    import numpy as np
    import torch
    lib = load_library()
    k, v, p, cb, pb = tm_kv_raw(cache)
    for ptr, nbytes, host in ((k, cb, kbuf), (v, cb, vbuf), (p, pb, szbuf)):
        t = torch.from_numpy(np.ascontiguousarray(host).view(np.uint8).reshape(-1)).cuda()
        if t.numel() != nbytes:
            raise ValueError("buffer size does not match the cache")
        _check(lib.tm_bench_copy(ctypes.c_void_p(ptr), ctypes.c_void_p(t.data_ptr()), nbytes, _stream_ptr(None)))
    torch.cuda.synchronize()
