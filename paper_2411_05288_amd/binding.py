"""ctypes binding of libvp.so.  Function names and argument order follow include/vp.h.

Tensors are torch tensors on the GPU; bf16 data may be passed as torch.bfloat16 or as
int16/uint16 bit patterns.  Nothing here computes: the functions check dtype / device /
contiguity, take raw pointers and the current HIP stream, and call the library.  There is no
fallback: if libvp.so is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

VP_F32 = 0
VP_BF16 = 1
VP_SAVE_LOGITS = 1
VP_SKIP_DH = 2
VP_DH_OVERWRITE = 4

VP_CALL_OUTPUT_FWD = 0
VP_CALL_COMBINE_STATS = 1
VP_CALL_OUTPUT_BWD = 2
VP_CALL_EMBED_FWD = 3
VP_CALL_EMBED_BWD = 4
VP_CALL_OUTPUT_FWD_ALG2 = 5
VP_CALL_OUTPUT_DX_ALG2 = 6

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class VPError(RuntimeError):
    pass


def lib_path() -> str:
    return os.path.join(_HERE, "libvp.so")


def load_library() -> ctypes.CDLL:
    """Loads libvp.so (built by ``python -m paper_2411_05288_amd.build``)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise VPError("libvp.so not found at %s: build it with `python -m paper_2411_05288_amd.build`" % path)
    lib = ctypes.CDLL(path)
    c = ctypes
    vp, i64, i32, u32, sz, fl = c.c_void_p, c.c_int64, c.c_int32, c.c_uint32, c.c_size_t, c.c_float
    lib.vp_version.restype = c.c_int
    lib.vp_version.argtypes = []
    lib.vp_status_string.restype = c.c_char_p
    lib.vp_status_string.argtypes = [c.c_int]
    lib.vp_workspace_bytes.restype = sz
    lib.vp_workspace_bytes.argtypes = [c.c_int, i64, i64, i64, c.c_int, u32]
    lib.vp_dlogits_row_stride.restype = i64
    lib.vp_dlogits_row_stride.argtypes = [i64, c.c_int]
    lib.vp_output_fwd.restype = c.c_int
    lib.vp_output_fwd.argtypes = [vp, vp, vp, i64, i64, i64, i64, c.c_int, u32, vp, vp, vp, vp, vp, sz, vp]
    lib.vp_output_fwd_noalloc.restype = c.c_int
    lib.vp_output_fwd_noalloc.argtypes = [vp, vp, vp, i64, i64, i64, i64, c.c_int, u32, vp, vp, vp, vp, vp]
    lib.vp_output_fwd_noalloc_max_scratch.restype = sz
    lib.vp_output_fwd_noalloc_max_scratch.argtypes = []
    lib.vp_combine_stats.restype = c.c_int
    lib.vp_combine_stats.argtypes = [vp, vp, vp, i32, i64, vp, vp, vp, vp, vp]
    lib.vp_output_bwd.restype = c.c_int
    lib.vp_output_bwd.argtypes = [vp, vp, vp, i64, i64, i64, i64, c.c_int, u32, vp, vp, vp, fl, vp, vp, vp, sz, vp]
    lib.vp_output_fwd_alg2.restype = c.c_int
    lib.vp_output_fwd_alg2.argtypes = [vp, vp, vp, i64, i64, i64, i64, c.c_int, u32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.vp_output_dx_alg2.restype = c.c_int
    lib.vp_output_dx_alg2.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, c.c_int, u32, fl, vp, vp]
    lib.vp_embed_fwd.restype = c.c_int
    lib.vp_embed_fwd.argtypes = [vp, vp, i64, i64, i64, i64, c.c_int, vp, vp]
    lib.vp_embed_bwd.restype = c.c_int
    lib.vp_embed_bwd.argtypes = [vp, vp, i64, i64, i64, i64, c.c_int, vp, vp, sz, vp]
    lib.vp_profile_mfma_loop.restype = c.c_int
    lib.vp_profile_mfma_loop.argtypes = [vp, vp, i32, i32, vp]
    lib.vp_profile_mfma_variant.restype = c.c_int
    lib.vp_profile_mfma_variant.argtypes = [vp, vp, i32, i32, i32, vp]
    lib.vp_profile_mfma_variant_count.restype = c.c_int
    lib.vp_profile_mfma_variant_count.argtypes = []
    lib.vp_profile_mfma_variant_flops.restype = c.c_double
    lib.vp_profile_mfma_variant_flops.argtypes = [i32]
    lib.vp_profile_force_generic_gemm.restype = c.c_int
    lib.vp_profile_force_generic_gemm.argtypes = [c.c_int]
    lib.vp_profile_gemm_trace.restype = c.c_int
    lib.vp_profile_gemm_trace.argtypes = [vp, sz, c.c_int]
    lib.vp_profile_kernel_count.restype = c.c_int
    lib.vp_profile_kernel_count.argtypes = []
    lib.vp_profile_kernel_name.restype = c.c_char_p
    lib.vp_profile_kernel_name.argtypes = [c.c_int]
    lib.vp_profile_enable.restype = c.c_int
    lib.vp_profile_enable.argtypes = [c.c_int]
    lib.vp_profile_read.restype = c.c_int
    lib.vp_profile_read.argtypes = [c.POINTER(c.c_double), c.POINTER(c.c_int64), c.c_int]
    _LIB = lib
    return lib


def _check(status: int, what: str) -> None:
    if status != 0:
        name = load_library().vp_status_string(status).decode()
        raise VPError("%s failed: %s" % (what, name))


_BF16_LIKE = (torch.bfloat16, torch.int16, torch.uint16)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return VP_F32
    if t.dtype in _BF16_LIKE:
        return VP_BF16
    raise VPError("unsupported tensor dtype %s" % t.dtype)


def _ptr(t: Optional[torch.Tensor], name: str, dtypes=None, shape=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise VPError("%s must be a GPU tensor" % name)
    if not t.is_contiguous():
        raise VPError("%s must be contiguous" % name)
    if dtypes is not None and t.dtype not in dtypes:
        raise VPError("%s has dtype %s, expected one of %s" % (name, t.dtype, dtypes))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise VPError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def vp_version() -> int:
    return load_library().vp_version()


def vp_workspace_bytes(which: int, N: int, h: int, Vs: int, dt: int, flags: int = 0) -> int:
    n = load_library().vp_workspace_bytes(which, N, h, Vs, dt, flags)
    if n == ctypes.c_size_t(-1).value:
        raise VPError("vp_workspace_bytes: invalid arguments")
    return n


def vp_dlogits_row_stride(Vs: int, dt: int) -> int:
    n = load_library().vp_dlogits_row_stride(Vs, dt)
    if n < 0:
        raise VPError("vp_dlogits_row_stride: invalid arguments")
    return n


def _ws(workspace: Optional[torch.Tensor]):
    if workspace is None:
        return None, 0
    return _ptr(workspace, "workspace"), workspace.numel() * workspace.element_size()


def vp_output_fwd(H, W_shard, labels, shard_offset: int, local_max, local_sumexp, local_target,
                  logits_out=None, workspace=None, stream=None) -> None:
    """Pass S for one shard; writes local_max / local_sumexp / local_target ([N] fp32 each)."""
    N, h = H.shape
    Vs = W_shard.shape[0]
    dt = _dtype_code(H)
    if _dtype_code(W_shard) != dt or W_shard.shape[1] != h:
        raise VPError("W_shard must be [Vs, h] with the dtype of H")
    same = (torch.float32,) if dt == VP_F32 else _BF16_LIKE
    wp, wb = _ws(workspace)
    st = load_library().vp_output_fwd(
        _ptr(H, "H"), _ptr(W_shard, "W_shard"), _ptr(labels, "labels", (torch.int64,), (N,)),
        N, h, Vs, shard_offset, dt, VP_SAVE_LOGITS if logits_out is not None else 0,
        _ptr(local_max, "local_max", (torch.float32,), (N,)),
        _ptr(local_sumexp, "local_sumexp", (torch.float32,), (N,)),
        _ptr(local_target, "local_target", (torch.float32,), (N,)),
        _ptr(logits_out, "logits_out", same, (N, Vs)), wp, wb, _stream(stream))
    _check(st, "vp_output_fwd")


def vp_output_fwd_noalloc(H, W_shard, labels, shard_offset: int, local_max, local_sumexp, local_target,
                          logits_out=None, stream=None) -> None:
    """vp_output_fwd with the scratch in a static device array of the library: no workspace argument,
    nothing allocated.  Sizes whose scratch exceeds vp_output_fwd_noalloc_max_scratch() are refused."""
    N, h = H.shape
    Vs = W_shard.shape[0]
    dt = _dtype_code(H)
    if _dtype_code(W_shard) != dt or W_shard.shape[1] != h:
        raise VPError("W_shard must be [Vs, h] with the dtype of H")
    same = (torch.float32,) if dt == VP_F32 else _BF16_LIKE
    st = load_library().vp_output_fwd_noalloc(
        _ptr(H, "H"), _ptr(W_shard, "W_shard"), _ptr(labels, "labels", (torch.int64,), (N,)),
        N, h, Vs, shard_offset, dt, VP_SAVE_LOGITS if logits_out is not None else 0,
        _ptr(local_max, "local_max", (torch.float32,), (N,)),
        _ptr(local_sumexp, "local_sumexp", (torch.float32,), (N,)),
        _ptr(local_target, "local_target", (torch.float32,), (N,)),
        _ptr(logits_out, "logits_out", same, (N, Vs)), _stream(stream))
    _check(st, "vp_output_fwd_noalloc")


def vp_output_fwd_noalloc_max_scratch() -> int:
    return load_library().vp_output_fwd_noalloc_max_scratch()


def vp_combine_stats(local_max, local_sumexp, local_target, global_max, global_sumexp, loss_per_row,
                     loss_mean, stream=None) -> None:
    """Barrier C1 over the p rows of the [p, N] statistics."""
    p, N = local_max.shape
    f = (torch.float32,)
    st = load_library().vp_combine_stats(
        _ptr(local_max, "local_max", f, (p, N)), _ptr(local_sumexp, "local_sumexp", f, (p, N)),
        _ptr(local_target, "local_target", f, (p, N)), p, N,
        _ptr(global_max, "global_max", f, (N,)), _ptr(global_sumexp, "global_sumexp", f, (N,)),
        _ptr(loss_per_row, "loss_per_row", f, (N,)), _ptr(loss_mean, "loss_mean", f, (1,)), _stream(stream))
    _check(st, "vp_combine_stats")


def vp_output_bwd(H, W_shard, labels, shard_offset: int, global_max, global_sumexp, logits_saved,
                  grad_scale: float, dH_accum, dW_shard, workspace, stream=None, dh_overwrite: bool = False) -> None:
    """Pass T for one shard: dH_accum += D W_shard, dW_shard = D^T H.  dH_accum=None selects pass T of
    Algorithm 2 (flag VP_SKIP_DH): only dW_shard is formed.  dh_overwrite=True (flag VP_DH_OVERWRITE)
    writes dH_accum = D W_shard: the first term of the reduce, no zero-fill needed."""
    N, h = H.shape
    Vs = W_shard.shape[0]
    dt = _dtype_code(H)
    if _dtype_code(W_shard) != dt or W_shard.shape[1] != h:
        raise VPError("W_shard must be [Vs, h] with the dtype of H")
    same = (torch.float32,) if dt == VP_F32 else _BF16_LIKE
    f = (torch.float32,)
    wp, wb = _ws(workspace)
    st = load_library().vp_output_bwd(
        _ptr(H, "H"), _ptr(W_shard, "W_shard"), _ptr(labels, "labels", (torch.int64,), (N,)),
        N, h, Vs, shard_offset, dt,
        (VP_SAVE_LOGITS if logits_saved is not None else 0) | (VP_SKIP_DH if dH_accum is None else 0)
        | (VP_DH_OVERWRITE if (dh_overwrite and dH_accum is not None) else 0),
        _ptr(global_max, "global_max", f, (N,)), _ptr(global_sumexp, "global_sumexp", f, (N,)),
        _ptr(logits_saved, "logits_saved", same, (N, Vs)), float(grad_scale),
        _ptr(dH_accum, "dH_accum", f, (N, h)), _ptr(dW_shard, "dW_shard", f, (Vs, h)),
        wp, wb, _stream(stream))
    _check(st, "vp_output_bwd")


def vp_output_fwd_alg2(H, W_shard, labels, shard_offset: int, local_max, local_sumexp, local_target,
                       A_out, B_out, logits_out=None, workspace=None, stream=None) -> None:
    """Pass S of Algorithm 2 for one shard: the outputs of vp_output_fwd plus A = softmax' W_shard
    ([N, h] fp32) and B = G W_shard ([N, h], dtype of W)."""
    N, h = H.shape
    Vs = W_shard.shape[0]
    dt = _dtype_code(H)
    if _dtype_code(W_shard) != dt or W_shard.shape[1] != h:
        raise VPError("W_shard must be [Vs, h] with the dtype of H")
    same = (torch.float32,) if dt == VP_F32 else _BF16_LIKE
    f = (torch.float32,)
    wp, wb = _ws(workspace)
    st = load_library().vp_output_fwd_alg2(
        _ptr(H, "H"), _ptr(W_shard, "W_shard"), _ptr(labels, "labels", (torch.int64,), (N,)),
        N, h, Vs, shard_offset, dt, VP_SAVE_LOGITS if logits_out is not None else 0,
        _ptr(local_max, "local_max", f, (N,)), _ptr(local_sumexp, "local_sumexp", f, (N,)),
        _ptr(local_target, "local_target", f, (N,)), _ptr(logits_out, "logits_out", same, (N, Vs)),
        _ptr(A_out, "A_out", f, (N, h)), _ptr(B_out, "B_out", same, (N, h)), wp, wb, _stream(stream))
    _check(st, "vp_output_fwd_alg2")


def vp_output_dx_alg2(A, B, local_max, local_sumexp, global_max, global_sumexp, grad_scale: float, dH_accum,
                      stream=None, dh_overwrite: bool = False) -> None:
    """dH_accum += (A * sum' e^{m'-m} / sum - B) * grad_scale: this shard's term of Algorithm 2's input gradient
    (dh_overwrite=True, flag VP_DH_OVERWRITE: = instead of +=, the first term of the reduce)."""
    N, h = A.shape
    f = (torch.float32,)
    dt = _dtype_code(B)
    st = load_library().vp_output_dx_alg2(
        _ptr(A, "A", f, (N, h)), _ptr(B, "B", None, (N, h)), _ptr(local_max, "local_max", f, (N,)),
        _ptr(local_sumexp, "local_sumexp", f, (N,)), _ptr(global_max, "global_max", f, (N,)),
        _ptr(global_sumexp, "global_sumexp", f, (N,)), N, h, dt, VP_DH_OVERWRITE if dh_overwrite else 0,
        float(grad_scale), _ptr(dH_accum, "dH_accum", f, (N, h)), _stream(stream))
    _check(st, "vp_output_dx_alg2")


def vp_embed_fwd(table_shard, ids, shard_offset: int, out, stream=None) -> None:
    Vs, h = table_shard.shape
    N = ids.shape[0]
    dt = _dtype_code(table_shard)
    st = load_library().vp_embed_fwd(
        _ptr(table_shard, "table_shard"), _ptr(ids, "ids", (torch.int64,), (N,)), N, h, Vs, shard_offset, dt,
        _ptr(out, "out", (table_shard.dtype,), (N, h)), _stream(stream))
    _check(st, "vp_embed_fwd")


def vp_embed_bwd(grad_out, ids, shard_offset: int, dtable_shard, workspace, stream=None) -> None:
    N, h = grad_out.shape
    Vs = dtable_shard.shape[0]
    dt = _dtype_code(grad_out)
    wp, wb = _ws(workspace)
    st = load_library().vp_embed_bwd(
        _ptr(grad_out, "grad_out"), _ptr(ids, "ids", (torch.int64,), (N,)), N, h, Vs, shard_offset, dt,
        _ptr(dtable_shard, "dtable_shard", (torch.float32,), (Vs, h)), wp, wb, _stream(stream))
    _check(st, "vp_embed_bwd")


def vp_profile_mfma_loop(operands, out, iters: int, blocks: int, stream=None) -> None:
    """Measurement aid: back-to-back MFMAs on register operands (see include/vp.h)."""
    if operands.numel() * operands.element_size() < 8 * 256 * 16 or out.numel() < blocks * 256:
        raise VPError("vp_profile_mfma_loop: buffers too small")
    st = load_library().vp_profile_mfma_loop(_ptr(operands, "operands", _BF16_LIKE), _ptr(out, "out", (torch.float32,)),
                                             iters, blocks, _stream(stream))
    _check(st, "vp_profile_mfma_loop")


def vp_profile_mfma_variant(operands, out, iters: int, blocks: int, variant: int, stream=None) -> float:
    """Measurement aid: the MFMA loop in another instruction shape / issue order (see include/vp.h).
    Returns the flop count of the launch."""
    lib = load_library()
    if operands.numel() * operands.element_size() < 32 * 256 * 16 or out.numel() < blocks * 256:
        raise VPError("vp_profile_mfma_variant: buffers too small")
    st = lib.vp_profile_mfma_variant(_ptr(operands, "operands", _BF16_LIKE), _ptr(out, "out", (torch.float32,)),
                                     iters, blocks, variant, _stream(stream))
    _check(st, "vp_profile_mfma_variant")
    return lib.vp_profile_mfma_variant_flops(variant) * blocks * 4 * iters


def vp_profile_mfma_variant_count() -> int:
    return load_library().vp_profile_mfma_variant_count()


def vp_profile_force_generic_gemm(on: bool) -> None:
    """Test switch: route every bf16 product through the generic GEMM kernel."""
    _check(load_library().vp_profile_force_generic_gemm(1 if on else 0), "vp_profile_force_generic_gemm")


def vp_profile_gemm_trace(buffer, kernel: Optional[str] = None) -> None:
    """Measurement aid: phase stamps of the fast GEMM kernel into `buffer` (a GPU tensor of int64; None = off),
    optionally only for launches timed under the kernel name `kernel` (see vp_profile_read)."""
    lib = load_library()
    if buffer is None:
        _check(lib.vp_profile_gemm_trace(None, 0, -1), "vp_profile_gemm_trace")
        return
    kid = -1
    if kernel is not None:
        names = [lib.vp_profile_kernel_name(i).decode() for i in range(lib.vp_profile_kernel_count())]
        if kernel not in names:
            raise VPError("unknown kernel name %r" % kernel)
        kid = names.index(kernel)
    _check(lib.vp_profile_gemm_trace(_ptr(buffer, "buffer", (torch.int64,)), buffer.numel() * 8, kid),
           "vp_profile_gemm_trace")


def vp_profile_enable(on: bool) -> None:
    _check(load_library().vp_profile_enable(1 if on else 0), "vp_profile_enable")


def vp_profile_read() -> dict:
    """{kernel name: (total milliseconds, launches)} since the last read; clears the records."""
    lib = load_library()
    n = lib.vp_profile_kernel_count()
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    _check(lib.vp_profile_read(ms, cnt, n), "vp_profile_read")
    return {lib.vp_profile_kernel_name(i).decode(): (ms[i], cnt[i]) for i in range(n) if cnt[i] > 0}
