"""Thin ctypes binding of libqzo.so (include/qzo.h): argument marshalling only.

Every function has the name of the C entry point it calls and takes torch CUDA
tensors for device memory.  PyTorch supplies memory and streams; every step of
the QZO path runs in the library's HIP kernels.  There is no fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqzo.so")
_lib = None

QZO_OK = 0
QZO_ERR_ARG, QZO_ERR_SHAPE, QZO_ERR_ALIGN, QZO_ERR_WORKSPACE = -1, -2, -3, -4
QZO_ERR_NONFINITE, QZO_ERR_HIP, QZO_ERR_UNSUPPORTED = -5, -6, -7

EXPORTS = [
    "qzo_model_create", "qzo_model_destroy", "qzo_model_scale_count", "qzo_workspace_bytes",
    "qzo_forward_loss", "qzo_step", "qzo_model_apply_update",
    "qzo_model_dense_count", "qzo_model_joint_table_bytes", "qzo_model_enable_joint", "qzo_step_joint",
    "qzo_linear_scratch_bytes", "qzo_dequant_gemm", "qzo_dequant_gemm_static", "qzo_dequant_gemm_zp", "qzo_apply_update",
    "qzo_rtn_quantize", "qzo_rtn_quantize_asym", "qzo_repack_kmajor",
    "qzo_int4_expand", "qzo_int4_scratch_bytes", "qzo_int4_gemm_expanded", "qzo_model_set_int4_path",
    "qzo_nf4_expand", "qzo_nf4_scratch_bytes", "qzo_nf4_gemm",
    "qzo_codebook_scratch_bytes", "qzo_codebook_gemm", "qzo_apply_update_channel",
    "qzo_debug_philox", "qzo_debug_normal_pairs", "qzo_debug_normals", "qzo_debug_dequant", "qzo_debug_dequant_zp",
    "qzo_debug_forward", "qzo_debug_bf16_gemm", "qzo_debug_mfma_rate",
    "qzo_profile_begin", "qzo_profile_collect", "qzo_profile_stride",
    "qzo_last_error",
]


class QzoError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"qzo status {status}: {msg}")
        self.status = status


class qzo_model_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("arch", C.c_uint32), ("n_layers", C.c_uint32),
                ("d_model", C.c_uint32), ("n_heads", C.c_uint32), ("d_ffn", C.c_uint32),
                ("vocab", C.c_uint32), ("max_seq", C.c_uint32), ("group_size", C.c_uint32),
                ("quant", C.c_uint32), ("norm_eps", C.c_float), ("rope_theta", C.c_float),
                ("scale_fp16", C.c_uint32), ("act_order", C.c_uint32)]


class qzo_buf(C.Structure):
    _fields_ = [("ptr_dev", C.c_void_p), ("bytes", C.c_uint64)]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -c 'import __graft_entry__ as g; g.build()'`")
        _lib = C.CDLL(LIB_PATH)
        _lib.qzo_last_error.restype = C.c_char_p
        for name in EXPORTS[:-1]:
            getattr(_lib, name).restype = C.c_int
    return _lib


def _check(status):
    if status != QZO_OK:
        raise QzoError(status, lib().qzo_last_error().decode())


def _ptr(t):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def make_config(shape: dict) -> qzo_model_config:
    return qzo_model_config(C.sizeof(qzo_model_config), 0 if shape["arch"] == "llama" else 1,
                            shape["n_layers"], shape["d_model"], shape["n_heads"], shape["d_ffn"],
                            shape["vocab"], shape["max_seq"], shape.get("group", 128), shape.get("quant", 0),
                            shape.get("norm_eps", 1e-5), shape.get("rope_theta", 10000.0),
                            int(shape.get("scale_fp16", 0)), int(shape.get("act_order", 0)))


def qzo_model_scale_count(shape: dict) -> int:
    cfg = make_config(shape)
    out = C.c_uint64(0)
    _check(lib().qzo_model_scale_count(C.byref(cfg), C.byref(out)))
    return out.value


def qzo_model_create(shape: dict, tensors, scale_arena):
    cfg = make_config(shape)
    bufs = (qzo_buf * len(tensors))(*[qzo_buf(t.data_ptr(), t.numel() * t.element_size())
                                      for t in tensors])
    handle = C.c_void_p(0)
    _check(lib().qzo_model_create(C.byref(cfg), bufs, C.c_uint32(len(tensors)), _ptr(scale_arena),
                                  C.c_uint64(scale_arena.numel()), C.byref(handle)))
    return handle


def qzo_model_destroy(model):
    _check(lib().qzo_model_destroy(model))


def qzo_workspace_bytes(model, batch, seq) -> int:
    out = C.c_uint64(0)
    _check(lib().qzo_workspace_bytes(model, C.c_uint32(batch), C.c_uint32(seq), C.byref(out)))
    return out.value


def qzo_forward_loss(model, tokens, seed, eps, sign, workspace, loss_out, stream=None):
    B, S = tokens.shape
    _check(lib().qzo_forward_loss(model, _ptr(tokens), C.c_uint32(B), C.c_uint32(S),
                                  C.c_uint64(seed), C.c_float(eps), C.c_int(sign), _ptr(workspace),
                                  C.c_uint64(workspace.numel() * workspace.element_size()),
                                  _ptr(loss_out), _stream(stream)))


def qzo_step(model, tokens, seed, eps, eta, clip, workspace, result, stream=None):
    """result: 8 x 4-byte device tensor receiving qzo_step_result."""
    B, S = tokens.shape
    _check(lib().qzo_step(model, _ptr(tokens), C.c_uint32(B), C.c_uint32(S), C.c_uint64(seed),
                          C.c_float(eps), C.c_float(eta), C.c_float(clip), _ptr(workspace),
                          C.c_uint64(workspace.numel() * workspace.element_size()), _ptr(result),
                          _stream(stream)))


def qzo_model_dense_count(shape: dict) -> int:
    cfg = make_config(shape)
    out = C.c_uint64(0)
    _check(lib().qzo_model_dense_count(C.byref(cfg), C.byref(out)))
    return out.value


def qzo_model_joint_table_bytes(shape: dict) -> int:
    cfg = make_config(shape)
    out = C.c_uint64(0)
    _check(lib().qzo_model_joint_table_bytes(C.byref(cfg), C.byref(out)))
    return out.value


def qzo_model_enable_joint(model, dense_master, table):
    """table: uint8 device tensor of qzo_model_joint_table_bytes bytes, kept alive by the caller."""
    assert dense_master.dtype == torch.float32
    _check(lib().qzo_model_enable_joint(model, _ptr(dense_master), C.c_uint64(dense_master.numel()),
                                        _ptr(table), C.c_uint64(table.numel() * table.element_size())))


def qzo_step_joint(model, tokens, seed, eps, eta, eta_dense, clip, workspace, result, stream=None):
    B, S = tokens.shape
    _check(lib().qzo_step_joint(model, _ptr(tokens), C.c_uint32(B), C.c_uint32(S), C.c_uint64(seed),
                                C.c_float(eps), C.c_float(eta), C.c_float(eta_dense), C.c_float(clip),
                                _ptr(workspace), C.c_uint64(workspace.numel() * workspace.element_size()),
                                _ptr(result), _stream(stream)))


def read_step_result(result) -> dict:
    """Host copy of a qzo_step_result (synchronises)."""
    raw = result.cpu()
    f = raw.view(torch.float32)
    i = raw.view(torch.int32)
    return dict(loss_plus=float(f[0]), loss_minus=float(f[1]), d=float(f[2]),
                d_clipped=float(f[3]), status=int(i[4]))


def qzo_model_apply_update(model, seed, eta, d_clipped, stream=None):
    _check(lib().qzo_model_apply_update(model, C.c_uint64(seed), C.c_float(eta),
                                        C.c_float(d_clipped), _stream(stream)))


def qzo_linear_scratch_bytes(M, N, K, with_sumsq) -> int:
    out = C.c_uint64(0)
    _check(lib().qzo_linear_scratch_bytes(C.c_uint32(M), C.c_uint32(N), C.c_uint32(K), C.c_int(int(with_sumsq)),
                                          C.byref(out)))
    return out.value


_scratch = {}


def scratch_for(device, nbytes):
    """Device-memory plumbing for the single-linear calls: one cached uint8 tensor per device, grown
    on demand (torch allocations are 256-byte aligned).  Calls that use it must not overlap."""
    t = _scratch.get(device)
    if t is None or t.numel() < nbytes:
        t = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        _scratch[device] = t
    return t


def _scratch_args(scratch):
    if scratch is None:
        return C.c_void_p(0), C.c_uint64(0)
    return _ptr(scratch), C.c_uint64(scratch.numel() * scratch.element_size())


def qzo_dequant_gemm(x, q, s, row_base, seed, eps, sign, y, sumsq=None, group=128, stream=None, scratch="auto"):
    M, K = x.shape
    N = q.shape[0]
    if isinstance(scratch, str):
        scratch = scratch_for(x.device, qzo_linear_scratch_bytes(M, N, K, sumsq is not None)) if K % 128 == 0 and K else None
    _check(lib().qzo_dequant_gemm(_ptr(x), _ptr(q), _ptr(s), C.c_uint32(row_base), C.c_uint32(M),
                                  C.c_uint32(N), C.c_uint32(K), C.c_uint32(group), C.c_uint64(seed),
                                  C.c_float(eps), C.c_int(sign), _ptr(y), _ptr(sumsq),
                                  *_scratch_args(scratch), _stream(stream)))


def qzo_dequant_gemm_static(x, q, s, row_base, seed, eps, sign, y, sumsq=None, group=128, stream=None):
    M, K = x.shape
    N = q.shape[0]
    _check(lib().qzo_dequant_gemm_static(_ptr(x), _ptr(q), _ptr(s), C.c_uint32(row_base), C.c_uint32(M),
                                         C.c_uint32(N), C.c_uint32(K), C.c_uint32(group), C.c_uint64(seed),
                                         C.c_float(eps), C.c_int(sign), _ptr(y), _ptr(sumsq), _stream(stream)))


def qzo_dequant_gemm_zp(x, q, s, zp, row_base, seed, eps, sign, y, sumsq=None, group=128, stream=None,
                        scratch="auto", scale_fp16=None):
    """s: bf16 or fp16 scales (scale_fp16 defaults to the tensor's dtype)."""
    if scale_fp16 is None:
        scale_fp16 = s.dtype == torch.float16
    M, K = x.shape
    N = q.shape[0]
    if isinstance(scratch, str):
        scratch = scratch_for(x.device, qzo_linear_scratch_bytes(M, N, K, sumsq is not None)) if K % 128 == 0 and K else None
    _check(lib().qzo_dequant_gemm_zp(_ptr(x), _ptr(q), _ptr(s), _ptr(zp), C.c_uint32(int(scale_fp16)),
                                     C.c_uint32(row_base), C.c_uint32(M), C.c_uint32(N), C.c_uint32(K), C.c_uint32(group),
                                     C.c_uint64(seed), C.c_float(eps), C.c_int(sign), _ptr(y),
                                     _ptr(sumsq), *_scratch_args(scratch), _stream(stream)))


def qzo_repack_kmajor(qweight, qzeros, scales, zero_add, q, zp, s, group=128, stream=None):
    K, N = qweight.shape[0] * 8, qweight.shape[1]
    _check(lib().qzo_repack_kmajor(_ptr(qweight), _ptr(qzeros), _ptr(scales), C.c_uint32(N),
                                   C.c_uint32(K), C.c_uint32(group), C.c_uint32(zero_add),
                                   C.c_uint32(int(s.dtype == torch.float16)), _ptr(q),
                                   _ptr(zp), _ptr(s), _stream(stream)))


def qzo_apply_update(s, row_base, seed, eta, d_clipped, stream=None):
    n_rows, G = s.shape
    _check(lib().qzo_apply_update(_ptr(s), C.c_uint32(n_rows), C.c_uint32(G), C.c_uint32(row_base),
                                  C.c_uint64(seed), C.c_float(eta), C.c_float(d_clipped),
                                  C.c_uint32(int(s.dtype == torch.float16)), _stream(stream)))


def qzo_rtn_quantize(w, q, s, group=128, stream=None):
    N, K = w.shape
    _check(lib().qzo_rtn_quantize(_ptr(w), C.c_uint32(N), C.c_uint32(K), C.c_uint32(group), _ptr(q),
                                  _ptr(s), _stream(stream)))


def qzo_rtn_quantize_asym(w, q, zp, s, group=128, stream=None):
    """s: bf16 or fp16 output tensor; its dtype selects the scale's storage type."""
    N, K = w.shape
    _check(lib().qzo_rtn_quantize_asym(_ptr(w), C.c_uint32(N), C.c_uint32(K), C.c_uint32(group),
                                       C.c_uint32(int(s.dtype == torch.float16)), _ptr(q), _ptr(zp), _ptr(s),
                                       _stream(stream)))


def qzo_debug_normals(seed, stream_id, row0, out, stream=None):
    n_rows, G = out.shape
    _check(lib().qzo_debug_normals(C.c_uint64(seed), C.c_uint32(stream_id), C.c_uint32(row0),
                                   C.c_uint32(n_rows), C.c_uint32(G), _ptr(out), _stream(stream)))


def qzo_debug_philox(seed, ctr, out, stream=None):
    _check(lib().qzo_debug_philox(C.c_uint64(seed), _ptr(ctr), C.c_uint32(ctr.shape[0]), _ptr(out),
                                  _stream(stream)))


def qzo_debug_normal_pairs(words, out, stream=None):
    _check(lib().qzo_debug_normal_pairs(_ptr(words), C.c_uint32(words.numel()), _ptr(out),
                                        _stream(stream)))


def qzo_debug_dequant(q, s, row_base, seed, eps, sign, w_eff, group=128, stream=None):
    N, K = w_eff.shape
    _check(lib().qzo_debug_dequant(_ptr(q), _ptr(s), C.c_uint32(row_base), C.c_uint32(N),
                                   C.c_uint32(K), C.c_uint32(group), C.c_uint64(seed),
                                   C.c_float(eps), C.c_int(sign), _ptr(w_eff), _stream(stream)))


def qzo_int4_expand(q, s, zp, row_base, seed, eps, sign, se_out, w_out, g_idx=None, stream=None):
    N, K = q.shape[0], q.shape[1] * 2
    _check(lib().qzo_int4_expand(_ptr(q), _ptr(s), _ptr(zp), _ptr(g_idx), C.c_uint32(row_base), C.c_uint32(N),
                                 C.c_uint32(K), C.c_uint32(128), C.c_uint64(seed), C.c_float(eps), C.c_int(sign),
                                 _ptr(se_out), _ptr(w_out), _stream(stream)))


def qzo_int4_scratch_bytes(N, K) -> int:
    out = C.c_uint64(0)
    _check(lib().qzo_int4_scratch_bytes(C.c_uint32(N), C.c_uint32(K), C.byref(out)))
    return out.value


def qzo_int4_gemm_expanded(x, q, s, zp, g_idx, row_base, seed, eps, sign, y, scratch, stream=None):
    M, K = x.shape
    N = q.shape[0]
    _check(lib().qzo_int4_gemm_expanded(_ptr(x), _ptr(q), _ptr(s), _ptr(zp), _ptr(g_idx), C.c_uint32(row_base),
                                        C.c_uint32(M), C.c_uint32(N), C.c_uint32(K), C.c_uint32(128),
                                        C.c_uint64(seed), C.c_float(eps), C.c_int(sign), _ptr(y), _ptr(scratch),
                                        C.c_uint64(scratch.numel() * scratch.element_size()), _stream(stream)))


def qzo_nf4_expand(q, s, row_base, seed, eps, sign, se_out, w_out, stream=None):
    N, K = q.shape[0], q.shape[1] * 2
    _check(lib().qzo_nf4_expand(_ptr(q), _ptr(s), C.c_uint32(row_base), C.c_uint32(N), C.c_uint32(K),
                                C.c_uint32(64), C.c_uint64(seed), C.c_float(eps), C.c_int(sign),
                                _ptr(se_out), _ptr(w_out), _stream(stream)))


def qzo_nf4_scratch_bytes(N, K) -> int:
    out = C.c_uint64(0)
    _check(lib().qzo_nf4_scratch_bytes(C.c_uint32(N), C.c_uint32(K), C.byref(out)))
    return out.value


def qzo_nf4_gemm(x, q, s, row_base, seed, eps, sign, y, scratch, stream=None):
    M, K = x.shape
    N = q.shape[0]
    _check(lib().qzo_nf4_gemm(_ptr(x), _ptr(q), _ptr(s), C.c_uint32(row_base), C.c_uint32(M), C.c_uint32(N),
                              C.c_uint32(K), C.c_uint32(64), C.c_uint64(seed), C.c_float(eps), C.c_int(sign),
                              _ptr(y), _ptr(scratch), C.c_uint64(scratch.numel() * scratch.element_size()),
                              _stream(stream)))


def qzo_model_set_int4_path(model, mode: int):
    _check(lib().qzo_model_set_int4_path(model, C.c_int(mode)))


def qzo_debug_bf16_gemm(x, w, y, pipe=2, stream=None):
    M, K = x.shape
    N = w.shape[0]
    _check(lib().qzo_debug_bf16_gemm(_ptr(x), _ptr(w), C.c_uint32(M), C.c_uint32(N), C.c_uint32(K),
                                     C.c_int(pipe), _ptr(y), _stream(stream)))


def qzo_debug_dequant_zp(q, s, zp, row_base, seed, eps, sign, w_eff, group=128, stream=None):
    N, K = w_eff.shape
    _check(lib().qzo_debug_dequant_zp(_ptr(q), _ptr(s), _ptr(zp), C.c_uint32(int(s.dtype == torch.float16)),
                                      C.c_uint32(row_base), C.c_uint32(N),
                                      C.c_uint32(K), C.c_uint32(group), C.c_uint64(seed),
                                      C.c_float(eps), C.c_int(sign), _ptr(w_eff), _stream(stream)))


def qzo_debug_forward(model, tokens, seed, eps, sign, workspace, loss_out, hidden_out, stream=None):
    B, S = tokens.shape
    _check(lib().qzo_debug_forward(model, _ptr(tokens), C.c_uint32(B), C.c_uint32(S),
                                   C.c_uint64(seed), C.c_float(eps), C.c_int(sign), _ptr(workspace),
                                   C.c_uint64(workspace.numel() * workspace.element_size()),
                                   _ptr(loss_out), _ptr(hidden_out), _stream(stream)))


PROFILE_KINDS = {"w4a16_gemm": 0, "lmhead_ce": 1, "attention": 2, "scale_update": 3, "embed": 4, "expand": 5}


def qzo_profile_stride(stride: int):
    _check(lib().qzo_profile_stride(C.c_uint32(stride)))


def qzo_debug_mfma_rate(iters: int, random_operands: bool, sink, stream=None) -> int:
    """Launches the matrix-pipe rate probe; returns the number of workgroups (8 wavefronts each)."""
    wgs = C.c_uint32(0)
    assert sink.numel() >= 512 * 512
    _check(lib().qzo_debug_mfma_rate(C.c_uint32(iters), C.c_int(int(random_operands)), _ptr(sink),
                                     C.byref(wgs), _stream(stream)))
    return wgs.value


def qzo_profile_begin(max_records: int):
    _check(lib().qzo_profile_begin(C.c_uint32(max_records)))


def qzo_profile_collect(kind: int) -> dict:
    ms, n, work = C.c_double(0), C.c_uint64(0), C.c_double(0)
    _check(lib().qzo_profile_collect(C.c_uint32(kind), C.byref(ms), C.byref(n), C.byref(work)))
    return dict(total_ms=ms.value, launches=n.value, work=work.value)


def qzo_codebook_scratch_bytes(M, N, with_sumsq) -> int:
    out = C.c_uint64(0)
    _check(lib().qzo_codebook_scratch_bytes(C.c_uint32(M), C.c_uint32(N), C.c_int(int(with_sumsq)), C.byref(out)))
    return out.value


def qzo_codebook_gemm(x, codes, codebook, c, row_base, seed, eps, sign, y, sumsq=None, stream=None,
                      scratch="auto"):
    M, K = x.shape
    N = codes.shape[0]
    if isinstance(scratch, str):
        scratch = scratch_for(x.device, qzo_codebook_scratch_bytes(M, N, sumsq is not None))
    _check(lib().qzo_codebook_gemm(_ptr(x), _ptr(codes), _ptr(codebook), _ptr(c), C.c_uint32(row_base),
                                   C.c_uint32(M), C.c_uint32(N), C.c_uint32(K), C.c_uint64(seed),
                                   C.c_float(eps), C.c_int(sign), _ptr(y), _ptr(sumsq),
                                   *_scratch_args(scratch), _stream(stream)))


def qzo_apply_update_channel(c, row_base, seed, eta, d_clipped, stream=None):
    _check(lib().qzo_apply_update_channel(_ptr(c), C.c_uint32(c.numel()), C.c_uint32(row_base),
                                          C.c_uint64(seed), C.c_float(eta), C.c_float(d_clipped),
                                          _stream(stream)))
