"""ctypes face of the CPU oracle (oracle/qzo_oracle.cpp) -- TEST INFRASTRUCTURE ONLY.

Imported by tests/, the smoke check and the benchmark's cpu_baseline leg; never
by the product.  It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        _lib = C.CDLL(path)
        _lib.orc_bf16_rne.restype = C.c_float
        _lib.orc_bf16_rne.argtypes = [C.c_float]
        _lib.orc_sumsq_bf16.restype = C.c_double
        _lib.orc_next_token_ce.restype = C.c_double
        _lib.orc_forward_loss.restype = C.c_double
        _lib.orc_spsa_d.restype = C.c_float
        _lib.orc_spsa_d.argtypes = [C.c_float, C.c_float, C.c_float]
        _lib.orc_clip.restype = C.c_float
        _lib.orc_clip.argtypes = [C.c_float, C.c_float]
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


# ----------------------------------------------------------------- RNG -----
def philox4x32_10(ctr, key):
    ctr = np.asarray(ctr, dtype=np.uint32)
    key = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(ctr), _p(key), _p(out))
    return out


def normal_pairs(words):
    w = np.ascontiguousarray(words, dtype=np.uint32)
    out = np.zeros((w.size, 2), dtype=np.float32)
    lib().orc_normal_pairs(_p(w), C.c_uint64(w.size), _p(out))
    return out


def scale_normals(seed, row0, n_rows, G, stream=0):
    out = np.zeros((n_rows, G), dtype=np.float32)
    lib().orc_scale_normals(C.c_uint64(seed), C.c_uint32(stream), C.c_uint32(row0),
                            C.c_uint32(n_rows), C.c_uint32(G), _p(out))
    return out


def flat_normals(seed, first, n, stream=1):
    out = np.zeros(n, dtype=np.float32)
    lib().orc_flat_normals(C.c_uint64(seed), C.c_uint32(stream), C.c_uint64(first),
                           C.c_uint64(n), _p(out))
    return out


def bf16_rne(x):
    a = _f32(x).copy()
    lib().orc_bf16_rne_array(_p(a), C.c_uint64(a.size))
    return a


# --------------------------------------------------------- quantization ----
def rtn_quantize(w, group=128):
    w = _f32(w)
    N, K = w.shape
    qp = np.zeros((N, K // 2), dtype=np.uint8)
    s = np.zeros((N, K // group), dtype=np.float32)
    lib().orc_rtn_quantize(_p(w), C.c_uint64(N), C.c_uint64(K), C.c_uint32(group), _p(qp), _p(s))
    return qp, s


def unpack_int4(qp, K):
    qp = np.ascontiguousarray(qp, dtype=np.uint8)
    N = qp.shape[0]
    q = np.zeros((N, K), dtype=np.int8)
    lib().orc_unpack_int4(_p(qp), C.c_uint64(N), C.c_uint64(K), _p(q))
    return q


def effective_scales(s, row_base, seed, eps_signed):
    s = _f32(s)
    n_rows, G = s.shape
    out = np.zeros((n_rows, G), dtype=np.float64)
    lib().orc_effective_scales(_p(s), C.c_uint32(n_rows), C.c_uint32(G), C.c_uint32(row_base),
                               C.c_uint64(seed), C.c_float(eps_signed), _p(out))
    return out


def dequant(qp, s, seed, row_base, eps_signed, group=128, to_bf16=False):
    qp = np.ascontiguousarray(qp, dtype=np.uint8)
    s = _f32(s)
    N, K = qp.shape[0], qp.shape[1] * 2
    out = np.zeros((N, K), dtype=np.float32)
    lib().orc_dequant(_p(qp), _p(s), C.c_uint64(N), C.c_uint64(K), C.c_uint32(group),
                      C.c_uint64(seed), C.c_uint32(row_base), C.c_float(eps_signed),
                      C.c_int(1 if to_bf16 else 0), _p(out))
    return out


def dequant_zp(qp, s, zp, seed, row_base, eps_signed, group=128, to_bf16=False, g_idx=None):
    """Asymmetric groups: W_eff[n,k] = (s + eps z) * (u[n,k] - zp[n,g(k)]), g(k) = k/group or g_idx[k]."""
    gi = None if g_idx is None else np.ascontiguousarray(g_idx, dtype=np.int32)
    qp = np.ascontiguousarray(qp, dtype=np.uint8)
    s = _f32(s)
    zp = np.ascontiguousarray(zp, dtype=np.uint8)
    N, K = qp.shape[0], qp.shape[1] * 2
    out = np.zeros((N, K), dtype=np.float32)
    lib().orc_dequant_zp(_p(qp), _p(s), _p(zp), C.c_uint64(N), C.c_uint64(K), C.c_uint32(group),
                         C.c_uint64(seed), C.c_uint32(row_base), C.c_float(eps_signed),
                         C.c_int(1 if to_bf16 else 0), _p(gi) if gi is not None else None, _p(out))
    return out


def qlinear_zp(x, qp, s_eff, zp, group=128, g_idx=None):
    gi = None if g_idx is None else np.ascontiguousarray(g_idx, dtype=np.int32)
    x = _f64(x)
    qp = np.ascontiguousarray(qp, dtype=np.uint8)
    s_eff = _f64(s_eff)
    zp = np.ascontiguousarray(zp, dtype=np.uint8)
    M, K = x.shape
    N = qp.shape[0]
    y = np.zeros((M, N), dtype=np.float64)
    lib().orc_qlinear_zp(_p(x), C.c_uint64(M), C.c_uint64(K), _p(qp), _p(s_eff), _p(zp), C.c_uint64(N),
                         C.c_uint32(group), None, _p(gi) if gi is not None else None, _p(y))
    return y


def rtn_quantize_asym(w, group=128, scale_fmt=0, g_idx=None):
    """Asymmetric RTN groups: (nibbles [N,K/2], zero-points [N,G], scales [N,G] rounded to bf16
    (scale_fmt 0) or fp16 (1)).  g_idx: int32 [K], the group of every input column (None: k // group)."""
    w = _f32(w)
    N, K = w.shape
    gi = None if g_idx is None else np.ascontiguousarray(g_idx, dtype=np.int32)
    qp = np.zeros((N, K // 2), dtype=np.uint8)
    zp = np.zeros((N, K // group), dtype=np.uint8)
    s = np.zeros((N, K // group), dtype=np.float32)
    lib().orc_rtn_quantize_asym(_p(w), C.c_uint64(N), C.c_uint64(K), C.c_uint32(group), C.c_int(scale_fmt),
                                _p(gi) if gi is not None else None, _p(qp), _p(zp), _p(s))
    return qp, zp, s


def nf4_levels():
    out = np.zeros(16, dtype=np.float32)
    lib().orc_nf4_levels(_p(out))
    return out


def nf4_quantize(w, block=64):
    """NormalFloat-4 blocks: (indices [N,K/2], bf16 absmax scales [N,K/block])."""
    w = _f32(w)
    N, K = w.shape
    qp = np.zeros((N, K // 2), dtype=np.uint8)
    s = np.zeros((N, K // block), dtype=np.float32)
    lib().orc_nf4_quantize(_p(w), C.c_uint64(N), C.c_uint64(K), C.c_uint32(block), _p(qp), _p(s))
    return qp, s


def dequant_nf4(qp, s, seed, row_base, eps_signed, block=64, to_bf16=False):
    qp = np.ascontiguousarray(qp, dtype=np.uint8)
    s = _f32(s)
    N, K = qp.shape[0], qp.shape[1] * 2
    out = np.zeros((N, K), dtype=np.float32)
    lib().orc_dequant_nf4(_p(qp), _p(s), C.c_uint64(N), C.c_uint64(K), C.c_uint32(block), C.c_uint64(seed),
                          C.c_uint32(row_base), C.c_float(eps_signed), C.c_int(1 if to_bf16 else 0), _p(out))
    return out


def qlinear_nf4(x, qp, s_eff, block=64, bias=None):
    x = _f64(x)
    qp = np.ascontiguousarray(qp, dtype=np.uint8)
    s_eff = _f64(s_eff)
    M, K = x.shape
    N = qp.shape[0]
    y = np.zeros((M, N), dtype=np.float64)
    b = _f32(bias) if bias is not None else None
    lib().orc_qlinear_nf4(_p(x), C.c_uint64(M), C.c_uint64(K), _p(qp), _p(s_eff), C.c_uint64(N),
                          C.c_uint32(block), _p(b) if b is not None else None, _p(y))
    return y


def repack_kmajor(qweight, qzeros, scales_f16, zero_add, group=128):
    """K-major checkpoint layout -> (nibbles [N,K/2], zero-points [N,G], bf16 scales [N,G])."""
    qweight = np.ascontiguousarray(qweight, dtype=np.uint32)
    qzeros = np.ascontiguousarray(qzeros, dtype=np.uint32)
    sc = _f32(scales_f16)
    K, N = qweight.shape[0] * 8, qweight.shape[1]
    G = K // group
    qp = np.zeros((N, K // 2), dtype=np.uint8)
    zp = np.zeros((N, G), dtype=np.uint8)
    s = np.zeros((N, G), dtype=np.float32)
    lib().orc_repack_kmajor(_p(qweight), _p(qzeros), _p(sc), C.c_uint64(N), C.c_uint64(K), C.c_uint32(group),
                            C.c_uint32(zero_add), _p(qp), _p(zp), _p(s))
    return qp, zp, s


def qlinear(x, qp, s_eff, group=128, bias=None):
    x = _f64(x)
    qp = np.ascontiguousarray(qp, dtype=np.uint8)
    s_eff = _f64(s_eff)
    M, K = x.shape
    N = qp.shape[0]
    y = np.zeros((M, N), dtype=np.float64)
    b = _f32(bias) if bias is not None else None
    lib().orc_qlinear(_p(x), C.c_uint64(M), C.c_uint64(K), _p(qp), _p(s_eff), C.c_uint64(N),
                      C.c_uint32(group), _p(b) if b is not None else None, _p(y))
    return y


def linear(x, w, bias=None):
    x = _f64(x)
    w = _f32(w)
    M, K = x.shape
    N = w.shape[0]
    y = np.zeros((M, N), dtype=np.float64)
    b = _f32(bias) if bias is not None else None
    lib().orc_linear(_p(x), C.c_uint64(M), C.c_uint64(K), _p(w), C.c_uint64(N),
                     _p(b) if b is not None else None, _p(y))
    return y


def sumsq_bf16(y):
    y = _f64(y)
    return float(lib().orc_sumsq_bf16(_p(y), C.c_uint64(y.size)))


# --------------------------------------------------------------- blocks ----
def rmsnorm(x, gain, eps=1e-5):
    x = _f64(x)
    g = _f32(gain)
    y = np.zeros_like(x)
    lib().orc_rmsnorm(_p(x), C.c_uint64(x.shape[0]), C.c_uint64(x.shape[1]), _p(g),
                      C.c_double(eps), _p(y))
    return y


def layernorm(x, gain, bias, eps=1e-5):
    x = _f64(x)
    g, b = _f32(gain), _f32(bias)
    y = np.zeros_like(x)
    lib().orc_layernorm(_p(x), C.c_uint64(x.shape[0]), C.c_uint64(x.shape[1]), _p(g), _p(b),
                        C.c_double(eps), _p(y))
    return y


def rope(x, B, S, col0, n_heads, dh, theta=10000.0):
    x = _f64(x).copy()
    lib().orc_rope(_p(x), C.c_uint64(B), C.c_uint64(S), C.c_uint64(x.shape[1]), C.c_uint64(col0),
                   C.c_uint64(n_heads), C.c_uint64(dh), C.c_double(theta))
    return x


def attention(qkv, B, S, n_heads, dh):
    qkv = _f64(qkv)
    out = np.zeros((B * S, n_heads * dh), dtype=np.float64)
    lib().orc_attention(_p(qkv), C.c_uint64(B), C.c_uint64(S), C.c_uint64(n_heads),
                        C.c_uint64(dh), _p(out))
    return out


def swiglu(gu, F):
    gu = _f64(gu)
    out = np.zeros((gu.shape[0], F), dtype=np.float64)
    lib().orc_swiglu(_p(gu), C.c_uint64(gu.shape[0]), C.c_uint64(F), _p(out))
    return out


def next_token_ce(logits, tok):
    logits = _f64(logits)
    tok = np.ascontiguousarray(tok, dtype=np.int32)
    B, S = tok.shape
    return float(lib().orc_next_token_ce(_p(logits), _p(tok), C.c_uint64(B), C.c_uint64(S),
                                         C.c_uint64(logits.shape[-1])))


# ---------------------------------------------------------------- model ----
class _Cfg(C.Structure):
    _fields_ = [("arch", C.c_uint32), ("n_layers", C.c_uint32), ("d_model", C.c_uint32),
                ("n_heads", C.c_uint32), ("d_ffn", C.c_uint32), ("vocab", C.c_uint32),
                ("max_seq", C.c_uint32), ("group", C.c_uint32),
                ("norm_eps", C.c_double), ("rope_theta", C.c_double), ("quant", C.c_uint32),
                ("act_order", C.c_uint32)]


@dataclass
class Segment:
    """One quantized linear's slice of the scale arena."""
    name: str
    offset: int      # first scale in the arena
    rows: int        # N
    G: int           # K / group
    row_base: int    # model-wide index of its first output row


@dataclass
class Model:
    shape: dict
    tensors: list            # numpy arrays in forward order (fp32 bf16-valued, or uint8 packed)
    names: list
    scales: np.ndarray       # flat fp32 arena of bf16-valued scales
    segments: list = field(default_factory=list)
    group: int = 128
    quant: int = 0           # 0: int4 + group scales; 1: codebook + per-channel scales; 2: int4 + zero-points;
                             # 3: NormalFloat-4 blocks of 64
    scale_fmt: int = 0       # storage type of the group scales: 0 bf16, 1 fp16 (quant = 2 checkpoints)
    act_order: bool = False  # quant = 2: every zero-point tensor is followed by g_idx int32 [K]

    @property
    def n_rows(self):
        return sum(s.rows for s in self.segments)


def build_model(shape: dict, table, group=128, asym=False, nf4=False, fp16_scales=False, g_idx=None) -> Model:
    """Quantize the 'w' entries of a (name, kind, array) table with RTN
    (Eq. 3 with the absmax scale; asym: with zero-points, each packed weight then followed by
    its zero-point tensor; nf4: NormalFloat-4 blocks of 64) and lay the scales out in arena order.
    fp16_scales (asym only): the scales are stored in fp16, as in the 4-bit checkpoints of Sec. 4.1.
    g_idx (asym only): a function K -> int32 [K] giving the group of every input column of a linear with
    K inputs (activation reordering); each zero-point tensor is then followed by that array."""
    if nf4:
        group = 64
    assert asym or (not fp16_scales and g_idx is None)
    tensors, names, segs, scales = [], [], [], []
    off = 0
    row = 0
    for name, kind, arr in table:
        if kind == "w":
            if asym:
                gi = None if g_idx is None else np.ascontiguousarray(g_idx(arr.shape[1]), dtype=np.int32)
                qp, zp, s = rtn_quantize_asym(arr, group, 1 if fp16_scales else 0, gi)
                tensors += [qp, zp]
                names += [name, name + ".zp"]
                if gi is not None:
                    tensors.append(gi)
                    names.append(name + ".g_idx")
            elif nf4:
                qp, s = nf4_quantize(arr, group)
                tensors.append(qp)
                names.append(name)
            else:
                qp, s = rtn_quantize(arr, group)
                tensors.append(qp)
                names.append(name)
            segs.append(Segment(name, off, s.shape[0], s.shape[1], row))
            scales.append(s.reshape(-1))
            off += s.size
            row += s.shape[0]
        else:
            tensors.append(_f32(arr))
            names.append(name)
    return Model(shape, tensors, names, np.concatenate(scales).astype(np.float32), segs, group,
                 3 if nf4 else (2 if asym else 0), 1 if fp16_scales else 0, g_idx is not None)


def fp16_rne(x):
    a = _f32(x).copy()
    lib().orc_fp16_rne_array(_p(a), C.c_uint64(a.size))
    return a


def codebook_linear(x, idx, cb, c_eff, bias=None):
    x = _f64(x)
    idx = np.ascontiguousarray(idx, dtype=np.uint16)
    cb = _f32(cb)
    c_eff = _f64(c_eff)
    M, K = x.shape
    N = idx.shape[0]
    y = np.zeros((M, N), dtype=np.float64)
    b = _f32(bias) if bias is not None else None
    lib().orc_codebook_linear(_p(x), C.c_uint64(M), C.c_uint64(K), _p(idx), _p(cb), _p(c_eff),
                              C.c_uint64(N), _p(b) if b is not None else None, _p(y))
    return y


def channel_effective_scales(c, row_base, seed, eps_signed):
    c = _f32(c).reshape(-1)
    out = np.zeros(c.size, dtype=np.float64)
    lib().orc_channel_effective_scales(_p(c), C.c_uint32(c.size), C.c_uint32(row_base),
                                       C.c_uint64(seed), C.c_float(eps_signed), _p(out))
    return out


def update_channel_scales(c, row_base, seed, eta, d_clipped):
    c = _f32(c).reshape(-1).copy()
    lib().orc_update_channel_scales(_p(c), C.c_uint32(c.size), C.c_uint32(row_base), C.c_uint64(seed),
                                    C.c_float(eta), C.c_float(d_clipped))
    return c


def build_codebook_model(shape: dict, table) -> Model:
    """table entries: (name, 'bf16', array) | (name, 'codes', u16 [N,K/8]) |
    (name, 'codebook', fp32 [65536,8] holding fp16 values) | (name, 'chscale', fp32 [N])."""
    tensors, names, segs, scales = [], [], [], []
    off = 0
    for name, kind, arr in table:
        if kind == "chscale":
            n = arr.size
            segs.append(Segment(name, off, n, 1, off))
            scales.append(_f32(arr).reshape(-1))
            off += n
            continue
        tensors.append(np.ascontiguousarray(arr, dtype=np.uint16) if kind == "codes" else _f32(arr))
        names.append(name)
    return Model(shape, tensors, names, np.concatenate(scales).astype(np.float32), segs, 128, 1)


def perturbed_scales(model: Model, seed: int, eps_signed: float, scales=None) -> np.ndarray:
    """Delta + (sigma*eps) z over the whole arena (PERTURB_SCALES, functional form)."""
    sc = model.scales if scales is None else scales
    if model.quant == 1:
        return channel_effective_scales(sc, 0, seed, eps_signed)
    out = np.zeros(sc.size, dtype=np.float64)
    for sg in model.segments:
        sl = slice(sg.offset, sg.offset + sg.rows * sg.G)
        out[sl] = effective_scales(sc[sl].reshape(sg.rows, sg.G), sg.row_base, seed,
                                   eps_signed).reshape(-1)
    return out


def forward_loss(model: Model, s_eff, tok, act_bf16=True, want_hidden=False, want_logits=False):
    sh = model.shape
    cfg = _Cfg(0 if sh["arch"] == "llama" else 1, sh["n_layers"], sh["d_model"], sh["n_heads"],
               sh["d_ffn"], sh["vocab"], sh["max_seq"], model.group,
               sh.get("norm_eps", 1e-5), sh.get("rope_theta", 10000.0), model.quant,
               1 if model.act_order else 0)
    tok = np.ascontiguousarray(tok, dtype=np.int32)
    B, S = tok.shape
    s_eff = _f64(s_eff)
    ptrs = (C.c_void_p * len(model.tensors))(*[t.ctypes.data for t in model.tensors])
    hid = np.zeros((B * S, sh["d_model"]), dtype=np.float64) if want_hidden else None
    lg = np.zeros((B * S, sh["vocab"]), dtype=np.float64) if want_logits else None
    loss = lib().orc_forward_loss(C.byref(cfg), ptrs, _p(s_eff), _p(tok), C.c_uint32(B),
                                  C.c_uint32(S), C.c_int(1 if act_bf16 else 0),
                                  _p(hid) if hid is not None else None,
                                  _p(lg) if lg is not None else None)
    extra = tuple(x for x in (hid, lg) if x is not None)
    return (float(loss),) + extra if extra else float(loss)


# ---- joint SPSA on the un-quantized parameters (Sec. 3.2, Sec. 4.1 2-bit runs) ----
def dense_slots(model: Model):
    """(tensor index, first flat index, size, format) of every 16-bit tensor of the table, in table
    order: together they are the un-quantized parameters theta_u.  Codebooks hold fp16 values."""
    out, first = [], 0
    for i, (name, t) in enumerate(zip(model.names, model.tensors)):
        if t.dtype != np.float32:
            continue
        fmt = 1 if name.endswith(".cb") else 0
        out.append((i, first, t.size, fmt))
        first += t.size
    return out


def dense_master(model: Model) -> np.ndarray:
    """fp32 master vector initialised from the 16-bit tensors."""
    return np.concatenate([model.tensors[i].reshape(-1) for i, _, _, _ in dense_slots(model)]).astype(np.float32)


def dense_effective(master, first, seed, eps_signed, fmt=0):
    master = _f32(master).reshape(-1)
    out = np.zeros(master.size, dtype=np.float32)
    lib().orc_dense_effective(_p(master), C.c_uint64(first), C.c_uint64(master.size), C.c_uint64(seed),
                              C.c_float(eps_signed), C.c_int(fmt), _p(out))
    return out


def dense_update(master, first, seed, eta, d_clipped):
    master = _f32(master).reshape(-1).copy()
    lib().orc_dense_update(_p(master), C.c_uint64(first), C.c_uint64(master.size), C.c_uint64(seed),
                           C.c_float(eta), C.c_float(d_clipped))
    return master


def with_dense(model: Model, master, seed, eps_signed) -> Model:
    """The model a perturbed pass sees: every 16-bit tensor replaced by round16(theta_u + eps z)."""
    tensors = list(model.tensors)
    for i, first, n, fmt in dense_slots(model):
        tensors[i] = dense_effective(master[first:first + n], first, seed, eps_signed, fmt).reshape(
            model.tensors[i].shape)
    return Model(model.shape, tensors, model.names, model.scales, model.segments, model.group, model.quant)


def qzo_step_joint(model: Model, master, tok, seed, eps, eta, eta_dense, Cthr, act_bf16=True):
    """One iteration of Algorithm 1 with the scales (Q-SPSA) and the un-quantized parameters (SPSA)
    perturbed together: one direction z over both, one scalar d', two updates."""
    lp = forward_loss(with_dense(model, master, seed, +eps), perturbed_scales(model, seed, +eps), tok, act_bf16)
    lm = forward_loss(with_dense(model, master, seed, -eps), perturbed_scales(model, seed, -eps), tok, act_bf16)
    d = spsa_d(np.float32(lp), np.float32(lm), np.float32(eps))
    if not np.isfinite(d):
        return dict(loss_plus=lp, loss_minus=lm, d=d, d_clipped=0.0, status=1,
                    scales=model.scales.copy(), master=_f32(master).copy())
    dc = clip(d, Cthr)
    return dict(loss_plus=lp, loss_minus=lm, d=d, d_clipped=dc, status=0,
                scales=update_scales(model, seed, eta, dc),
                master=dense_update(master, 0, seed, eta_dense, dc))


def spsa_d(loss_plus, loss_minus, eps):
    return float(lib().orc_spsa_d(loss_plus, loss_minus, eps))


def clip(d, Cthr):
    return float(lib().orc_clip(d, Cthr))


def update_scales(model: Model, seed: int, eta: float, d_clipped: float, scales=None) -> np.ndarray:
    """Returns the updated arena (Algorithm 1's update loop); input untouched."""
    if model.quant == 1:
        return update_channel_scales(model.scales if scales is None else scales, 0, seed, eta, d_clipped)
    sc = (model.scales if scales is None else scales).astype(np.float32).copy()
    for sg in model.segments:
        view = sc[sg.offset:sg.offset + sg.rows * sg.G]
        lib().orc_update_scales(_p(view), C.c_uint32(sg.rows), C.c_uint32(sg.G),
                                C.c_uint32(sg.row_base), C.c_uint64(seed), C.c_float(eta),
                                C.c_float(d_clipped), C.c_int(model.scale_fmt))
    return sc


def qzo_step(model: Model, tok, seed, eps, eta, Cthr, act_bf16=True):
    """One iteration of Algorithm 1.  Returns dict(loss_plus, loss_minus, d,
    d_clipped, status, scales) and leaves `model` untouched.  A non-finite d
    skips the update (status 1): the paper's clip is undefined there."""
    lp = forward_loss(model, perturbed_scales(model, seed, +eps), tok, act_bf16)
    lm = forward_loss(model, perturbed_scales(model, seed, -eps), tok, act_bf16)
    d = spsa_d(np.float32(lp), np.float32(lm), np.float32(eps))
    if not np.isfinite(d):
        return dict(loss_plus=lp, loss_minus=lm, d=d, d_clipped=0.0, status=1,
                    scales=model.scales.copy())
    dc = clip(d, Cthr)
    return dict(loss_plus=lp, loss_minus=lm, d=d, d_clipped=dc, status=0,
                scales=update_scales(model, seed, eta, dc))
