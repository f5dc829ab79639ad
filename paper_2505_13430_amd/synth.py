"""Seeded synthetic inputs shared by the HIP path's tests, the benchmark and the CPU oracle.

Only shapes and random draws live here: no quantization, no RNG of the method,
no forward arithmetic.  Values that are stored as bf16 downstream are produced
already exactly representable in bf16 (low 16 bits of the fp32 pattern cleared),
so every consumer sees the same numbers whatever its own rounding routine is.

The shapes stand in for the checkpoints the paper fine-tunes (OPT and Llama
families, Sec. 4.1) and the token batches stand in for its prompt batches; the
paper's datasets and weights are not used.
"""
from __future__ import annotations

import numpy as np

GROUP = 128

# name -> architecture; the five workloads of this build.
SHAPES = {
    "tiny": dict(arch="llama", n_layers=2, d_model=256, n_heads=4, d_ffn=1024, vocab=1024,
                 max_seq=64, batch=4, seq=64),
    "tiny_opt": dict(arch="opt", n_layers=2, d_model=256, n_heads=4, d_ffn=1024, vocab=1024,
                     max_seq=64, batch=4, seq=64),
    "opt-1.3b": dict(arch="opt", n_layers=24, d_model=2048, n_heads=32, d_ffn=8192, vocab=50272,
                     max_seq=256, batch=16, seq=256),
    "llama-2-7b": dict(arch="llama", n_layers=32, d_model=4096, n_heads=32, d_ffn=11008,
                       vocab=32000, max_seq=512, batch=16, seq=512),
    "llama-2-13b": dict(arch="llama", n_layers=40, d_model=5120, n_heads=40, d_ffn=13824,
                        vocab=32000, max_seq=512, batch=8, seq=512),
}
LINEAR_SHAPE = dict(M=2048, N=11008, K=4096)   # single linear at a Llama-7B MLP shape


def bf16_exact(x: np.ndarray) -> np.ndarray:
    """Clear the low 16 bits so the fp32 value is exactly a bf16 value."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


def quantized_linears(shape: dict):
    """[(name, N, K)] of one decoder block, in scale-arena order."""
    d, F = shape["d_model"], shape["d_ffn"]
    if shape["arch"] == "llama":
        return [("wqkv", 3 * d, d), ("wo", d, d), ("wgu", 2 * F, d), ("wdown", d, F)]
    return [("wqkv", 3 * d, d), ("wo", d, d), ("wfc1", F, d), ("wfc2", d, F)]


def n_scales(shape: dict, group: int = GROUP) -> int:
    return shape["n_layers"] * sum(N * (K // group) for _, N, K in quantized_linears(shape))


def tensor_table(shape: dict, seed: int):
    """Ordered list of (name, kind, fp32 array).  kind: 'bf16' = used as is
    (bf16-exact values), 'w' = float weight [N,K] ~ N(0, 0.02) to be quantized."""
    rng = np.random.default_rng(seed)
    d, V = shape["d_model"], shape["vocab"]
    llama = shape["arch"] == "llama"

    def normal(*sz):
        return bf16_exact(rng.standard_normal(sz, dtype=np.float32) * np.float32(0.02))

    def weight(N, K):
        return rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)

    def gain(n):   # norm gains near 1 so a dropped gain shows up
        return bf16_exact(1.0 + 0.1 * rng.standard_normal(n, dtype=np.float32))

    out = [("tok_emb", "bf16", normal(V, d))]
    if not llama:
        out.append(("pos_emb", "bf16", normal(shape["max_seq"], d)))
    for l in range(shape["n_layers"]):
        lin = quantized_linears(shape)
        if llama:
            out.append((f"l{l}.attn_norm", "bf16", gain(d)))
            out.append((f"l{l}.wqkv", "w", weight(*lin[0][1:])))
            out.append((f"l{l}.wo", "w", weight(*lin[1][1:])))
            out.append((f"l{l}.ffn_norm", "bf16", gain(d)))
            out.append((f"l{l}.wgu", "w", weight(*lin[2][1:])))
            out.append((f"l{l}.wdown", "w", weight(*lin[3][1:])))
        else:
            out.append((f"l{l}.ln1_g", "bf16", gain(d)))
            out.append((f"l{l}.ln1_b", "bf16", normal(d)))
            out.append((f"l{l}.wqkv", "w", weight(*lin[0][1:])))
            out.append((f"l{l}.bqkv", "bf16", normal(lin[0][1])))
            out.append((f"l{l}.wo", "w", weight(*lin[1][1:])))
            out.append((f"l{l}.bo", "bf16", normal(d)))
            out.append((f"l{l}.ln2_g", "bf16", gain(d)))
            out.append((f"l{l}.ln2_b", "bf16", normal(d)))
            out.append((f"l{l}.wfc1", "w", weight(*lin[2][1:])))
            out.append((f"l{l}.bfc1", "bf16", normal(lin[2][1])))
            out.append((f"l{l}.wfc2", "w", weight(*lin[3][1:])))
            out.append((f"l{l}.bfc2", "bf16", normal(d)))
    if llama:
        out.append(("final_norm", "bf16", gain(d)))
    else:
        out.append(("lnf_g", "bf16", gain(d)))
        out.append(("lnf_b", "bf16", normal(d)))
    out.append(("lm_head", "bf16", normal(V, d)))
    return out


def tokens(shape: dict, seed: int, batch: int | None = None, seq: int | None = None) -> np.ndarray:
    rng = np.random.default_rng(seed)
    B = batch or shape["batch"]
    S = seq or shape["seq"]
    return rng.integers(0, shape["vocab"], size=(B, S), dtype=np.int32)


def linear_case(M: int, N: int, K: int, seed: int, group: int = GROUP):
    """Single perturbed linear: X ~ N(0,1) (bf16-exact) [M,K]; packed nibbles
    uniform over 0..15 as bytes [N,K/2]; scales ~ U(0.005, 0.02) (bf16-exact) [N,K/group]."""
    rng = np.random.default_rng(seed)
    x = bf16_exact(rng.standard_normal((M, K), dtype=np.float32))
    qp = rng.integers(0, 256, size=(N, K // 2), dtype=np.uint8)
    s = bf16_exact(rng.uniform(0.005, 0.02, size=(N, K // group)).astype(np.float32))
    return x, qp, s


def kmajor_case(N: int, K: int, seed: int, group: int = GROUP):
    """An asymmetric 4-bit linear in the K-major checkpoint layout: qweight uint32 [K/8, N]
    (8 consecutive k per word, lowest nibble first), qzeros uint32 [K/group, N/8] (8 consecutive
    n per word), scales [K/group, N] ~ U(0.005, 0.02) exactly representable in fp16.  All nibbles
    uniform."""
    rng = np.random.default_rng(seed)
    qweight = rng.integers(0, 1 << 32, size=(K // 8, N), dtype=np.uint64).astype(np.uint32)
    qzeros = rng.integers(0, 1 << 32, size=(K // group, N // 8), dtype=np.uint64).astype(np.uint32)
    scales = rng.uniform(0.005, 0.02, size=(K // group, N)).astype(np.float32).astype(np.float16).astype(np.float32)
    return qweight, qzeros, scales


def act_order_g_idx(K: int, seed: int = 0, group: int = GROUP) -> np.ndarray:
    """A group assignment as activation-reordering quantizers produce it: int32 [K], every group
    of `group` columns scattered over the input dimension (a random permutation of k // group)."""
    return np.random.default_rng(seed + K).permutation(np.arange(K) // group).astype(np.int32)


def fp16_exact(x: np.ndarray) -> np.ndarray:
    """Values exactly representable in IEEE binary16, as fp32."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


def codebook_linear_case(M: int, N: int, K: int, seed: int):
    """Single codebook-quantized linear: X ~ N(0,1) (bf16-exact) [M,K]; one 16-bit code per 8
    weights, uniform [N,K/8]; codebook ~ N(0, 0.02) (fp16-exact) [65536,8]; per-output-channel
    scales ~ U(0.5, 1.5) (fp16-exact) [N]."""
    rng = np.random.default_rng(seed)
    x = bf16_exact(rng.standard_normal((M, K), dtype=np.float32))
    idx = rng.integers(0, 65536, size=(N, K // 8), dtype=np.uint16)
    cb = fp16_exact(rng.standard_normal((65536, 8), dtype=np.float32) * np.float32(0.02))
    c = fp16_exact(rng.uniform(0.5, 1.5, size=N).astype(np.float32))
    return x, idx, cb, c


def codebook_tensor_table(shape: dict, seed: int):
    """Llama-shaped model in the codebook variant: (name, kind, array) with kind in
    'bf16' | 'codes' | 'codebook' | 'chscale' (see the oracle's build_codebook_model)."""
    assert shape["arch"] == "llama"
    rng = np.random.default_rng(seed)
    d, V = shape["d_model"], shape["vocab"]

    def normal(*sz):
        return bf16_exact(rng.standard_normal(sz, dtype=np.float32) * np.float32(0.02))

    def gain(n):
        return bf16_exact(1.0 + 0.1 * rng.standard_normal(n, dtype=np.float32))

    def lin(name, N, K):
        # codebook entries ~ N(0, 0.02) times channel scales ~ U(0.5, 1.5)
        return [(name, "codes", rng.integers(0, 65536, size=(N, K // 8), dtype=np.uint16)),
                (name + ".cb", "codebook",
                 fp16_exact(rng.standard_normal((65536, 8), dtype=np.float32) * np.float32(0.02))),
                (name + ".c", "chscale", fp16_exact(rng.uniform(0.5, 1.5, size=N).astype(np.float32)))]

    out = [("tok_emb", "bf16", normal(V, d))]
    for l in range(shape["n_layers"]):
        ql = quantized_linears(shape)
        out.append((f"l{l}.attn_norm", "bf16", gain(d)))
        out += lin(f"l{l}.wqkv", *ql[0][1:])
        out += lin(f"l{l}.wo", *ql[1][1:])
        out.append((f"l{l}.ffn_norm", "bf16", gain(d)))
        out += lin(f"l{l}.wgu", *ql[2][1:])
        out += lin(f"l{l}.wdown", *ql[3][1:])
    out.append(("final_norm", "bf16", gain(d)))
    out.append(("lm_head", "bf16", normal(V, d)))
    return out
