"""HIP path vs the CPU oracle, through the C ABI (needs an MI355X).

Bit-exact: Philox words, the normal recipe, z(row, group), int4 unpack +
indexing + perturbation (the bf16 weight tile), RTN, the update given d'.
Floating point: |err| <= tol relative, tolerances stated per test (the bar for
losses and updated scales is 2e-2 relative, bf16 operands with fp32 accumulate).
"""
import math

import numpy as np
import pytest
import torch

from paper_2505_13430_amd import binding as qb
from paper_2505_13430_amd import synth
from paper_2505_13430_amd.model import DeviceModel

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return t.to(dtype) if dtype is not None else t


def _bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


# ------------------------------------------------------------------ RNG ----
def test_philox_words_bit_exact(oracle):
    rng = np.random.default_rng(1)
    ctr = rng.integers(0, 1 << 32, size=(4099, 4), dtype=np.uint64).astype(np.uint32)
    ctr[0] = 0
    ctr[1] = 0xFFFFFFFF
    ctr[2] = [0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344]
    for seed in (0, 0xFFFFFFFFFFFFFFFF, 0x299F31D0A4093822, 1234):
        out = torch.zeros(ctr.shape, dtype=torch.int32, device=DEV)
        qb.qzo_debug_philox(seed, _dev(ctr.view(np.int32)), out)
        got = out.cpu().numpy().view(np.uint32)
        key = [seed & 0xFFFFFFFF, seed >> 32]
        for i in list(range(8)) + list(range(8, 4099, 97)):
            assert np.array_equal(got[i], oracle.philox4x32_10(ctr[i], key)), (seed, i)
    # the published vectors, on the device
    kat = {0: (0, "6627e8d5 e169c58d bc57ac4c 9b00dbd8"),
           0xFFFFFFFFFFFFFFFF: (1, "408f276d 41c83b0e a20bc7c6 6d5451fd"),
           0x299F31D0A4093822: (2, "d16cfe09 94fdcceb 5001e420 24126ea1")}
    for seed, (row, words) in kat.items():
        out = torch.zeros(ctr.shape, dtype=torch.int32, device=DEV)
        qb.qzo_debug_philox(seed, _dev(ctr.view(np.int32)), out)
        assert [f"{x:08x}" for x in out.cpu().numpy().view(np.uint32)[row]] == words.split()


def test_normal_recipe_bit_exact_over_both_factors(oracle):
    # the radius depends on the top 16 bits only, the angle and signs on the low
    # 16 only, and the variate is one IEEE product of the two: every value of
    # each factor, plus a stride through all 2^32 words.
    ws = [np.arange(65536, dtype=np.uint64) << 16 | a for a in (0, 0x3FFF, 0x9ABC, 0x4001, 0xFFFF)]
    ws += [np.arange(65536, dtype=np.uint64) | (h << 16) for h in (0, 1, 0x7FFF, 0xFFFF, 0x1234, 0x8000)]
    ws.append(np.arange(0, 1 << 32, 1021, dtype=np.uint64))
    w = np.concatenate(ws).astype(np.uint32)
    out = torch.zeros((w.size, 2), dtype=torch.float32, device=DEV)
    qb.qzo_debug_normal_pairs(_dev(w.view(np.int32)), out)
    assert np.array_equal(_bits(out.cpu().numpy()), _bits(oracle.normal_pairs(w)))


@pytest.mark.parametrize("rows,G,row0,seed", [(70, 86, 0, 1), (64, 32, 1000, 2), (5, 1, 7, 3),
                                             (33, 3, 0xFFFFFF00, 0xDEADBEEF12345678),
                                             (9, 108, 123456, 5), (300, 8, 0, 6)])
def test_scale_noise_bit_exact(oracle, rows, G, row0, seed):
    out = torch.zeros((rows, G), dtype=torch.float32, device=DEV)
    qb.qzo_debug_normals(seed, 0, row0, out)
    assert np.array_equal(_bits(out.cpu().numpy()), _bits(oracle.scale_normals(seed, row0, rows, G)))


# --------------------------------------------- unpack + index + perturb ----
@pytest.mark.parametrize("N,K,row_base,sign", [(24, 384, 0, 1), (40, 1024 + 128, 77, -1), (8, 128, 5, 1)])
def test_weight_tile_bit_exact(oracle, N, K, row_base, sign):
    _, qp, s = synth.linear_case(1, N, K, seed=N + K)
    out = torch.zeros((N, K), dtype=torch.bfloat16, device=DEV)
    qb.qzo_debug_dequant(_dev(qp), _dev(s, torch.bfloat16), row_base, 99, 1e-3, sign, out)
    want = oracle.dequant(qp, s, 99, row_base, sign * np.float32(1e-3), to_bf16=True)
    assert np.array_equal(_bits(out.float().cpu().numpy()), _bits(want))


@pytest.mark.parametrize("M", [16, 32, 64, 256], ids=["few16", "few32", "few64", "tile"])
@pytest.mark.parametrize("zp", [False, True], ids=["sym", "zp"])
def test_gemm_kernels_reproduce_the_perturbed_weights_bit_for_bit(oracle, M, zp):
    """The GEMM kernels' own unpacking and perturbation, read out through one-hot activations: row m
    of X is the unit vector of column k_m, so y[m, n] is the perturbed weight (n, k_m) itself, one
    fp32 product rounded to bf16 (Eq. 4-5).  256 tokens take the tile kernel (every column), fewer the
    few-token kernel in each of its variants (64 columns spread over both groups and all nibble
    positions): its integer-code products and fp32 group scaling round like the definition here."""
    N, K = 72, 256
    _, qp, s = synth.linear_case(1, N, K, seed=77)
    cols = np.arange(K) if M == K else (np.arange(M) * (K // M) + np.arange(M) % (K // M))
    x = np.zeros((M, K), dtype=np.float32)
    x[np.arange(M), cols] = 1.0
    y = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    eps = np.float32(1e-3)
    if zp:
        zo = np.random.default_rng(3).integers(0, 16, size=(N, K // 128), dtype=np.uint8)
        qb.qzo_dequant_gemm_zp(_dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16), _dev(zo), 11, 99, 1e-3, -1, y)
        want = oracle.dequant_zp(qp, s, zo, 99, 11, -eps, to_bf16=True)
    else:
        qb.qzo_dequant_gemm(_dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16), 11, 99, 1e-3, -1, y)
        want = oracle.dequant(qp, s, 99, 11, -eps, to_bf16=True)
    got = y.float().cpu().numpy()                      # [M, N] = W_eff[:, cols]^T
    assert len(set(cols.tolist())) == M
    assert np.array_equal(_bits(got), _bits(np.ascontiguousarray(want[:, cols].T)))


@pytest.mark.parametrize("fp16", [False, True], ids=["bf16", "fp16"])
def test_asymmetric_rtn_quantizer_bit_exact(oracle, fp16):
    rng = np.random.default_rng(4)
    w = (rng.standard_normal((136, 640)) * 0.02 + 0.03 * np.sin(np.arange(136))[:, None]).astype(np.float32)
    w[5, 128:256] = 0
    w[6, :128] = np.abs(w[6, :128])
    q = torch.zeros((136, 320), dtype=torch.uint8, device=DEV)
    zp = torch.zeros((136, 5), dtype=torch.uint8, device=DEV)
    s = torch.zeros((136, 5), dtype=torch.float16 if fp16 else torch.bfloat16, device=DEV)
    qb.qzo_rtn_quantize_asym(_dev(w), q, zp, s)
    qp, zo, sc = oracle.rtn_quantize_asym(w, scale_fmt=1 if fp16 else 0)
    assert np.array_equal(q.cpu().numpy(), qp) and np.array_equal(zp.cpu().numpy(), zo)
    assert np.array_equal(s.float().cpu().numpy(), sc)
    assert zo.min() <= 3 and zo.max() >= 12 and zo[6, 0] == 0 and sc[5, 1] == 0


def test_rtn_quantizer_bit_exact(oracle):
    rng = np.random.default_rng(3)
    w = (rng.standard_normal((136, 640)) * 0.02).astype(np.float32)
    w[5, 128:256] = 0
    q = torch.zeros((136, 320), dtype=torch.uint8, device=DEV)
    s = torch.zeros((136, 5), dtype=torch.bfloat16, device=DEV)
    qb.qzo_rtn_quantize(_dev(w), q, s)
    qp, sc = oracle.rtn_quantize(w)
    assert np.array_equal(q.cpu().numpy(), qp)
    assert np.array_equal(s.float().cpu().numpy(), sc)


# --------------------------------------------------------------- update ----
@pytest.mark.parametrize("fp16", [False, True], ids=["bf16", "fp16"])
@pytest.mark.parametrize("rows,G", [(257, 32), (128, 86), (33, 3), (64, 8), (100, 108), (7, 1), (1, 16)])
def test_update_given_d_bit_exact(oracle, rows, G, fp16):
    rng = np.random.default_rng(rows * G)
    s = rng.uniform(0.0, 0.02, (rows, G)).astype(np.float32)
    s = synth.fp16_exact(s) if fp16 else synth.bf16_exact(s)
    s[0, 0] = 0.0
    for eta, dc in ((1e-5, 37.5), (1e-3, -100.0), (0.0, 5.0), (1e-5, 0.0), (1e-7, 100.0)):
        sd = _dev(s, torch.float16 if fp16 else torch.bfloat16)
        guard = sd.clone()
        qb.qzo_apply_update(sd, 4242, 17, eta, dc)

        class Seg:
            pass
        sg = Seg()
        sg.name, sg.offset, sg.rows, sg.G, sg.row_base = "t", 0, rows, G, 4242
        m = oracle.Model(shape={}, tensors=[], names=[], scales=s.reshape(-1).copy(), segments=[sg],
                         scale_fmt=1 if fp16 else 0)
        want = oracle.update_scales(m, 17, eta, dc).reshape(rows, G)
        got = sd.float().cpu().numpy()
        assert np.array_equal(_bits(got), _bits(want)), (eta, dc)
        if eta == 0.0 or dc == 0.0:
            assert torch.equal(sd, guard)
        assert got.min() >= 0
        if fp16 and eta == 1e-7 and rows * G > 1000:      # the paper's step is visible in fp16 storage
            assert float((sd != guard).float().mean()) > 0.3


# ----------------------------------------------------- perturbed linear ----
def _gemm_case(oracle, M, N, K, seed, eps, sign, row_base=0):
    x, qp, s = synth.linear_case(M, N, K, seed)
    y = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    ssq = torch.zeros(1, dtype=torch.float32, device=DEV)
    qb.qzo_dequant_gemm(_dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16), row_base, 31,
                        eps, sign, y, ssq)
    se = oracle.effective_scales(s, row_base, 31, sign * np.float32(eps))
    ref = oracle.qlinear(x, qp, se)
    return y.float().cpu().numpy().astype(np.float64), float(ssq.item()), ref


@pytest.mark.parametrize("M,N,K", [(300, 520, 384), (256, 256, 128), (1, 8, 128), (513, 264, 1280),
                                   (64, 1024, 256), (65, 136, 256),
                                   # few-token path (M <= 64): ragged rows, odd group counts, K slices
                                   (7, 264, 384), (16, 520, 1280), (33, 4104, 1152), (64, 136, 4096),
                                   (32, 8, 128), (5, 12288, 512)])
def test_perturbed_linear_matches_oracle(oracle, M, N, K):
    for sign in (1, -1):
        got, ssq, ref = _gemm_case(oracle, M, N, K, seed=M + N, eps=1e-3, sign=sign, row_base=11)
        rms = math.sqrt((ref ** 2).mean())
        # bf16 unit roundoff is 2^-8: the weight tile's rounding gives an error of std
        # ~1.6e-3 rms (independent over K), the stored output one of <= 2^-8 |y|.
        bad = np.abs(got - ref) > 6e-3 * np.abs(ref) + 1.2e-2 * rms
        assert not bad.any(), (int(bad.sum()), np.abs(got - ref).max() / rms)
        assert math.sqrt(((got - ref) ** 2).mean()) <= 4e-3 * rms
        assert abs(ssq - oracle.sumsq_bf16(ref)) <= 5e-3 * oracle.sumsq_bf16(ref)
        assert abs(ssq - (got ** 2).sum()) <= 1e-4 * ssq      # the sum is of the stored outputs


def test_perturbed_linear_sign_and_eps_identities(oracle):
    x, qp, s = synth.linear_case(130, 264, 512, 8)
    xd, qd, sd = _dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16)

    def run(eps, sign, seed=5):
        y = torch.zeros((130, 264), dtype=torch.bfloat16, device=DEV)
        qb.qzo_dequant_gemm(xd, qd, sd, 0, seed, eps, sign, y, None)
        return y
    assert torch.equal(run(1e-3, 1), run(-1e-3, -1))          # only sign*eps matters
    assert torch.equal(run(0.0, 1), run(0.0, -1))             # eps = 0: both passes coincide
    assert torch.equal(run(0.0, 1), run(0.0, 1, seed=6))      # ... and the seed is irrelevant
    assert not torch.equal(run(1e-3, 1), run(1e-3, -1))
    assert torch.equal(run(1e-3, 1), run(1e-3, 1))            # run-to-run deterministic


def test_few_token_path_is_deterministic_and_close_to_the_tile_path(oracle):
    """The same rows computed as a 64-token call (few-token kernel) and inside a 200-token call
    (tile kernel) agree; repeated calls are bit-identical.  The tile kernel rounds every perturbed
    weight to bf16 (relative error up to 2^-9, independent from weight to weight), the few-token
    kernel multiplies the integer codes and scales the group sums in fp32: per output the two
    differ by about 2^-9 / sqrt(3) = 1.1e-3 of the outputs' rms (a sum of K independent terms),
    bounded here at six times that, plus one bf16 rounding of the output itself."""
    x, qp, s = synth.linear_case(200, 520, 1280, seed=9)
    xd, qd, sd = _dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16)
    big = torch.zeros((200, 520), dtype=torch.bfloat16, device=DEV)
    qb.qzo_dequant_gemm(xd, qd, sd, 3, 31, 1e-3, 1, big)
    outs = []
    for _ in range(2):
        y = torch.zeros((64, 520), dtype=torch.bfloat16, device=DEV)
        qb.qzo_dequant_gemm(xd[:64].contiguous(), qd, sd, 3, 31, 1e-3, 1, y)
        outs.append(y)
    assert torch.equal(outs[0], outs[1])
    a, b = outs[0].float(), big[:64].float()
    assert ((a - b).abs() <= 2.0 ** -7 * b.abs() + 7e-3 * b.pow(2).mean().sqrt()).all()


def test_boundary_rejects_bad_arguments():
    x = torch.zeros((4, 128), dtype=torch.bfloat16, device=DEV)
    q = torch.zeros((8, 64), dtype=torch.uint8, device=DEV)
    s = torch.zeros((8, 1), dtype=torch.bfloat16, device=DEV)
    y = torch.zeros((4, 8), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(qb.QzoError) as e:
        qb.qzo_dequant_gemm(x, q, s, 0, 1, 1e-3, 2, y)
    assert e.value.status == qb.QZO_ERR_ARG
    with pytest.raises(qb.QzoError) as e:
        qb.qzo_dequant_gemm(x, q, s, 0, 1, 1e-3, 1, y, group=64)
    assert e.value.status == qb.QZO_ERR_SHAPE
    with pytest.raises(qb.QzoError) as e:
        qb.qzo_dequant_gemm(x.view(-1)[1:].view(-1)[:384].view(3, 128), q, s, 0, 1, 1e-3, 1, y)
    assert e.value.status == qb.QZO_ERR_ALIGN


# ------------------------------------------------------------ the model ----
SHARP = dict(arch="llama", n_layers=2, d_model=256, n_heads=2, d_ffn=512, vocab=520, max_seq=96,
             batch=3, seq=80)     # head size 128, ragged vocab, seq not a multiple of 32/128


def _models(oracle, shape, seed, gain=1.0, asym=False, nf4=False, route=None, fp16=False, act_order=False):
    """route: None = the library's choice by token count, 1 = fused kernel, 2 = expand-then-multiply.
    fp16 / act_order (zero-point format): fp16 scale arena; a group index per input column."""
    table = synth.tensor_table(shape, seed)
    if gain != 1.0:   # larger weights: logits far from uniform, loss far from ln V
        table = [(n, k, synth.bf16_exact(a * gain) if (k == "w" or n in ("tok_emb", "lm_head")) else a)
                 for n, k, a in table]
    if asym:          # rows with off-centre weights, so that the zero-points spread over 2..13
        table = [(n, k, (a + 0.03 * gain * np.sin(np.arange(a.shape[0]))[:, None]).astype(np.float32)
                  if k == "w" else a) for n, k, a in table]
    om = oracle.build_model(shape, table, asym=asym, nf4=nf4, fp16_scales=fp16,
                            g_idx=(lambda K: synth.act_order_g_idx(K, seed)) if act_order else None)
    dm = DeviceModel.from_host(dict(shape, quant=om.quant, group=om.group, scale_fp16=om.scale_fmt,
                                    act_order=int(om.act_order)), om.tensors, om.scales, DEV)
    if route is not None:
        dm.set_int4_path(route)
    return om, dm



def _case(name):
    """'<shape>', '<shape>+zp' (zero-points) or '<shape>+nf4' (NormalFloat-4) -> (shape, variant flag)."""
    base, _, var = name.partition("+")
    shape = SHARP if base == "sharp" else (FEW.get(base) or MANY.get(base) or LONG.get(base) or synth.SHAPES[base])
    return shape, {"": False, "zp": True, "nf4": "nf4", "zp16": "zp16", "zpao": "zpao"}[var]


def _variant_args(var):
    """Keyword arguments of _models for a case's variant flag: zero-points (True), NormalFloat-4 ('nf4'),
    zero-points with an fp16 scale arena ('zp16'), the same plus a group index per column ('zpao')."""
    return dict(asym=var in (True, "zp16", "zpao"), nf4=var == "nf4", fp16=var in ("zp16", "zpao"),
                act_order=var == "zpao")


def _route(name):
    """Cases named many_* force the expand-then-multiply route (mode 2) on their model."""
    return 2 if name.startswith("many_") else None


# 576 tokens with the model's int4 route set to 2: the int4 linears run expand-then-multiply (by default
# only from several thousand tokens on, more than the oracle handles in a test)
MANY = {"many_llama": dict(synth.SHAPES["tiny"], batch=9, seq=64),
        "many_opt": dict(synth.SHAPES["tiny_opt"], batch=9, seq=64)}
# Sequences as long as the benchmark's: the attention kernel's steady state (a key tile refills an LDS
# buffer that was already read, loads run two tiles ahead, several 128-query blocks per sequence that
# are dispatched last-first).  long_llama: head size 128, 512 positions = 8 key tiles, 4 query blocks;
# long_opt: head size 64, 256 positions; long_ragged: 300 positions (a ragged last query block and key tile)
LONG = {"long_llama": dict(arch="llama", n_layers=2, d_model=256, n_heads=2, d_ffn=512, vocab=520, max_seq=512,
                           batch=2, seq=512),
        "long_opt": dict(arch="opt", n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=520, max_seq=256,
                         batch=3, seq=256),
        "long_ragged": dict(arch="llama", n_layers=1, d_model=256, n_heads=2, d_ffn=512, vocab=520, max_seq=320,
                            batch=2, seq=300)}
FEW = {"few_llama": dict(synth.SHAPES["tiny"], batch=1, seq=24),        # 24 tokens: one token tile
       "few_opt": dict(synth.SHAPES["tiny_opt"], batch=2, seq=32)}      # 64 tokens: two token tiles


@pytest.mark.parametrize("name,gain", [("tiny", 1.0), ("tiny_opt", 1.0), ("tiny", 4.0), ("tiny_opt", 4.0),
                                       ("sharp", 4.0), ("few_llama", 4.0), ("few_opt", 4.0),
                                       ("tiny+zp", 4.0), ("tiny_opt+zp", 4.0), ("sharp+zp", 4.0),
                                       ("few_llama+zp", 4.0), ("few_opt+zp", 1.0),
                                       ("tiny+nf4", 4.0), ("tiny_opt+nf4", 4.0), ("sharp+nf4", 4.0),
                                       ("few_llama+nf4", 1.0),
                                       ("many_llama", 4.0), ("many_opt", 4.0), ("many_llama+zp", 4.0),
                                       ("long_llama", 4.0), ("long_opt", 4.0), ("long_ragged", 4.0),
                                       ("long_llama+zp", 1.0),
                                       # the checkpoints' own scale type (fp16), and a group index per column
                                       ("tiny+zp16", 1.0), ("tiny_opt+zp16", 1.0), ("few_llama+zp16", 1.0),
                                       ("many_llama+zp16", 1.0), ("tiny+zpao", 1.0), ("tiny_opt+zpao", 1.0),
                                       ("sharp+zpao", 1.0), ("few_llama+zpao", 1.0)])
def test_forward_matches_oracle(oracle, name, gain):
    shape, asym = _case(name)
    om, dm = _models(oracle, shape, 1234, gain, route=_route(name), **_variant_args(asym))
    if asym is True:
        zps = np.concatenate([t.reshape(-1) for n, t in zip(om.names, om.tensors) if n.endswith(".zp")])
        assert zps.min() <= 3 and zps.max() >= 12
    tok = synth.tokens(shape, 5678)
    tokd = _dev(tok)
    B, S = tok.shape
    for sign in (1, -1):
        se = oracle.perturbed_scales(om, 9, sign * np.float32(1e-3))
        ref_loss, ref_hid = oracle.forward_loss(om, se, tok, act_bf16=True, want_hidden=True)
        hid = torch.zeros((B * S, shape["d_model"]), dtype=torch.bfloat16, device=DEV)
        loss = torch.zeros(1, dtype=torch.float32, device=DEV)
        qb.qzo_debug_forward(dm.handle, tokd, 9, 1e-3, sign, dm.workspace(B, S), loss, hid)
        got_loss = float(loss.item())
        assert abs(got_loss - ref_loss) <= 2e-2 * abs(ref_loss), (got_loss, ref_loss)
        if gain > 1:
            assert abs(ref_loss - math.log(shape["vocab"])) > 0.05      # the case is not degenerate
        h = hid.float().cpu().numpy().astype(np.float64)
        rms = math.sqrt((ref_hid ** 2).mean())
        # final hidden states after 2 layers of bf16 storage.  The noise floor of 16-bit
        # activations is what the oracle itself moves by when its A16 rounding is switched
        # off (5e-3 .. 1.3e-2 rms here); the kernels round the weight tile and the attention
        # probabilities to bf16 as well, so they may sit up to twice that floor away.
        _, exact_hid = oracle.forward_loss(om, se, tok, act_bf16=False, want_hidden=True)
        floor_rms = math.sqrt(((exact_hid - ref_hid) ** 2).mean())
        floor_max = np.abs(exact_hid - ref_hid).max()
        err = np.abs(h - ref_hid)
        assert math.sqrt((err ** 2).mean()) <= 2 * floor_rms + 2e-3 * rms, (math.sqrt((err ** 2).mean()) / rms, floor_rms / rms)
        # the largest single deviation: a maximum over 10^4 .. 10^5 elements of the sum of three rounding
        # sources (activations, weight tile, probabilities) against the maximum of one of them, so the
        # ratio scatters around sqrt(3): three times the floor's maximum bounds it (the rms bound above,
        # which carries the comparison, stays at twice the floor)
        assert err.max() <= 3 * floor_max + 2e-2 * rms, (err.max() / rms, floor_max / rms)
        again = torch.zeros(1, dtype=torch.float32, device=DEV)
        qb.qzo_forward_loss(dm.handle, tokd, 9, 1e-3, sign, dm.workspace(B, S), again)
        assert again.item() == got_loss                                  # deterministic
    dm.close()


def _d_noise_floor(oracle, om, tok, seeds, eps=1e-3):
    """What the oracle's own projected gradient d = (l+ - l-)/(2 eps) (Eq. 5, Algorithm 1) moves by when
    its 16-bit activation rounding is switched off, largest over a few directions: the size of the
    rounding noise that 1/(2 eps) = 500 amplifies into d."""
    return max(abs(oracle.qzo_step(om, tok, seed=sd, eps=eps, eta=0.0, Cthr=1e9)["d"] -
                   oracle.qzo_step(om, tok, seed=sd, eps=eps, eta=0.0, Cthr=1e9, act_bf16=False)["d"])
               for sd in seeds)


@pytest.mark.parametrize("name", ["tiny", "tiny_opt", "few_llama", "few_opt",
                                  "tiny+zp", "tiny_opt+zp", "few_llama+zp", "few_opt+zp",
                                  "tiny+nf4", "tiny_opt+nf4", "few_llama+nf4",
                                  "many_llama", "many_opt", "many_llama+zp",
                                  "long_llama", "long_opt", "long_ragged",
                                  "tiny+zp16", "tiny_opt+zp16", "few_llama+zp16", "many_llama+zp16",
                                  "tiny+zpao", "tiny_opt+zpao", "few_llama+zpao"])
def test_step_matches_oracle(oracle, name):
    shape, asym = _case(name)
    om, dm = _models(oracle, shape, 1234, route=_route(name), **_variant_args(asym))
    tok = synth.tokens(shape, 5678)
    tokd = _dev(tok)
    # NormalFloat-4 scales are a block's absmax, ten times larger (the 24-token case has a larger |d|)
    eta = (1e-4 if name.startswith("few") else 3e-4) if asym == "nf4" else 1e-5
    if name.startswith("long"):       # 1024 / 768 / 600 tokens: |d| is below 2, a larger step makes it visible
        eta = 1e-4
    seed = 3 if asym else 1           # a direction whose |d| is large enough to move the scales
    ref = oracle.qzo_step(om, tok, seed=seed, eps=1e-3, eta=eta, Cthr=100.0)
    before = dm.scales.clone()
    res = qb.read_step_result(dm.step(tokd, seed, 1e-3, eta, 100.0))
    assert res["status"] == 0
    print(name, "d gpu", res["d"], "d oracle", ref["d"], "losses", res["loss_plus"], ref["loss_plus"])
    for k in ("loss_plus", "loss_minus"):
        assert abs(res[k] - ref[k]) <= 2e-2 * abs(ref[k])
    assert res["d"] == np.float32((np.float32(res["loss_plus"]) - np.float32(res["loss_minus"]))
                                  / (np.float32(2) * np.float32(1e-3)))
    assert res["d_clipped"] == max(-100.0, min(100.0, res["d"]))
    # the projected gradient itself: within four times the 16-bit noise floor of the oracle's own d
    # (the floor holds the rounding of the activations; the kernels also round the weight tile to bf16,
    # an error of the same size per linear)
    floor = _d_noise_floor(oracle, om, tok, [seed + 100 * i for i in range(5)])
    print(name, "d error", abs(res["d"] - ref["d"]), "floor", floor)
    assert abs(res["d"] - ref["d"]) <= 4 * floor + 1e-3 * abs(ref["d"]), (res["d"], ref["d"], floor)
    got = dm.scales.float().cpu().numpy()
    assert (np.abs(got - ref["scales"]) <= 2e-2 * np.abs(ref["scales"]) + 1e-7).all()
    assert not torch.equal(dm.scales, before)
    # exactly the oracle's update for the d' the device found
    want = oracle.update_scales(om, seed, eta, res["d_clipped"])
    assert np.array_equal(_bits(got), _bits(want))
    dm.close()


@pytest.mark.parametrize("name", ["tiny", "tiny_opt", "tiny+zp", "tiny+zp16"])
def test_stacked_passes_equal_separate_passes(oracle, name):
    """With at most 32 tokens qzo_step runs both perturbed passes as one stacked forward (the
    weights are read once); its losses are bit-identical to two separate forward passes."""
    base, asym = _case(name)
    shape = dict(base, batch=2, seq=13)
    om, dm = _models(oracle, shape, 1234, 4.0, **_variant_args(asym))
    tokd = _dev(synth.tokens(shape, 5678))
    res = qb.read_step_result(dm.step(tokd, 21, 1e-3, 0.0, 100.0))       # eta = 0: scales untouched
    lp = float(dm.forward_loss(tokd, 21, 1e-3, 1).item())
    lm = float(dm.forward_loss(tokd, 21, 1e-3, -1).item())
    assert res["loss_plus"] == lp and res["loss_minus"] == lm and lp != lm
    dm.close()


@pytest.mark.parametrize("name,batch,seq", [("tiny", 4, 64), ("long_opt+zp", 3, 256), ("long_ragged", 2, 300),
                                            ("tiny_opt", 3, 40), ("tiny+zp", 3, 40)])
def test_stacked_tile_passes_match_separate_passes(oracle, name, batch, seq):
    """Beyond the few-token kernel's range qzo_step runs both perturbed passes as one stacked forward
    through the tile kernel, the second pass's token tiles with -eps; the second pass starts on a
    256-row tile boundary, with padding rows in between when a pass is not a whole number of tiles
    (600 -> 768, 120 -> 256 here).  The K split of a linear depends on the number of token tiles, so
    the sums are ordered differently than in two separate passes: equal to within the 16-bit
    activations' noise, not bit for bit."""
    base, asym = _case(name)
    shape = dict(base, batch=batch, seq=seq)
    om, dm = _models(oracle, shape, 1234, 4.0, **_variant_args(asym))
    tokd = _dev(synth.tokens(shape, 5678))
    res = qb.read_step_result(dm.step(tokd, 21, 1e-3, 0.0, 100.0))       # eta = 0: scales untouched
    lp = float(dm.forward_loss(tokd, 21, 1e-3, 1).item())
    lm = float(dm.forward_loss(tokd, 21, 1e-3, -1).item())
    assert abs(res["loss_plus"] - lp) <= 2e-3 * lp and abs(res["loss_minus"] - lm) <= 2e-3 * lm
    assert res["loss_plus"] != res["loss_minus"]
    # the sign of each pass is the right one: the stacked losses are closer to their own pass than to the other
    if abs(lp - lm) > 8e-3 * lp:
        assert abs(res["loss_plus"] - lp) < abs(res["loss_plus"] - lm)
        assert abs(res["loss_minus"] - lm) < abs(res["loss_minus"] - lp)
    # and they are the oracle's losses
    tok = synth.tokens(shape, 5678)
    want = oracle.qzo_step(om, tok, seed=21, eps=1e-3, eta=0.0, Cthr=100.0)
    assert abs(res["loss_plus"] - want["loss_plus"]) <= 2e-2 * want["loss_plus"]
    assert abs(res["loss_minus"] - want["loss_minus"]) <= 2e-2 * want["loss_minus"]
    dm.close()


def test_step_special_cases(oracle):
    shape = synth.SHAPES["tiny"]
    om, dm = _models(oracle, shape, 1234)
    tokd = _dev(synth.tokens(shape, 5678))
    before = dm.scales.clone()
    r = qb.read_step_result(dm.step(tokd, 1, 0.0, 1e-5, 100.0))          # eps = 0: 0/0, skipped
    assert r["loss_plus"] == r["loss_minus"] and r["status"] == qb.QZO_ERR_NONFINITE
    assert torch.equal(dm.scales, before)
    r = qb.read_step_result(dm.step(tokd, 1, 1e-3, 1e-5, 0.0))           # C = 0: zero-shot
    assert r["status"] == 0 and r["d_clipped"] == 0.0 and torch.equal(dm.scales, before)
    r = qb.read_step_result(dm.step(tokd, 1, 1e-3, 0.0, 100.0))          # eta = 0
    assert torch.equal(dm.scales, before)
    with pytest.raises(qb.QzoError):
        dm.step(tokd, 1, 1e-3, 1e-5, -1.0)                               # C must be >= 0
    # update over the whole arena given the oracle's d', bit-exact
    dm.apply_update(77, 1e-5, -12.5)
    want = oracle.update_scales(om, 77, 1e-5, -12.5)
    assert np.array_equal(_bits(dm.scales.float().cpu().numpy()), _bits(want))
    dm.close()


def test_device_built_model_runs_and_is_near_ln_vocab():
    shape = synth.SHAPES["tiny"]
    dm = DeviceModel.synthetic(shape, seed=3, device=DEV)
    tokd = _dev(synth.tokens(shape, 5))
    r = qb.read_step_result(dm.step(tokd, 2, 1e-3, 1e-5, 100.0))
    assert r["status"] == 0 and abs(r["loss_plus"] - math.log(shape["vocab"])) < 0.3
    dm.close()


# ------------------------------------------------- full-size configurations ----
def test_single_linear_full_size_sampled(oracle):
    # the single-linear workload at its real size (2048 x 11008 x 4096), both signs:
    # sampled outputs recomputed by the oracle, and the loss against its closed form
    M, N, K = synth.LINEAR_SHAPE["M"], synth.LINEAR_SHAPE["N"], synth.LINEAR_SHAPE["K"]
    x, qp, s = synth.linear_case(M, N, K, seed=2)
    xd, qd, sd = _dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16)
    rng = np.random.default_rng(0)
    ms = np.sort(rng.choice(M, 24, replace=False))
    ns = np.sort(np.concatenate([rng.choice(N, 60, replace=False), [0, 255, 256, N - 1]]))
    losses = {}
    for sign in (1, -1):
        y = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
        ssq = torch.zeros(1, dtype=torch.float32, device=DEV)
        qb.qzo_dequant_gemm(xd, qd, sd, 0, 1, 1e-3, sign, y, ssq)
        se = oracle.effective_scales(s, 0, 1, sign * np.float32(1e-3))
        ref = oracle.qlinear(x[ms], qp[ns], se[ns])
        got = y.float().cpu().numpy().astype(np.float64)[np.ix_(ms, ns)]
        rms = math.sqrt((ref ** 2).mean())
        assert (np.abs(got - ref) <= 6e-3 * np.abs(ref) + 1.2e-2 * rms).all()
        losses[sign] = float(ssq.item())
        # E[loss] = M N K E[q^2] (E[s^2] + eps^2), q uniform on -8..7, s ~ U(0.005, 0.02)
        closed = M * N * K * 21.5 * ((0.005 ** 2 + 0.005 * 0.02 + 0.02 ** 2) / 3 + 1e-6)
        assert abs(losses[sign] - closed) <= 2e-2 * closed
        assert abs(losses[sign] - float((y.float() ** 2).sum().item())) <= 1e-3 * losses[sign]
    assert losses[1] != losses[-1]


def test_expand_then_multiply_full_size_sampled(oracle):
    # the route the benchmark's linears take (8192 tokens per pass), at a real layer shape
    # (8192 x 11008 x 4096): sampled outputs recomputed by the oracle, and equality with the fused kernel
    M, N, K = 8192, synth.LINEAR_SHAPE["N"], synth.LINEAR_SHAPE["K"]
    x, qp, s = synth.linear_case(M, N, K, seed=3)
    xd, qd, sd = _dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16)
    rng = np.random.default_rng(1)
    ms = np.sort(np.concatenate([rng.choice(M, 20, replace=False), [0, 255, 256, M - 1]]))
    ns = np.sort(np.concatenate([rng.choice(N, 60, replace=False), [0, 255, 256, N - 1]]))
    scratch = torch.empty(qb.qzo_int4_scratch_bytes(N, K), dtype=torch.uint8, device=DEV)
    y = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    qb.qzo_int4_gemm_expanded(xd, qd, sd, None, None, 5, 1, 1e-3, -1, y, scratch)
    se = oracle.effective_scales(s, 5, 1, -np.float32(1e-3))
    ref = oracle.qlinear(x[ms], qp[ns], se[ns])
    got = y.float().cpu().numpy().astype(np.float64)[np.ix_(ms, ns)]
    rms = math.sqrt((ref ** 2).mean())
    assert (np.abs(got - ref) <= 6e-3 * np.abs(ref) + 1.2e-2 * rms).all()
    y2 = torch.zeros_like(y)
    qb.qzo_dequant_gemm(xd, qd, sd, 5, 1, 1e-3, -1, y2)
    assert torch.equal(y, y2)


@pytest.mark.parametrize("rows,G,row_base", [(38400, 32, 31 * 42496), (4096, 86, 31 * 42496 + 38400),
                                             (48128, 40, 0), (5120, 108, 1877000),
                                             # beyond a million counters the update runs as one persistent
                                             # workgroup per compute unit with the angle factors in an LDS table
                                             (300000, 32, 7), (131072, 86, 1000000), (1100000, 3, 5)])
def test_update_at_real_tensor_sizes_bit_exact(oracle, rows, G, row_base):
    # one decoder layer's update segments of the Llama-2-7B / 13B shapes
    rng = np.random.default_rng(rows + G)
    s = synth.bf16_exact(rng.uniform(0.003, 0.012, (rows, G)).astype(np.float32))
    sd = _dev(s, torch.bfloat16)
    qb.qzo_apply_update(sd, row_base, 2025, 1e-5, -63.0)

    class Seg:
        pass
    sg = Seg()
    sg.name, sg.offset, sg.rows, sg.G, sg.row_base = "t", 0, rows, G, row_base
    m = oracle.Model(shape={}, tensors=[], names=[], scales=s.reshape(-1).copy(), segments=[sg])
    want = oracle.update_scales(m, 2025, 1e-5, -63.0).reshape(rows, G)
    assert np.array_equal(_bits(sd.float().cpu().numpy()), _bits(want))


@pytest.mark.parametrize("name,batch,seq,eta", [("opt-1.3b", 1, 24, 1e-5), ("llama-2-7b", 1, 16, 1e-7),
                                                ("llama-2-13b", 1, 16, 1e-7),      # few-token path
                                                # few-token path with the block sums of the activations delivered
                                                # by the norm and by the SwiGLU reduction: 24 tokens (stacked
                                                # passes), 48 tokens (two passes, two token tiles)
                                                ("llama-2-7b", 1, 24, 1e-7), ("llama-2-7b", 2, 24, 1e-7),
                                                ("opt-1.3b", 3, 24, 1e-5), ("llama-2-7b", 3, 24, 1e-7)])
def test_real_width_one_layer_step(oracle, name, batch, seq, eta):
    # depth-reduced copy: real widths (incl. the ragged OPT vocabulary), one layer, short batch.
    # d = (l+ - l-)/(2 eps) amplifies the losses' rounding noise 500 times, so the 2e-2 bound on
    # the updated scales is checked at the paper's learning rate for the 7B width (eta 1e-7,
    # Sec. 4.1) and at 1e-5 for the narrower model; the update itself is checked bit for bit
    # against the oracle for the d' the device found.
    shape = dict(synth.SHAPES[name], n_layers=1, batch=batch, seq=seq, max_seq=32)
    om, dm = _models(oracle, shape, 77)
    tok = synth.tokens(shape, 78)
    ref = oracle.qzo_step(om, tok, seed=3, eps=1e-3, eta=eta, Cthr=100.0)
    res = qb.read_step_result(dm.step(_dev(tok), 3, 1e-3, eta, 100.0))
    assert res["status"] == 0
    for k in ("loss_plus", "loss_minus"):
        assert abs(res[k] - ref[k]) <= 2e-2 * abs(ref[k]), (k, res[k], ref[k])
    got = dm.scales.float().cpu().numpy()
    assert (np.abs(got - ref["scales"]) <= 2e-2 * np.abs(ref["scales"]) + 1e-7).all()
    assert np.array_equal(_bits(got), _bits(oracle.update_scales(om, 3, eta, res["d_clipped"])))
    dm.apply_update(9, 1e-5, 55.0)       # a visible update on top, bit for bit
    want = oracle.update_scales(om, 9, 1e-5, 55.0, scales=got)
    assert np.array_equal(_bits(dm.scales.float().cpu().numpy()), _bits(want))
    print(name, "loss", res["loss_plus"], ref["loss_plus"], "d", res["d"], ref["d"])
    dm.close()


@pytest.mark.parametrize("name,asym", [("llama-2-7b", False), ("llama-2-13b", False), ("opt-1.3b", False),
                                       ("llama-2-7b", True)])
def test_real_width_one_layer_expanded_route(oracle, name, asym):
    """The route the benchmark's linears take (perturbed scales of the whole arena in one launch, the
    perturbed bf16 matrix written out, plain GEMM), at real widths: 86 / 108 groups per row in the
    down projection, the gate/up row interleave at 11008 / 13824 features, K = 11008 / 13824 in the
    plain GEMM, two token tiles (272 tokens).  One layer, a short vocabulary for the Llama shapes."""
    shape = dict(synth.SHAPES[name], n_layers=1, batch=2, seq=136, max_seq=136)
    if shape["arch"] == "llama":
        shape["vocab"] = 1000
    om, dm = _models(oracle, shape, 77, asym=asym, route=2)
    tok = synth.tokens(shape, 78)
    B, S = tok.shape
    se = oracle.perturbed_scales(om, 3, np.float32(1e-3))
    ref_loss, ref_hid = oracle.forward_loss(om, se, tok, act_bf16=True, want_hidden=True)
    _, exact_hid = oracle.forward_loss(om, se, tok, act_bf16=False, want_hidden=True)
    hid = torch.zeros((B * S, shape["d_model"]), dtype=torch.bfloat16, device=DEV)
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    qb.qzo_debug_forward(dm.handle, _dev(tok), 3, 1e-3, 1, dm.workspace(B, S), loss, hid)
    assert abs(loss.item() - ref_loss) <= 2e-2 * abs(ref_loss), (loss.item(), ref_loss)
    rms = math.sqrt((ref_hid ** 2).mean())
    err = np.abs(hid.float().cpu().numpy().astype(np.float64) - ref_hid)
    floor_rms = math.sqrt(((exact_hid - ref_hid) ** 2).mean())
    print(name, "hidden rms err", math.sqrt((err ** 2).mean()) / rms, "floor", floor_rms / rms)
    assert math.sqrt((err ** 2).mean()) <= 2 * floor_rms + 2e-3 * rms
    assert err.max() <= 2 * np.abs(exact_hid - ref_hid).max() + 2e-2 * rms
    eta = 1e-5 if name == "opt-1.3b" else 1e-7
    ref = oracle.qzo_step(om, tok, seed=3, eps=1e-3, eta=eta, Cthr=100.0)
    res = qb.read_step_result(dm.step(_dev(tok), 3, 1e-3, eta, 100.0))
    assert res["status"] == 0
    assert res["loss_plus"] == loss.item()                   # the step's first pass is that forward
    for k in ("loss_plus", "loss_minus"):
        assert abs(res[k] - ref[k]) <= 2e-2 * abs(ref[k]), (k, res[k], ref[k])
    got = dm.scales.float().cpu().numpy()
    assert (np.abs(got - ref["scales"]) <= 2e-2 * np.abs(ref["scales"]) + 1e-7).all()
    assert np.array_equal(_bits(got), _bits(oracle.update_scales(om, 3, eta, res["d_clipped"])))
    print(name, "loss", res["loss_plus"], ref["loss_plus"], "d", res["d"], ref["d"])
    dm.close()


@pytest.mark.parametrize("name,asym", [("llama-2-7b", False), ("opt-1.3b", True)])
def test_real_width_one_layer_stacked_tile_step(oracle, name, asym):
    """The step of the paper's batch regime at real widths: 272 tokens per pass on the default route,
    i.e. both passes in one forward through the fused tile kernel (the second pass from row 512 on, 240
    padding rows), K split of the 4096- / 2048-wide projections, RoPE inside the attention kernel.
    Losses, and the scales after the update, against the oracle."""
    shape = dict(synth.SHAPES[name], n_layers=1, batch=2, seq=136, max_seq=136)
    if shape["arch"] == "llama":
        shape["vocab"] = 1000
    om, dm = _models(oracle, shape, 77, asym=asym)
    tok = synth.tokens(shape, 78)
    eta = 1e-5 if name == "opt-1.3b" else 1e-7
    ref = oracle.qzo_step(om, tok, seed=3, eps=1e-3, eta=eta, Cthr=100.0)
    res = qb.read_step_result(dm.step(_dev(tok), 3, 1e-3, eta, 100.0))
    assert res["status"] == 0
    for k in ("loss_plus", "loss_minus"):
        assert abs(res[k] - ref[k]) <= 2e-2 * abs(ref[k]), (k, res[k], ref[k])
    assert res["loss_plus"] != res["loss_minus"]
    got = dm.scales.float().cpu().numpy()
    assert (np.abs(got - ref["scales"]) <= 2e-2 * np.abs(ref["scales"]) + 1e-7).all()
    assert np.array_equal(_bits(got), _bits(oracle.update_scales(om, 3, eta, res["d_clipped"])))
    print(name, "loss", res["loss_plus"], ref["loss_plus"], "d", res["d"], ref["d"])
    dm.close()


def test_failing_calls_enqueue_nothing(oracle):
    """Every error that the library finds itself (anything but a failing HIP call) is found before
    the first launch: outputs, workspace and scales are untouched afterwards."""
    import ctypes as C
    shape = synth.SHAPES["tiny"]
    om, dm = _models(oracle, shape, 1234)
    tok = synth.tokens(shape, 5678)
    tokd = _dev(tok)
    B, S = tok.shape
    ws = dm.workspace(B, S)
    ws.fill_(0x5A)
    dm.result.fill_(0x7B7B7B7B)
    scales0 = dm.scales.clone()
    lib = qb.lib()

    def step(tokens=tokd, batch=B, seq=S, ws_bytes=ws.numel(), wsp=ws.data_ptr(), clip=100.0, eps=1e-3):
        return lib.qzo_step(dm.handle, C.c_void_p(tokens.data_ptr()), C.c_uint32(batch), C.c_uint32(seq),
                            C.c_uint64(1), C.c_float(eps), C.c_float(1e-5), C.c_float(clip), C.c_void_p(wsp),
                            C.c_uint64(ws_bytes), C.c_void_p(dm.result.data_ptr()), None)
    assert step(ws_bytes=ws.numel() - 256) == qb.QZO_ERR_WORKSPACE
    assert step(seq=S + 1) == qb.QZO_ERR_SHAPE                     # beyond max_seq
    assert step(seq=1) == qb.QZO_ERR_SHAPE
    assert step(batch=0) == qb.QZO_ERR_SHAPE
    assert step(wsp=ws.data_ptr() + 4) == qb.QZO_ERR_ALIGN
    assert step(clip=-1.0) == qb.QZO_ERR_ARG
    assert step(eps=float("nan")) == qb.QZO_ERR_ARG
    assert step(batch=1 << 20, seq=S) == qb.QZO_ERR_SHAPE          # activations beyond 32-bit byte offsets
    assert "2^31" in lib.qzo_last_error().decode()
    loss = torch.full((1,), 7.0, device=DEV)
    assert lib.qzo_forward_loss(dm.handle, C.c_void_p(tokd.data_ptr()), C.c_uint32(B), C.c_uint32(S), C.c_uint64(1),
                                C.c_float(1e-3), C.c_int(0), C.c_void_p(ws.data_ptr()), C.c_uint64(ws.numel()),
                                C.c_void_p(loss.data_ptr()), None) == qb.QZO_ERR_ARG      # sign 0
    torch.cuda.synchronize()
    assert bool((ws == 0x5A).all()) and bool((dm.result == 0x7B7B7B7B).all()) and loss.item() == 7.0
    assert torch.equal(dm.scales, scales0)
    # a single linear: scratch too small / missing / misaligned, operands too large
    x, qp, s = synth.linear_case(16, 520, 1280, seed=4)
    xd, qd, sd = _dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16)
    y = torch.full((16, 520), 3.0, dtype=torch.bfloat16, device=DEV)
    need = qb.qzo_linear_scratch_bytes(16, 520, 1280, True)
    scratch = torch.full((need + 256,), 0x33, dtype=torch.uint8, device=DEV)
    ssq = torch.full((1,), -1.0, device=DEV)
    for bad, status in ((scratch[:need - 256], qb.QZO_ERR_WORKSPACE), (None, qb.QZO_ERR_ARG),
                        (scratch[16:], qb.QZO_ERR_ALIGN)):
        with pytest.raises(qb.QzoError) as e:
            qb.qzo_dequant_gemm(xd, qd, sd, 0, 1, 1e-3, 1, y, ssq, scratch=bad)
        assert e.value.status == status
    assert lib.qzo_dequant_gemm(C.c_void_p(xd.data_ptr()), C.c_void_p(qd.data_ptr()), C.c_void_p(sd.data_ptr()),
                                C.c_uint32(0), C.c_uint32(1 << 20), C.c_uint32(520), C.c_uint32(1280),
                                C.c_uint32(128), C.c_uint64(1), C.c_float(1e-3), C.c_int(1),
                                C.c_void_p(y.data_ptr()), None, C.c_void_p(scratch.data_ptr()),
                                C.c_uint64(scratch.numel()), None) == qb.QZO_ERR_SHAPE
    torch.cuda.synchronize()
    assert bool((y == 3.0).all()) and bool((scratch == 0x33).all()) and ssq.item() == -1.0
    qb.qzo_dequant_gemm(xd, qd, sd, 0, 1, 1e-3, 1, y, ssq, scratch=scratch[:need])      # exactly enough
    torch.cuda.synchronize()
    assert not bool((y == 3.0).all()) and ssq.item() > 0 and bool((scratch[need:] == 0x33).all())
    # joint mode: a wrong count and a table that is too small are refused, the model stays usable
    n_dense = qb.qzo_model_dense_count(dm.shape)
    master = torch.zeros(n_dense, dtype=torch.float32, device=DEV)
    table = torch.zeros(qb.qzo_model_joint_table_bytes(dm.shape), dtype=torch.uint8, device=DEV)
    with pytest.raises(qb.QzoError) as e:
        qb.qzo_model_enable_joint(dm.handle, master[:-8], table)
    assert e.value.status == qb.QZO_ERR_SHAPE
    with pytest.raises(qb.QzoError) as e:
        qb.qzo_model_enable_joint(dm.handle, master, table[:64])
    assert e.value.status == qb.QZO_ERR_WORKSPACE
    with pytest.raises(qb.QzoError) as e:
        dm.step_joint(tokd, 1, 1e-3, 1e-5, 1e-5, 100.0)
    assert e.value.status == qb.QZO_ERR_ARG
    assert bool((table == 0).all())
    assert qb.read_step_result(dm.step(tokd, 1, 1e-3, 0.0, 100.0))["status"] == 0
    with pytest.raises(qb.QzoError) as e:
        dm.set_int4_path(3)
    assert e.value.status == qb.QZO_ERR_ARG
    dm.close()


# ----------------------------------- asymmetric groups (zero-points) ----
def _zp_case(oracle, N, K, seed, fp16=False):
    qweight, qzeros, scales = synth.kmajor_case(N, K, seed)
    q = torch.zeros((N, K // 2), dtype=torch.uint8, device=DEV)
    zp = torch.zeros((N, K // 128), dtype=torch.uint8, device=DEV)
    s = torch.zeros((N, K // 128), dtype=torch.float16 if fp16 else torch.bfloat16, device=DEV)
    qb.qzo_repack_kmajor(_dev(qweight.view(np.int32)), _dev(qzeros.view(np.int32)),
                         _dev(scales, torch.float16), 1, q, zp, s)
    return (qweight, qzeros, scales), (q, zp, s)


@pytest.mark.parametrize("fp16", [False, True], ids=["bf16", "fp16"])
@pytest.mark.parametrize("N,K", [(24, 384), (264, 1280), (8, 128)])
def test_kmajor_repack_and_zero_point_tile_bit_exact(oracle, N, K, fp16):
    host, (q, zp, s) = _zp_case(oracle, N, K, seed=N + K, fp16=fp16)
    qp, zpo, so = oracle.repack_kmajor(*host, zero_add=1)
    if fp16:                       # the checkpoint's fp16 scales are kept as they are
        so = host[2].T.copy()
    assert np.array_equal(q.cpu().numpy(), qp) and np.array_equal(zp.cpu().numpy(), zpo)
    assert np.array_equal(_bits(s.float().cpu().numpy()), _bits(so))
    for sign in (1, -1):
        out = torch.zeros((N, K), dtype=torch.bfloat16, device=DEV)
        qb.qzo_debug_dequant_zp(q, s, zp, 9, 99, 1e-3, sign, out)
        want = oracle.dequant_zp(qp, so, zpo, 99, 9, sign * np.float32(1e-3), to_bf16=True)
        assert np.array_equal(_bits(out.float().cpu().numpy()), _bits(want))


@pytest.mark.parametrize("fp16", [False, True], ids=["bf16", "fp16"])
@pytest.mark.parametrize("M,N,K", [(300, 520, 384), (256, 264, 1280), (16, 520, 1280), (64, 136, 512),
                                   (1, 8, 128)])
def test_zero_point_linear_matches_oracle(oracle, M, N, K, fp16):
    host, (q, zp, s) = _zp_case(oracle, N, K, seed=M + N + K, fp16=fp16)
    qp, zpo, so = oracle.repack_kmajor(*host, zero_add=1)
    if fp16:
        so = host[2].T.copy()
    x = synth.linear_case(M, 8, K, seed=M)[0]
    xd = _dev(x, torch.bfloat16)
    for sign in (1, -1):
        y = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
        ssq = torch.zeros(1, dtype=torch.float32, device=DEV)
        qb.qzo_dequant_gemm_zp(xd, q, s, zp, 11, 31, 1e-3, sign, y, ssq)
        se = oracle.effective_scales(so, 11, 31, sign * np.float32(1e-3))
        ref = oracle.qlinear_zp(x, qp, se, zpo)
        got = y.float().cpu().numpy().astype(np.float64)
        rms = math.sqrt((ref ** 2).mean())
        bad = np.abs(got - ref) > 6e-3 * np.abs(ref) + 1.2e-2 * rms
        assert not bad.any(), (int(bad.sum()), np.abs(got - ref).max() / rms)
        assert abs(float(ssq.item()) - oracle.sumsq_bf16(ref)) <= 5e-3 * oracle.sumsq_bf16(ref)
    # zero-point 8 everywhere reproduces the symmetric entry point bit for bit
    if not fp16:
        zp8 = torch.full_like(zp, 8)
        a = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
        b = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
        qb.qzo_dequant_gemm_zp(xd, q, s, zp8, 11, 31, 1e-3, 1, a)
        qb.qzo_dequant_gemm(xd, q, s, 11, 31, 1e-3, 1, b)
        assert torch.equal(a, b)


# ------------------------------------------------------ codebook variant ----
@pytest.mark.parametrize("n,row_base", [(1000, 0), (4096, 128), (37, 5), (8, 0xFFFFF000)])
def test_channel_update_bit_exact(oracle, n, row_base):
    rng = np.random.default_rng(n)
    c = synth.fp16_exact(rng.uniform(0.0, 1.5, n).astype(np.float32))
    c[0] = 0.0
    for eta, dc in ((1e-3, 40.0), (1.0, -100.0), (0.0, 3.0)):
        cd = _dev(c, torch.float16)
        qb.qzo_apply_update_channel(cd, row_base, 11, eta, dc)
        want = oracle.update_channel_scales(c, row_base, 11, eta, dc)
        got = cd.float().cpu().numpy()
        assert np.array_equal(_bits(got), _bits(want)), (eta, dc)
        assert got.min() >= 0


@pytest.mark.parametrize("M,N,K", [(300, 520, 384), (256, 256, 128), (513, 264, 1280)])
def test_codebook_linear_matches_oracle(oracle, M, N, K):
    x, idx, cb, c = synth.codebook_linear_case(M, N, K, seed=M + K)
    xd, cd = _dev(x, torch.bfloat16), _dev(c, torch.float16)
    idxd, cbd = _dev(idx.view(np.int16)), _dev(cb, torch.float16)
    outs = {}
    for sign in (1, -1):
        y = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
        ssq = torch.zeros(1, dtype=torch.float32, device=DEV)
        qb.qzo_codebook_gemm(xd, idxd, cbd, cd, 24, 5, 1e-2, sign, y, ssq)
        ce = oracle.channel_effective_scales(c, 24, 5, sign * np.float32(1e-2))
        ref = oracle.codebook_linear(x, idx, cb, ce)
        got = y.float().cpu().numpy().astype(np.float64)
        rms = math.sqrt((ref ** 2).mean())
        assert (np.abs(got - ref) <= 6e-3 * np.abs(ref) + 1.2e-2 * rms).all(), np.abs(got - ref).max() / rms
        assert abs(float(ssq.item()) - oracle.sumsq_bf16(ref)) <= 5e-3 * oracle.sumsq_bf16(ref)
        outs[sign] = y
    assert not torch.equal(outs[1], outs[-1])
    y0 = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    y1 = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    qb.qzo_codebook_gemm(xd, idxd, cbd, cd, 24, 5, 0.0, 1, y0)
    qb.qzo_codebook_gemm(xd, idxd, cbd, cd, 24, 6, 0.0, -1, y1)
    assert torch.equal(y0, y1)                      # eps = 0: seed and sign are irrelevant


@pytest.mark.parametrize("shape,eta", [
    (dict(arch="llama", n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=520, max_seq=48, batch=3, seq=40), 1e-1),
    # Llama-2-13B widths, one layer, short batch (a smaller step: d carries the losses' noise x 500)
    # more tokens (several token tiles)
    (dict(arch="llama", n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=520, max_seq=48, batch=12, seq=48), 1e-1),
    (dict(synth.SHAPES["llama-2-13b"], n_layers=1, batch=1, seq=16, max_seq=32), 1e-5)],
    ids=["tiny", "tiny-576-tokens", "13b-width"])
def test_codebook_model_step(oracle, shape, eta):
    table = synth.codebook_tensor_table(shape, 31)
    om = oracle.build_codebook_model(shape, table)
    dm = DeviceModel.from_host_codebook(shape, table, DEV)
    assert dm.scales.numel() == qb.qzo_model_scale_count(dict(shape, quant=1)) == om.scales.size
    tok = synth.tokens(shape, 32)
    # final hidden states of one perturbed forward, to twice the oracle's own 16-bit noise floor
    B, S = tok.shape
    se = oracle.perturbed_scales(om, 4, np.float32(1e-3))
    ref_loss, ref_hid = oracle.forward_loss(om, se, tok, act_bf16=True, want_hidden=True)
    _, exact_hid = oracle.forward_loss(om, se, tok, act_bf16=False, want_hidden=True)
    hid = torch.zeros((B * S, shape["d_model"]), dtype=torch.bfloat16, device=DEV)
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    qb.qzo_debug_forward(dm.handle, _dev(tok), 4, 1e-3, 1, dm.workspace(B, S), loss, hid)
    assert abs(loss.item() - ref_loss) <= 2e-2 * abs(ref_loss)
    rms = math.sqrt((ref_hid ** 2).mean())
    err = np.abs(hid.float().cpu().numpy().astype(np.float64) - ref_hid)
    floor_rms = math.sqrt(((exact_hid - ref_hid) ** 2).mean())
    assert math.sqrt((err ** 2).mean()) <= 2 * floor_rms + 2e-3 * rms, (math.sqrt((err ** 2).mean()) / rms, floor_rms / rms)
    assert err.max() <= 2 * np.abs(exact_hid - ref_hid).max() + 2e-2 * rms
    ref = oracle.qzo_step(om, tok, seed=4, eps=1e-3, eta=eta, Cthr=100.0)
    res = qb.read_step_result(dm.step(_dev(tok), 4, 1e-3, eta, 100.0))
    assert res["status"] == 0
    for k in ("loss_plus", "loss_minus"):
        assert abs(res[k] - ref[k]) <= 2e-2 * abs(ref[k]), (k, res[k], ref[k])
    got = dm.scales.float().cpu().numpy()
    assert (np.abs(got - ref["scales"]) <= 2e-2 * np.abs(ref["scales"]) + 1e-6).all()
    assert np.array_equal(_bits(got), _bits(oracle.update_scales(om, 4, eta, res["d_clipped"])))
    print("codebook d gpu", res["d"], "oracle", ref["d"], "changed", float((got != om.scales).mean()))
    dm.close()


# ------------------- joint SPSA on the un-quantized parameters (Sec. 3.2 / 4.1) ----
def _t16_bits(t):
    return t.view(torch.int16).cpu().numpy()


def _host16_bits(a, fmt):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.float16 if fmt == 1 else torch.bfloat16).view(torch.int16).numpy()


def _joint_models(oracle, name):
    if name == "codebook":
        shape = dict(arch="llama", n_layers=2, d_model=256, n_heads=4, d_ffn=512, vocab=520, max_seq=48,
                     batch=3, seq=40)
        table = synth.codebook_tensor_table(shape, 31)
        return shape, oracle.build_codebook_model(shape, table), DeviceModel.from_host_codebook(shape, table, DEV)
    shape, asym = _case(name)
    om, dm = _models(oracle, shape, 1234, **_variant_args(asym))
    return shape, om, dm


@pytest.mark.parametrize("name", ["tiny", "tiny_opt", "few_llama", "tiny+zp", "tiny+nf4", "codebook"])
def test_joint_step_matches_oracle(oracle, name):
    shape, om, dm = _joint_models(oracle, name)
    tok = synth.tokens(shape, 5678)
    tokd = _dev(tok)
    slots = oracle.dense_slots(om)
    master0 = oracle.dense_master(om)
    md = dm.enable_joint()
    assert md.numel() == master0.size and np.array_equal(_bits(md.cpu().numpy()), _bits(master0))
    dev16 = [t for t in dm.tensors if t.dtype in (torch.bfloat16, torch.float16)]
    assert len(dev16) == len(slots)
    seed, eps, eta, eta_u = 3, 1e-3, 1e-5, 1e-4
    # one perturbed pass: the 16-bit tensors it leaves behind are the oracle's, bit for bit
    for sign in (1, -1):
        loss = float(dm.forward_loss(tokd, seed, eps, sign).item())
        pert = oracle.with_dense(om, master0, seed, sign * np.float32(eps))
        for t, (i, first, n, fmt) in zip(dev16, slots):
            assert np.array_equal(_t16_bits(t).reshape(-1), _host16_bits(pert.tensors[i], fmt).reshape(-1)), om.names[i]
        ref_loss = oracle.forward_loss(pert, oracle.perturbed_scales(om, seed, sign * np.float32(eps)), tok)
        assert abs(loss - ref_loss) <= 2e-2 * abs(ref_loss)
    with pytest.raises(qb.QzoError):
        dm.step(tokd, seed, eps, eta, 100.0)                      # plain step refused in joint mode
    ref = oracle.qzo_step_joint(om, master0, tok, seed, eps, eta, eta_u, 100.0)
    res = qb.read_step_result(dm.step_joint(tokd, seed, eps, eta, eta_u, 100.0))
    assert res["status"] == 0
    print(name, "joint d gpu", res["d"], "oracle", ref["d"])
    for k in ("loss_plus", "loss_minus"):
        assert abs(res[k] - ref[k]) <= 2e-2 * abs(ref[k])
    got_s = dm.scales.float().cpu().numpy()
    assert (np.abs(got_s - ref["scales"]) <= 2e-2 * np.abs(ref["scales"]) + 1e-6).all()
    assert np.array_equal(_bits(got_s), _bits(oracle.update_scales(om, seed, eta, res["d_clipped"])))
    # the master: exactly the oracle's update for the d' the device found, and close to the oracle's own
    got_m = md.cpu().numpy()
    assert np.array_equal(_bits(got_m), _bits(oracle.dense_update(master0, 0, seed, eta_u, res["d_clipped"])))
    assert not np.array_equal(got_m, master0)
    assert np.abs(got_m - ref["master"]).max() <= eta_u * abs(res["d_clipped"] - ref["d_clipped"]) * 6 + 1e-7
    # and the 16-bit tensors are back at round16(master)
    for t, (i, first, n, fmt) in zip(dev16, slots):
        assert np.array_equal(_t16_bits(t).reshape(-1), _host16_bits(got_m[first:first + n], fmt))
    dm.close()


@pytest.mark.parametrize("M,N,K,pipe", [(300, 520, 384, 1), (513, 264, 1280, 0), (64, 136, 512, 1),
                                          (300, 520, 384, 2), (513, 264, 1280, 2), (1, 8, 128, 2), (700, 776, 256, 2)])
def test_plain_bf16_gemm_matches_oracle(oracle, M, N, K, pipe):
    rng = np.random.default_rng(M + N + K)
    x = synth.bf16_exact(rng.standard_normal((M, K), dtype=np.float32))
    w = synth.bf16_exact(rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.05))
    y = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    qb.qzo_debug_bf16_gemm(_dev(x, torch.bfloat16), _dev(w, torch.bfloat16), y, pipe)
    ref = oracle.linear(x.astype(np.float64), w)
    err = np.abs(y.float().cpu().numpy() - ref)
    assert (err <= 2e-2 * np.abs(ref) + 2e-2 * math.sqrt(K) * 0.05).all()
    assert err.max() <= 1e-2 * np.abs(ref).max()


def test_plain_bf16_gemm_deferred_stores_ragged_edges(oracle):
    """More output tiles than compute units and a k-loop of 16 k-tiles: the kernel of the expanded route keeps
    the packed output of a workgroup's first tile in registers and stores it during its second tile's k-loop.
    Ragged on both sides (rows past M fall outside the buffer, columns past N are masked per piece).  Checked
    against the oracle, and bit for bit against the register-staged kernel, which sums in the same order."""
    M, N, K = 4400, 3848, 1024
    rng = np.random.default_rng(5)
    x = synth.bf16_exact(rng.standard_normal((M, K), dtype=np.float32))
    w = synth.bf16_exact(rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.05))
    xd, wd = _dev(x, torch.bfloat16), _dev(w, torch.bfloat16)
    guard = 4096
    buf = torch.full((M * N + guard,), 7.0, dtype=torch.bfloat16, device=DEV)
    y = buf[:M * N].view(M, N)
    qb.qzo_debug_bf16_gemm(xd, wd, y, 2)
    y1 = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    qb.qzo_debug_bf16_gemm(xd, wd, y1, 1)
    assert torch.equal(y, y1)
    assert bool((buf[M * N:] == 7.0).all())                      # nothing written past the last row
    ref = oracle.linear(x.astype(np.float64), w)
    err = np.abs(y.float().cpu().numpy() - ref)
    assert (err <= 2e-2 * np.abs(ref) + 2e-2 * math.sqrt(K) * 0.05).all()


# ------------------------------------- NormalFloat-4 blocks (the quantizer of Sec. 4.3) ----
@pytest.mark.parametrize("N,K,row_base", [(24, 384, 0), (264, 1280, 77), (8, 128, 5), (40, 11008, 3)])
def test_nf4_perturbed_scales_and_matrix_bit_exact(oracle, N, K, row_base):
    rng = np.random.default_rng(N + K)
    w = (rng.standard_normal((N, K)) * 0.03).astype(np.float32)
    qp, s = oracle.nf4_quantize(w)
    q, sd = _dev(qp), _dev(s, torch.bfloat16)
    for sign in (1, -1):
        se = torch.zeros((N, K // 64), dtype=torch.float32, device=DEV)
        out = torch.zeros((N, K), dtype=torch.bfloat16, device=DEV)
        qb.qzo_nf4_expand(q, sd, row_base, 99, 1e-3, sign, se, out)
        want_se = oracle.effective_scales(s, row_base, 99, sign * np.float32(1e-3)).astype(np.float32)
        assert np.array_equal(_bits(se.cpu().numpy()), _bits(want_se))
        want = oracle.dequant_nf4(qp, s, 99, row_base, sign * np.float32(1e-3), to_bf16=True)
        assert np.array_equal(_bits(out.float().cpu().numpy()), _bits(want))


@pytest.mark.parametrize("M,N,K", [(300, 520, 384), (256, 264, 1280), (16, 136, 512), (513, 256, 128)])
def test_nf4_linear_matches_oracle(oracle, M, N, K):
    rng = np.random.default_rng(M * 7 + N + K)
    x = synth.bf16_exact(rng.standard_normal((M, K), dtype=np.float32))
    w = (rng.standard_normal((N, K)) * 0.03).astype(np.float32)
    qp, s = oracle.nf4_quantize(w)
    scratch = torch.empty(qb.qzo_nf4_scratch_bytes(N, K), dtype=torch.uint8, device=DEV)
    for sign in (1, -1):
        y = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
        qb.qzo_nf4_gemm(_dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16), 11, 31, 1e-3, sign, y, scratch)
        se = oracle.effective_scales(s, 11, 31, sign * np.float32(1e-3))
        ref = oracle.qlinear_nf4(x.astype(np.float64), qp, se)
        err = np.abs(y.float().cpu().numpy() - ref)
        scale = math.sqrt(K) * 0.03
        assert (err <= 2e-2 * np.abs(ref) + 2e-2 * scale).all()
        assert err.max() <= 1e-2 * np.abs(ref).max() + 4e-3 * scale
    with pytest.raises(qb.QzoError):
        qb.qzo_nf4_gemm(_dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16), 11, 31, 1e-3, 1, y, scratch[:256])


@pytest.mark.parametrize("name", ["many_llama", "many_opt+zp", "long_llama", "long_llama+zp"])
def test_int4_expand_then_multiply_equals_the_fused_path(oracle, name):
    """Both routes form the same bf16 weights (one rounding of scale x integer) and accumulate each
    output over k in the same order, so losses and hidden states agree bit for bit.  (d_ffn = 256 keeps
    every K at 256, too short for the fused kernel's split-K, which would change the order.)
    On the expanded route the rotary embedding is applied by the qkv GEMM's epilogue (heads of 64 in
    many_llama, heads of 128 with the permuted weight rows in long_llama), on the fused route by its own
    kernel: the same arithmetic on the same bf16 values, so this equality covers it too."""
    base, asym = _case(name)
    shape = dict(base, d_ffn=256)
    om, dm = _models(oracle, shape, 1234, 4.0, **_variant_args(asym))
    tok = synth.tokens(shape, 5678)
    B, S = tok.shape
    outs, ws_bytes = [], []
    for mode in (2, 1):
        dm.set_int4_path(mode)                   # the workspace layout depends on the route
        ws_bytes.append(qb.qzo_workspace_bytes(dm.handle, B, S))
        hid = torch.zeros((B * S, shape["d_model"]), dtype=torch.bfloat16, device=DEV)
        loss = torch.zeros(1, dtype=torch.float32, device=DEV)
        qb.qzo_debug_forward(dm.handle, _dev(tok), 9, 1e-3, -1, dm.workspace(B, S), loss, hid)
        outs.append((float(loss.item()), hid.float().cpu().numpy()))
    assert outs[0][0] == outs[1][0]
    assert np.array_equal(outs[0][1], outs[1][1])
    # the expanded route keeps one linear in bf16 and every perturbed scale in fp32 in the workspace
    # (the fused route's workspace is not smaller any more: at this token count its step stacks both passes)
    n_scales = qb.qzo_model_scale_count(dict(shape, quant=2) if asym is True else shape)
    largest = max(N * K for _, N, K in synth.quantized_linears(shape))
    assert ws_bytes[0] >= 4 * n_scales + 2 * largest + 2 * B * S * shape["d_model"]
    dm.close()


def test_full_size_token_count_sampled_sequence_matches_oracle(oracle):
    """The benchmark's launch configuration (16 x 512 tokens, the default route: expansion, plain GEMM at
    32 token tiles, RoPE in the qkv epilogue at positions up to 511, attention over 8 key tiles) through
    one decoder layer at Llama-2-7B widths, checked on a sample the oracle can afford: a decoder treats
    the sequences of a batch independently, so the oracle runs sequence 11 alone and its final hidden
    states are compared with rows 11*512 .. 12*512-1 of the batch's."""
    shape = dict(synth.SHAPES["llama-2-7b"], n_layers=1, vocab=1000)
    om, dm = _models(oracle, shape, 77)
    tok = synth.tokens(shape, 78)
    B, S = tok.shape
    assert (B, S) == (16, 512)
    hid = torch.zeros((B * S, shape["d_model"]), dtype=torch.bfloat16, device=DEV)
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    qb.qzo_debug_forward(dm.handle, _dev(tok), 3, 1e-3, 1, dm.workspace(B, S), loss, hid)
    b = 11
    se = oracle.perturbed_scales(om, 3, np.float32(1e-3))
    _, ref_hid = oracle.forward_loss(om, se, tok[b:b + 1], act_bf16=True, want_hidden=True)
    _, exact_hid = oracle.forward_loss(om, se, tok[b:b + 1], act_bf16=False, want_hidden=True)
    got = hid[b * S:(b + 1) * S].float().cpu().numpy().astype(np.float64)
    rms = math.sqrt((ref_hid ** 2).mean())
    err = np.abs(got - ref_hid)
    floor_rms = math.sqrt(((exact_hid - ref_hid) ** 2).mean())
    print("hidden rms err", math.sqrt((err ** 2).mean()) / rms, "floor", floor_rms / rms)
    assert math.isfinite(loss.item())
    assert math.sqrt((err ** 2).mean()) <= 2 * floor_rms + 2e-3 * rms
    assert err.max() <= 2 * np.abs(exact_hid - ref_hid).max() + 2e-2 * rms
    dm.close()


def test_llama_13b_width_column_tail_split(oracle):
    """8 x 512 tokens through one decoder layer at Llama-2-13B widths: the o and down projections have
    16 x 20 = 320 output tiles, a quarter more than one round of the chip, so their launch is cut in two: the
    first 4096 columns as they are, the last 1024 along K in four slices whose partial sums a reduction adds
    (bias-free, residual epilogue, K = 5120 and 13824).  Fused and expanded routes must agree bit for bit, and
    one sequence of the batch must match the oracle run on that sequence alone."""
    shape = dict(synth.SHAPES["llama-2-13b"], n_layers=1, vocab=1000)
    om, dm = _models(oracle, shape, 55)
    tok = synth.tokens(shape, 56)
    B, S = tok.shape
    assert (B, S) == (8, 512)
    outs = []
    for mode in (2, 1):
        dm.set_int4_path(mode)
        hid = torch.zeros((B * S, shape["d_model"]), dtype=torch.bfloat16, device=DEV)
        loss = torch.zeros(1, dtype=torch.float32, device=DEV)
        qb.qzo_debug_forward(dm.handle, _dev(tok), 3, 1e-3, 1, dm.workspace(B, S), loss, hid)
        outs.append((float(loss.item()), hid))
    assert math.isfinite(outs[0][0]) and outs[0][0] == outs[1][0]
    assert torch.equal(outs[0][1], outs[1][1])
    b = 5
    se = oracle.perturbed_scales(om, 3, np.float32(1e-3))
    _, ref_hid = oracle.forward_loss(om, se, tok[b:b + 1], act_bf16=True, want_hidden=True)
    _, exact_hid = oracle.forward_loss(om, se, tok[b:b + 1], act_bf16=False, want_hidden=True)
    got = outs[0][1][b * S:(b + 1) * S].float().cpu().numpy().astype(np.float64)
    rms = math.sqrt((ref_hid ** 2).mean())
    err = np.abs(got - ref_hid)
    floor_rms = math.sqrt(((exact_hid - ref_hid) ** 2).mean())
    assert math.sqrt((err ** 2).mean()) <= 2 * floor_rms + 2e-3 * rms
    assert err.max() <= 2 * np.abs(exact_hid - ref_hid).max() + 2e-2 * rms
    dm.close()


def test_opt_width_token_count_routes_agree_bit_for_bit():
    """16 x 256 tokens through one decoder layer at OPT-1.3B widths: on the expanded route the qkv (bias) and
    fc1 (bias + ReLU) GEMMs have more output tiles than compute units, so the one-wavefront-per-SIMD kernel
    defers a tile's stores into the next tile's k-loop with those epilogues; the narrow o and fc2 projections
    are cut along K.  Loss and hidden states must equal the fused route's bit for bit."""
    shape = dict(synth.SHAPES["opt-1.3b"], n_layers=1, vocab=2000)
    dm = DeviceModel.synthetic(shape, seed=8, device=DEV)
    B, S = shape["batch"], shape["seq"]
    tok = _dev(synth.tokens(shape, 9))
    outs = []
    for mode in (2, 1):
        dm.set_int4_path(mode)
        hid = torch.zeros((B * S, shape["d_model"]), dtype=torch.bfloat16, device=DEV)
        loss = torch.zeros(1, dtype=torch.float32, device=DEV)
        qb.qzo_debug_forward(dm.handle, tok, 4, 1e-3, 1, dm.workspace(B, S), loss, hid)
        outs.append((float(loss.item()), hid))
    assert math.isfinite(outs[0][0]) and outs[0][0] == outs[1][0]
    assert torch.equal(outs[0][1], outs[1][1])
    dm.close()


@pytest.mark.parametrize("S", [256, 300])
def test_attention_per_head_walk_head_size_64_sampled_sequence_matches_oracle(oracle, S):
    """16 sequences x 32 heads of 64 features fill the chip twice over, so the attention workgroups walk the
    query blocks of their (batch, head) themselves: one workgroup the 2 blocks at 256 positions, two
    workgroups in snake order the 3 at 300 (the last one ragged, 44 rows).
    One decoder layer at OPT-1.3B widths (LayerNorm, bias, ReLU, learned positions); the oracle runs one
    sequence of the batch alone, whose final hidden states are compared with the batch's rows."""
    shape = dict(synth.SHAPES["opt-1.3b"], n_layers=1, vocab=1000, max_seq=S, seq=S)
    _walk_case(oracle, shape, 16, S, 6)


def test_attention_shared_walk_five_blocks_odd_pair_count_matches_oracle(oracle):
    """86 sequences x 6 heads of 64 features: 516 (batch, head) pairs, not a multiple of the 8 XCDs (the launch
    index is then not remapped), 640 positions = 5 query blocks, which two workgroups share as 4, 1, 0 | 3, 2.
    One decoder layer (OPT kind, d_model 384); a late sequence of the batch against the oracle."""
    S = 640
    shape = dict(synth.SHAPES["tiny_opt"], n_layers=1, d_model=384, n_heads=6, d_ffn=1024, vocab=1000,
                 max_seq=S, seq=S, batch=86)
    _walk_case(oracle, shape, 86, S, 85)


def _walk_case(oracle, shape, n_seq, S, b):
    om, dm = _models(oracle, shape, 91)
    tok = synth.tokens(shape, 92)
    B = tok.shape[0]
    assert tok.shape == (n_seq, S)
    hid = torch.zeros((B * S, shape["d_model"]), dtype=torch.bfloat16, device=DEV)
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    qb.qzo_debug_forward(dm.handle, _dev(tok), 5, 1e-3, -1, dm.workspace(B, S), loss, hid)
    se = oracle.perturbed_scales(om, 5, np.float32(-1e-3))
    _, ref_hid = oracle.forward_loss(om, se, tok[b:b + 1], act_bf16=True, want_hidden=True)
    _, exact_hid = oracle.forward_loss(om, se, tok[b:b + 1], act_bf16=False, want_hidden=True)
    got = hid[b * S:(b + 1) * S].float().cpu().numpy().astype(np.float64)
    rms = math.sqrt((ref_hid ** 2).mean())
    err = np.abs(got - ref_hid)
    floor_rms = math.sqrt(((exact_hid - ref_hid) ** 2).mean())
    assert math.isfinite(loss.item())
    assert math.sqrt((err ** 2).mean()) <= 2 * floor_rms + 2e-3 * rms
    assert err.max() <= 2 * np.abs(exact_hid - ref_hid).max() + 2e-2 * rms
    dm.close()


def test_full_size_token_count_one_layer_routes_agree_bit_for_bit():
    """The benchmark's token count (16 x 512) through one decoder layer at Llama-2-7B widths, once on the
    route the benchmark times (perturbed scales of the arena, expanded bf16 weights, plain GEMM with the
    rotary embedding in the qkv epilogue: 6 / 2 / 10.75 / 2 rounds of output tiles per CU) and once on
    the fused dequantizing GEMM with the separate RoPE kernel: the same bf16 weights, the same order of
    the sums, so loss and final hidden states agree bit for bit.  (The fused route is the one that the
    smaller cases compare with the oracle element by element.)"""
    shape = dict(synth.SHAPES["llama-2-7b"], n_layers=1, vocab=2000)
    dm = DeviceModel.synthetic(shape, seed=5, device=DEV)
    B, S = shape["batch"], shape["seq"]
    tok = _dev(synth.tokens(shape, 6))
    outs = []
    for mode in (2, 1):
        dm.set_int4_path(mode)
        hid = torch.zeros((B * S, shape["d_model"]), dtype=torch.bfloat16, device=DEV)
        loss = torch.zeros(1, dtype=torch.float32, device=DEV)
        qb.qzo_debug_forward(dm.handle, tok, 9, 1e-3, -1, dm.workspace(B, S), loss, hid)
        outs.append((float(loss.item()), hid))
    assert math.isfinite(outs[0][0]) and outs[0][0] == outs[1][0]
    assert torch.equal(outs[0][1], outs[1][1])
    dm.close()


@pytest.mark.parametrize("N,K,row_base,with_zp", [(24, 384, 0, False), (40, 1024 + 128, 77, True), (8, 128, 5, False),
                                                  (16, 11008, 3, True)])
def test_int4_expanded_matrix_bit_exact(oracle, N, K, row_base, with_zp):
    rng = np.random.default_rng(N + K)
    qp = rng.integers(0, 256, (N, K // 2), dtype=np.uint8)
    s = synth.bf16_exact(rng.uniform(0.002, 0.02, (N, K // 128)).astype(np.float32))
    zp = rng.integers(0, 16, (N, K // 128), dtype=np.uint8) if with_zp else None
    for sign in (1, -1):
        se = torch.zeros((N, K // 128), dtype=torch.float32, device=DEV)
        out = torch.zeros((N, K), dtype=torch.bfloat16, device=DEV)
        qb.qzo_int4_expand(_dev(qp), _dev(s, torch.bfloat16), _dev(zp) if with_zp else None, row_base, 99, 1e-3,
                           sign, se, out)     # no activation reordering
        e = sign * np.float32(1e-3)
        assert np.array_equal(_bits(se.cpu().numpy()),
                              _bits(oracle.effective_scales(s, row_base, 99, e).astype(np.float32)))
        want = (oracle.dequant_zp(qp, s, zp, 99, row_base, e, to_bf16=True) if with_zp
                else oracle.dequant(qp, s, 99, row_base, e, to_bf16=True))
        assert np.array_equal(_bits(out.float().cpu().numpy()), _bits(want))


@pytest.mark.parametrize("M,N,K", [(300, 520, 384), (64, 136, 1280)])
def test_activation_reordering_matrix_bit_exact_and_linear(oracle, M, N, K):
    rng = np.random.default_rng(M + N + K)
    G = K // 128
    qp = rng.integers(0, 256, (N, K // 2), dtype=np.uint8)
    s = synth.bf16_exact(rng.uniform(0.002, 0.02, (N, G)).astype(np.float32))
    zp = rng.integers(0, 16, (N, G), dtype=np.uint8)
    g_idx = rng.permutation(np.arange(K) // 128).astype(np.int32)      # every group keeps 128 columns
    x = synth.bf16_exact(rng.standard_normal((M, K), dtype=np.float32))
    gd = _dev(g_idx)
    se = torch.zeros((N, G), dtype=torch.float32, device=DEV)
    out = torch.zeros((N, K), dtype=torch.bfloat16, device=DEV)
    qb.qzo_int4_expand(_dev(qp), _dev(s, torch.bfloat16), _dev(zp), 11, 31, 1e-3, -1, se, out, g_idx=gd)
    want = oracle.dequant_zp(qp, s, zp, 31, 11, -np.float32(1e-3), to_bf16=True, g_idx=g_idx)
    assert np.array_equal(_bits(out.float().cpu().numpy()), _bits(want))
    scratch = torch.empty(qb.qzo_int4_scratch_bytes(N, K), dtype=torch.uint8, device=DEV)
    y = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
    qb.qzo_int4_gemm_expanded(_dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16), _dev(zp), gd, 11, 31,
                              1e-3, -1, y, scratch)
    ref = oracle.linear(x.astype(np.float64), oracle.dequant_zp(qp, s, zp, 31, 11, -np.float32(1e-3), g_idx=g_idx))
    err = np.abs(y.float().cpu().numpy() - ref)
    scale = math.sqrt(K) * 0.011 * 4.6
    assert (err <= 2e-2 * np.abs(ref) + 2e-2 * scale).all() and err.max() <= 1e-2 * np.abs(ref).max() + 4e-3 * scale
    # without a group index the entry point is the plain zero-point linear
    qb.qzo_int4_gemm_expanded(_dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16), _dev(zp), None, 11, 31,
                              1e-3, -1, y, scratch)
    y2 = torch.zeros_like(y)
    qb.qzo_dequant_gemm_zp(_dev(x, torch.bfloat16), _dev(qp), _dev(s, torch.bfloat16), _dev(zp), 11, 31, 1e-3, -1, y2)
    if M > 64:          # the tile kernel accumulates in the same order; the few-token kernel does not
        assert torch.equal(y, y2)


@pytest.mark.parametrize("name", ["tiny", "few_llama"])
def test_step_replays_from_a_captured_graph(oracle, name):
    """qzo_step allocates nothing and never synchronises, so after one eager call (which sets the
    kernels' LDS attributes) it can be captured into a HIP graph.  Every replay, with eager work and
    synchronisations in between, gives the eager step's scalars; a replay with eta > 0 leaves the
    eager step's scales."""
    shape, _ = _case(name)
    om, dm = _models(oracle, shape, 1234)
    tokd = _dev(synth.tokens(shape, 5678))
    start = dm.scales.clone()
    eager0 = qb.read_step_result(dm.step(tokd, 7, 1e-3, 0.0, 100.0))          # eta = 0: scales untouched
    dm.step(tokd, 7, 1e-3, 1e-5, 100.0)
    torch.cuda.synchronize()
    eager_scales = dm.scales.clone()
    dm.scales.copy_(start)
    side = torch.cuda.Stream()
    graphs = {}
    for eta in (0.0, 1e-5):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            dm.step(tokd, 7, 1e-3, eta, 100.0)
        graphs[eta] = g
    for rep in range(3):
        graphs[0.0].replay()
        torch.cuda.synchronize()
        got = qb.read_step_result(dm.result)
        assert got == eager0, (rep, got, eager0)
        assert torch.equal(dm.scales, start)
        # eager work between the replays
        again = qb.read_step_result(dm.step(tokd, 7, 1e-3, 0.0, 100.0))
        assert again == eager0
    graphs[1e-5].replay()
    torch.cuda.synchronize()
    assert torch.equal(dm.scales, eager_scales) and not torch.equal(dm.scales, start)
    dm.close()
