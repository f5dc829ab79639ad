// C ABI of the QZO hot path (include/qzo.h): argument checking, the decoder
// forward as a sequence of kernel launches on the caller's stream, and the
// step of Algorithm 1 (two perturbed forwards, SPSA scalar + clipping, update).
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>
#include "../../include/qzo.h"
#include "qzo_kernels.hpp"
#include <algorithm>

using namespace qzo;

namespace {

thread_local std::string g_err;

qzo_status fail(qzo_status st, const std::string& msg) {
  g_err = msg;
  return st;
}
qzo_status hip_fail(hipError_t e, const char* what) {
  return fail(QZO_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}
#define QZO_HIP(call)                                         \
  do {                                                        \
    hipError_t e_ = (call);                                   \
    if (e_ != hipSuccess) return hip_fail(e_, #call);         \
  } while (0)

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
// The GEMM kernels address X [M,K], a bf16 W [N,K] and Y [M,N] with 32-bit byte offsets.
bool bf16_gemm_fits(uint64_t M, uint64_t N, uint64_t K) {
  return M * K * 2 < (1ull << 31) && N * K * 2 < (1ull << 31) && M * N * 2 < (1ull << 31);
}
uint64_t up256(uint64_t x) { return (x + 255u) & ~uint64_t(255); }

struct Linear {           // one quantized linear of a layer
  uint32_t N, K;
  uint64_t s_off;         // first scale within the layer's arena slice
  uint32_t row_base;      // first noise row within the layer
};

struct Workspace {
  unsigned char *h, *a, *qkv, *att, *ff, *act;
  float *ce_part, *tgt, *rowloss, *losses, *skinny;
  float *xs_a, *xs_act;     // few-token path: block sums of the norm output and of the MLP's hidden activation
  float* split;             // K-slice partial sums of the int4 tile kernel (too few tiles for the chip)
  unsigned char* wexp;      // one linear's expanded bf16 weights (expand-then-multiply paths)
  float* se;                // expand-then-multiply of int4 / NormalFloat-4: every perturbed scale of the model, fp32
  float* rope;              // Llama: (cos, sin) of every (position < seq, pair of the head), rebuilt by every pass
  uint64_t total;
};

}  // namespace

struct qzo_model {
  qzo_model_config cfg;
  std::vector<qzo_buf> T;
  void* arena;
  uint64_t n_scales;
  Linear lin[4];
  uint64_t scales_per_layer;
  uint32_t rows_per_layer;
  UpdPlan plan;
  uint32_t tensors_per_layer, first_layer_tensor;
  // int4 linears: 0 = expand-then-multiply from expand_min_m_int4(N, K) tokens on, 1 = always the
  // fused kernel, 2 = always expand-then-multiply
  int int4_path = 0;
  // joint SPSA on the un-quantized parameters (off until qzo_model_enable_joint)
  float* dense_master = nullptr;       // caller-owned fp32 [n_dense]
  uint64_t n_dense = 0;
  DenseSeg* dense_segs = nullptr;      // device, caller-owned (qzo_model_enable_joint's table_dev)
  uint32_t n_dense_segs = 0;
};

namespace {

qzo_status check_cfg(const qzo_model_config* c) {
  if (!c) return fail(QZO_ERR_ARG, "config is null");
  if (c->struct_size != sizeof(qzo_model_config))
    return fail(QZO_ERR_ARG, "config.struct_size does not match this library");
  if (c->arch > 1) return fail(QZO_ERR_ARG, "config.arch must be 0 (Llama) or 1 (OPT)");
  if (c->quant > 3)
    return fail(QZO_ERR_UNSUPPORTED,
                "quant must be 0 (int4 group scales), 1 (codebook), 2 (int4 with zero-points) or 3 (NormalFloat-4)");
  if (c->quant == 1 && c->arch != 0)
    return fail(QZO_ERR_UNSUPPORTED, "the codebook variant is built for the Llama family only");
  if (c->quant == 3 ? c->group_size != 64 : c->group_size != 128)
    return fail(QZO_ERR_SHAPE, "group_size must be 128 (64 for the NormalFloat-4 format)");
  if (!c->n_layers || !c->d_model || !c->n_heads || !c->d_ffn || !c->vocab || !c->max_seq)
    return fail(QZO_ERR_SHAPE, "zero dimension in config");
  if (c->d_model % 128 || c->d_ffn % 128)
    return fail(QZO_ERR_SHAPE, "d_model and d_ffn must be multiples of 128");
  if (c->d_model % c->n_heads) return fail(QZO_ERR_SHAPE, "d_model not divisible by n_heads");
  uint32_t dh = c->d_model / c->n_heads;
  if (dh != 64 && dh != 128) return fail(QZO_ERR_SHAPE, "head size must be 64 or 128");
  if (c->scale_fp16 > 1 || c->act_order > 1) return fail(QZO_ERR_ARG, "scale_fp16 and act_order must be 0 or 1");
  if (c->scale_fp16 && c->quant != 0 && c->quant != 2)
    return fail(QZO_ERR_UNSUPPORTED, "fp16 group scales are built for the int4 formats (quant 0 and 2)");
  if (c->act_order && c->quant != 2)
    return fail(QZO_ERR_UNSUPPORTED, "a group index per column belongs to the zero-point format (quant 2)");
  return QZO_OK;
}

void layer_linears(const qzo_model_config& c, Linear lin[4]) {
  const uint32_t d = c.d_model, F = c.d_ffn;
  const uint32_t N[4] = {3 * d, d, c.arch == 0 ? 2 * F : F, d};
  const uint32_t K[4] = {d, d, d, F};
  uint64_t off = 0;
  uint32_t row = 0;
  for (int i = 0; i < 4; ++i) {
    lin[i] = {N[i], K[i], off, row};
    off += (uint64_t)N[i] * (K[i] / c.group_size);
    row += N[i];
  }
}

// Merge a layer's consecutive linears with equal groups-per-row into update segments.
qzo_status build_plan(const Linear* lin, int n_lin, uint32_t n_layers, UpdPlan& p, uint32_t group = 128,
                      uint32_t scale_fp16 = 0) {
  std::memset(&p, 0, sizeof(p));
  p.fp16 = scale_fp16;
  uint32_t wg = 0;
  for (int i = 0; i < n_lin; ++i) {
    const uint32_t G = lin[i].K / group;
    if (p.n_seg && p.seg[p.n_seg - 1].G == G) {
      p.seg[p.n_seg - 1].rows += lin[i].N;
    } else {
      if (lin[i].s_off > 0xffffffffull) return fail(QZO_ERR_SHAPE, "layer has too many scales");
      p.seg[p.n_seg++] = {(uint32_t)lin[i].s_off, lin[i].N, G, lin[i].row_base, 0};
    }
    p.layer_stride = lin[i].s_off + (uint64_t)lin[i].N * G;
    p.rows_per_layer = lin[i].row_base + lin[i].N;
  }
  for (uint32_t i = 0; i < p.n_seg; ++i) {
    const uint64_t units = (uint64_t)p.seg[i].rows * ((p.seg[i].G + 7) / 8);
    if (units >= (1u << 24)) return fail(QZO_ERR_SHAPE, "update segment exceeds 2^24 counters");
    p.seg[i].first_wg = wg;
    wg += (uint32_t)((units + 255) / 256);
  }
  p.wgs_per_layer = wg;
  p.n_layers = n_layers;
  return QZO_OK;
}

// Bytes and kind (0: bf16, 1: fp16, 2: packed integers) of every tensor of the model table.
void table_layout(const qzo_model_config& c, std::vector<uint64_t>& need, std::vector<uint8_t>& kind) {
  const bool llama = c.arch == 0, codebook = c.quant == 1, asym = c.quant == 2;
  const uint64_t d = c.d_model, F = c.d_ffn, V = c.vocab;
  auto b16 = [&](uint64_t n) { need.push_back(n * 2); kind.push_back(0); };
  auto packed = [&](uint64_t bytes) { need.push_back(bytes); kind.push_back(2); };
  b16(V * d);
  if (!llama) b16((uint64_t)c.max_seq * d);
  // a packed weight [N,K/2]; with zero-points, followed by its uint8 [N,K/128] tensor;
  // codebook variant: uint16 codes [N,K/8], then the linear's fp16 [65536,8] codebook
  auto weight = [&](uint64_t N, uint64_t K) {
    if (codebook) {
      packed(N * K / 4);
      need.push_back(65536 * 16); kind.push_back(1);
      return;
    }
    packed(N * K / 2);
    if (asym) packed(N * K / 128);
    if (asym && c.act_order) packed(K * 4);       // int32 group index of every input column
  };
  for (uint32_t l = 0; l < c.n_layers; ++l) {
    if (llama) {
      b16(d); weight(3 * d, d); weight(d, d);
      b16(d); weight(2 * F, d); weight(d, F);
    } else {
      b16(d); b16(d);
      weight(3 * d, d); b16(3 * d); weight(d, d); b16(d);
      b16(d); b16(d);
      weight(F, d); b16(F); weight(d, F); b16(d);
    }
  }
  b16(d);
  if (!llama) b16(d);
  b16(V * d);
}

// Whether qzo_step runs its two perturbed passes as one forward over 2 * batch sequences.  With at
// most 32 tokens the few-token kernel reads the int4 weights once for both.  Beyond the few-token
// kernel's range and as long as the fused kernel serves (at most 4096 tokens per pass), a launch of
// the tile kernel holds both passes' token tiles, the second pass's with -eps: twice the tiles per
// launch for a chip that such token counts do not fill, half the launches.  The second pass starts
// on a tile boundary (stacked_pass_stride); the rows in between are padding (zeros at the embedding,
// never read back).
bool passes_stacked(const qzo_model* m, uint64_t M1) {
  const qzo_model_config& c = m->cfg;
  if (!(c.quant == 0 || c.quant == 2) || m->dense_master || c.act_order) return false;
  if (M1 <= SKINNY_MAX_M_DUAL) return true;
  if (M1 <= SKINNY_MAX_M || M1 > STACK_TILE_MAX_M || m->int4_path == 2) return false;
  // Stacked, the fused kernel stays ahead of expand-then-multiply for a fifth more tokens than the
  // break-even of separate passes (7B widths: 72.2 against 74.9 ms per step at 2560 tokens, 83.8
  // against 85.0 at 3072, 103.5 against 100.1 at 4096).
  if (m->int4_path == 0)
    for (int i = 0; i < 4; ++i)
      if (M1 * 5 >= (uint64_t)expand_min_m_int4(m->lin[i].N, m->lin[i].K) * 6) return false;
  return true;
}
// Row at which the second pass of a stacked forward starts.
uint64_t stacked_pass_stride(uint64_t M1) { return M1 <= SKINNY_MAX_M_DUAL ? M1 : (M1 + 255) / 256 * 256; }

Workspace carve(const qzo_model* m, uint32_t batch, uint32_t seq, void* base) {
  const qzo_model_config& c = m->cfg;
  const uint64_t M1 = (uint64_t)batch * seq;
  const bool int4 = c.quant == 0 || c.quant == 2;
  const bool stack = passes_stacked(m, M1);
  const uint64_t M = stack ? stacked_pass_stride(M1) + M1 : M1, d = c.d_model, F = c.d_ffn;
  const uint64_t n_slices = ((c.vocab + 255) / 256) * 4;
  Workspace w;
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) {
    unsigned char* p = base ? (unsigned char*)base + off : nullptr;
    off += up256(bytes);
    return p;
  };
  w.h = take(M * d * 2);
  w.a = take(M * d * 2);
  w.qkv = take(M * 3 * d * 2);
  w.att = take(M * d * 2);
  w.ff = take(c.arch == 0 ? 0 : M * F * 2);     // Llama: SwiGLU is folded into the gate/up GEMM
  w.act = take(c.arch == 0 ? M * F * 2 : 0);
  w.ce_part = (float*)take(M * n_slices * 8);
  w.tgt = (float*)take(M * 4);
  w.rowloss = (float*)take(M * 4);
  w.losses = (float*)take(256);
  // few-token path of the int4 GEMM: fp32 partial sums of the K slices of the largest linear
  uint64_t sk = 0;
  if (M1 <= SKINNY_MAX_M && int4 && !c.act_order)
    for (int i = 0; i < 4; ++i)
      sk = std::max<uint64_t>(sk, skinny_ws_floats((uint32_t)M, m->lin[i].N, m->lin[i].K));
  w.skinny = (float*)take(sk * 4);
  if (sk == 0) w.skinny = nullptr;
  w.xs_a = sk ? (float*)take((d / 128) * M * 4) : nullptr;
  w.xs_act = sk ? (float*)take((F / 128) * M * 4) : nullptr;
  // more tokens than that but still too few output tiles for the chip: split-K partial sums
  uint64_t sp = 0;
  if ((M1 > SKINNY_MAX_M && int4) || c.act_order || c.quant == 3 || (c.quant == 1 && M1 >= EXPAND_MIN_M_CODEBOOK))
    for (int i = 0; i < 4; ++i) {
      sp = std::max<uint64_t>(sp, tile_split_ws_floats((uint32_t)M, m->lin[i].N, m->lin[i].K));
      // a single pass (qzo_forward_loss) of a batch whose step stacks its two passes
      if (stack) sp = std::max<uint64_t>(sp, tile_split_ws_floats((uint32_t)M1, m->lin[i].N, m->lin[i].K));
    }
  w.split = (float*)take(sp * 4);
  if (sp == 0) w.split = nullptr;
  // codebook variant with many tokens: the largest linear written out as bf16
  // and the NormalFloat-4 format at any token count (with its perturbed block scales, fp32)
  uint64_t ex = 0, sx = 0;
  for (int i = 0; i < 4; ++i) {
    const bool expanded = c.quant == 3 || c.act_order || (c.quant == 1 && M1 >= EXPAND_MIN_M_CODEBOOK) ||
                          (int4 && m->int4_path != 1 && !stack &&
                           (m->int4_path == 2 || M1 >= expand_min_m_int4(m->lin[i].N, m->lin[i].K)));
    if (expanded) ex = std::max<uint64_t>(ex, (uint64_t)m->lin[i].N * m->lin[i].K * 2);
  }
  if (ex && c.quant != 1) sx = m->n_scales * 4;     // every perturbed scale of the model, fp32
  w.wexp = take(ex);
  if (ex == 0) w.wexp = nullptr;
  w.se = (float*)take(sx);
  if (sx == 0) w.se = nullptr;
  w.rope = c.arch == 0 ? (float*)take((uint64_t)seq * (c.d_model / c.n_heads / 2) * 8) : nullptr;
  w.total = off;
  return w;
}

qzo_status check_batch(const qzo_model* m, const void* tok, uint32_t batch, uint32_t seq,
                       const void* ws, uint64_t ws_bytes) {
  if (!m) return fail(QZO_ERR_ARG, "model is null");
  if (!tok || !ws) return fail(QZO_ERR_ARG, "tokens or workspace is null");
  if (!aligned16(tok) || !aligned16(ws)) return fail(QZO_ERR_ALIGN, "tokens/workspace not 16-byte aligned");
  if (batch == 0 || seq < 2) return fail(QZO_ERR_SHAPE, "need batch >= 1 and seq >= 2");
  if (seq > m->cfg.max_seq) return fail(QZO_ERR_SHAPE, "seq exceeds max_seq");
  if ((uint64_t)batch * seq > 0x7fffffffull) return fail(QZO_ERR_SHAPE, "batch*seq too large");
  {
    // the kernels address every operand with 32-bit byte offsets: tokens x widest tensor row, in
    // bf16, must stay below 2^31 bytes (stacked passes count twice)
    const qzo_model_config& c = m->cfg;
    const uint64_t M1 = (uint64_t)batch * seq +
                        (passes_stacked(m, (uint64_t)batch * seq) ? stacked_pass_stride((uint64_t)batch * seq) : 0);
    const uint64_t widest = std::max<uint64_t>({3ull * c.d_model, (c.arch == 0 ? 2ull : 1ull) * c.d_ffn});
    if (M1 * widest * 2 >= (1ull << 31))
      return fail(QZO_ERR_SHAPE, "batch*seq too large for this model: an activation tensor would exceed 2^31 bytes");
  }
  Workspace w = carve(m, batch, seq, nullptr);
  if (ws_bytes < w.total) return fail(QZO_ERR_WORKSPACE, "workspace smaller than qzo_workspace_bytes");
  return QZO_OK;
}

// Optional per-kernel-class timing with HIP events recorded on the caller's
// stream around each launch (qzo_profile_begin / qzo_profile_collect).
struct ProfRec { hipEvent_t a, b; uint32_t kind; double work; };
struct Profiler {
  bool on = false;
  std::vector<ProfRec> pool;
  size_t used = 0;
  uint32_t stride = 1;          // every stride-th launch of a class is bracketed
  uint32_t seen[8] = {};
} g_prof;

struct ProfScope {
  ProfRec* r = nullptr;
  hipStream_t st;
  ProfScope(uint32_t kind, double work, hipStream_t s) : st(s) {
    if (!g_prof.on || g_prof.used >= g_prof.pool.size()) return;
    if (g_prof.seen[kind & 7u]++ % g_prof.stride) return;
    r = &g_prof.pool[g_prof.used++];
    r->kind = kind;
    r->work = work;
    (void)hipEventRecord(r->a, st);
  }
  ~ProfScope() {
    if (r) (void)hipEventRecord(r->b, st);
  }
};
enum { PK_W4GEMM = 0, PK_LMHEAD = 1, PK_ATTN = 2, PK_UPDATE = 3, PK_OTHER = 4, PK_EXPAND = 5, PK_COUNT = 6 };


// The decoder forward with every quantized linear perturbed by sign*eps*z.
// n_pass = 2 (int4 only; see passes_stacked): both passes of a step stacked, rows [0,M1) perturbed by
// +eps_signed and rows [P, P + M1) by -eps_signed, P = stacked_pass_stride(M1); their losses go to
// loss_out and loss_out2.
qzo_status forward(qzo_model* m, const int32_t* tok, uint32_t batch1, uint32_t seq, uint64_t seed,
                   float eps_signed, const Workspace& w, float* loss_out, hipStream_t st,
                   void* hidden_out = nullptr, uint32_t n_pass = 1, float* loss_out2 = nullptr) {
  const qzo_model_config& c = m->cfg;
  const uint32_t batch = batch1 * n_pass, M1 = batch1 * seq;
  const uint32_t P = n_pass == 2 ? (uint32_t)stacked_pass_stride(M1) : M1;     // rows per pass
  const bool padded = P != M1;                                                // rows [M1, P) are padding
  const uint32_t M = n_pass == 2 ? P + M1 : M1;                               // rows of every activation
  const uint32_t d = c.d_model, F = c.d_ffn, H = c.n_heads, dh = d / H;
  const bool llama = c.arch == 0, asym = c.quant == 2;
  const uint32_t seed_lo = (uint32_t)seed, seed_hi = (uint32_t)(seed >> 32);
  const unsigned char* arena = (const unsigned char*)m->arena;

  if (m->dense_master) {      // joint mode: the 16-bit tensors become round16(theta_u + eps_signed z)
    ProfScope ps(PK_OTHER, 0, st);
    QZO_HIP(launch_dense_perturb(m->dense_master, m->dense_segs, m->n_dense_segs, m->n_dense, seed_lo,
                                 seed_hi, eps_signed, st));
  }
  if (w.se) {   // some linear takes the expansion route: one launch perturbs every scale of the model
    ProfScope ps(PK_EXPAND, 0, st);
    QZO_HIP(launch_perturbed_scales_all(m->arena, m->plan, seed_lo, seed_hi, eps_signed, w.se, st));
  }
  {
    ProfScope ps(PK_OTHER, 0, st);
    if (llama) QZO_HIP(launch_rope_table(w.rope, seq, dh, c.rope_theta, st));
    QZO_HIP(launch_embed(tok, M1, P, m->T[0].ptr_dev, llama ? nullptr : m->T[1].ptr_dev, M, seq, d, w.h, st));
  }
  const double attn_flops = 2.0 * batch * H * (double)seq * seq * dh;   // causal: half of 4 B H S^2 dh
  const double Mreal = (double)n_pass * M1;                             // rows that count as work
  // attention over both passes: one launch when they are contiguous, one per pass otherwise
  // short sequences: no RoPE launch, the attention kernel rotates q and k itself
  const bool rope_in_attention = llama && seq <= ATTENTION_ROPE_MAX_S;
  auto attention = [&](bool rotated) {
    ProfScope ps(PK_ATTN, attn_flops, st);
    const float* tb = (llama && !rotated) ? w.rope : nullptr;
    if (!padded) return launch_attention(w.qkv, batch, seq, H, dh, w.att, tb, st);
    hipError_t e = launch_attention(w.qkv, batch1, seq, H, dh, w.att, tb, st);
    if (e != hipSuccess) return e;
    return launch_attention((const unsigned char*)w.qkv + (size_t)P * 3 * d * 2, batch1, seq, H, dh,
                            (unsigned char*)w.att + (size_t)P * d * 2, tb, st);
  };
  auto other = [&](hipError_t e) { return e; };
  (void)other;
  bool rope_fused = false;     // set by a qkv linear whose GEMM applied the rotary embedding itself
  // few-token linears take the block sums of their input from its producer
  const bool few = w.skinny && M1 <= SKINNY_MAX_M && (c.quant == 0 || c.quant == 2) && !c.act_order;
  float* const xs_a = few ? w.xs_a : nullptr;
  for (uint32_t l = 0; l < c.n_layers; ++l) {
    const qzo_buf* T = &m->T[m->first_layer_tensor + (size_t)l * m->tensors_per_layer];
    const uint64_t layer_off = (uint64_t)l * m->scales_per_layer;
    // Position of a tensor of the symmetric table (and of the li-th weight) within this layer: with
    // zero-points every packed weight is followed by one more tensor.
    static const uint32_t wpos_llama[4] = {1, 2, 4, 5}, wpos_opt[4] = {2, 4, 8, 10};
    const uint32_t* wpos = llama ? wpos_llama : wpos_opt;
    const uint32_t extra = (asym ? 1u : 0u) + (c.act_order ? 1u : 0u);    // tensors that follow a packed weight
    auto tpos = [&](uint32_t k) {
      uint32_t shift = 0;
      for (int i = 0; i < 4; ++i) shift += wpos[i] < k ? extra : 0u;
      return k + shift;
    };
    auto ti = [&](uint32_t k) { return T[tpos(k)].ptr_dev; };
    auto gemm = [&](int li, const void* x, const void* bias, const void* resid, void* y, uint32_t epi) {
      GemmArgs g = {};
      g.x = x; g.w = ti(wpos[li]); g.zp = asym ? T[tpos(wpos[li]) + 1].ptr_dev : nullptr;
      g.s = arena + (layer_off + m->lin[li].s_off) * 2;
      g.bias = bias; g.resid = resid; g.y = y;
      g.M = M1; g.N = m->lin[li].N; g.K = m->lin[li].K;
      g.dual = n_pass == 2;
      g.pass_stride = n_pass == 2 ? P : 0;
      g.row_base = l * m->rows_per_layer + m->lin[li].row_base;
      g.seed_lo = seed_lo; g.seed_hi = seed_hi; g.eps_signed = eps_signed;
      g.epi = epi & ~EPI_ROPE;                // a request: only the plain GEMM of the int4 expansion route serves it
      g.s_fp16 = c.scale_fp16;
      g.skinny_ws = w.skinny;
      g.split_ws = w.split;
      if (few) {     // the few-token kernel takes the block sums of its input from the kernel that wrote it
        g.xsum = (li == 0 || li == 2) ? w.xs_a : (li == 3 ? w.xs_act : nullptr);
        g.xsum_out = li == 2 ? w.xs_act : nullptr;
      }
      if (c.act_order) {
        // a group index per column: scale and zero-point are looked up per weight while the perturbed
        // matrix is written out; the fused kernels, whose k-tile shares one scale per row, cannot serve it
        const int32_t* g_idx = (const int32_t*)T[tpos(wpos[li]) + 2].ptr_dev;
        const bool split = w.split && tile_ksplit(g.M, g.N, g.K, nullptr) > 1;
        {
          ProfScope pe(PK_EXPAND, 2.5 * (double)g.N * g.K, st);
          hipError_t e = launch_expand_int4_from(g.w, w.se + layer_off + m->lin[li].s_off, g.zp, g_idx, g.N, g.K,
                                                 (epi & EPI_SWIGLU) != 0 && !split, w.wexp, st);
          if (e != hipSuccess) return e;
        }
        g.w = w.wexp; g.s = nullptr; g.zp = nullptr; g.skinny_ws = nullptr; g.split_ws = (split || (w.split && tile_tail_cols(g.M, g.N, g.K, g.epi))) ? w.split : nullptr;
        ProfScope ps(PK_W4GEMM, 2.0 * Mreal * (double)g.N * g.K, st);
        return launch_bf16_gemm(g, PLAIN_GEMM_PIPE, st);
      }
      if (c.quant == 3) {
        // NormalFloat-4: table lookup and scaling once per weight, then a plain bf16 GEMM
        const bool split = w.split && tile_ksplit(g.M, g.N, g.K, nullptr) > 1;
        int order = ((epi & EPI_SWIGLU) && !split) ? ROW_ORDER_SWIGLU : ROW_ORDER_NATURAL;
        if (epi == EPI_ROPE && !split && (dh == 64 || (dh == 128 && g.N % 256 == 0))) {   // as for int4 below
          if (dh == 128) order = ROW_ORDER_ROPE128;
          g.epi = EPI_ROPE; g.rope = w.rope; g.rope_S = seq; g.rope_dh = dh;
          rope_fused = true;
        }
        {
          ProfScope pe(PK_EXPAND, 2.5 * (double)g.N * g.K, st);
          hipError_t e = launch_expand_nf4_from(g.w, w.se + layer_off + m->lin[li].s_off, g.N, g.K, order, w.wexp, st);
          if (e != hipSuccess) return e;
        }
        g.w = w.wexp; g.s = nullptr; g.skinny_ws = nullptr; g.split_ws = (split || (w.split && tile_tail_cols(g.M, g.N, g.K, g.epi))) ? w.split : nullptr;
        ProfScope ps(PK_W4GEMM, 2.0 * Mreal * (double)g.N * g.K, st);
        return launch_bf16_gemm(g, PLAIN_GEMM_PIPE, st);
      }
      if (w.wexp && m->int4_path != 1 && n_pass == 1 &&
          (m->int4_path == 2 || M >= expand_min_m_int4(g.N, g.K))) {
        // many tokens: write the perturbed matrix out once, then a plain bf16 GEMM.  The rotary embedding
        // of a qkv linear rides on that GEMM's epilogue (heads of 64 or 128; with 128 the matrix is
        // written in the row order that puts feature i and i + 64 of a head into one lane).
        int order = (epi & EPI_SWIGLU) ? ROW_ORDER_SWIGLU : ROW_ORDER_NATURAL;
        if (epi == EPI_ROPE && (dh == 64 || (dh == 128 && g.N % 256 == 0))) {
          if (dh == 128) order = ROW_ORDER_ROPE128;
          g.epi = EPI_ROPE; g.rope = w.rope; g.rope_S = seq; g.rope_dh = dh;
          rope_fused = true;
        }
        {
          ProfScope pe(PK_EXPAND, 2.5 * (double)g.N * g.K, st);
          hipError_t e = launch_expand_int4_from(g.w, w.se + layer_off + m->lin[li].s_off, g.zp, nullptr, g.N,
                                                 g.K, order, w.wexp, st);
          if (e != hipSuccess) return e;
        }
        g.w = w.wexp; g.s = nullptr; g.zp = nullptr; g.skinny_ws = nullptr;
        // (plain epilogues: the launcher cuts K where the output tiles do not fill the chip, or the last
        // columns' K where they are a little more than whole rounds, exactly as it does for the fused kernel)
        g.split_ws = (g.epi & (EPI_SWIGLU | EPI_ROPE)) ? nullptr : w.split;
        ProfScope ps(PK_W4GEMM, 2.0 * Mreal * (double)g.N * g.K, st);
        return launch_bf16_gemm(g, PLAIN_GEMM_PIPE, st);
      }
      ProfScope ps(PK_W4GEMM, 2.0 * Mreal * (double)g.N * g.K, st);
      return launch_w4a16_gemm(g, st);
    };
    auto cgemm = [&](int li, const void* x, const void* codes, const void* cb, const void* resid,
                     void* y, uint32_t epi) {
      GemmArgs g = {};
      g.x = x; g.w = codes; g.cb = cb;
      g.s = arena + ((uint64_t)l * m->rows_per_layer + m->lin[li].row_base) * 2;   // fp16 channel scales
      g.resid = resid; g.y = y;
      g.M = M; g.N = m->lin[li].N; g.K = m->lin[li].K;
      g.row_base = l * m->rows_per_layer + m->lin[li].row_base;
      g.seed_lo = seed_lo; g.seed_hi = seed_hi; g.eps_signed = eps_signed;
      g.epi = epi & ~EPI_ROPE;                // a request, served by the plain GEMM below when it does not split K
      if (w.wexp) {
        // many tokens: reconstruct the perturbed matrix once, then a plain bf16 GEMM
        // (rows in natural order when the GEMM will split K: its reduction applies SwiGLU)
        const bool split = w.split && tile_ksplit(g.M, g.N, g.K, nullptr) > 1;
        int order = ((epi & EPI_SWIGLU) && !split) ? ROW_ORDER_SWIGLU : ROW_ORDER_NATURAL;
        if (epi == EPI_ROPE && !split && (dh == 64 || (dh == 128 && g.N % 256 == 0))) {   // as for int4
          if (dh == 128) order = ROW_ORDER_ROPE128;
          g.epi = EPI_ROPE; g.rope = w.rope; g.rope_S = seq; g.rope_dh = dh;
          rope_fused = true;
        }
        {
          ProfScope pe(PK_EXPAND, 2.25 * (double)g.N * g.K, st);
          hipError_t e = launch_expand_codebook(codes, cb, g.s, g.N, g.K, g.row_base, seed_lo, seed_hi,
                                                eps_signed, order, w.wexp, st);
          if (e != hipSuccess) return e;
        }
        g.w = w.wexp; g.cb = nullptr; g.s = nullptr; g.split_ws = (split || (w.split && tile_tail_cols(g.M, g.N, g.K, g.epi))) ? w.split : nullptr;
        ProfScope ps(PK_W4GEMM, 2.0 * Mreal * (double)g.N * g.K, st);
        return launch_bf16_gemm(g, PLAIN_GEMM_PIPE, st);
      }
      ProfScope ps(PK_W4GEMM, 2.0 * Mreal * (double)g.N * g.K, st);
      return launch_codebook_gemm(g, st);
    };
    if (llama && c.quant == 1) {
      // attn_norm, codes/cb qkv, codes/cb o, ffn_norm, codes/cb gate+up, codes/cb down
      QZO_HIP(launch_rmsnorm(w.h, T[0].ptr_dev, M, d, c.norm_eps, w.a, st));
      rope_fused = false;
      QZO_HIP(cgemm(0, w.a, T[1].ptr_dev, T[2].ptr_dev, nullptr, w.qkv, EPI_ROPE));
      if (!rope_fused && !rope_in_attention) QZO_HIP(launch_rope(w.qkv, w.rope, M, seq, P, d, H, st));
      QZO_HIP(attention(rope_fused || !rope_in_attention));
      QZO_HIP(cgemm(1, w.att, T[3].ptr_dev, T[4].ptr_dev, w.h, w.h, EPI_RESIDUAL));
      QZO_HIP(launch_rmsnorm(w.h, T[5].ptr_dev, M, d, c.norm_eps, w.a, st));
      QZO_HIP(cgemm(2, w.a, T[6].ptr_dev, T[7].ptr_dev, nullptr, w.act, EPI_SWIGLU));
      QZO_HIP(cgemm(3, w.act, T[8].ptr_dev, T[9].ptr_dev, w.h, w.h, EPI_RESIDUAL));
    } else if (llama) {
      // attn_norm, wqkv, wo, ffn_norm, wgu, wdown (symmetric-table positions)
      QZO_HIP(launch_rmsnorm(w.h, ti(0), M, d, c.norm_eps, w.a, st, xs_a));
      rope_fused = false;
      QZO_HIP(gemm(0, w.a, nullptr, nullptr, w.qkv, EPI_ROPE));
      if (!rope_fused && !rope_in_attention) QZO_HIP(launch_rope(w.qkv, w.rope, M, seq, P, d, H, st));
      QZO_HIP(attention(rope_fused || !rope_in_attention));
      QZO_HIP(gemm(1, w.att, nullptr, w.h, w.h, EPI_RESIDUAL));
      QZO_HIP(launch_rmsnorm(w.h, ti(3), M, d, c.norm_eps, w.a, st, xs_a));
      QZO_HIP(gemm(2, w.a, nullptr, nullptr, w.act, EPI_SWIGLU));
      QZO_HIP(gemm(3, w.act, nullptr, w.h, w.h, EPI_RESIDUAL));
    } else {
      // ln1_g, ln1_b, wqkv, bqkv, wo, bo, ln2_g, ln2_b, wfc1, bfc1, wfc2, bfc2 (symmetric-table positions)
      QZO_HIP(launch_layernorm(w.h, ti(0), ti(1), M, d, c.norm_eps, w.a, st, xs_a));
      QZO_HIP(gemm(0, w.a, ti(3), nullptr, w.qkv, EPI_BIAS));
      QZO_HIP(attention(true));
      QZO_HIP(gemm(1, w.att, ti(5), w.h, w.h, EPI_BIAS | EPI_RESIDUAL));
      QZO_HIP(launch_layernorm(w.h, ti(6), ti(7), M, d, c.norm_eps, w.a, st, xs_a));
      QZO_HIP(gemm(2, w.a, ti(9), nullptr, w.ff, EPI_BIAS | EPI_RELU));
      QZO_HIP(gemm(3, w.ff, ti(11), w.h, w.h, EPI_BIAS | EPI_RESIDUAL));
    }
  }
  const size_t tail = m->first_layer_tensor + (size_t)c.n_layers * m->tensors_per_layer;
  const void* lm_head;
  if (llama) {
    QZO_HIP(launch_rmsnorm(w.h, m->T[tail].ptr_dev, M, d, c.norm_eps, w.a, st));
    lm_head = m->T[tail + 1].ptr_dev;
  } else {
    QZO_HIP(launch_layernorm(w.h, m->T[tail].ptr_dev, m->T[tail + 1].ptr_dev, M, d, c.norm_eps, w.a, st));
    lm_head = m->T[tail + 2].ptr_dev;
  }
  if (hidden_out)
    QZO_HIP(hipMemcpyAsync(hidden_out, w.a, (size_t)M * d * 2, hipMemcpyDeviceToDevice, st));
  CeArgs ce = {};
  ce.w = lm_head; ce.tok = tok; ce.tok_rows = M1;
  ce.V = c.vocab; ce.K = d; ce.S = seq; ce.n_slices = ((c.vocab + 255) / 256) * 4;
  // both passes in one launch when they are contiguous, one launch per pass otherwise
  for (uint32_t r0 = 0; r0 < M; r0 += P) {
    ce.x = (const unsigned char*)w.a + (size_t)r0 * d * 2;
    ce.part = w.ce_part + (size_t)r0 * ce.n_slices * 2;
    ce.tgt = w.tgt + r0;
    ce.M = padded ? M1 : M;
    ProfScope ps(PK_LMHEAD, 2.0 * ce.M * (double)c.vocab * d, st);
    QZO_HIP(launch_lmhead_ce(ce, st));
    if (!padded) break;
  }
  QZO_HIP(launch_ce_reduce(w.ce_part, w.tgt, M1, seq, ce.n_slices, w.rowloss, loss_out, st));
  if (n_pass == 2)
    QZO_HIP(launch_ce_reduce(w.ce_part + (size_t)P * ce.n_slices * 2, w.tgt + P, M1, seq, ce.n_slices,
                             w.rowloss + P, loss_out2, st));
  return QZO_OK;
}

}  // namespace

extern "C" {

const char* qzo_last_error(void) { return g_err.c_str(); }

qzo_status qzo_model_scale_count(const qzo_model_config* cfg, uint64_t* out) {
  qzo_status st = check_cfg(cfg);
  if (st != QZO_OK) return st;
  if (!out) return fail(QZO_ERR_ARG, "out is null");
  Linear lin[4];
  layer_linears(*cfg, lin);
  if (cfg->quant == 1)
    *out = (uint64_t)(lin[3].row_base + lin[3].N) * cfg->n_layers;     // one scale per output row
  else
    *out = (lin[3].s_off + (uint64_t)lin[3].N * (lin[3].K / cfg->group_size)) * cfg->n_layers;
  return QZO_OK;
}

qzo_status qzo_model_create(const qzo_model_config* cfg, const qzo_buf* tensors, uint32_t n_tensors,
                            void* scale_arena_dev, uint64_t n_scales, qzo_model** out) {
  qzo_status st = check_cfg(cfg);
  if (st != QZO_OK) return st;
  if (!tensors || !scale_arena_dev || !out) return fail(QZO_ERR_ARG, "null argument");
  if (!aligned16(scale_arena_dev)) return fail(QZO_ERR_ALIGN, "scale arena not 16-byte aligned");
  const bool llama = cfg->arch == 0;
  const bool codebook = cfg->quant == 1;
  const bool asym = cfg->quant == 2;
  const uint32_t per_layer = codebook ? 10 : (llama ? 6 : 12) + (asym ? 4 : 0) + (cfg->act_order ? 4 : 0),
                 head = llama ? 1 : 2, tail = llama ? 2 : 3;
  if (n_tensors != head + per_layer * cfg->n_layers + tail)
    return fail(QZO_ERR_ARG, "tensor count does not match the architecture's table");
  uint64_t want = 0;
  qzo_model_scale_count(cfg, &want);
  if (n_scales != want) return fail(QZO_ERR_SHAPE, "n_scales does not match the config");
  if ((uint64_t)cfg->n_layers * (4 * (uint64_t)cfg->d_model + (llama ? 2 : 1) * (uint64_t)cfg->d_ffn) >
      0xffffffffull)
    return fail(QZO_ERR_SHAPE, "too many quantized rows");

  std::vector<uint64_t> need;
  std::vector<uint8_t> kind;
  table_layout(*cfg, need, kind);
  for (uint32_t i = 0; i < n_tensors; ++i) {
    if (!tensors[i].ptr_dev) return fail(QZO_ERR_ARG, "tensor " + std::to_string(i) + " is null");
    if (!aligned16(tensors[i].ptr_dev))
      return fail(QZO_ERR_ALIGN, "tensor " + std::to_string(i) + " not 16-byte aligned");
    if (tensors[i].bytes != need[i])
      return fail(QZO_ERR_SHAPE, "tensor " + std::to_string(i) + " has " +
                                     std::to_string(tensors[i].bytes) + " bytes, expected " +
                                     std::to_string(need[i]));
  }

  qzo_model* m = new qzo_model();
  m->cfg = *cfg;
  m->T.assign(tensors, tensors + n_tensors);
  m->arena = scale_arena_dev;
  m->n_scales = n_scales;
  layer_linears(*cfg, m->lin);
  m->scales_per_layer = m->lin[3].s_off + (uint64_t)m->lin[3].N * (m->lin[3].K / cfg->group_size);
  m->rows_per_layer = m->lin[3].row_base + m->lin[3].N;
  m->tensors_per_layer = per_layer;
  m->first_layer_tensor = head;
  st = build_plan(m->lin, 4, cfg->n_layers, m->plan, cfg->group_size, cfg->scale_fp16);
  if (st != QZO_OK) { delete m; return st; }
  for (int i = 0; i < 4; ++i)       // one linear written out in bf16 must fit 32-bit byte offsets
    if ((uint64_t)m->lin[i].N * m->lin[i].K * 2 >= (1ull << 31)) {
      delete m;
      return fail(QZO_ERR_SHAPE, "a linear of this model exceeds 2^31 bytes in bf16");
    }
  if ((uint64_t)cfg->vocab * cfg->d_model * 2 >= (1ull << 31)) {
    delete m;
    return fail(QZO_ERR_SHAPE, "lm_head exceeds 2^31 bytes");
  }
  *out = m;
  return QZO_OK;
}

qzo_status qzo_model_destroy(qzo_model* m) {
  if (!m) return QZO_OK;
  delete m;
  return QZO_OK;
}

qzo_status qzo_model_dense_count(const qzo_model_config* cfg, uint64_t* out) {
  qzo_status st = check_cfg(cfg);
  if (st != QZO_OK) return st;
  if (!out) return fail(QZO_ERR_ARG, "out is null");
  std::vector<uint64_t> need;
  std::vector<uint8_t> kind;
  table_layout(*cfg, need, kind);
  uint64_t n = 0;
  for (size_t i = 0; i < need.size(); ++i)
    if (kind[i] != 2) n += need[i] / 2;
  *out = n;
  return QZO_OK;
}

qzo_status qzo_model_joint_table_bytes(const qzo_model_config* cfg, uint64_t* out) {
  qzo_status st = check_cfg(cfg);
  if (st != QZO_OK) return st;
  if (!out) return fail(QZO_ERR_ARG, "out is null");
  std::vector<uint64_t> need;
  std::vector<uint8_t> kind;
  table_layout(*cfg, need, kind);
  uint64_t n = 0;
  for (size_t i = 0; i < need.size(); ++i) n += kind[i] != 2;
  *out = up256(n * sizeof(DenseSeg));
  return QZO_OK;
}

qzo_status qzo_model_enable_joint(qzo_model* m, float* dense_master_dev, uint64_t n_dense, void* table_dev,
                                  uint64_t table_bytes) {
  if (!m || !dense_master_dev || !table_dev) return fail(QZO_ERR_ARG, "null argument");
  if (m->dense_master) return fail(QZO_ERR_ARG, "joint mode is already on");
  if (!aligned16(dense_master_dev) || !aligned16(table_dev))
    return fail(QZO_ERR_ALIGN, "dense master or table not 16-byte aligned");
  uint64_t want = 0;
  qzo_model_dense_count(&m->cfg, &want);
  if (n_dense != want) return fail(QZO_ERR_SHAPE, "n_dense does not match the config");
  std::vector<uint64_t> need;
  std::vector<uint8_t> kind;
  table_layout(m->cfg, need, kind);
  std::vector<DenseSeg> segs;
  uint64_t first = 0;
  for (size_t i = 0; i < need.size(); ++i) {
    if (kind[i] == 2) continue;
    const uint64_t n = need[i] / 2;
    if (n % 8) return fail(QZO_ERR_SHAPE, "a 16-bit tensor's size is not a multiple of 8");
    DenseSeg sg = {};
    sg.first8 = first / 8;
    sg.out = const_cast<void*>(m->T[i].ptr_dev);
    sg.fmt = kind[i];
    segs.push_back(sg);
    first += n;
  }
  if (table_bytes < segs.size() * sizeof(DenseSeg))
    return fail(QZO_ERR_WORKSPACE, "table smaller than qzo_model_joint_table_bytes");
  QZO_HIP(hipMemcpy(table_dev, segs.data(), segs.size() * sizeof(DenseSeg), hipMemcpyHostToDevice));
  m->dense_segs = (DenseSeg*)table_dev;
  m->n_dense_segs = (uint32_t)segs.size();
  m->n_dense = n_dense;
  m->dense_master = dense_master_dev;
  return QZO_OK;
}

qzo_status qzo_workspace_bytes(const qzo_model* m, uint32_t batch, uint32_t seq, uint64_t* out) {
  if (!m || !out) return fail(QZO_ERR_ARG, "null argument");
  if (batch == 0 || seq < 2 || seq > m->cfg.max_seq) return fail(QZO_ERR_SHAPE, "bad batch/seq");
  *out = carve(m, batch, seq, nullptr).total;
  return QZO_OK;
}

qzo_status qzo_forward_loss(qzo_model* m, const int32_t* tokens_dev, uint32_t batch, uint32_t seq,
                            uint64_t seed, float eps, int sign, void* workspace_dev,
                            uint64_t workspace_bytes, float* loss_dev, void* stream) {
  qzo_status st = check_batch(m, tokens_dev, batch, seq, workspace_dev, workspace_bytes);
  if (st != QZO_OK) return st;
  if (!loss_dev) return fail(QZO_ERR_ARG, "loss_dev is null");
  if (sign != 1 && sign != -1) return fail(QZO_ERR_ARG, "sign must be +1 or -1");
  if (!std::isfinite(eps)) return fail(QZO_ERR_ARG, "eps not finite");
  Workspace w = carve(m, batch, seq, workspace_dev);
  return forward(m, tokens_dev, batch, seq, seed, sign > 0 ? eps : -eps, w, loss_dev,
                 (hipStream_t)stream);
}

qzo_status qzo_debug_forward(qzo_model* m, const int32_t* tokens_dev, uint32_t batch, uint32_t seq,
                             uint64_t seed, float eps, int sign, void* workspace_dev,
                             uint64_t workspace_bytes, float* loss_dev, void* hidden_dev,
                             void* stream) {
  qzo_status st = check_batch(m, tokens_dev, batch, seq, workspace_dev, workspace_bytes);
  if (st != QZO_OK) return st;
  if (!loss_dev || !hidden_dev) return fail(QZO_ERR_ARG, "null output");
  if (sign != 1 && sign != -1) return fail(QZO_ERR_ARG, "sign must be +1 or -1");
  Workspace w = carve(m, batch, seq, workspace_dev);
  return forward(m, tokens_dev, batch, seq, seed, sign > 0 ? eps : -eps, w, loss_dev,
                 (hipStream_t)stream, hidden_dev);
}

static qzo_status step_impl(qzo_model* m, const int32_t* tokens_dev, uint32_t batch, uint32_t seq,
                            uint64_t seed, float eps, float eta, float eta_dense, float clip,
                            void* workspace_dev, uint64_t workspace_bytes, qzo_step_result* result_dev,
                            void* stream) {
  qzo_status st = check_batch(m, tokens_dev, batch, seq, workspace_dev, workspace_bytes);
  if (st != QZO_OK) return st;
  if (!result_dev) return fail(QZO_ERR_ARG, "result_dev is null");
  if (!(clip >= 0.0f)) return fail(QZO_ERR_ARG, "clip must be >= 0");
  if (!std::isfinite(eps) || !std::isfinite(eta) || !std::isfinite(eta_dense))
    return fail(QZO_ERR_ARG, "eps/eta not finite");
  hipStream_t s = (hipStream_t)stream;
  Workspace w = carve(m, batch, seq, workspace_dev);
  if (passes_stacked(m, (uint64_t)batch * seq)) {
    // one forward over both passes
    st = forward(m, tokens_dev, batch, seq, seed, eps, w, w.losses, s, nullptr, 2, w.losses + 1);
    if (st != QZO_OK) return st;
  } else {
    st = forward(m, tokens_dev, batch, seq, seed, eps, w, w.losses, s);
    if (st != QZO_OK) return st;
    st = forward(m, tokens_dev, batch, seq, seed, -eps, w, w.losses + 1, s);
    if (st != QZO_OK) return st;
  }
  QZO_HIP(launch_spsa_clip(w.losses, eps, clip, result_dev, s));
  {
    ProfScope ps(PK_UPDATE, 4.0 * (double)m->n_scales, s);
    if (m->cfg.quant == 1)
      QZO_HIP(launch_channel_update(m->arena, (uint32_t)m->n_scales, 0u, (uint32_t)seed,
                                    (uint32_t)(seed >> 32), eta, 0.0f, result_dev, s));
    else
      QZO_HIP(launch_scale_update(m->arena, m->plan, (uint32_t)seed, (uint32_t)(seed >> 32), eta, 0.0f,
                                  result_dev, s));
  }
  if (m->dense_master) {
    // SPSA part of the joint step, then the 16-bit tensors are brought back to round16(theta_u)
    ProfScope ps(PK_OTHER, 0, s);
    QZO_HIP(launch_dense_update(m->dense_master, m->n_dense, (uint32_t)seed, (uint32_t)(seed >> 32),
                                eta_dense, 0.0f, result_dev, s));
    QZO_HIP(launch_dense_perturb(m->dense_master, m->dense_segs, m->n_dense_segs, m->n_dense,
                                 (uint32_t)seed, (uint32_t)(seed >> 32), 0.0f, s));
  }
  return QZO_OK;
}

qzo_status qzo_step(qzo_model* m, const int32_t* tokens_dev, uint32_t batch, uint32_t seq,
                    uint64_t seed, float eps, float eta, float clip, void* workspace_dev,
                    uint64_t workspace_bytes, qzo_step_result* result_dev, void* stream) {
  if (m && m->dense_master) return fail(QZO_ERR_ARG, "the model is in joint mode: call qzo_step_joint");
  return step_impl(m, tokens_dev, batch, seq, seed, eps, eta, 0.0f, clip, workspace_dev, workspace_bytes,
                   result_dev, stream);
}

qzo_status qzo_step_joint(qzo_model* m, const int32_t* tokens_dev, uint32_t batch, uint32_t seq,
                          uint64_t seed, float eps, float eta, float eta_dense, float clip,
                          void* workspace_dev, uint64_t workspace_bytes, qzo_step_result* result_dev,
                          void* stream) {
  if (m && !m->dense_master) return fail(QZO_ERR_ARG, "joint mode is off: call qzo_model_enable_joint first");
  return step_impl(m, tokens_dev, batch, seq, seed, eps, eta, eta_dense, clip, workspace_dev,
                   workspace_bytes, result_dev, stream);
}

qzo_status qzo_model_apply_update(qzo_model* m, uint64_t seed, float eta, float d_clipped,
                                  void* stream) {
  if (!m) return fail(QZO_ERR_ARG, "model is null");
  if (!std::isfinite(eta) || !std::isfinite(d_clipped)) return fail(QZO_ERR_ARG, "eta/d' not finite");
  if (m->cfg.quant == 1)
    QZO_HIP(launch_channel_update(m->arena, (uint32_t)m->n_scales, 0u, (uint32_t)seed,
                                  (uint32_t)(seed >> 32), eta, d_clipped, nullptr, (hipStream_t)stream));
  else
    QZO_HIP(launch_scale_update(m->arena, m->plan, (uint32_t)seed, (uint32_t)(seed >> 32), eta,
                                d_clipped, nullptr, (hipStream_t)stream));
  return QZO_OK;
}

qzo_status qzo_apply_update(void* s_dev, uint32_t n_rows, uint32_t G, uint32_t row_base,
                            uint64_t seed, float eta, float d_clipped, uint32_t scale_fp16, void* stream) {
  if (!s_dev) return fail(QZO_ERR_ARG, "s_dev is null");
  if (scale_fp16 > 1) return fail(QZO_ERR_ARG, "scale_fp16 must be 0 or 1");
  if (!aligned16(s_dev)) return fail(QZO_ERR_ALIGN, "s_dev not 16-byte aligned");
  if (!std::isfinite(eta) || !std::isfinite(d_clipped)) return fail(QZO_ERR_ARG, "eta/d' not finite");
  if (n_rows == 0 || G == 0) return QZO_OK;
  Linear lin = {n_rows, G * 128, 0, row_base};
  UpdPlan plan;
  qzo_status st = build_plan(&lin, 1, 1, plan, 128, scale_fp16);
  if (st != QZO_OK) return st;
  QZO_HIP(launch_scale_update(s_dev, plan, (uint32_t)seed, (uint32_t)(seed >> 32), eta, d_clipped,
                              nullptr, (hipStream_t)stream));
  return QZO_OK;
}

// Scratch of a single perturbed linear: [per-tile sums of y^2][K-slice partial sums], each part
// rounded up to 256 bytes.
struct LinearScratch { uint32_t tiles; uint64_t part_floats; uint64_t part_off, total; bool skinny, split; };
static LinearScratch linear_scratch(uint32_t M, uint32_t N, uint32_t K, bool with_sumsq) {
  LinearScratch ls = {};
  if (M == 0 || N == 0) return ls;
  ls.skinny = M <= SKINNY_MAX_M;
  ls.split = !ls.skinny && tile_ksplit(M, N, K, nullptr) > 1;     // too few tiles for the chip
  ls.tiles = (ls.skinny || ls.split) ? skinny_reduce_blocks(M, N, 0) : ((M + 255) / 256) * ((N + 255) / 256);
  ls.part_floats = ls.skinny ? skinny_ws_floats(M, N, K) : (ls.split ? tile_split_ws_floats(M, N, K) : 0);
  ls.part_off = with_sumsq ? up256((uint64_t)ls.tiles * 4) : 0;
  ls.total = ls.part_off + up256(ls.part_floats * 4);
  return ls;
}

static qzo_status linear_check(const void* x_dev, const void* q_dev, const void* s_dev, const void* y_dev,
                               uint32_t M, uint32_t N, uint32_t K, uint32_t group, float eps, int sign) {
  if (!x_dev || !q_dev || !s_dev || !y_dev) return fail(QZO_ERR_ARG, "null device pointer");
  if (!aligned16(x_dev) || !aligned16(q_dev) || !aligned16(s_dev) || !aligned16(y_dev))
    return fail(QZO_ERR_ALIGN, "device pointer not 16-byte aligned");
  if (group != 128) return fail(QZO_ERR_SHAPE, "group must be 128");
  if (K == 0 || K % 128) return fail(QZO_ERR_SHAPE, "K must be a positive multiple of 128");
  if (N % 8) return fail(QZO_ERR_SHAPE, "N must be a multiple of 8");
  if (sign != 1 && sign != -1) return fail(QZO_ERR_ARG, "sign must be +1 or -1");
  if (!std::isfinite(eps)) return fail(QZO_ERR_ARG, "eps not finite");
  // buffer loads and stores address each operand with 32-bit byte offsets
  if ((uint64_t)M * K * 2 >= (1ull << 31) || (uint64_t)N * K / 2 >= (1ull << 31) ||
      (uint64_t)M * N * 2 >= (1ull << 31))
    return fail(QZO_ERR_SHAPE, "an operand exceeds 2^31 bytes");
  return QZO_OK;
}

// The launches of a single perturbed linear; scratch (ls.total bytes) is known to be large enough.
static qzo_status dequant_gemm_run(const void* x_dev, const void* q_dev, const void* s_dev, const void* zp_dev,
                                   uint32_t scale_fp16, uint32_t row_base, uint32_t M, uint32_t N, uint32_t K, uint64_t seed,
                                   float eps, int sign, void* y_dev, float* sumsq_dev, void* scratch,
                                   const LinearScratch& ls, hipStream_t st) {
  if (M == 0 || N == 0) {
    if (sumsq_dev) QZO_HIP(launch_sum_partials(nullptr, 0, sumsq_dev, st));
    return QZO_OK;
  }
  GemmArgs g = {};
  g.x = x_dev; g.w = q_dev; g.s = s_dev; g.zp = zp_dev; g.y = y_dev;
  g.M = M; g.N = N; g.K = K; g.row_base = row_base;
  g.seed_lo = (uint32_t)seed; g.seed_hi = (uint32_t)(seed >> 32);
  g.eps_signed = sign > 0 ? eps : -eps;
  g.s_fp16 = scale_fp16;
  float* part = (float*)((unsigned char*)scratch + ls.part_off);
  if (ls.skinny) g.skinny_ws = part;
  if (ls.split) g.split_ws = part;
  if (sumsq_dev) {
    g.epi = EPI_SUMSQ;
    g.partials = (float*)scratch;
  }
  QZO_HIP(launch_w4a16_gemm(g, st));
  if (sumsq_dev) QZO_HIP(launch_sum_partials((const float*)scratch, ls.tiles, sumsq_dev, st));
  return QZO_OK;
}

static qzo_status dequant_gemm(const void* x_dev, const void* q_dev, const void* s_dev,
                               const void* zp_dev, uint32_t scale_fp16, uint32_t row_base, uint32_t M, uint32_t N,
                               uint32_t K, uint32_t group, uint64_t seed, float eps, int sign,
                               void* y_dev, float* sumsq_dev, void* scratch_dev, uint64_t scratch_bytes,
                               void* stream) {
  qzo_status st = linear_check(x_dev, q_dev, s_dev, y_dev, M, N, K, group, eps, sign);
  if (st != QZO_OK) return st;
  const LinearScratch ls = linear_scratch(M, N, K, sumsq_dev != nullptr);
  if (ls.total) {
    if (!scratch_dev) return fail(QZO_ERR_ARG, "scratch_dev is null");
    if ((uintptr_t)scratch_dev & 255u) return fail(QZO_ERR_ALIGN, "scratch not 256-byte aligned");
    if (scratch_bytes < ls.total) return fail(QZO_ERR_WORKSPACE, "scratch too small: see qzo_linear_scratch_bytes");
  }
  return dequant_gemm_run(x_dev, q_dev, s_dev, zp_dev, scale_fp16, row_base, M, N, K, seed, eps, sign, y_dev,
                          sumsq_dev, scratch_dev, ls, (hipStream_t)stream);
}

qzo_status qzo_linear_scratch_bytes(uint32_t M, uint32_t N, uint32_t K, int with_sumsq, uint64_t* out) {
  if (!out) return fail(QZO_ERR_ARG, "out is null");
  if (K == 0 || K % 128) return fail(QZO_ERR_SHAPE, "K must be a positive multiple of 128");
  *out = linear_scratch(M, N, K, with_sumsq != 0).total;
  return QZO_OK;
}

qzo_status qzo_dequant_gemm(const void* x_dev, const void* q_dev, const void* s_dev,
                            uint32_t row_base, uint32_t M, uint32_t N, uint32_t K, uint32_t group,
                            uint64_t seed, float eps, int sign, void* y_dev, float* sumsq_dev,
                            void* scratch_dev, uint64_t scratch_bytes, void* stream) {
  return dequant_gemm(x_dev, q_dev, s_dev, nullptr, 0u, row_base, M, N, K, group, seed, eps, sign, y_dev,
                      sumsq_dev, scratch_dev, scratch_bytes, stream);
}

// ---- qzo_dequant_gemm for callers that cannot allocate: the scratch is a fixed array of this library ----
// Every GPU the library runs on holds its own copy of the array at its own address; the name below is
// a host-side stand-in, so host code only ever uses the per-device address that hipGetSymbolAddress
// returned (looked up once per device, with that device current).
constexpr uint64_t STATIC_SCRATCH_BYTES = 32ull << 20;
static __device__ __align__(256) unsigned char static_scratch[STATIC_SCRATCH_BYTES];
constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
static void* g_static_scratch_ptr[STATIC_SCRATCH_MAX_DEVICES] = {};
static std::mutex g_static_scratch_mutex;

qzo_status qzo_dequant_gemm_static(const void* x_dev, const void* q_dev, const void* s_dev,
                                   uint32_t row_base, uint32_t M, uint32_t N, uint32_t K, uint32_t group,
                                   uint64_t seed, float eps, int sign, void* y_dev, float* sumsq_dev,
                                   void* stream) {
  qzo_status st = linear_check(x_dev, q_dev, s_dev, y_dev, M, N, K, group, eps, sign);
  if (st != QZO_OK) return st;
  const LinearScratch ls = linear_scratch(M, N, K, sumsq_dev != nullptr);
  if (ls.total > STATIC_SCRATCH_BYTES)
    return fail(QZO_ERR_WORKSPACE, "this size needs " + std::to_string(ls.total) +
                                       " bytes of scratch, the fixed array holds " +
                                       std::to_string(STATIC_SCRATCH_BYTES) +
                                       ": call qzo_dequant_gemm with scratch of your own");
  int dev = -1;
  QZO_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES) return fail(QZO_ERR_UNSUPPORTED, "device ordinal out of range");
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (!g_static_scratch_ptr[dev]) {
      void* p = nullptr;
      QZO_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch)));
      if (!p) return fail(QZO_ERR_HIP, "hipGetSymbolAddress returned a null address");
      g_static_scratch_ptr[dev] = p;
    }
    ptr = g_static_scratch_ptr[dev];
  }
  // nothing in the scratch has to start at zero: every partial sum that is read was written by this call
  return dequant_gemm_run(x_dev, q_dev, s_dev, nullptr, 0u, row_base, M, N, K, seed, eps, sign, y_dev, sumsq_dev,
                          ptr, ls, (hipStream_t)stream);
}

qzo_status qzo_dequant_gemm_zp(const void* x_dev, const void* q_dev, const void* s_dev,
                               const void* zp_dev, uint32_t scale_fp16, uint32_t row_base, uint32_t M,
                               uint32_t N, uint32_t K, uint32_t group, uint64_t seed, float eps, int sign,
                               void* y_dev, float* sumsq_dev, void* scratch_dev, uint64_t scratch_bytes,
                               void* stream) {
  if (!zp_dev) return fail(QZO_ERR_ARG, "zp_dev is null");
  if (scale_fp16 > 1) return fail(QZO_ERR_ARG, "scale_fp16 must be 0 or 1");
  return dequant_gemm(x_dev, q_dev, s_dev, zp_dev, scale_fp16, row_base, M, N, K, group, seed, eps, sign, y_dev,
                      sumsq_dev, scratch_dev, scratch_bytes, stream);
}

qzo_status qzo_repack_kmajor(const void* qweight_dev, const void* qzeros_dev, const void* scales_dev,
                             uint32_t N, uint32_t K, uint32_t group, uint32_t zero_add, uint32_t scale_fp16,
                             void* q_dev, void* zp_dev, void* s_dev, void* stream) {
  if (!qweight_dev || !qzeros_dev || !scales_dev || !q_dev || !zp_dev || !s_dev)
    return fail(QZO_ERR_ARG, "null device pointer");
  if (group != 128 || K == 0 || K % 128) return fail(QZO_ERR_SHAPE, "group must be 128 and divide K");
  if (N == 0 || N % 8) return fail(QZO_ERR_SHAPE, "N must be a positive multiple of 8");
  if (zero_add > 15) return fail(QZO_ERR_ARG, "zero_add must be 0 .. 15");
  if (scale_fp16 > 1) return fail(QZO_ERR_ARG, "scale_fp16 must be 0 or 1");
  if (!aligned16(q_dev) || !aligned16(s_dev)) return fail(QZO_ERR_ALIGN, "output not 16-byte aligned");
  QZO_HIP(launch_repack_kmajor(qweight_dev, qzeros_dev, scales_dev, N, K, zero_add, scale_fp16 != 0, q_dev,
                               zp_dev, s_dev, (hipStream_t)stream));
  return QZO_OK;
}

qzo_status qzo_codebook_scratch_bytes(uint32_t M, uint32_t N, int with_sumsq, uint64_t* out) {
  if (!out) return fail(QZO_ERR_ARG, "out is null");
  *out = (with_sumsq && M && N) ? up256((uint64_t)((M + 255) / 256) * ((N + 255) / 256) * 4) : 0;
  return QZO_OK;
}

qzo_status qzo_codebook_gemm(const void* x_dev, const void* codes_dev, const void* codebook_dev,
                             const void* c_dev, uint32_t row_base, uint32_t M, uint32_t N, uint32_t K,
                             uint64_t seed, float eps, int sign, void* y_dev, float* sumsq_dev,
                             void* scratch_dev, uint64_t scratch_bytes, void* stream) {
  if (!x_dev || !codes_dev || !codebook_dev || !c_dev || !y_dev) return fail(QZO_ERR_ARG, "null device pointer");
  if (!aligned16(x_dev) || !aligned16(codes_dev) || !aligned16(codebook_dev) || !aligned16(c_dev) ||
      !aligned16(y_dev))
    return fail(QZO_ERR_ALIGN, "device pointer not 16-byte aligned");
  if (K == 0 || K % 128) return fail(QZO_ERR_SHAPE, "K must be a positive multiple of 128");
  if (N % 8) return fail(QZO_ERR_SHAPE, "N must be a multiple of 8");
  if (sign != 1 && sign != -1) return fail(QZO_ERR_ARG, "sign must be +1 or -1");
  if (!std::isfinite(eps)) return fail(QZO_ERR_ARG, "eps not finite");
  if ((uint64_t)M * K * 2 >= (1ull << 31) || (uint64_t)N * K / 4 >= (1ull << 31) ||
      (uint64_t)M * N * 2 >= (1ull << 31))
    return fail(QZO_ERR_SHAPE, "an operand exceeds 2^31 bytes");
  uint64_t need = 0;
  qzo_codebook_scratch_bytes(M, N, sumsq_dev != nullptr, &need);
  if (need) {
    if (!scratch_dev) return fail(QZO_ERR_ARG, "scratch_dev is null");
    if ((uintptr_t)scratch_dev & 255u) return fail(QZO_ERR_ALIGN, "scratch not 256-byte aligned");
    if (scratch_bytes < need) return fail(QZO_ERR_WORKSPACE, "scratch too small: see qzo_codebook_scratch_bytes");
  }
  hipStream_t st = (hipStream_t)stream;
  if (M == 0 || N == 0) {
    if (sumsq_dev) QZO_HIP(launch_sum_partials(nullptr, 0, sumsq_dev, st));
    return QZO_OK;
  }
  GemmArgs g = {};
  g.x = x_dev; g.w = codes_dev; g.cb = codebook_dev; g.s = c_dev; g.y = y_dev;
  g.M = M; g.N = N; g.K = K; g.row_base = row_base;
  g.seed_lo = (uint32_t)seed; g.seed_hi = (uint32_t)(seed >> 32);
  g.eps_signed = sign > 0 ? eps : -eps;
  const uint32_t tiles = ((M + 255) / 256) * ((N + 255) / 256);
  if (sumsq_dev) {
    g.epi = EPI_SUMSQ;
    g.partials = (float*)scratch_dev;
  }
  QZO_HIP(launch_codebook_gemm(g, st));
  if (sumsq_dev) QZO_HIP(launch_sum_partials((const float*)scratch_dev, tiles, sumsq_dev, st));
  return QZO_OK;
}

static qzo_status int4_expand_check(const void* q_dev, const void* s_dev, const int32_t* g_idx_dev,
                                    uint32_t K, uint32_t group, float eps, int sign) {
  if (!q_dev || !s_dev) return fail(QZO_ERR_ARG, "null device pointer");
  if (!aligned16(q_dev) || !aligned16(s_dev) || !aligned16(g_idx_dev))
    return fail(QZO_ERR_ALIGN, "device pointer not 16-byte aligned");
  if (group != 128 || K == 0 || K % 128) return fail(QZO_ERR_SHAPE, "group must be 128 and divide K");
  if (sign != 1 && sign != -1) return fail(QZO_ERR_ARG, "sign must be +1 or -1");
  if (!std::isfinite(eps)) return fail(QZO_ERR_ARG, "eps not finite");
  return QZO_OK;
}

qzo_status qzo_int4_expand(const void* q_dev, const void* s_dev, const void* zp_dev,
                           const int32_t* g_idx_dev, uint32_t row_base, uint32_t N, uint32_t K,
                           uint32_t group, uint64_t seed, float eps, int sign, float* se_dev, void* w_dev,
                           void* stream) {
  qzo_status st = int4_expand_check(q_dev, s_dev, g_idx_dev, K, group, eps, sign);
  if (st != QZO_OK) return st;
  if (!se_dev || !w_dev) return fail(QZO_ERR_ARG, "null output");
  if (!aligned16(se_dev) || !aligned16(w_dev)) return fail(QZO_ERR_ALIGN, "output not 16-byte aligned");
  QZO_HIP(launch_expand_int4(q_dev, s_dev, zp_dev, g_idx_dev, N, K, row_base, (uint32_t)seed,
                             (uint32_t)(seed >> 32), sign > 0 ? eps : -eps, false, se_dev, w_dev,
                             (hipStream_t)stream));
  return QZO_OK;
}

qzo_status qzo_int4_scratch_bytes(uint32_t N, uint32_t K, uint64_t* out) {
  if (!out) return fail(QZO_ERR_ARG, "out is null");
  *out = up256((uint64_t)N * K * 2) + up256((uint64_t)N * (K / 128) * 4);
  return QZO_OK;
}

qzo_status qzo_int4_gemm_expanded(const void* x_dev, const void* q_dev, const void* s_dev, const void* zp_dev,
                                  const int32_t* g_idx_dev, uint32_t row_base, uint32_t M, uint32_t N,
                                  uint32_t K, uint32_t group, uint64_t seed, float eps, int sign, void* y_dev,
                                  void* scratch_dev, uint64_t scratch_bytes, void* stream) {
  qzo_status st = int4_expand_check(q_dev, s_dev, g_idx_dev, K, group, eps, sign);
  if (st != QZO_OK) return st;
  if (!x_dev || !y_dev || !scratch_dev) return fail(QZO_ERR_ARG, "null device pointer");
  if (!aligned16(x_dev) || !aligned16(y_dev) || ((uintptr_t)scratch_dev & 255u))
    return fail(QZO_ERR_ALIGN, "x/y need 16-byte, scratch 256-byte alignment");
  if (N % 8) return fail(QZO_ERR_SHAPE, "N must be a multiple of 8");
  uint64_t need = 0;
  qzo_int4_scratch_bytes(N, K, &need);
  if (scratch_bytes < need) return fail(QZO_ERR_WORKSPACE, "scratch too small: see qzo_int4_scratch_bytes");
  if (!bf16_gemm_fits(M, N, K)) return fail(QZO_ERR_SHAPE, "an operand exceeds 2^31 bytes");
  if (M == 0 || N == 0) return QZO_OK;
  hipStream_t s = (hipStream_t)stream;
  unsigned char* wexp = (unsigned char*)scratch_dev;
  float* se = (float*)(wexp + up256((uint64_t)N * K * 2));
  QZO_HIP(launch_expand_int4(q_dev, s_dev, zp_dev, g_idx_dev, N, K, row_base, (uint32_t)seed,
                             (uint32_t)(seed >> 32), sign > 0 ? eps : -eps, false, se, wexp, s));
  GemmArgs g = {};
  g.x = x_dev; g.w = wexp; g.y = y_dev; g.M = M; g.N = N; g.K = K;
  QZO_HIP(launch_bf16_gemm(g, PLAIN_GEMM_PIPE, s));
  return QZO_OK;
}

static qzo_status nf4_check(const void* q_dev, const void* s_dev, uint32_t N, uint32_t K, uint32_t block,
                            float eps, int sign) {
  if (!q_dev || !s_dev) return fail(QZO_ERR_ARG, "null device pointer");
  if (!aligned16(q_dev) || !aligned16(s_dev)) return fail(QZO_ERR_ALIGN, "device pointer not 16-byte aligned");
  if (block != 64 || K == 0 || K % 128) return fail(QZO_ERR_SHAPE, "block must be 64 and K a positive multiple of 128");
  if (N % 8) return fail(QZO_ERR_SHAPE, "N must be a multiple of 8");
  if (sign != 1 && sign != -1) return fail(QZO_ERR_ARG, "sign must be +1 or -1");
  if (!std::isfinite(eps)) return fail(QZO_ERR_ARG, "eps not finite");
  return QZO_OK;
}

qzo_status qzo_nf4_expand(const void* q_dev, const void* s_dev, uint32_t row_base, uint32_t N, uint32_t K,
                          uint32_t block, uint64_t seed, float eps, int sign, float* se_dev, void* w_dev,
                          void* stream) {
  qzo_status st = nf4_check(q_dev, s_dev, N, K, block, eps, sign);
  if (st != QZO_OK) return st;
  if (!se_dev || !w_dev) return fail(QZO_ERR_ARG, "null output");
  if (!aligned16(se_dev) || !aligned16(w_dev)) return fail(QZO_ERR_ALIGN, "output not 16-byte aligned");
  QZO_HIP(launch_expand_nf4(q_dev, s_dev, N, K, row_base, (uint32_t)seed, (uint32_t)(seed >> 32),
                            sign > 0 ? eps : -eps, false, se_dev, w_dev, (hipStream_t)stream));
  return QZO_OK;
}

qzo_status qzo_nf4_scratch_bytes(uint32_t N, uint32_t K, uint64_t* out) {
  if (!out) return fail(QZO_ERR_ARG, "out is null");
  *out = up256((uint64_t)N * K * 2) + up256((uint64_t)N * (K / 64) * 4);
  return QZO_OK;
}

qzo_status qzo_nf4_gemm(const void* x_dev, const void* q_dev, const void* s_dev, uint32_t row_base,
                        uint32_t M, uint32_t N, uint32_t K, uint32_t block, uint64_t seed, float eps,
                        int sign, void* y_dev, void* scratch_dev, uint64_t scratch_bytes, void* stream) {
  qzo_status st = nf4_check(q_dev, s_dev, N, K, block, eps, sign);
  if (st != QZO_OK) return st;
  if (!x_dev || !y_dev || !scratch_dev) return fail(QZO_ERR_ARG, "null device pointer");
  if (!aligned16(x_dev) || !aligned16(y_dev) || ((uintptr_t)scratch_dev & 255u))
    return fail(QZO_ERR_ALIGN, "x/y need 16-byte, scratch 256-byte alignment");
  uint64_t need = 0;
  qzo_nf4_scratch_bytes(N, K, &need);
  if (scratch_bytes < need) return fail(QZO_ERR_WORKSPACE, "scratch too small: see qzo_nf4_scratch_bytes");
  if (!bf16_gemm_fits(M, N, K)) return fail(QZO_ERR_SHAPE, "an operand exceeds 2^31 bytes");
  if (M == 0 || N == 0) return QZO_OK;
  hipStream_t s = (hipStream_t)stream;
  unsigned char* wexp = (unsigned char*)scratch_dev;
  float* se = (float*)(wexp + up256((uint64_t)N * K * 2));
  QZO_HIP(launch_expand_nf4(q_dev, s_dev, N, K, row_base, (uint32_t)seed, (uint32_t)(seed >> 32),
                            sign > 0 ? eps : -eps, false, se, wexp, s));
  GemmArgs g = {};
  g.x = x_dev; g.w = wexp; g.y = y_dev; g.M = M; g.N = N; g.K = K;
  QZO_HIP(launch_bf16_gemm(g, PLAIN_GEMM_PIPE, s));
  return QZO_OK;
}

qzo_status qzo_model_set_int4_path(qzo_model* m, int mode) {
  if (!m) return fail(QZO_ERR_ARG, "model is null");
  if (mode < 0 || mode > 2) return fail(QZO_ERR_ARG, "mode must be 0 (by token count), 1 (fused) or 2 (expanded)");
  if (m->cfg.quant != 0 && m->cfg.quant != 2) return fail(QZO_ERR_UNSUPPORTED, "the model's format is not int4");
  m->int4_path = mode;
  return QZO_OK;
}

qzo_status qzo_debug_bf16_gemm(const void* x_dev, const void* w_dev, uint32_t M, uint32_t N, uint32_t K,
                               int pipe, void* y_dev, void* stream) {
  if (!x_dev || !w_dev || !y_dev) return fail(QZO_ERR_ARG, "null device pointer");
  if (!aligned16(x_dev) || !aligned16(w_dev) || !aligned16(y_dev))
    return fail(QZO_ERR_ALIGN, "device pointer not 16-byte aligned");
  if (K == 0 || K % 128) return fail(QZO_ERR_SHAPE, "K must be a positive multiple of 128");
  if (N % 8) return fail(QZO_ERR_SHAPE, "N must be a multiple of 8");
  if (pipe < 0 || pipe > 2) return fail(QZO_ERR_ARG, "pipe must be 0, 1 or 2");
  if (!bf16_gemm_fits(M, N, K)) return fail(QZO_ERR_SHAPE, "an operand exceeds 2^31 bytes");
  GemmArgs g = {};
  g.x = x_dev; g.w = w_dev; g.y = y_dev; g.M = M; g.N = N; g.K = K;
  QZO_HIP(launch_bf16_gemm(g, pipe, (hipStream_t)stream));
  return QZO_OK;
}

qzo_status qzo_apply_update_channel(void* c_dev, uint32_t n_rows, uint32_t row_base, uint64_t seed,
                                    float eta, float d_clipped, void* stream) {
  if (!c_dev) return fail(QZO_ERR_ARG, "c_dev is null");
  if (!std::isfinite(eta) || !std::isfinite(d_clipped)) return fail(QZO_ERR_ARG, "eta/d' not finite");
  QZO_HIP(launch_channel_update(c_dev, n_rows, row_base, (uint32_t)seed, (uint32_t)(seed >> 32), eta,
                                d_clipped, nullptr, (hipStream_t)stream));
  return QZO_OK;
}

qzo_status qzo_debug_mfma_rate(uint32_t iters, int random_operands, float* sink_dev,
                               uint32_t* workgroups_out, void* stream) {
  if (!sink_dev || !workgroups_out) return fail(QZO_ERR_ARG, "null pointer");
  if (iters == 0 || iters > (1u << 20)) return fail(QZO_ERR_ARG, "iters must be 1 .. 2^20");
  const uint32_t wgs = gemm_workgroups(1u << 20, 1u << 20);      // one per compute unit
  *workgroups_out = wgs;
  QZO_HIP(launch_mfma_rate(sink_dev, wgs, iters, random_operands != 0, (hipStream_t)stream));
  return QZO_OK;
}

qzo_status qzo_profile_begin(uint32_t max_records) {
  while (g_prof.pool.size() < max_records) {
    ProfRec r = {};
    QZO_HIP(hipEventCreate(&r.a));
    QZO_HIP(hipEventCreate(&r.b));
    g_prof.pool.push_back(r);
  }
  g_prof.used = 0;
  for (uint32_t& c : g_prof.seen) c = 0;
  g_prof.on = true;
  return QZO_OK;
}

qzo_status qzo_profile_stride(uint32_t stride) {
  if (stride == 0) return fail(QZO_ERR_ARG, "stride must be >= 1");
  g_prof.stride = stride;
  return QZO_OK;
}

qzo_status qzo_profile_collect(uint32_t kind, double* total_ms, uint64_t* launches, double* work) {
  if (!total_ms || !launches || !work) return fail(QZO_ERR_ARG, "null output");
  if (kind >= PK_COUNT) return fail(QZO_ERR_ARG, "unknown kernel class");
  g_prof.on = false;
  double ms = 0, wk = 0;
  uint64_t n = 0;
  for (size_t i = 0; i < g_prof.used; ++i) {
    ProfRec& r = g_prof.pool[i];
    if (r.kind != kind) continue;
    QZO_HIP(hipEventSynchronize(r.b));
    float t = 0;
    QZO_HIP(hipEventElapsedTime(&t, r.a, r.b));
    ms += t;
    wk += r.work;
    ++n;
  }
  *total_ms = ms; *launches = n; *work = wk;
  return QZO_OK;
}

qzo_status qzo_rtn_quantize(const float* w_dev, uint32_t N, uint32_t K, uint32_t group, void* q_dev,
                            void* s_dev, void* stream) {
  if (!w_dev || !q_dev || !s_dev) return fail(QZO_ERR_ARG, "null device pointer");
  if (!aligned16(w_dev) || !aligned16(q_dev) || !aligned16(s_dev))
    return fail(QZO_ERR_ALIGN, "device pointer not 16-byte aligned");
  if (group != 128 || K % 128) return fail(QZO_ERR_SHAPE, "group must be 128 and divide K");
  QZO_HIP(launch_rtn_quantize(w_dev, N, K, q_dev, s_dev, (hipStream_t)stream));
  return QZO_OK;
}

qzo_status qzo_rtn_quantize_asym(const float* w_dev, uint32_t N, uint32_t K, uint32_t group,
                                 uint32_t scale_fp16, void* q_dev, void* zp_dev, void* s_dev, void* stream) {
  if (!w_dev || !q_dev || !zp_dev || !s_dev) return fail(QZO_ERR_ARG, "null device pointer");
  if (!aligned16(w_dev) || !aligned16(q_dev) || !aligned16(s_dev))
    return fail(QZO_ERR_ALIGN, "device pointer not 16-byte aligned");
  if (group != 128 || K % 128) return fail(QZO_ERR_SHAPE, "group must be 128 and divide K");
  if (scale_fp16 > 1) return fail(QZO_ERR_ARG, "scale_fp16 must be 0 or 1");
  QZO_HIP(launch_rtn_quantize_asym(w_dev, N, K, scale_fp16 != 0, q_dev, zp_dev, s_dev, (hipStream_t)stream));
  return QZO_OK;
}

qzo_status qzo_debug_normals(uint64_t seed, uint32_t stream_id, uint32_t row0, uint32_t n_rows,
                             uint32_t G, float* out_dev, void* stream) {
  if (!out_dev) return fail(QZO_ERR_ARG, "out_dev is null");
  QZO_HIP(launch_debug_normals((uint32_t)seed, (uint32_t)(seed >> 32), stream_id, row0, n_rows, G,
                               out_dev, (hipStream_t)stream));
  return QZO_OK;
}
qzo_status qzo_debug_philox(uint64_t seed, const uint32_t* ctr_dev, uint32_t n, uint32_t* out_dev,
                            void* stream) {
  if (!ctr_dev || !out_dev) return fail(QZO_ERR_ARG, "null device pointer");
  QZO_HIP(launch_debug_philox((uint32_t)seed, (uint32_t)(seed >> 32), ctr_dev, n, out_dev,
                              (hipStream_t)stream));
  return QZO_OK;
}
qzo_status qzo_debug_normal_pairs(const uint32_t* words_dev, uint32_t n, float* out_dev,
                                  void* stream) {
  if (!words_dev || !out_dev) return fail(QZO_ERR_ARG, "null device pointer");
  QZO_HIP(launch_debug_normal_pairs(words_dev, n, out_dev, (hipStream_t)stream));
  return QZO_OK;
}
qzo_status qzo_debug_dequant(const void* q_dev, const void* s_dev, uint32_t row_base, uint32_t N,
                             uint32_t K, uint32_t group, uint64_t seed, float eps, int sign,
                             void* w_eff_dev, void* stream) {
  return qzo_debug_dequant_zp(q_dev, s_dev, nullptr, 0u, row_base, N, K, group, seed, eps, sign, w_eff_dev,
                              stream);
}

qzo_status qzo_debug_dequant_zp(const void* q_dev, const void* s_dev, const void* zp_dev,
                                uint32_t scale_fp16, uint32_t row_base, uint32_t N, uint32_t K,
                                uint32_t group, uint64_t seed, float eps, int sign, void* w_eff_dev,
                                void* stream) {
  if (scale_fp16 > 1) return fail(QZO_ERR_ARG, "scale_fp16 must be 0 or 1");
  if (!q_dev || !s_dev || !w_eff_dev) return fail(QZO_ERR_ARG, "null device pointer");
  if (!aligned16(q_dev) || !aligned16(s_dev) || !aligned16(w_eff_dev))
    return fail(QZO_ERR_ALIGN, "device pointer not 16-byte aligned");
  if (group != 128 || K == 0 || K % 128) return fail(QZO_ERR_SHAPE, "group must be 128 and divide K");
  if (sign != 1 && sign != -1) return fail(QZO_ERR_ARG, "sign must be +1 or -1");
  QZO_HIP(launch_debug_dequant(q_dev, s_dev, zp_dev, scale_fp16 != 0, row_base, N, K, (uint32_t)seed, (uint32_t)(seed >> 32),
                               sign > 0 ? eps : -eps, w_eff_dev, (hipStream_t)stream));
  return QZO_OK;
}

}  // extern "C"
