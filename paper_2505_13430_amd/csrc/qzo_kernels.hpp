// Host-side launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/qzo.h"

namespace qzo {

// One run of consecutive rows with the same number of groups per row, inside
// one decoder layer's slice of the scale arena.
struct UpdSeg {
  uint32_t off;        // first scale, relative to the layer's slice
  uint32_t rows, G;    // rows x G scales
  uint32_t row_base;   // noise row id of its first row, relative to the layer
  uint32_t first_wg;   // first workgroup (of 256 units) serving this segment
};
struct UpdPlan {
  UpdSeg seg[4];
  uint32_t n_seg;
  uint32_t wgs_per_layer;
  uint32_t n_layers;
  uint64_t layer_stride;     // scales per layer
  uint32_t rows_per_layer;
  uint32_t fp16;             // storage type of the arena: 0 bf16, 1 fp16
};

// Epilogue selection of the GEMM.
enum : uint32_t {
  EPI_BIAS = 1u,       // + bias[n]
  EPI_RESIDUAL = 2u,   // y = resid[m,n] + acc
  EPI_RELU = 4u,
  EPI_SUMSQ = 8u,      // per-workgroup sum of bf16(y)^2 into partials
  EPI_SWIGLU = 16u,    // W is [gate rows | up rows] (N = 2F): y[M,F] = silu(gate) * up
  EPI_ROPE = 32u,      // plain bf16 GEMM only: y is qkv [M, 3d] of heads of 64 or 128 features; the rotary embedding
                       // is applied to the q and k thirds on the way out (rope, rope_S); with heads of 128 the rows
                       // of W must be in ROW_ORDER_ROPE128 order
};

struct GemmArgs {
  const void* x;        // bf16 [M,K]
  const void* w;        // packed int4 [N,K/2] (W4) or bf16 [N,K] (dense)
  const void* s;        // bf16 [N,K/128] (W4) or fp16 [N] per-channel scales (codebook)
  const void* cb;       // fp16 [65536,8] codebook (codebook only)
  const void* zp;       // uint8 [N,K/128] zero-points (int4 only; null = symmetric, zero-point 8)
  const void* bias;     // bf16 [N] or null
  const void* resid;    // bf16 [M,N] or null
  void* y;              // bf16 [M,N]
  float* partials;      // EPI_SUMSQ: one float per workgroup
  float* skinny_ws;     // fp32 scratch of skinny_ws_floats(rows, N, K) floats: enables the few-token path (M <= 64)
  float* split_ws;      // fp32 scratch of tile_split_ws_floats(M, N, K) floats: enables split-K of the int4 tile kernel
  uint32_t ksplit, kt_per;   // set by the launcher: K slices and k-tiles per slice
  const float* rope;    // EPI_ROPE: (cos, sin) of [rope_S positions][dh/2 pairs]; row m sits at position m % rope_S
  uint32_t rope_S, rope_dh;
  uint32_t dual;        // both passes of a step stacked: x, y, resid hold 2 M rows; rows [0,M) use +eps_signed,
                        // [M,2M) -eps_signed (few-token path: M <= 32; tile path: see pass_stride)
  uint32_t pass_stride; // dual, tile path: the second pass starts at this row (a multiple of 256 >= M; x, y, resid
                        // hold pass_stride + M rows, the rows in between are padding); 0: at row M
  uint32_t flip_row;    // set by the launcher for the tile kernel: rows from here on take -eps_signed (0: none)
  uint32_t M, N, K;
  uint32_t ldy;         // row stride of y and resid in elements when the call covers a column block of a wider
                        // matrix (0: N); plain epilogues only (bias, residual, ReLU)
  uint32_t row_base;
  uint32_t seed_lo, seed_hi;
  float eps_signed;
  uint32_t epi;
  uint32_t s_fp16;      // int4 formats: s holds fp16 instead of bf16
  // Few-token path: block sums X[g][row] = sum of x[row, 128 g .. 128 g + 127] (fp32, [K/128][rows], rows = M or
  // 2 M when dual), delivered by the kernel that wrote x (null: the kernel sums them itself), and the same for
  // the output y of the K-slice reduction ([N_out/128][rows], N_out % 128 == 0; null: not wanted).
  const float* xsum;
  float* xsum_out;
};
hipError_t launch_w4a16_gemm(const GemmArgs& a, hipStream_t st);
// Order of the rows of an expanded (bf16) weight matrix: natural; the fused-SwiGLU consumer's tile order;
// the fused-RoPE consumer's order for heads of 128 features (within every 256 rows, so that a lane of the
// GEMM holds feature i and feature i + 64 of a head).
enum : int { ROW_ORDER_NATURAL = 0, ROW_ORDER_SWIGLU = 1, ROW_ORDER_ROPE128 = 2 };
// Few-token path (M <= 64): weights streamed once, K split over workgroups, partial sums in ws.
constexpr uint32_t SKINNY_MAX_M = 64;
constexpr uint32_t STACK_TILE_MAX_M = 4096;  // tile kernel: the two passes share a launch up to this many tokens per pass
constexpr uint32_t SKINNY_MAX_M_DUAL = 32;   // per sign, when both perturbed passes share one launch
uint32_t skinny_ksplit(uint32_t N, uint32_t K);
uint64_t skinny_ws_floats(uint32_t M, uint32_t N, uint32_t K);
uint32_t skinny_reduce_blocks(uint32_t M, uint32_t N, uint32_t epi);   // EPI_SUMSQ partial count
hipError_t launch_skinny_gemm(const GemmArgs& a, float* ws, hipStream_t st);
// Adds K-slice partial sums part[slice][M][N] in slice order and applies a's epilogue.
hipError_t launch_partial_reduce(const GemmArgs& a, const float* part, uint32_t ksplit, hipStream_t st);
// Split-K of the int4 tile kernel when an M x N output has too few 256 x 256 tiles for the chip:
// number of K slices (1: none) and k-tiles per slice.
uint32_t tile_ksplit(uint32_t M, uint32_t N, uint32_t K, uint32_t* kt_per);
// Column split of a launch whose output tiles are a little more than whole rounds of the chip: the first
// tile_tail_cols(...) columns (whole rounds, ordinary launch) and the rest (at most half a round of tiles,
// cut along K so that they fill the chip); 0: no split.  Plain epilogues only.
uint32_t tile_tail_cols(uint32_t M, uint32_t N, uint32_t K, uint32_t epi);
uint64_t tile_split_ws_floats(uint32_t M, uint32_t N, uint32_t K);
// w = uint16 codes [N,K/8]; cb and s as above; N % 8 == 0, K % 128 == 0.
hipError_t launch_codebook_gemm(const GemmArgs& a, hipStream_t st);
// pipe: 0 / 1 = operand tiles staged through registers (compiler's / explicit issue order),
// 2 = loaded from memory straight into the LDS.
hipError_t launch_bf16_gemm(const GemmArgs& a, int pipe, hipStream_t st);
// The plain bf16 GEMM with one wavefront per SIMD and deferred output stores (no split-K): what
// launch_bf16_gemm(pipe = 2) runs when the output tiles fill the chip.
hipError_t launch_bf16_gemm_wide(const GemmArgs& a, hipStream_t st);
constexpr int PLAIN_GEMM_PIPE = 2;     // the route the models take: 3 % faster than 1 on a full step
// One linear's perturbed weights written out as bf16 [N,K] (rows in the GEMM's tile order
// when the consumer fuses SwiGLU), for launch_bf16_gemm.
hipError_t launch_expand_codebook(const void* codes, const void* cb, const void* c_fp16, uint32_t N,
                                  uint32_t K, uint32_t row_base, uint32_t seed_lo, uint32_t seed_hi,
                                  float eps_signed, int swiglu, void* out_bf16, hipStream_t st);
// NormalFloat-4 blocks of 64: se_scratch receives the perturbed scales, fp32 [N, K/64].
hipError_t launch_expand_nf4(const void* q, const void* s_bf16, uint32_t N, uint32_t K, uint32_t row_base,
                             uint32_t seed_lo, uint32_t seed_hi, float eps_signed, int swiglu,
                             float* se_scratch, void* out_bf16, hipStream_t st);
// int4 groups of 128 (zp: uint8 [N, K/128] or null = 8; g_idx: int32 [K] group of each column, or
// null = k / 128): se_scratch fp32 [N, K/128].
hipError_t launch_expand_int4(const void* q, const void* s_bf16, const void* zp, const int32_t* g_idx,
                              uint32_t N, uint32_t K, uint32_t row_base, uint32_t seed_lo, uint32_t seed_hi, float eps_signed,
                              int swiglu, float* se_scratch, void* out_bf16, hipStream_t st);
// Inside a model the perturbed scales of every linear are written by one launch per pass (fp32, laid
// out like the scale arena) and the expansions read them from there.
hipError_t launch_perturbed_scales_all(const void* arena, const UpdPlan& plan, uint32_t seed_lo, uint32_t seed_hi,
                                       float eps_signed, float* se_all, hipStream_t st);
hipError_t launch_expand_int4_from(const void* q, const float* se, const void* zp, const int32_t* g_idx,
                                   uint32_t N, uint32_t K, int swiglu, void* out_bf16, hipStream_t st);
hipError_t launch_expand_nf4_from(const void* q, const float* se, uint32_t N, uint32_t K, int swiglu,
                                  void* out_bf16, hipStream_t st);
// Tokens per pass from which an int4 linear [N,K] is expanded first.  The expansion costs two short
// launches (about 8 us) plus 2.5 bytes per weight at about 4.5 TB/s; the fused kernel needs about 13.6 %
// more time than the plain GEMM on the expanded weights, a time that grows with the tokens
// (2 M N K flop at about 1.3 PFLOP/s).  Setting the two equal gives M = a + b / (N K) with a near
// 2700 and b near 4e10; fitted to the measurements (Llama-2-7B widths: a tie at 2560 tokens, the
// expansion 3 % ahead at 3072; 13B widths: 4.5 % ahead at 4096; OPT-1.3B widths, d = 2048: 7 % behind
// at 4096) a = 2300, b = 3.3e10.
// The codebook format is always expanded inside a model: its fused kernel is 45 % slower than the
// plain GEMM and cannot split K.
inline uint32_t expand_min_m_int4(uint32_t N, uint32_t K) {
  return 2300u + (uint32_t)(3.3e10 / ((double)N * (double)K));
}
constexpr uint32_t EXPAND_MIN_M_CODEBOOK = 1;
hipError_t launch_channel_update(void* c_fp16, uint32_t n, uint32_t row_base, uint32_t seed_lo,
                                 uint32_t seed_hi, float eta, float d_clipped,
                                 const qzo_step_result* res, hipStream_t st);
// One 16-bit tensor of the model table inside the flat vector of un-quantized parameters.
struct DenseSeg {
  uint64_t first8;     // first entry / 8
  void* out;           // the tensor (device), written by the perturbation
  uint32_t fmt;        // 0: bf16, 1: fp16
  uint32_t pad;
};
hipError_t launch_dense_perturb(const float* master, const DenseSeg* segs_dev, uint32_t n_seg,
                                uint64_t n_dense, uint32_t seed_lo, uint32_t seed_hi, float eps_signed,
                                hipStream_t st);
hipError_t launch_dense_update(float* master, uint64_t n_dense, uint32_t seed_lo, uint32_t seed_hi,
                               float eta, float d_clipped, const qzo_step_result* res, hipStream_t st);
uint32_t gemm_workgroups(uint32_t M, uint32_t N);

// lm_head GEMM with the cross-entropy folded into the epilogue: for every row
// m and every 64-column slice it writes (max, sum exp(l - max)) and, where the
// target column falls in the slice, the target logit.
struct CeArgs {
  const void* x;        // bf16 [M,K]  final hidden states
  const void* w;        // bf16 [V,K]  lm_head
  const int32_t* tok;   // [B,S]; row m takes its target from tok[(m % tok_rows) + 1]
  uint32_t tok_rows;    // B*S (M is a multiple of it: the same batch may be stacked twice)
  float* part;          // [M, n_slices, 2]
  float* tgt;           // [M]
  uint32_t M, V, K, S;
  uint32_t n_slices;    // ceil(V/256)*4
};
hipError_t launch_lmhead_ce(const CeArgs& a, hipStream_t st);
hipError_t launch_mfma_rate(float* sink, uint32_t workgroups, uint32_t iters, int random_operands,
                            hipStream_t st);
hipError_t launch_ce_reduce(const float* part, const float* tgt, uint32_t M, uint32_t S,
                            uint32_t n_slices, float* rowloss, float* loss_out, hipStream_t st);

hipError_t launch_sum_partials(const float* partials, uint32_t n, float* out, hipStream_t st);

// pass_stride: rows per pass of a stacked forward (M for a single pass); rows m % pass_stride >= tok_rows get zeros.
hipError_t launch_embed(const int32_t* tok, uint32_t tok_rows, uint32_t pass_stride, const void* tok_emb,
                        const void* pos_emb, uint32_t M, uint32_t S, uint32_t d, void* h, hipStream_t st);
// xsum_t (nullable, d % 128 == 0): receives the block sums of the output, [d/128][M] fp32 (see GemmArgs::xsum)
hipError_t launch_rmsnorm(const void* x, const void* gain, uint32_t M, uint32_t d, float eps,
                          void* y, hipStream_t st, float* xsum_t = nullptr);
hipError_t launch_layernorm(const void* x, const void* gain, const void* bias, uint32_t M,
                            uint32_t d, float eps, void* y, hipStream_t st, float* xsum_t = nullptr);
hipError_t launch_rope_table(float* table, uint32_t max_seq, uint32_t dh, float theta,
                             hipStream_t st);
hipError_t launch_rope(void* qkv, const float* table, uint32_t M, uint32_t S, uint32_t pass_stride, uint32_t d,
                       uint32_t n_heads, hipStream_t st);
// rope (nullable): the (cos, sin) table; with it the kernel rotates q and k itself (qkv holds them unrotated).
constexpr uint32_t ATTENTION_ROPE_MAX_S = 256;   // up to this sequence length the models let it do so
hipError_t launch_attention(const void* qkv, uint32_t B, uint32_t S, uint32_t n_heads,
                            uint32_t dh, void* out, const float* rope, hipStream_t st);
hipError_t launch_spsa_clip(const float* losses, float eps, float clip, qzo_step_result* res,
                            hipStream_t st);
hipError_t launch_scale_update(void* arena, const UpdPlan& plan, uint32_t seed_lo,
                               uint32_t seed_hi, float eta, float d_clipped,
                               const qzo_step_result* res, hipStream_t st);
hipError_t launch_rtn_quantize(const float* w, uint32_t N, uint32_t K, void* q, void* s,
                               hipStream_t st);
hipError_t launch_rtn_quantize_asym(const float* w, uint32_t N, uint32_t K, bool s_fp16, void* q, void* zp,
                                    void* s, hipStream_t st);
hipError_t launch_debug_normals(uint32_t seed_lo, uint32_t seed_hi, uint32_t stream_id,
                                uint32_t row0, uint32_t n_rows, uint32_t G, float* out,
                                hipStream_t st);
hipError_t launch_debug_philox(uint32_t seed_lo, uint32_t seed_hi, const uint32_t* ctr,
                               uint32_t n, uint32_t* out, hipStream_t st);
hipError_t launch_debug_normal_pairs(const uint32_t* words, uint32_t n, float* out,
                                     hipStream_t st);
hipError_t launch_repack_kmajor(const void* qweight, const void* qzeros, const void* scales,
                                uint32_t N, uint32_t K, uint32_t zero_add, bool s_fp16, void* q_out,
                                void* zp_out, void* s_out, hipStream_t st);
hipError_t launch_debug_dequant(const void* q, const void* s, const void* zp, bool s_fp16, uint32_t row_base,
                                uint32_t N, uint32_t K, uint32_t seed_lo, uint32_t seed_hi, float eps_signed,
                                void* w_eff, hipStream_t st);

}  // namespace qzo
