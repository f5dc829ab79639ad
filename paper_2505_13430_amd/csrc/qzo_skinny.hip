// Perturbed W4A16 linear for few tokens (M <= 64): Y[M,N] = X[M,K] * W_eff^T with
//   W_eff[n,k] = (s[n,k/128] + sigma*eps*z(row_base+n, k/128)) * (u[n,k] - zp[n,k/128])   (paper Eq. 4-5;
// zp = 8 without zero-points).  At this size every weight is used once per token tile, so the kernel
// is bound by streaming the int4 weights from HBM and by the work of turning them into MFMA
// operands, not by the matrix pipe.
//
// A workgroup of four wavefronts owns 128 output rows and one slice of K; each wavefront owns 32
// rows.  The weights of a row are contiguous in memory, and a load instruction costs the memory
// pipeline one access per cache line it touches, so eight neighbouring lanes read one whole 128-byte
// line of a row (two groups): an instruction touches 8 lines, not 64 (a lane per row costs 11 us
// for the 25 MB of a 12288 x 4096 matrix whatever else the kernel does).  A round of four such
// instructions brings two groups of the wavefront's 32 rows into registers, two rounds ahead;
// the MFMA wants a lane per row, so each round passes through a 4 KB LDS buffer that only its
// wavefront uses (16-byte chunks swizzled by the row: neither side has bank conflicts; a
// wavefront's LDS instructions execute in order, so no barrier is involved).
//
// The scale is applied to the group's partial sums, not to the weights: a dword of eight nibbles
// becomes eight bf16 values 128 + u with seven integer operations (0x4300 | u is the bf16 pattern
// of 128 + u), the MFMAs accumulate P[n,m] = sum_k (128 + u[n,k]) x[m,k] over the group's 128
// inputs (products of bf16 values are exact, fp32 accumulation), and once per group
//   y[n,m] += s_eff[n,g] * (P[n,m] - (128 + zp[n,g]) * X[m,g]),   X[m,g] = sum_k x[m,k]
// in fp32, with X[m,g] summed while the activation block goes to LDS.  The weights are not
// rounded to bf16 at all (the result is closer to Eq. 4-5 than a bf16 weight tile's), the work per
// weight is a third of unpack + fma + round, and the two perturbed passes of a QZO step, which
// differ in s_eff only, share everything but the last line.
// The unpack yields the k order 0,4,1,5,2,6,3,7 inside a dword; the activation block is stored to LDS
// in the same order (the contraction index of an MFMA k-step is free as long as both operands agree).
//
// Partial sums of the K slices go to a scratch buffer in fp32; a second kernel adds them in slice
// order and applies the epilogue: deterministic.  (Letting the workgroup that finishes an output
// block last do the reduction - an arrival counter per block, the partial sums stored and loaded
// past the per-XCD L2 caches - was measured: 25.7 us per linear against 17.5 + 4.7 us for the
// two launches at 1 x 16 tokens on the 7B shapes; store acknowledgement, counter round trip and
// uncached loads all sit on the last workgroup's path.)
//
// Dual mode: the +eps and the -eps pass of one QZO step read the same int4 weights and the same
// noise, so for very few tokens they share one launch.  X and Y then hold the two passes stacked
// (rows [0,M) and [M,2M)).
#include "qzo_device.hpp"
#include "qzo_kernels.hpp"

namespace qzo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int SK_ROWS = 128;      // output rows per workgroup
constexpr int SK_WD = 8;          // groups per pass of the K loop: four rounds of two groups, all in flight

// 8 nibbles of one dword -> the bf16 values 128 + u, in the order k = 0,4,1,5,2,6,3,7.
// One bitfield insert per pair ((mask & w) | (~mask & 0x43004300)) with the two constants in
// registers; written as "and, or" with literals the compiler spends two instructions on it.
__device__ __forceinline__ uint32_t bias_pair(uint32_t w, uint32_t mask, uint32_t magic) {
  uint32_t r;
  asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(r) : "s"(mask), "v"(w), "v"(magic));
  return r;
}
__device__ __forceinline__ bf16x8 unpack8_biased(uint32_t w, uint32_t mask, uint32_t magic) {
  union { bf16x8 v; uint32_t u[4]; } r;
  r.u[0] = bias_pair(w, mask, magic);
  r.u[1] = bias_pair(w >> 4, mask, magic);
  r.u[2] = bias_pair(w >> 8, mask, magic);
  r.u[3] = bias_pair(w >> 12, mask, magic);
  return r.v;
}
// 8 consecutive bf16 (4 dwords) -> the same order 0,4,1,5,2,6,3,7
__device__ __forceinline__ u32x4 permute8(u32x4 x) {
  u32x4 r;
  r.x = __builtin_amdgcn_perm(x.z, x.x, 0x05040100u);    // (x0, x4): low halves of dwords 0 and 2
  r.y = __builtin_amdgcn_perm(x.z, x.x, 0x07060302u);    // (x1, x5): high halves
  r.z = __builtin_amdgcn_perm(x.w, x.y, 0x05040100u);    // (x2, x6)
  r.w = __builtin_amdgcn_perm(x.w, x.y, 0x07060302u);    // (x3, x7)
  return r;
}
// sum of 8 bf16 values in fp32
__device__ __forceinline__ float sum8_bf16(u32x4 x) {
  const uint32_t d[4] = {x.x, x.y, x.z, x.w};
  float lo = 0.0f, hi = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    lo += __uint_as_float(d[i] << 16);
    hi += __uint_as_float(d[i] & 0xffff0000u);
  }
  return lo + hi;
}

__device__ __forceinline__ uint32_t x_lds_off(uint32_t row, uint32_t chunk) {   // 256-byte rows, 16 chunks
  return row * 256u + ((chunk ^ (row & 15u)) << 4);
}

// One output item of the slice reduction: 4 consecutive output features f .. f+3 of token m.
// Adds the K-slice partials in slice order and applies the epilogue; returns the sum of the squares
// of the stored bf16 values (and their plain sum in `sum`).
__device__ __forceinline__ float reduce_item(const GemmArgs& a, const float* __restrict__ part, uint32_t ksplit,
                                             uint32_t m, uint32_t f, float& sum) {
  const bool swiglu = (a.epi & EPI_SWIGLU) != 0;
  const uint32_t NO = swiglu ? a.N >> 1 : a.N;
  auto load4 = [&](uint32_t ks, uint32_t col) {
    return *reinterpret_cast<const float4*>(part + ((uint64_t)ks * a.M + m) * a.N + col);
  };
  // four slices' loads in flight at a time (one at a time, the loop is a chain of memory
  // latencies); the additions stay in slice order
  float v[4] = {0, 0, 0, 0}, u[4] = {0, 0, 0, 0};
  for (uint32_t k0 = 0; k0 < ksplit; k0 += 4) {
    float4 p[4], pu[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t ks = min(k0 + i, ksplit - 1);
      p[i] = load4(ks, f);
      if (swiglu) pu[i] = load4(ks, NO + f);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (k0 + i < ksplit) {
        v[0] += p[i].x; v[1] += p[i].y; v[2] += p[i].z; v[3] += p[i].w;
        if (swiglu) { u[0] += pu[i].x; u[1] += pu[i].y; u[2] += pu[i].z; u[3] += pu[i].w; }
      }
    }
  }
  if (swiglu) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      v[c] = v[c] * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504f * v[c])) * u[c];
  }
  if (a.epi & EPI_BIAS) {
    const uint2 bb = *reinterpret_cast<const uint2*>((const bf16_t*)a.bias + f);
    v[0] += __uint_as_float(bb.x << 16); v[1] += __uint_as_float(bb.x & 0xffff0000u);
    v[2] += __uint_as_float(bb.y << 16); v[3] += __uint_as_float(bb.y & 0xffff0000u);
  }
  const uint64_t o = (uint64_t)m * (a.ldy ? a.ldy : NO) + f;
  if (a.epi & EPI_RESIDUAL) {
    const uint2 rr = *reinterpret_cast<const uint2*>((const bf16_t*)a.resid + o);
    v[0] += __uint_as_float(rr.x << 16); v[1] += __uint_as_float(rr.x & 0xffff0000u);
    v[2] += __uint_as_float(rr.y << 16); v[3] += __uint_as_float(rr.y & 0xffff0000u);
  }
  if (a.epi & EPI_RELU) {
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = fmaxf(v[c], 0.0f);
  }
  uint2 out;
  out.x = pack_bf16x2(v[0], v[1]);
  out.y = pack_bf16x2(v[2], v[3]);
  *reinterpret_cast<uint2*>((bf16_t*)a.y + o) = out;
  const float q0 = __uint_as_float(out.x << 16), q1 = __uint_as_float(out.x & 0xffff0000u);
  const float q2 = __uint_as_float(out.y << 16), q3 = __uint_as_float(out.y & 0xffff0000u);
  sum = (q0 + q2) + (q1 + q3);
  return q0 * q0 + q1 * q1 + q2 * q2 + q3 * q3;
}

// MT = 32-row activation tiles (1 or 2).  grid = (ceil(N/128), ksplit); part is [ksplit, rows, N]
// fp32 with rows = M, or 2 M in dual mode.  In dual mode the tile rows are split between the
// passes: rows [0, 16 MT) are tokens of the +eps pass, rows [16 MT, 32 MT) the same tokens of
// the -eps pass (M <= 16 MT).
// XSUM_BY_MFMA (one token tile, at most 16 tokens per pass: the stacked and the separate passes of
// a step then sum alike, bit for bit): the block sums come from the matrix unit, see below.
// XIN: the block sums come from memory (GemmArgs::xsum, written by the kernel that wrote x); a pass's 8 groups
// x tile rows are fetched one pass ahead, one or two values per thread, and handed on through the LDS.
// (One token tile with XIN fits 168 registers: three workgroups per CU, which holds the 688 workgroups of a
// 22016-row gate/up linear in one round.)
template <int MT, bool DUAL, bool ZP, bool XSUM_BY_MFMA, bool XIN>
__global__ __launch_bounds__(256, (MT == 1 && XIN) ? 3 : 2) void skinny_gemm_kernel(GemmArgs a, float* part,
                                                             uint32_t groups_per_split) {
  constexpr uint32_t TPP = DUAL ? MT * 16 : MT * 32;      // tile rows per pass
  __shared__ __attribute__((aligned(16))) unsigned char xs[2][MT * 32 * 256];
  __shared__ __attribute__((aligned(16))) float xsum[2][MT * 32];          // X[m,g] of the block in the same buffer
  __shared__ __attribute__((aligned(16))) unsigned char wt[4][32 * 128];   // per wavefront: a round of its 32 rows
  __shared__ __attribute__((aligned(16))) float xin[2][XIN ? SK_WD : 1][MT * 32];   // XIN: X[g][tile row] of two passes
  const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
  const uint32_t lrow = lane & 31u, half = lane >> 5;     // MFMA operand: row of the wavefront, half of the k-step
  const uint32_t lr = lane >> 3, lc = lane & 7u;          // loads: row within an instruction's 8 rows, 16-byte chunk
  const uint32_t K = a.K, ngrp = K >> 7;
  const uint32_t g0 = blockIdx.y * groups_per_split, g1 = min(g0 + groups_per_split, ngrp);   // g0 is even
  const uint32_t nb = blockIdx.x * SK_ROWS + wave * 32;   // the wavefront's first row
  const uint32_t n_own = nb + lrow;
  const uint32_t n = min(n_own, a.N - 1);                 // the row this lane feeds to the MFMA
  const bool s_fp16 = a.s_fp16 != 0;
  const uint32_t nib_mask = 0x000f000fu;
  uint32_t nib_magic;
  asm volatile("v_mov_b32 %0, 0x43004300" : "=v"(nib_magic));      // kept in a vector register

  // y[m][4 b + c]: weight row n, tile row 32 m + 8 b + 4 half + c
  floatx16 y[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int r = 0; r < 16; ++r) y[m][r] = 0.0f;

  if (g0 < g1) {
    // All loads of the K loop are buffer loads whose offset is pushed out of range for groups
    // beyond the slice (and is out of range by itself for rows beyond N): such a load returns zero
    // and moves no data, and every pass issues the same instructions, so the wait for a load
    // counts the loads issued after it and nothing more.
    constexpr uint32_t OUT_OF_RANGE = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(a.x), 0, (int)((uint64_t)(DUAL ? 2 * a.M : a.M) * K * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(a.w), 0, (int)((uint64_t)a.N * (K >> 1)), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(a.s), 0, (int)((uint64_t)a.N * ngrp * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(ZP ? a.zp : a.s), 0, (int)((uint64_t)a.N * ngrp), 0x00020000);
    const uint32_t woff = (nb + lr) * (K >> 1) + lc * 16;           // instruction i: + 8 i rows
    const uint32_t wstep = 8 * (K >> 1);
    const uint32_t soff = n * ngrp;
    // scales (zero-points) of eight groups in one load when every row starts on a dword
    const bool s_wide = (ngrp & 1u) == 0, z_wide = (ngrp & 3u) == 0;

    // activation staging: a group's block is MT*32 rows x 16 chunks of 16 bytes; a thread moves MT*2 chunks.
    // Tile row -> row of x: clamped to the pass's last token.
    static_assert(!XSUM_BY_MFMA || MT == 1, "no registers for it with two token tiles");
    static_assert(!(XIN && XSUM_BY_MFMA), "one source of the block sums");
    constexpr int NX = MT * 2;
    uint32_t xoff[NX];
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      const uint32_t c = t + 256u * i, row = c >> 4, ch = c & 15u;
      const uint32_t xrow = DUAL ? (row / TPP) * a.M + min(row % TPP, a.M - 1) : min(row, a.M - 1);
      xoff[i] = xrow * K * 2 + ch * 16;
    }
    // The counter of outstanding loads retires in issue order: waiting for a load waits for every
    // older one.  So the activation blocks are requested as far ahead as the weights (four groups);
    // a block requested just in time would cut the weights' lead down to its own.
    // With two token tiles the registers do not allow it: two groups ahead there, and also where one tile
    // runs three workgroups per CU (XIN).
    constexpr int XD = (MT == 1 && !XIN) ? 4 : 2;
    u32x4 xr[XD][NX];           // the next XD blocks on their way: block g0 + j in slot j % XD
#define QZO_SK_XLOAD(SLOT, G_)                                                               \
  do {                                                                                       \
    const uint32_t go_ = (G_) < g1 ? (G_) * 256u : OUT_OF_RANGE;                             \
    _Pragma("unroll") for (int i = 0; i < NX; ++i)                                           \
      xr[SLOT][i] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(xoff[i] + go_), 0, 0);   \
  } while (0)
    // The block sums X[m,g] = sum_k x[m,k]: with few tokens the matrix unit computes them (a second
    // MFMA per k-step on the same activation fragment, against a fragment of ones: its accumulator
    // holds X of exactly the tile rows the lane rescales, and the matrix unit has the time); with two
    // tiles there are no registers for that, and the staging threads add them up:
    // the 16 threads of a row are 16 consecutive lanes: their chunk sums meet in four exchange steps.
    // The K loop holds no divergent branch, so that its uniform branches stay plain scalar branches.
#define QZO_SK_XSTORE(SLOT, BUF)                                                             \
  do {                                                                                       \
    _Pragma("unroll") for (int i = 0; i < NX; ++i) {                                         \
      const uint32_t c = t + 256u * i, row = c >> 4, ch = c & 15u;                           \
      *reinterpret_cast<u32x4*>(xs[BUF] + x_lds_off(row, ch)) = permute8(xr[SLOT][i]);       \
      if (!XSUM_BY_MFMA && !XIN) {                                                           \
        float sx_ = sum8_bf16(xr[SLOT][i]);                                                  \
        sx_ += __shfl_xor(sx_, 1, 64); sx_ += __shfl_xor(sx_, 2, 64);                        \
        sx_ += __shfl_xor(sx_, 4, 64); sx_ += __shfl_xor(sx_, 8, 64);                        \
        xsum[BUF][row] = sx_;         /* all 16 lanes of the row hold the sum */             \
      }                                                                                      \
    }                                                                                        \
  } while (0)

    // weights in flight: the round of groups g0 + 2 j, g0 + 2 j + 1 in slot j % 2; instruction i
    // of a round holds rows 8 i + lr, bytes [16 lc, 16 lc + 16) of the two groups' 128
    u32x4 wq[2][4];
#define QZO_SK_WLOAD(SLOT, G_)                                                               \
  do {                                                                                       \
    const uint32_t wo_ = woff + ((G_) < g1 ? (G_) * 64u : OUT_OF_RANGE);                     \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                            \
      wq[SLOT][i] = __builtin_amdgcn_raw_buffer_load_b128(rw, (int)(wo_ + i * wstep), 0, 0); \
  } while (0)
    // a round to the wavefront's LDS buffer: row r, chunk c at 128 r + 16 (c ^ r % 8)
    unsigned char* wtw = wt[wave];
#define QZO_SK_WSTORE(SLOT)                                                                  \
  do {                                                                                       \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                            \
      *reinterpret_cast<u32x4*>(wtw + (8 * i + lr) * 128 + ((lc ^ lr) << 4)) = wq[SLOT][i];  \
  } while (0)
    // scales and zero-points of the eight groups from G_ on, 16 (8) bits each, for row n
    u32x4 sv, sv_next;
    uint32_t zv[2] = {0, 0}, zv_next[2] = {0, 0};
#define QZO_SK_SLOAD(G_)                                                                     \
  do {                                                                                       \
    const bool in_ = (G_) < g1;                                                              \
    const uint32_t so_ = in_ ? (soff + (G_)) * 2u : OUT_OF_RANGE;                            \
    if (s_wide) {                                                                            \
      sv_next = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)so_, 0, 0);                   \
    } else {                                                                                 \
      uint32_t h_[8];                                                                        \
      _Pragma("unroll") for (int j = 0; j < 8; ++j)                                          \
        h_[j] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs, (int)so_, 2 * j, 0); \
      sv_next.x = h_[0] | (h_[1] << 16); sv_next.y = h_[2] | (h_[3] << 16);                  \
      sv_next.z = h_[4] | (h_[5] << 16); sv_next.w = h_[6] | (h_[7] << 16);                  \
    }                                                                                        \
    if (ZP) {                                                                                \
      const uint32_t zo_ = in_ ? soff + (G_) : OUT_OF_RANGE;                                 \
      if (z_wide) {                                                                          \
        typedef uint32_t u32x2_ __attribute__((ext_vector_type(2)));                         \
        const u32x2_ z2_ = __builtin_amdgcn_raw_buffer_load_b64(rz, (int)zo_, 0, 0);         \
        zv_next[0] = z2_.x; zv_next[1] = z2_.y;                                              \
      } else {                                                                               \
        uint32_t b_[8];                                                                      \
        _Pragma("unroll") for (int j = 0; j < 8; ++j)                                        \
          b_[j] = (uint32_t)(uint8_t)__builtin_amdgcn_raw_buffer_load_b8(rz, (int)zo_, j, 0); \
        zv_next[0] = b_[0] | (b_[1] << 8) | (b_[2] << 16) | (b_[3] << 24);                   \
        zv_next[1] = b_[4] | (b_[5] << 8) | (b_[6] << 16) | (b_[7] << 24);                   \
      }                                                                                      \
    }                                                                                        \
  } while (0)

    // XIN: element e = t + 256 i of a pass is (group e / (32 MT), tile row e % (32 MT)); X is [K/128][rows]
    const uint32_t xrows = DUAL ? 2 * a.M : a.M;
    const __amdgpu_buffer_rsrc_t rxs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(XIN ? a.xsum : (const float*)a.x), 0, (int)((uint64_t)xrows * ngrp * 4), 0x00020000);
    uint32_t xin_off[MT];
    float xin_next[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const uint32_t e = t + 256u * i, row = e % (MT * 32u);
      const uint32_t xrow = DUAL ? (row / TPP) * a.M + min(row % TPP, a.M - 1) : min(row, a.M - 1);
      xin_off[i] = ((e / (MT * 32u)) * xrows + xrow) * 4u;
      xin_next[i] = 0.0f;
    }
#define QZO_SK_XINLOAD(G_)                                                                   \
  do {                                                                                       \
    if (XIN) {                                                                               \
      _Pragma("unroll") for (int i = 0; i < MT; ++i) {                                       \
        const uint32_t gi_ = (G_) + (t + 256u * i) / (MT * 32u);                             \
        xin_next[i] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(                  \
            rxs, (int)(gi_ < g1 ? xin_off[i] + (G_) * xrows * 4u : OUT_OF_RANGE), 0, 0));    \
      }                                                                                      \
    }                                                                                        \
  } while (0)
    union { bf16x8 v; uint32_t u[4]; } ones;
    ones.u[0] = ones.u[1] = ones.u[2] = ones.u[3] = 0x3f803f80u;
    // noise: one Philox counter per 8 groups, one Box-Muller pair per 2 groups
    uint32_t zw[4] = {0, 0, 0, 0};
    float z_even = 0.0f, z_odd = 0.0f;
    bool fresh = true;

    // Memory returns in issue order: block g0 first, then the weights in the order of their use
    // with the activation blocks in between.
    QZO_SK_XLOAD(0, g0);
    QZO_SK_WLOAD(0, g0);
    QZO_SK_SLOAD(g0);
    QZO_SK_XINLOAD(g0);
    QZO_SK_XLOAD(1, g0 + 1);
    QZO_SK_WLOAD(1, g0 + 2);
#pragma unroll
    for (int j = 2; j < XD; ++j) QZO_SK_XLOAD(j, g0 + j);
    QZO_SK_XSTORE(0, 0);
    QZO_SK_XLOAD(0, g0 + XD);

    // Whole passes of SK_WD groups, no way out in between (a loop with one exit keeps the wait for
    // a load at "the loads issued after it", whichever path led here): for groups past the slice's
    // end the loads are still issued (out of range: they move nothing) and the arithmetic is skipped.
    for (uint32_t gb = g0; gb < g1; gb += SK_WD) {
      sv = sv_next;
      zv[0] = zv_next[0]; zv[1] = zv_next[1];
      QZO_SK_SLOAD(gb + SK_WD);
      const uint32_t xpp = ((gb - g0) / SK_WD) & 1u;      // XIN: this pass's LDS buffer (visible after the barrier of d = 0)
      if (XIN) {
#pragma unroll
        for (int i = 0; i < MT; ++i) (&xin[xpp][0][0])[t + 256u * i] = xin_next[i];
      }
      QZO_SK_XINLOAD(gb + SK_WD);
#pragma unroll
      for (int d = 0; d < SK_WD; ++d) {
        const uint32_t g = gb + d;
        const bool live = g < g1;
        const uint32_t buf = (uint32_t)d & 1u;            // (g - g0) % 2: SK_WD is even
        if ((d & 1) == 0) {                               // a new round: through the LDS, its slot refilled
          if (d & 2) { QZO_SK_WSTORE(1); QZO_SK_WLOAD(1, g + 4); }
          else { QZO_SK_WSTORE(0); QZO_SK_WLOAD(0, g + 4); }
        }
        __syncthreads();                                  // block g is complete, block g-1 has been read
        // block g+1 to the other buffer (if the slice has one), block g+1+XD requested.  Beyond the
        // slice's end only the loads are issued (they move nothing): the wait counts stay the same.
        if (g + 1 < g1) QZO_SK_XSTORE((d + 1) % XD, (d + 1) & 1);
        QZO_SK_XLOAD((d + 1) % XD, g + 1 + XD);
        if (live) {
          // perturbed scales of (row, g): s + eps z for the first pass, s - eps z for the second
          if (fresh || (g & 7u) == 0u) {
            const u32x4_t pw = philox4x32_10(a.row_base + n, g >> 3, 0u, 0u, a.seed_lo, a.seed_hi);
            zw[0] = pw.x; zw[1] = pw.y; zw[2] = pw.z; zw[3] = pw.w;
          }
          if (fresh || (g & 1u) == 0u) {
            const uint32_t p = (g & 7u) >> 1;
            normal_pair(p == 0 ? zw[0] : (p == 1 ? zw[1] : (p == 2 ? zw[2] : zw[3])), z_even, z_odd);
          }
          fresh = false;
          const uint32_t sw = (d >> 1) == 0 ? sv.x : ((d >> 1) == 1 ? sv.y : ((d >> 1) == 2 ? sv.z : sv.w));
          const float zz = (g & 1u) ? z_odd : z_even;
          const float s0 = scale_to_f32((d & 1) ? sw >> 16 : sw & 0xffffu, s_fp16);
          const float se_p = __builtin_fmaf(a.eps_signed, zz, s0);
          const float se_m = __builtin_fmaf(-a.eps_signed, zz, s0);
          const float cz = ZP ? -(128.0f + (float)((zv[d >> 2] >> (8 * (d & 3))) & 0xffu)) : -136.0f;
          // this lane's 64 nibbles of the group: chunks 4 (d % 2) + 2 half and the next of row lrow
          const uint32_t c0 = 4 * (d & 1) + 2 * half;
          const u32x4 w0 = *reinterpret_cast<const u32x4*>(wtw + lrow * 128 + ((c0 ^ (lrow & 7u)) << 4));
          const u32x4 w1 = *reinterpret_cast<const u32x4*>(wtw + lrow * 128 + (((c0 + 1) ^ (lrow & 7u)) << 4));
          const uint32_t wd[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
          floatx16 pg[MT], px;                    // px: X[m,g] of tile rows 8 b + 4 half + c in every lane
#pragma unroll
          for (int j = 0; j < 8; ++j) {           // k-step j: inputs 64 half + 8 j .. + 7 of the group
            const bf16x8 wf = unpack8_biased(wd[j], nib_mask, nib_magic);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
              const bf16x8 xf = *reinterpret_cast<const bf16x8*>(xs[buf] + x_lds_off(m * 32 + lrow, half * 8 + j));
              const floatx16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
              pg[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, wf, j == 0 ? zero : pg[m], 0, 0, 0);
              if (XSUM_BY_MFMA) px = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, ones.v, j == 0 ? zero : px, 0, 0, 0);
            }
          }
          // y += s_eff * (P - (128 + zp) X)
#pragma unroll
          for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
              const float4 xg = XIN ? *reinterpret_cast<const float4*>(&xin[xpp][XIN ? d : 0][m * 32 + 8 * b + 4 * half])
                                : XSUM_BY_MFMA
                                    ? make_float4(px[4 * b], px[4 * b + 1], px[4 * b + 2], px[4 * b + 3])
                                    : *reinterpret_cast<const float4*>(&xsum[buf][m * 32 + 8 * b + 4 * half]);
              const float se = !DUAL ? se_p : ((MT == 2 ? m == 1 : b >= 2) ? se_m : se_p);
              y[m][4 * b + 0] = __builtin_fmaf(se, __builtin_fmaf(cz, xg.x, pg[m][4 * b + 0]), y[m][4 * b + 0]);
              y[m][4 * b + 1] = __builtin_fmaf(se, __builtin_fmaf(cz, xg.y, pg[m][4 * b + 1]), y[m][4 * b + 1]);
              y[m][4 * b + 2] = __builtin_fmaf(se, __builtin_fmaf(cz, xg.z, pg[m][4 * b + 2]), y[m][4 * b + 2]);
              y[m][4 * b + 3] = __builtin_fmaf(se, __builtin_fmaf(cz, xg.w, pg[m][4 * b + 3]), y[m][4 * b + 3]);
            }
        }
      }
    }
#undef QZO_SK_XLOAD
#undef QZO_SK_XSTORE
#undef QZO_SK_WLOAD
#undef QZO_SK_WSTORE
#undef QZO_SK_SLOAD
#undef QZO_SK_XINLOAD

    // partial sums of this slice
    const uint32_t rows = DUAL ? 2 * a.M : a.M;
    const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(
        part, 0, (int)((uint64_t)gridDim.y * rows * a.N * 4), 0x00020000);
    if (n_own < a.N) {
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const uint32_t tr = 32 * m + 8 * (r >> 2) + 4 * half + (r & 3);      // tile row
          const uint32_t tok = DUAL ? tr % TPP : tr;
          const uint32_t orow = DUAL ? (tr / TPP) * a.M + tok : tok;
          const uint32_t off = ((blockIdx.y * rows + orow) * a.N + n_own) * 4u;
          if (tok < a.M) __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(y[m][r]), rp, (int)off, 0, 0);
        }
    }
  }
}

// Adds the K-slice partials in slice order and applies the epilogue.  A thread owns 4
// consecutive output features of one token (of the output: [M, N], or [M, N/2] with SwiGLU).
__global__ __launch_bounds__(256) void skinny_reduce_kernel(GemmArgs a, const float* __restrict__ part,
                                                            uint32_t ksplit) {
  const uint32_t NO = (a.epi & EPI_SWIGLU) ? a.N >> 1 : a.N;                  // output width
  const uint32_t q = blockIdx.x * 256 + threadIdx.x, per_row = NO >> 2;
  float ssq = 0.0f, sx = 0.0f;
  const bool own = q < a.M * per_row;
  if (own) ssq = reduce_item(a, part, ksplit, q / per_row, (q % per_row) * 4, sx);
  if (a.xsum_out) {
    // block sums of the output for a few-token linear that reads it: 128 features = 32 consecutive
    // threads of one token (the output width is a multiple of 128)
    sx += __shfl_xor(sx, 1, 64); sx += __shfl_xor(sx, 2, 64); sx += __shfl_xor(sx, 4, 64);
    sx += __shfl_xor(sx, 8, 64); sx += __shfl_xor(sx, 16, 64);
    if (own && (threadIdx.x & 31u) == 0u) a.xsum_out[(uint64_t)((q % per_row) >> 5) * a.M + q / per_row] = sx;
  }
  if (a.epi & EPI_SUMSQ) {
    __shared__ float red[4];
    ssq = wave_sum(ssq);
    if ((threadIdx.x & 63u) == 0) red[threadIdx.x >> 6] = ssq;
    __syncthreads();
    if (threadIdx.x == 0) a.partials[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
  }
}

}  // namespace

// K slices, whole groups each (an even number, but for the last).  A workgroup works in passes of
// SK_WD groups; measured on the 7B shapes at 16 tokens, slices of 8 groups beat 4, 16 and 32
// (12288 x 4096: 17.5, 15.0, 19.1, 32.8 us; 22016 x 4096: 26.8, 23.6, 24.9, 33.3; 4096 x 11008:
// 17.4, 15.3, 19.3, 31.3) unless that leaves the chip half empty (4096 x 4096: 9.0, 12.0, 18.3, 32.1).
uint32_t skinny_ksplit(uint32_t N, uint32_t K) {
  const uint32_t row_blocks = (N + SK_ROWS - 1) / SK_ROWS, ngrp = K >> 7;
  uint32_t per = SK_WD;
  while (row_blocks * ((ngrp + per - 1) / per) > 1024 && per < ngrp) per += SK_WD;
  if (row_blocks * ((ngrp + SK_WD - 1) / SK_WD) < 256 && ngrp > SK_WD / 2) per = SK_WD / 2;
  if (per > ngrp) per = ngrp;
  return (ngrp + per - 1) / per;
}
uint64_t skinny_ws_floats(uint32_t rows, uint32_t N, uint32_t K) {     // rows = M, or 2 M in dual mode
  return (uint64_t)skinny_ksplit(N, K) * rows * N;
}
uint32_t skinny_reduce_blocks(uint32_t M, uint32_t N, uint32_t epi) {
  const uint32_t NO = (epi & EPI_SWIGLU) ? N >> 1 : N;
  return (uint32_t)(((uint64_t)M * (NO >> 2) + 255) / 256);
}

// a.M <= 64, a.N % 8 == 0 (N % 16 == 0 with SwiGLU), a.K % 128 == 0; ws holds skinny_ws_floats
// floats; with EPI_SUMSQ a.partials holds skinny_reduce_blocks floats.
template <int MT, bool DUAL, bool XMF>
static void skinny_launch(const GemmArgs& a, dim3 grid, float* ws, uint32_t per, hipStream_t st) {
  if (a.xsum) {       // block sums delivered by the kernel that wrote x
    if (a.zp)
      skinny_gemm_kernel<MT, DUAL, true, false, true><<<grid, 256, 0, st>>>(a, ws, per);
    else
      skinny_gemm_kernel<MT, DUAL, false, false, true><<<grid, 256, 0, st>>>(a, ws, per);
    return;
  }
  if (a.zp)
    skinny_gemm_kernel<MT, DUAL, true, XMF, false><<<grid, 256, 0, st>>>(a, ws, per);
  else
    skinny_gemm_kernel<MT, DUAL, false, XMF, false><<<grid, 256, 0, st>>>(a, ws, per);
}
hipError_t launch_skinny_gemm(const GemmArgs& a, float* ws, hipStream_t st) {
  if (a.M == 0 || a.N == 0) return hipSuccess;
  if (a.M > SKINNY_MAX_M || (a.dual && a.M > SKINNY_MAX_M_DUAL) || !ws) return hipErrorInvalidValue;
  // 32-bit byte offsets into the weights, the activations and the partial sums
  if ((uint64_t)a.N * (a.K >> 1) >= (1ull << 31) || (uint64_t)2 * SKINNY_MAX_M * a.K * 2 >= (1ull << 31) ||
      skinny_ws_floats(a.dual ? 2 * a.M : a.M, a.N, a.K) * 4 >= (1ull << 31))
    return hipErrorInvalidValue;
  const uint32_t ks = skinny_ksplit(a.N, a.K), ngrp = a.K >> 7, per = (ngrp + ks - 1) / ks;
  dim3 grid((a.N + SK_ROWS - 1) / SK_ROWS, ks);
  if (a.dual) {
    if (a.M <= 16) skinny_launch<1, true, true>(a, grid, ws, per, st);
    else skinny_launch<2, true, false>(a, grid, ws, per, st);
  } else if (a.M <= 16) {
    skinny_launch<1, false, true>(a, grid, ws, per, st);
  } else if (a.M <= 32) {
    skinny_launch<1, false, false>(a, grid, ws, per, st);
  } else {
    skinny_launch<2, false, false>(a, grid, ws, per, st);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  GemmArgs r = a;                               // the reduction sees the stacked rows as one matrix
  if (a.dual) r.M = 2 * a.M;
  if (r.ldy || ((r.epi & EPI_SWIGLU) ? r.N >> 1 : r.N) % 128) r.xsum_out = nullptr;
  skinny_reduce_kernel<<<skinny_reduce_blocks(r.M, r.N, r.epi), 256, 0, st>>>(r, ws, ks);
  return hipGetLastError();
}

hipError_t launch_partial_reduce(const GemmArgs& a, const float* part, uint32_t ksplit, hipStream_t st) {
  if (a.M == 0 || a.N == 0) return hipSuccess;
  GemmArgs r = a;
  r.xsum_out = nullptr;                         // block sums are a service of the few-token path only
  skinny_reduce_kernel<<<skinny_reduce_blocks(a.M, a.N, a.epi), 256, 0, st>>>(r, part, ksplit);
  return hipGetLastError();
}

}  // namespace qzo
