// Plain bf16 GEMM of the expand-then-multiply route (paper Eq. 4-5 with the perturbed weights already
// written out in bf16): Y[M,N] = X[M,K] W[N,K]^T with the tile kernel's full-width epilogues (bias,
// residual, ReLU, rotary embedding, sum of squares), one wavefront per SIMD.
//
// 256 threads = 4 wavefronts (2 along tokens x 2 along features) on the 256 x 256 x 64 workgroup tile,
// each 128 x 128 = 4 x 4 v_mfma_f32_32x32x16_bf16 tiles: 256 accumulator registers, which live in the
// AGPR half of the 512 registers a lone wavefront of a SIMD has.  Both operand tiles go from memory
// straight into the LDS (two stages), fragments are double buffered in registers.  Against the
// 512-thread tile kernel:
//  * a third less fragment traffic from the LDS per flop (8 fragment reads feed 16 MFMAs instead of 6
//    feeding 8);
//  * nothing else runs on the SIMD, so every fragment read and every load of the next k-tile is
//    slotted between two MFMAs in source order (scheduling fences keep it);
//  * 128 vector registers are free to keep the packed output of a finished tile, which is stored two
//    16-byte pieces per k-tile during the first 16 k-tiles of the next tile instead of in one burst from
//    every CU at once.  With ST_AUX = 2 these stores are non-temporal: a 128 KB tile per CU would
//    otherwise displace the operand lines that the workgroups of an XCD share through its 4 MB L2
//    while the k-loop is reading them.
// What it pays: a load that cannot be issued because the memory pipeline's queue is full stops the only
// wavefront of the SIMD, MFMAs included (the 512-thread kernel has a second wavefront to go on with), so
// it is the slower of the two where the operands come in slowly (the 22016-wide gate/up matrix) and is
// not used with the fused SwiGLU, whose half-width output makes the other kernel's store burst cheap.
// Results are bit-identical to the 512-thread kernel's: every output element sums the same k-steps in the
// same order.
#include "qzo_gemm_tile.hpp"

namespace qzo {

#define QW_DTL16(RSRC, LDSADDR, VOFF, SOFF)                                                  \
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"                \
               : : "s"(LDSADDR), "v"(VOFF), "s"(RSRC), "s"(SOFF) : "memory", "m0")

template <int ST_AUX>
__global__ __launch_bounds__(256, 1) void wide_gemm_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  TileWalk walk = tile_walk_init(a.M, a.N, 1);
  uint32_t tile_m, tile_n;
  if (!tile_walk_get(walk, tile_m, tile_n)) return;
  const uint32_t tiles_m = walk.tiles_m;
  const uint32_t t = threadIdx.x, lane = t & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const uint32_t wm = wave >> 1, wn = wave & 1u;
  const uint32_t K = a.K, nkt = K / BK, last = nkt - 1;
  typedef int i32x4 __attribute__((ext_vector_type(4)));
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const i32x4 rx4 = {(int)(uint32_t)(uintptr_t)a.x, (int)(uint32_t)((uintptr_t)a.x >> 32),
                     (int)((uint64_t)a.M * K * 2), 0x00020000};
  const i32x4 rw4 = {(int)(uint32_t)(uintptr_t)a.w, (int)(uint32_t)((uintptr_t)a.w >> 32),
                     (int)((uint64_t)a.N * K * 2), 0x00020000};
  const uint32_t ldy = a.ldy ? a.ldy : a.N;        // row stride of y and resid (a column block of a wider matrix)
  const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(
      a.y, 0, (int)(((uint64_t)(a.M - 1) * ldy + a.N) * 2), 0x00020000);
  const uint32_t lds_wave = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds + wave * 1024u;
  unsigned char* const lds_a = lds;
  unsigned char* const lds_b = lds + 2 * TILE_BYTES;

  // direct-to-LDS offsets: chunk i (0..7) of the thread is row t/8 + 32 i; the swizzle is applied on the memory side
  uint32_t xo[8], wo[8];
#define QW_TILE_PTRS(TM, TN)                                                                 \
  do {                                                                                       \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                          \
      const uint32_t row = (t >> 3) + 32 * i;                                                \
      const uint32_t c = (t & 7u) ^ ((row >> 1) & 7u);                                       \
      xo[i] = (min((TM) * BM + row, a.M - 1) * K + c * 8) * 2;                               \
      wo[i] = (min((TN) * BN + row, a.N - 1) * K + c * 8) * 2;                               \
    }                                                                                        \
  } while (0)
  QW_TILE_PTRS(tile_m, tile_n);
#define QW_DTL_ONE(KT, STAGE, D)                                                             \
  do {                                                                                       \
    const uint32_t so_ = (uint32_t)(KT) * (BK * 2);                                          \
    if (((D) & 1) == 0)                                                                      \
      QW_DTL16(rx4, lds_wave + (uint32_t)((STAGE) * TILE_BYTES + ((D) >> 1) * 32 * 128), xo[(D) >> 1], so_); \
    else                                                                                     \
      QW_DTL16(rw4, lds_wave + (uint32_t)((2 + (STAGE)) * TILE_BYTES + ((D) >> 1) * 32 * 128), wo[(D) >> 1], so_); \
  } while (0)
#define QW_DTL_TILE(KT, STAGE)                                                               \
  do {                                                                                       \
    _Pragma("unroll") for (int d_ = 0; d_ < 16; ++d_) QW_DTL_ONE(KT, STAGE, d_);             \
  } while (0)

  const uint32_t frow = lane & 31u, fhalf = lane >> 5, fsw = (frow >> 1) & 7u;
  uint32_t fa_k[4], fb_k[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const uint32_t co = ((uint32_t)(ks * 2 + fhalf) ^ fsw) << 4;
    fa_k[ks] = (wm * 128 + frow) * 128u + co;
    fb_k[ks] = (wn * 128 + frow) * 128u + co;
  }
  floatx16 acc[4][4];
  bf16x8 fa_[2][4], fb_[2][4];

  // the packed output of the tile before: piece (i, j, bp) = 8 features of one token per lane
  uint4 pend[32];
  uint32_t pend_cnt = 0, pend_base = 0, pend_istride = 0, pend_col = 0;
#define QW_PST(IDX)                                                                          \
  do {                                                                                       \
    const int i_ = (IDX) >> 3, j_ = ((IDX) >> 1) & 3, b_ = (IDX) & 1;                        \
    const bool ok_ = pend_col + j_ * 32 + b_ * 16 < a.N;                                     \
    const uint32_t o_ = pend_base + i_ * pend_istride + (uint32_t)(j_ * 64 + b_ * 32);       \
    __builtin_amdgcn_raw_buffer_store_b128(u32x4{pend[IDX].x, pend[IDX].y, pend[IDX].z, pend[IDX].w}, \
                                           ry, (int)(ok_ ? o_ : 0x80000000u), 0, ST_AUX);      \
  } while (0)
#define QW_PCASE(T_) case T_: QW_PST(2 * T_); QW_PST(2 * T_ + 1); break;
#define QW_PEND_FLUSH(T)                                                                     \
  do {                                                                                       \
    switch (T) {                                                                             \
      QW_PCASE(0) QW_PCASE(1) QW_PCASE(2) QW_PCASE(3) QW_PCASE(4) QW_PCASE(5) QW_PCASE(6) QW_PCASE(7) \
      QW_PCASE(8) QW_PCASE(9) QW_PCASE(10) QW_PCASE(11) QW_PCASE(12) QW_PCASE(13) QW_PCASE(14) QW_PCASE(15) \
      default: break;                                                                        \
    }                                                                                        \
  } while (0)

// Step: 16 MFMAs of the k-step read one step earlier (buffer 1 - RBUF) with, one per MFMA pair, the 8
// fragment reads of k-step KS into buffer RBUF (in the order the MFMAs first need them) and, in steps 0
// and 1, the 16 direct-to-LDS loads of the next k-tile.  MODE 0: no MFMAs (first step of an output
// tile), 1: accumulate, 2: first k-step of an output tile (accumulators start from zero).
#define QW_STEP(RBUF, KS, STAGE, MODE, DO_LOAD, LOAD_KT, D0)                                 \
  do {                                                                                       \
    _Pragma("unroll") for (int n_ = 0; n_ < 8; ++n_) {                                       \
      if (n_ == 0 || n_ > 4) fa_[RBUF][n_ ? n_ - 4 : 0] = *reinterpret_cast<const bf16x8*>(  \
          lds_a + fa_k[KS] + ((n_ ? n_ - 4 : 0) * 32 * 128 + (STAGE) * TILE_BYTES));         \
      else fb_[RBUF][n_ - 1] = *reinterpret_cast<const bf16x8*>(                             \
          lds_b + fb_k[KS] + ((n_ - 1) * 32 * 128 + (STAGE) * TILE_BYTES));                  \
      if ((MODE) != 0) {                                                                     \
        _Pragma("unroll") for (int q_ = 0; q_ < 2; ++q_) {                                   \
          const int m_ = 2 * n_ + q_, i_ = m_ >> 2, j_ = m_ & 3;                             \
          if ((MODE) == 2) acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb_[1 - (RBUF)][j_], fa_[1 - (RBUF)][i_], zero16, 0, 0, 0); \
          else acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb_[1 - (RBUF)][j_], fa_[1 - (RBUF)][i_], acc[i_][j_], 0, 0, 0); \
        }                                                                                    \
      }                                                                                      \
      if (DO_LOAD) QW_DTL_ONE(LOAD_KT, 1 - (STAGE), (D0) + n_);                              \
      __builtin_amdgcn_sched_barrier(0);                                                     \
    }                                                                                        \
  } while (0)
// One k-tile (index T of its output tile) in LDS stage STAGE; FIRST: k-tile 0.
#define QW_TILE(STAGE, FIRST, DO_LOAD, LOAD_KT, T)                                           \
  do {                                                                                       \
    const bool st_ = pend_cnt && (uint32_t)(T) < 16u;                                        \
    QW_STEP(0, 0, STAGE, (FIRST) ? 0 : 1, DO_LOAD, LOAD_KT, 0);                              \
    QW_STEP(1, 1, STAGE, (FIRST) ? 2 : 1, DO_LOAD, LOAD_KT, 8);                              \
    if (st_) QW_PEND_FLUSH(T);                                                               \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    QW_STEP(0, 2, STAGE, 1, false, 0u, 0);                                                   \
    QW_STEP(1, 3, STAGE, 1, false, 0u, 0);                                                   \
    /* the next k-tile has landed (this wavefront's loads; the two stores behind them may stay in flight) */ \
    if (st_) __builtin_amdgcn_s_waitcnt(0x0F72);                                             \
    else __builtin_amdgcn_s_waitcnt(0x0F70);                                                 \
    __syncthreads();                                                                         \
  } while (0)

  const floatx16 zero16 = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
  QW_DTL_TILE(0u, 0);
  QW_DTL_TILE(1u, 1);
  for (;;) {
    __builtin_amdgcn_s_waitcnt(0x0F70);   /* vmcnt(0): k-tiles 0 and 1 (and any store of an undeferred epilogue) */
    __syncthreads();
    QW_TILE(0, true, false, 0u, 0u);
    for (uint32_t kt = 1; kt + 2 < nkt; kt += 2) {
      QW_TILE(1, false, true, kt + 1, kt);
      QW_TILE(0, false, true, kt + 2, kt + 1);
    }
    QW_TILE(1, false, false, 0u, last);
    /* k-step 3 of the last k-tile */
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb_[1][j], fa_[1][i], acc[i][j], 0, 0, 0);
    pend_cnt = 0;

    const uint32_t m0 = tile_m * BM, n0 = tile_n * BN;
    const uint32_t done_m = tile_m, done_n = tile_n;
    walk.slot += walk.stride;
    const bool more = tile_walk_get(walk, tile_m, tile_n);
    if (more) {             /* every wavefront is past the barrier that ended the last k-tile */
      QW_TILE_PTRS(tile_m, tile_n);
      QW_DTL_TILE(0u, 0);
      QW_DTL_TILE(1u, 1);
    }
    // ---- epilogue: acc[i][j][4 b + c] = token 32 i + lane%32, feature 32 j + 8 b + 4 (lane/32) + c of the
    // wavefront's 128 x 128 sub-tile.  Pieces are packed into pend[]; with a next tile whose k-loop is long
    // enough to carry them they are stored there, otherwise right away.
    const bool defer = more && nkt >= 16u;
    const uint32_t mrow = m0 + wm * 128 + frow;
#define QW_ACC(I, J, R, DST) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(DST) : "a"(acc[I][J][R]))
#define QW_SWAP8(LO, HI)                                                                     \
  do {                                                                                       \
    _Pragma("unroll") for (int c_ = 0; c_ < 4; ++c_) {                                       \
      const auto r_ = __builtin_amdgcn_permlane32_swap(__float_as_uint((LO)[c_]),            \
                                                       __float_as_uint((HI)[c_]), false, false); \
      (LO)[c_] = __uint_as_float(r_[0]);                                                     \
      (HI)[c_] = __uint_as_float(r_[1]);                                                     \
    }                                                                                        \
  } while (0)
    if (a.epi & EPI_ROPE) {
      // qkv [M, 3d] with the rotary embedding on its q and k thirds: tiles (0,1) and (2,3) of the wavefront hold
      // feature f and feature f + dh/2 of a head for the same token (heads of 64: natural row order; heads of
      // 128: ROW_ORDER_ROPE128).  Each output is rounded to bf16 first (what a separate RoPE pass would read),
      // rotated in fp32 at position m % rope_S and rounded again.
      const uint32_t half = a.rope_dh >> 1, d2 = (a.N / 3u) * 2u;
      const float2* table = reinterpret_cast<const float2*>(a.rope);
      pend_col = n0 + wn * 128u + fhalf * 8u;
      pend_base = (mrow * a.N + pend_col) * 2u;
      pend_istride = 32u * a.N * 2u;
      // step u = (i, jp, bp): columns cb + (2 bp + fhalf) 8 .. + 7 and their partners half further on
      auto tb_of = [&](int u) {
        const int i = u >> 2, jp = (u >> 1) & 1, bp = u & 1;
        const uint32_t wq = wn * 2u + jp;
        const uint32_t idx_base = half == 64u ? (wq & 1u) * 32u : 0u;
        const uint32_t pos = min(mrow + i * 32, a.M - 1) % a.rope_S;
        return reinterpret_cast<const float4*>(table + (uint64_t)pos * half + idx_base + (2u * bp + fhalf) * 8u);
      };
      float4 tn[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) tn[q] = tb_of(0)[q];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int i = u >> 2, jp = (u >> 1) & 1, bp = u & 1;
        const uint32_t wq = wn * 2u + jp;
        const uint32_t na_base = half == 64u ? n0 + (wq >> 1) * 128u + (wq & 1u) * 32u : n0 + wq * 64u;
        const bool rotate = na_base < d2;
        // tile pair and slots: heads of 128 pair tiles (jp, jp + 2) of the permuted rows, heads of 64 tiles (2 jp, 2 jp + 1)
        float4 tcs[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) tcs[q] = tn[q];
        if (u < 15) {
#pragma unroll
          for (int q = 0; q < 4; ++q) tn[q] = tb_of(u + 1)[q];
        }
        float va[2][4], vb[2][4];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            QW_ACC(i, 2 * jp, 4 * (2 * bp + h) + c, va[h][c]);
            QW_ACC(i, 2 * jp + 1, 4 * (2 * bp + h) + c, vb[h][c]);
          }
        QW_SWAP8(va[0], va[1]);
        QW_SWAP8(vb[0], vb[1]);
        uint32_t oa[4], ob[4];
        oa[0] = pack_bf16x2(va[0][0], va[0][1]); oa[1] = pack_bf16x2(va[0][2], va[0][3]);
        oa[2] = pack_bf16x2(va[1][0], va[1][1]); oa[3] = pack_bf16x2(va[1][2], va[1][3]);
        ob[0] = pack_bf16x2(vb[0][0], vb[0][1]); ob[1] = pack_bf16x2(vb[0][2], vb[0][3]);
        ob[2] = pack_bf16x2(vb[1][0], vb[1][1]); ob[3] = pack_bf16x2(vb[1][2], vb[1][3]);
        if (rotate) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {                  // tcs[q]: (cos, sin) of pairs 2 q and 2 q + 1
            const float a0 = __uint_as_float(oa[q] << 16), a1 = __uint_as_float(oa[q] & 0xffff0000u);
            const float b0 = __uint_as_float(ob[q] << 16), b1 = __uint_as_float(ob[q] & 0xffff0000u);
            oa[q] = pack_bf16x2(a0 * tcs[q].x - b0 * tcs[q].y, a1 * tcs[q].z - b1 * tcs[q].w);
            ob[q] = pack_bf16x2(b0 * tcs[q].x + a0 * tcs[q].y, b1 * tcs[q].z + a1 * tcs[q].w);
          }
        }
        // output columns: heads of 128: the pair sits 64 columns apart (column blocks jp and jp + 2 of the
        // wavefront's 128); heads of 64: 32 apart (blocks 2 jp and 2 jp + 1)
        const uint4 outa = {oa[0], oa[1], oa[2], oa[3]}, outb = {ob[0], ob[1], ob[2], ob[3]};
        if (half == 64u) {
          pend[(i * 4 + jp) * 2 + bp] = outa;
          pend[(i * 4 + jp + 2) * 2 + bp] = outb;
        } else {
          pend[(i * 4 + 2 * jp) * 2 + bp] = outa;
          pend[(i * 4 + 2 * jp + 1) * 2 + bp] = outb;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      float ssq = 0.0f;
      const bf16_t* bias = (const bf16_t*)a.bias;
      const bf16_t* resid = (const bf16_t*)a.resid;
      pend_col = n0 + wn * 128u + fhalf * 8u;
      pend_base = (mrow * ldy + pend_col) * 2u;
      pend_istride = 32u * ldy * 2u;
      const __amdgpu_buffer_rsrc_t rr_ = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<bf16_t*>((a.epi & EPI_RESIDUAL) ? resid : (const bf16_t*)a.y), 0,
          (int)(((uint64_t)(a.M - 1) * ldy + a.N) * 2), 0x00020000);
      auto resid_of = [&](int u) {
        const int i = u >> 3, j = (u >> 1) & 3, bp = u & 1;
        const bool ok = pend_col + j * 32 + bp * 16 < a.N && (a.epi & EPI_RESIDUAL);
        return __builtin_amdgcn_raw_buffer_load_b128(rr_, (int)(ok ? pend_base + i * pend_istride + j * 64 + bp * 32 : 0x80000000u), 0, 0);
      };
      u32x4 rn = resid_of(0);
#pragma unroll
      for (int u = 0; u < 32; ++u) {
        const int i = u >> 3, j = (u >> 1) & 3, bp = u & 1;
        const u32x4 rr = rn;
        if (u < 31) rn = resid_of(u + 1);
        float v[2][4];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int c = 0; c < 4; ++c) QW_ACC(i, j, 4 * (2 * bp + h) + c, v[h][c]);
        QW_SWAP8(v[0], v[1]);
        const uint32_t n = pend_col + j * 32 + bp * 16;
        const bool inside = mrow + i * 32 < a.M && n < a.N;
        if (a.epi & EPI_BIAS) {
          const uint4 bb = *reinterpret_cast<const uint4*>(bias + min(n, a.N - 8));
          v[0][0] += __uint_as_float(bb.x << 16); v[0][1] += __uint_as_float(bb.x & 0xffff0000u);
          v[0][2] += __uint_as_float(bb.y << 16); v[0][3] += __uint_as_float(bb.y & 0xffff0000u);
          v[1][0] += __uint_as_float(bb.z << 16); v[1][1] += __uint_as_float(bb.z & 0xffff0000u);
          v[1][2] += __uint_as_float(bb.w << 16); v[1][3] += __uint_as_float(bb.w & 0xffff0000u);
        }
        if (a.epi & EPI_RESIDUAL) {
          v[0][0] += __uint_as_float(rr.x << 16); v[0][1] += __uint_as_float(rr.x & 0xffff0000u);
          v[0][2] += __uint_as_float(rr.y << 16); v[0][3] += __uint_as_float(rr.y & 0xffff0000u);
          v[1][0] += __uint_as_float(rr.z << 16); v[1][1] += __uint_as_float(rr.z & 0xffff0000u);
          v[1][2] += __uint_as_float(rr.w << 16); v[1][3] += __uint_as_float(rr.w & 0xffff0000u);
        }
        if (a.epi & EPI_RELU) {
#pragma unroll
          for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int c = 0; c < 4; ++c) v[h][c] = fmaxf(v[h][c], 0.0f);
        }
        const uint4 out = make_uint4(pack_bf16x2(v[0][0], v[0][1]), pack_bf16x2(v[0][2], v[0][3]),
                                     pack_bf16x2(v[1][0], v[1][1]), pack_bf16x2(v[1][2], v[1][3]));
        pend[u] = out;
        if ((a.epi & EPI_SUMSQ) && inside) {
          const uint32_t ow[4] = {out.x, out.y, out.z, out.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const float q0 = __uint_as_float(ow[q] << 16), q1 = __uint_as_float(ow[q] & 0xffff0000u);
            ssq = __builtin_fmaf(q0, q0, ssq);
            ssq = __builtin_fmaf(q1, q1, ssq);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (a.epi & EPI_SUMSQ) {
        float* red = reinterpret_cast<float*>(lds + LDS_BYTES);   /* behind the stages, which are being refilled */
        ssq = wave_sum(ssq);
        __syncthreads();
        if (lane == 0) red[wave] = ssq;
        __syncthreads();
        if (t == 0) a.partials[done_n * tiles_m + done_m] = ((red[0] + red[1]) + red[2]) + red[3];
      }
    }
    pend_cnt = 32;
    if (!defer) {
#pragma unroll
      for (int u = 0; u < 16; ++u) { QW_PST(2 * u); QW_PST(2 * u + 1); }
      pend_cnt = 0;
    }
    if (!more) break;
  }
#undef QW_SWAP8
#undef QW_ACC
#undef QW_TILE
#undef QW_STEP
#undef QW_PEND_FLUSH
#undef QW_PCASE
#undef QW_PST
#undef QW_DTL_TILE
#undef QW_DTL_ONE
#undef QW_TILE_PTRS
}
#undef QW_DTL16

// Output bytes from which the deferred stores are issued non-temporal (measured at 8192 tokens: 201 MB
// and 180-360 MB outputs gain 5-8 %, 67 MB outputs lose 5 % and stay on the default policy).
constexpr uint64_t WIDE_NT_MIN_BYTES = 96ull << 20;

hipError_t launch_bf16_gemm_wide(const GemmArgs& a, hipStream_t st) {
  static bool ready = false;
  if (!ready) {       // + 1 KB: the sum-of-squares scratch sits behind the stages
    hipError_t e = hipFuncSetAttribute((const void*)wide_gemm_kernel<0>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES + 1024);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void*)wide_gemm_kernel<2>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES + 1024);
    if (e != hipSuccess) return e;
    ready = true;
  }
  if (a.M == 0 || a.N == 0) return hipSuccess;
  // buffer loads and stores address the operands and the output with 32-bit byte offsets; K in whole groups
  if ((uint64_t)a.M * a.K * 2 >= (1ull << 31) || (uint64_t)a.N * a.K * 2 >= (1ull << 31) ||
      (uint64_t)a.M * (a.ldy ? a.ldy : a.N) * 2 >= (1ull << 31) || a.K % 128 != 0 || a.K == 0)
    return hipErrorInvalidValue;
  if (a.epi & EPI_SWIGLU) return hipErrorInvalidValue;      // the 512-thread kernel's epilogue
  if (a.ldy && (a.epi & EPI_ROPE)) return hipErrorInvalidValue;   // a column block has no thirds
  const uint64_t out_bytes = (uint64_t)a.M * a.N * 2;
  const uint32_t wgs = gemm_workgroups(a.M, a.N);
  if (out_bytes >= WIDE_NT_MIN_BYTES) wide_gemm_kernel<2><<<wgs, 256, LDS_BYTES + 1024, st>>>(a);
  else wide_gemm_kernel<0><<<wgs, 256, LDS_BYTES + 1024, st>>>(a);
  return hipGetLastError();
}

}  // namespace qzo
