// Perturbed W4A16 linear for few tokens (M <= 64): Y[M,N] = X[M,K] * W_eff^T with
//   W_eff[n,k] = (s[n,k/128] + sigma*eps*z(row_base+n, k/128)) * wbar[n,k]   (paper Eq. 4-5).
// At this size every weight is used once per token tile, so the kernel is bound by
// streaming the int4 weights from HBM, not by the matrix pipe.
//
// A workgroup of four wavefronts owns 128 output rows and one slice of K; each
// wavefront owns 32 rows.  A lane (row, half) reads 2 x 16 bytes of its row per
// 128-wide group straight into registers (no LDS for weights: nobody else needs
// them), several groups ahead, converts them to the MFMA's first operand and
// multiplies with the activation block, which the workgroup shares through LDS
// (double buffered, one barrier per group).  The contraction index of one MFMA
// k-step is {64 half + 32 c + 8 j + e}: any order is fine as long as both operands
// agree.  Partial sums of the K slices go to a scratch buffer in fp32 and a second
// kernel adds them in a fixed order (deterministic) and applies the epilogue.
//
// Dual mode: the +eps and the -eps pass of one QZO step read the same int4 weights
// and the same noise, so for very few tokens they share one launch.  X and Y then
// hold the two passes stacked (rows [0,M) and [M,2M)); a weight dword is converted
// twice (with s + eps z and s - eps z) and each token tile multiplies with its own.
#include "qzo_device.hpp"
#include "qzo_kernels.hpp"

namespace qzo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int SK_ROWS = 128;      // output rows per workgroup
constexpr int SK_DEPTH = 4;       // groups of weights in flight per lane

// 8 nibbles of one dword -> 8 bf16 of (nibble-8)*se in k order (see the tile GEMM).
// ZP: the parameters are the scale and the negated zero-point (u - zp exact, one rounding).
template <bool ZP>
__device__ __forceinline__ bf16x8 dequant8_frag(uint32_t w, float se512, float m8se) {
  typedef float f2 __attribute__((ext_vector_type(2)));
  const uint32_t lo = w & 0x0f0f0f0fu, hi = (w >> 4) & 0x0f0f0f0fu;
  const f2 l01 = __builtin_amdgcn_cvt_pk_f32_fp8(lo, false), l23 = __builtin_amdgcn_cvt_pk_f32_fp8(lo, true);
  const f2 h01 = __builtin_amdgcn_cvt_pk_f32_fp8(hi, false), h23 = __builtin_amdgcn_cvt_pk_f32_fp8(hi, true);
  float e0, e1, e2, e3, e4, e5, e6, e7;
  if (ZP) {
    e0 = __builtin_fmaf(l01.x, 512.0f, m8se) * se512; e1 = __builtin_fmaf(h01.x, 512.0f, m8se) * se512;
    e2 = __builtin_fmaf(l01.y, 512.0f, m8se) * se512; e3 = __builtin_fmaf(h01.y, 512.0f, m8se) * se512;
    e4 = __builtin_fmaf(l23.x, 512.0f, m8se) * se512; e5 = __builtin_fmaf(h23.x, 512.0f, m8se) * se512;
    e6 = __builtin_fmaf(l23.y, 512.0f, m8se) * se512; e7 = __builtin_fmaf(h23.y, 512.0f, m8se) * se512;
  } else {
    e0 = __builtin_fmaf(l01.x, se512, m8se); e1 = __builtin_fmaf(h01.x, se512, m8se);
    e2 = __builtin_fmaf(l01.y, se512, m8se); e3 = __builtin_fmaf(h01.y, se512, m8se);
    e4 = __builtin_fmaf(l23.x, se512, m8se); e5 = __builtin_fmaf(h23.x, se512, m8se);
    e6 = __builtin_fmaf(l23.y, se512, m8se); e7 = __builtin_fmaf(h23.y, se512, m8se);
  }
  union { bf16x8 v; uint32_t u[4]; } r;
  r.u[0] = pack_bf16x2(e0, e1); r.u[1] = pack_bf16x2(e2, e3);
  r.u[2] = pack_bf16x2(e4, e5); r.u[3] = pack_bf16x2(e6, e7);
  return r.v;
}

__device__ __forceinline__ uint32_t x_lds_off(uint32_t row, uint32_t chunk) {   // 256-byte rows, 16 chunks
  return row * 256u + ((chunk ^ (row & 15u)) << 4);
}

// MT = 32-token tiles (1 or 2).  grid = (ceil(N/128), ksplit); part is [ksplit, rows, N] fp32
// with rows = M, or 2 M in dual mode (MT = 2: tile 0 is the +eps pass, tile 1 the -eps pass).
template <int MT, bool DUAL, bool ZP>
__global__ __launch_bounds__(256, MT == 1 ? 3 : 2) void skinny_gemm_kernel(GemmArgs a, float* __restrict__ part,
                                                             uint32_t groups_per_split) {
  static_assert(!DUAL || MT == 2, "dual mode: one token tile per pass");
  __shared__ __attribute__((aligned(16))) unsigned char xs[2][MT * 32 * 256];
  const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
  const uint32_t lrow = lane & 31u, half = lane >> 5;
  const uint32_t K = a.K, ngrp = K >> 7;
  const uint32_t g0 = blockIdx.y * groups_per_split, g1 = min(g0 + groups_per_split, ngrp);
  if (g0 >= g1) return;
  const uint32_t n = min(blockIdx.x * SK_ROWS + wave * 32 + lrow, a.N - 1);      // this lane's weight row
  const unsigned char* wrow = (const unsigned char*)a.w + (uint64_t)n * (K >> 1) + half * 32;
  const bf16_t* srow = (const bf16_t*)a.s + (uint64_t)n * ngrp;
  const uint8_t* zrow = ZP ? (const uint8_t*)a.zp + (uint64_t)n * ngrp : nullptr;
  const bf16_t* x = (const bf16_t*)a.x;

  // activation staging: a group's block is MT*32 rows x 16 chunks; a thread moves MT*2 chunks
  // LDS row -> row of x: clamped to the last token; in dual mode LDS rows 32.. are the second pass
  auto xrow = [&](uint32_t row) {
    return DUAL ? (row >> 5) * a.M + min(row & 31u, a.M - 1) : min(row, a.M - 1);
  };
  // Memory returns in issue order, so whatever is consumed must be the oldest request in
  // flight: activations and weights are requested SK_DEPTH groups ahead, interleaved in
  // the order in which they are used (block g+1 goes to LDS, then the weights of group g).
  constexpr int NX = MT * 2;
  u32x4 xr[SK_DEPTH][NX];
#define QZO_SK_XLOAD(SLOT, G_)                                                               \
  do {                                                                                       \
    const uint32_t gx_ = min((uint32_t)(G_), ngrp - 1);                                      \
    _Pragma("unroll") for (int i = 0; i < NX; ++i) {                                         \
      const uint32_t c = t + 256u * i, row = c >> 4, ch = c & 15u;                           \
      xr[SLOT][i] = *reinterpret_cast<const u32x4*>(x + (uint64_t)xrow(row) * K + gx_ * 128u + ch * 8); \
    }                                                                                        \
  } while (0)
#define QZO_SK_XSTORE(SLOT, BUF)                                                             \
  do {                                                                                       \
    _Pragma("unroll") for (int i = 0; i < NX; ++i) {                                         \
      const uint32_t c = t + 256u * i, row = c >> 4, ch = c & 15u;                           \
      *reinterpret_cast<u32x4*>(xs[BUF] + x_lds_off(row, ch)) = xr[SLOT][i];                 \
    }                                                                                        \
  } while (0)

  // weights and scales in flight: slot g % SK_DEPTH
  u32x4 wq[SK_DEPTH][2];
  uint32_t zq[SK_DEPTH];     // zero-points (ZP)
  uint32_t sq[SK_DEPTH];     // one register each: 16-bit loads into shared registers would chain the slots
#define QZO_SK_WLOAD(SLOT, G_)                                                               \
  do {                                                                                       \
    const uint32_t gg_ = min((uint32_t)(G_), ngrp - 1);                                      \
    wq[SLOT][0] = *reinterpret_cast<const u32x4*>(wrow + (uint64_t)gg_ * 64);                \
    wq[SLOT][1] = *reinterpret_cast<const u32x4*>(wrow + (uint64_t)gg_ * 64 + 16);           \
    sq[SLOT] = (uint32_t)srow[gg_];                                                          \
    if (ZP) zq[SLOT] = (uint32_t)zrow[gg_];                                                  \
  } while (0)

  floatx16 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[m][r] = 0.0f;

  // noise: one Philox counter per 8 groups, one Box-Muller pair per 2 groups
  uint32_t zw[4] = {0, 0, 0, 0};
  float z_even = 0.0f, z_odd = 0.0f;
  bool fresh = true;

  // everything is requested before the first wait; block g0 travels in a slot of its own
  u32x4 x0[NX];
#pragma unroll
  for (int i = 0; i < NX; ++i) {
    const uint32_t c = t + 256u * i, row = c >> 4, ch = c & 15u;
    x0[i] = *reinterpret_cast<const u32x4*>(x + (uint64_t)xrow(row) * K + g0 * 128u + ch * 8);
  }
#pragma unroll
  for (int d = 0; d < SK_DEPTH; ++d) {        // slot of block g: (g - g0) % SK_DEPTH
    QZO_SK_XLOAD((d + 1) % SK_DEPTH, g0 + 1 + d);
    QZO_SK_WLOAD(d, g0 + d);
  }
#pragma unroll
  for (int i = 0; i < NX; ++i) {
    const uint32_t c = t + 256u * i, row = c >> 4, ch = c & 15u;
    *reinterpret_cast<u32x4*>(xs[0] + x_lds_off(row, ch)) = x0[i];
  }
  __syncthreads();

  for (uint32_t gb = g0; gb < g1; gb += SK_DEPTH) {
#pragma unroll
    for (int d = 0; d < SK_DEPTH; ++d) {
      const uint32_t g = gb + d;
      if (g < g1) {
        const uint32_t buf = (g - g0) & 1u;
        if (g > g0) __syncthreads();            // block g is complete, block g-1 has been read
        if (g + 1 < g1) {
          if (buf) QZO_SK_XSTORE((d + 1) % SK_DEPTH, 0); else QZO_SK_XSTORE((d + 1) % SK_DEPTH, 1);
        }
        QZO_SK_XLOAD((d + 1) % SK_DEPTH, g + 1 + SK_DEPTH);
        // perturbed scale of (row, g)
        if (fresh || (g & 7u) == 0u) {
          const u32x4_t pw = philox4x32_10(a.row_base + n, g >> 3, 0u, 0u, a.seed_lo, a.seed_hi);
          zw[0] = pw.x; zw[1] = pw.y; zw[2] = pw.z; zw[3] = pw.w;
        }
        if (fresh || (g & 1u) == 0u) {
          const uint32_t p = (g & 7u) >> 1;
          normal_pair(p == 0 ? zw[0] : (p == 1 ? zw[1] : (p == 2 ? zw[2] : zw[3])), z_even, z_odd);
        }
        fresh = false;
        const float zz = (g & 1u) ? z_odd : z_even, s0 = scale_to_f32(sq[d], a.s_fp16 != 0);
        const float se = __builtin_fmaf(a.eps_signed, zz, s0);
        const float nzp = ZP ? -(float)zq[d] : 0.0f;
        const float se512 = ZP ? se : 512.0f * se, m8se = ZP ? nzp : -8.0f * se;
        const float sn = __builtin_fmaf(-a.eps_signed, zz, s0);     // dual mode: the other pass
        const float sn512 = ZP ? sn : 512.0f * sn, m8sn = ZP ? nzp : -8.0f * sn;
        const u32x4 w0 = wq[d][0], w1 = wq[d][1];
        const uint32_t wd[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {           // k-step j: k = 64 half + 8 j + e of the group
          const bf16x8 af = dequant8_frag<ZP>(wd[j], se512, m8se);
          const bf16x8 an = DUAL ? dequant8_frag<ZP>(wd[j], sn512, m8sn) : af;
#pragma unroll
          for (int m = 0; m < MT; ++m) {
            const bf16x8 xf = *reinterpret_cast<const bf16x8*>(xs[buf] + x_lds_off(m * 32 + lrow, half * 8 + j));
            acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16((DUAL && m == 1) ? an : af, xf, acc[m], 0, 0, 0);
          }
        }
        // refill the slot SK_DEPTH groups ahead, after its last use so that the loads can
        // target the slot's own registers (no copy that would have to wait for them)
        QZO_SK_WLOAD(d, g + SK_DEPTH);
      }
    }
  }
#undef QZO_SK_XLOAD
#undef QZO_SK_XSTORE
#undef QZO_SK_WLOAD

  // acc[m][4 b + c]: token 32 m + lane%32, row 8 b + 4 half + c of the wavefront's 32 rows
  const uint32_t nb = blockIdx.x * SK_ROWS + wave * 32 + 4 * half;
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const uint32_t rows = DUAL ? 2 * a.M : a.M;
    const uint32_t tok = DUAL ? m * a.M + lrow : m * 32 + lrow;          // row of the stacked output
    if (DUAL ? lrow < a.M : tok < a.M) {
      float* dst = part + ((uint64_t)blockIdx.y * rows + tok) * a.N;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const uint32_t nn = nb + 8 * b;
        if (nn < a.N)                          // N % 4 == 0: the four rows are in range together
          *reinterpret_cast<float4*>(dst + nn) =
              make_float4(acc[m][4 * b], acc[m][4 * b + 1], acc[m][4 * b + 2], acc[m][4 * b + 3]);
      }
    }
  }
}

// Adds the K-slice partials in slice order and applies the epilogue.  A thread owns 4
// consecutive output features of one token (of the output: [M, N], or [M, N/2] with SwiGLU).
__global__ __launch_bounds__(256) void skinny_reduce_kernel(GemmArgs a, const float* __restrict__ part,
                                                            uint32_t ksplit) {
  const bool swiglu = (a.epi & EPI_SWIGLU) != 0;
  const uint32_t NO = swiglu ? a.N >> 1 : a.N;                  // output width
  const uint32_t q = blockIdx.x * 256 + threadIdx.x, per_row = NO >> 2;
  float ssq = 0.0f;
  if (q < a.M * per_row) {
    const uint32_t m = q / per_row, f = (q % per_row) * 4;
    float v[4] = {0, 0, 0, 0}, u[4] = {0, 0, 0, 0};
    for (uint32_t ks = 0; ks < ksplit; ++ks) {
      const float* src = part + ((uint64_t)ks * a.M + m) * a.N;
      const float4 p = *reinterpret_cast<const float4*>(src + f);
      v[0] += p.x; v[1] += p.y; v[2] += p.z; v[3] += p.w;
      if (swiglu) {
        const float4 pu = *reinterpret_cast<const float4*>(src + NO + f);
        u[0] += pu.x; u[1] += pu.y; u[2] += pu.z; u[3] += pu.w;
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
    const uint64_t o = (uint64_t)m * NO + f;
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
    ssq = q0 * q0 + q1 * q1 + q2 * q2 + q3 * q3;
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

// K slices: enough workgroups to keep every compute unit streaming, whole groups per slice.
uint32_t skinny_ksplit(uint32_t N, uint32_t K) {
  const uint32_t row_blocks = (N + SK_ROWS - 1) / SK_ROWS, ngrp = K >> 7;
  uint32_t ks = (384 + row_blocks - 1) / row_blocks;
  ks = ks < 1 ? 1 : (ks > 8 ? 8 : ks);
  if (ks > ngrp) ks = ngrp;
  const uint32_t per = (ngrp + ks - 1) / ks;
  return (ngrp + per - 1) / per;                // drop empty slices
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
hipError_t launch_skinny_gemm(const GemmArgs& a, float* ws, hipStream_t st) {
  if (a.M == 0 || a.N == 0) return hipSuccess;
  if (a.M > SKINNY_MAX_M || (a.dual && a.M > SKINNY_MAX_M_DUAL) || !ws) return hipErrorInvalidValue;
  const uint32_t ks = skinny_ksplit(a.N, a.K), ngrp = a.K >> 7, per = (ngrp + ks - 1) / ks;
  dim3 grid((a.N + SK_ROWS - 1) / SK_ROWS, ks);
  if (a.zp) {
    if (a.dual)
      skinny_gemm_kernel<2, true, true><<<grid, 256, 0, st>>>(a, ws, per);
    else if (a.M <= 32)
      skinny_gemm_kernel<1, false, true><<<grid, 256, 0, st>>>(a, ws, per);
    else
      skinny_gemm_kernel<2, false, true><<<grid, 256, 0, st>>>(a, ws, per);
  } else if (a.dual) {
    skinny_gemm_kernel<2, true, false><<<grid, 256, 0, st>>>(a, ws, per);
  } else if (a.M <= 32) {
    skinny_gemm_kernel<1, false, false><<<grid, 256, 0, st>>>(a, ws, per);
  } else {
    skinny_gemm_kernel<2, false, false><<<grid, 256, 0, st>>>(a, ws, per);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  GemmArgs r = a;                               // the reduction sees the stacked rows as one matrix
  if (a.dual) r.M = 2 * a.M;
  skinny_reduce_kernel<<<skinny_reduce_blocks(r.M, r.N, r.epi), 256, 0, st>>>(r, ws, ks);
  return hipGetLastError();
}

hipError_t launch_partial_reduce(const GemmArgs& a, const float* part, uint32_t ksplit, hipStream_t st) {
  if (a.M == 0 || a.N == 0) return hipSuccess;
  skinny_reduce_kernel<<<skinny_reduce_blocks(a.M, a.N, a.epi), 256, 0, st>>>(a, part, ksplit);
  return hipGetLastError();
}

}  // namespace qzo
