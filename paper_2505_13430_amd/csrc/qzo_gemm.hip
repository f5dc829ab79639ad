// W4A16 group-dequant GEMM with the Q-SPSA perturbation fused into the weight
// tile (paper Eq. 4-5): Y[M,N] = X[M,K] * W_eff^T,
//   W_eff[n,k] = (s[n,k/128] + sigma*eps*z(row_base+n, k/128)) * wbar[n,k],
// bf16 MFMA (v_mfma_f32_32x32x16_bf16) with fp32 accumulation, for gfx950.
// The same tiling serves the dense bf16 lm_head GEMM whose epilogue folds the
// cross-entropy partial reductions instead of writing logits.
//
// Tiling: 256x256 output tile per workgroup, BK = 64, eight wavefronts in a
// 2 (M) x 4 (N) arrangement, each owning 128x64 = 4x2 MFMA tiles.  Both
// operands are K-contiguous in LDS (128 B per row, 16-byte chunks XOR-swizzled
// by row so that fragment reads and tile writes spread over all banks), double
// buffered.  int4 weights are unpacked, scaled by the perturbed scale and
// rounded to bf16 once per workgroup while being written to LDS; the noise z
// is regenerated per row every eight groups from the Philox counter
// (row, g/8) and never touches memory.
#include "qzo_device.hpp"
#include "qzo_kernels.hpp"

namespace qzo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int THREADS = 512;
constexpr int TILE_BYTES = BM * BK * 2;            // 32 KB per operand per stage
constexpr int LDS_BYTES = 4 * TILE_BYTES;          // A0 B0 A1 B1

uint32_t gemm_workgroups(uint32_t M, uint32_t N) {
  uint32_t tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  return ((tiles + 7) / 8) * 8;
}

// Workgroup id -> output tile.  Hardware deals consecutive workgroup ids to the
// eight XCDs in turn; each XCD gets one contiguous eighth of a tile order in
// which groups of 8 M-tiles sweep the N-tiles, so the tiles resident on one
// XCD at a time share a few A row-panels and B row-panels in that XCD's L2.
__device__ __forceinline__ bool tile_of_block(uint32_t tiles_m, uint32_t tiles_n, uint32_t& tm,
                                              uint32_t& tn) {
  const uint32_t total = tiles_m * tiles_n;
  const uint32_t per = (total + 7) >> 3;
  const uint32_t id = (blockIdx.x & 7u) * per + (blockIdx.x >> 3);
  if (id >= total) return false;
  const uint32_t width = 8u * tiles_n;
  const uint32_t group = id / width;
  const uint32_t first = group * 8u;
  const uint32_t gsz = min(tiles_m - first, 8u);
  const uint32_t in = id - group * width;
  tm = first + in % gsz;
  tn = in / gsz;
  return true;
}

__device__ __forceinline__ uint32_t lds_off(uint32_t row, uint32_t chunk) {
  return row * 128u + ((chunk ^ (row & 7u)) << 4);
}

// 8 nibbles of one dword -> 8 bf16 of (nibble-8)*se, in k order.
__device__ __forceinline__ uint4 dequant8(uint32_t w, float se, float m8se) {
  const uint32_t lo = w & 0x0f0f0f0fu, hi = (w >> 4) & 0x0f0f0f0fu;
  float e0 = __builtin_fmaf((float)(lo & 0xffu), se, m8se);
  float e1 = __builtin_fmaf((float)(hi & 0xffu), se, m8se);
  float e2 = __builtin_fmaf((float)((lo >> 8) & 0xffu), se, m8se);
  float e3 = __builtin_fmaf((float)((hi >> 8) & 0xffu), se, m8se);
  float e4 = __builtin_fmaf((float)((lo >> 16) & 0xffu), se, m8se);
  float e5 = __builtin_fmaf((float)((hi >> 16) & 0xffu), se, m8se);
  float e6 = __builtin_fmaf((float)(lo >> 24), se, m8se);
  float e7 = __builtin_fmaf((float)(hi >> 24), se, m8se);
  return make_uint4(pack_bf16x2(e0, e1), pack_bf16x2(e2, e3), pack_bf16x2(e4, e5),
                    pack_bf16x2(e6, e7));
}

struct CeEpilogue {
  const int32_t* tok;
  float* part;
  float* tgt;
  uint32_t S, n_slices;
};

template <bool W4, bool CE>
__global__ __launch_bounds__(THREADS, 1) void gemm_kernel(GemmArgs a, CeEpilogue ce) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const uint32_t tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  uint32_t tile_m, tile_n;
  if (!tile_of_block(tiles_m, tiles_n, tile_m, tile_n)) return;
  const uint32_t m0 = tile_m * BM, n0 = tile_n * BN;
  const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
  const uint32_t wm = wave >> 2, wn = wave & 3u;
  const uint32_t K = a.K;

  // ---- global -> register staging ---------------------------------------
  // A (and dense B): 2048 16-byte chunks per tile, 4 per thread; 8 consecutive
  // threads cover one 128-byte row segment.
  const unsigned char* xa[4];
  uint32_t a_lds[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t cid = t + THREADS * i, row = cid >> 3, c = cid & 7u;
    const uint32_t gm = min(m0 + row, a.M - 1);
    xa[i] = (const unsigned char*)a.x + ((uint64_t)gm * K + c * 8) * 2;
    a_lds[i] = lds_off(row, c);
  }
  const unsigned char* wb[4];
  uint32_t b_lds[4];
  // W4: thread = (row t/2, half t%2): 16 bytes = 32 nibbles = 4 chunks.
  const uint32_t brow = t >> 1, bhalf = t & 1u;
  const uint32_t gn_w4 = min(n0 + brow, a.N - 1);
  const bf16_t* srow = nullptr;
  if (W4) {
    wb[0] = (const unsigned char*)a.w + (uint64_t)gn_w4 * (K >> 1) + bhalf * 16;
    srow = (const bf16_t*)a.s + (uint64_t)gn_w4 * (K >> 7);
#pragma unroll
    for (int j = 0; j < 4; ++j) b_lds[j] = lds_off(brow, bhalf * 4 + j);
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t cid = t + THREADS * i, row = cid >> 3, c = cid & 7u;
      const uint32_t gn = min(n0 + row, a.N - 1);
      wb[i] = (const unsigned char*)a.w + ((uint64_t)gn * K + c * 8) * 2;
      b_lds[i] = lds_off(row, c);
    }
  }

  uint4 ra[4], rb[4];
  float z8[8];
  float se = 0.0f, m8se = 0.0f;

  auto gload = [&](uint32_t kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) ra[i] = *reinterpret_cast<const uint4*>(xa[i] + (uint64_t)kt * (BK * 2));
    if (W4) {
      rb[0] = *reinterpret_cast<const uint4*>(wb[0] + (uint64_t)kt * (BK / 2));
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        rb[i] = *reinterpret_cast<const uint4*>(wb[i] + (uint64_t)kt * (BK * 2));
    }
  };
  auto lstore = [&](uint32_t kt, uint32_t stage) {
    unsigned char* As = lds + stage * (2 * TILE_BYTES);
    unsigned char* Bs = As + TILE_BYTES;
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(As + a_lds[i]) = ra[i];
    if (W4) {
      if ((kt & 1u) == 0u) {             // a new group of 128 starts every two k-tiles
        const uint32_t g = kt >> 1;
        if ((g & 7u) == 0u)
          scale_normals8(a.seed_lo, a.seed_hi, 0u, a.row_base + gn_w4, g >> 3, z8);
        float zz = z8[0];
#pragma unroll
        for (int j = 1; j < 8; ++j) zz = ((g & 7u) == (uint32_t)j) ? z8[j] : zz;
        se = __builtin_fmaf(a.eps_signed, zz, bf16_to_f32(srow[g]));
        m8se = -8.0f * se;
      }
      const uint32_t w[4] = {rb[0].x, rb[0].y, rb[0].z, rb[0].w};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        *reinterpret_cast<uint4*>(Bs + b_lds[j]) = dequant8(w[j], se, m8se);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(Bs + b_lds[i]) = rb[i];
    }
  };

  floatx16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const uint32_t frow = lane & 31u, fhalf = lane >> 5;
  auto compute = [&](uint32_t stage) {
    const unsigned char* As = lds + stage * (2 * TILE_BYTES);
    const unsigned char* Bs = As + TILE_BYTES;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 fa[4], fb[2];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(As + lds_off(wm * 128 + i * 32 + frow, ks * 2 + fhalf));
#pragma unroll
      for (int j = 0; j < 2; ++j)
        fb[j] = *reinterpret_cast<const bf16x8*>(Bs + lds_off(wn * 64 + j * 32 + frow, ks * 2 + fhalf));
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  };

  const uint32_t nkt = K / BK;
  gload(0);
  lstore(0, 0);
  __syncthreads();
  for (uint32_t kt = 0; kt < nkt; ++kt) {
    const uint32_t cur = kt & 1u;
    if (kt + 1 < nkt) gload(kt + 1);
    compute(cur);
    if (kt + 1 < nkt) lstore(kt + 1, cur ^ 1u);
    __syncthreads();
  }

  // ---- epilogue ----------------------------------------------------------
  // acc[i][j][r]: row = 32 i + 8 (r/4) + 4 (lane/32) + r%4, col = 32 j + lane%32
  // of the wavefront's 128x64 sub-tile.
  if (!CE) {
    float ssq = 0.0f;
    const bf16_t* bias = (const bf16_t*)a.bias;
    const bf16_t* resid = (const bf16_t*)a.resid;
    bf16_t* y = (bf16_t*)a.y;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint32_t n = n0 + wn * 64 + j * 32 + frow;
      const bool nok = n < a.N;
      const float bv = ((a.epi & EPI_BIAS) && nok) ? bf16_to_f32(bias[n]) : 0.0f;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const uint32_t m = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3);
          if (nok && m < a.M) {
            float v = acc[i][j][r] + bv;
            const uint64_t o = (uint64_t)m * a.N + n;
            if (a.epi & EPI_RESIDUAL) v += bf16_to_f32(resid[o]);
            if (a.epi & EPI_RELU) v = fmaxf(v, 0.0f);
            const bf16_t b = f32_to_bf16(v);
            y[o] = b;
            const float vb = bf16_to_f32(b);
            ssq = __builtin_fmaf(vb, vb, ssq);
          }
        }
    }
    if (a.epi & EPI_SUMSQ) {
      float* red = reinterpret_cast<float*>(lds);
      ssq = wave_sum(ssq);
      if (lane == 0) red[wave] = ssq;
      __syncthreads();
      if (t == 0) {
        float s = 0.0f;
        for (int w = 0; w < THREADS / 64; ++w) s += red[w];
        a.partials[tile_n * tiles_m + tile_m] = s;
      }
    }
  } else {
    // Cross-entropy partials: for each row, (max, sum exp(l - max)) over this
    // wavefront's 64 columns, and the target logit where it falls here.
    const uint32_t slice = tile_n * 4 + wn;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t m = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3);
        const uint32_t c0 = n0 + wn * 64 + frow, c1 = c0 + 32;
        const float l0 = c0 < a.N ? acc[i][0][r] : -INFINITY;
        const float l1 = c1 < a.N ? acc[i][1][r] : -INFINITY;
        float mx = fmaxf(l0, l1);
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
        float sum = 0.0f;
        if (mx > -INFINITY) sum = expf(l0 - mx) + expf(l1 - mx);
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
        if (m < a.M) {
          if (frow == 0)
            reinterpret_cast<float2*>(ce.part)[(uint64_t)m * ce.n_slices + slice] = make_float2(mx, sum);
          if ((m % ce.S) != ce.S - 1) {
            const uint32_t target = (uint32_t)ce.tok[m + 1];
            if (target == c0) ce.tgt[m] = l0;
            if (target == c1) ce.tgt[m] = l1;
          }
        }
      }
  }
}

static hipError_t set_lds_attr(const void* fn) {
  return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
}

hipError_t launch_w4a16_gemm(const GemmArgs& a, hipStream_t st) {
  static bool ready = false;
  if (!ready) {
    hipError_t e = set_lds_attr((const void*)gemm_kernel<true, false>);
    if (e != hipSuccess) return e;
    ready = true;
  }
  if (a.M == 0 || a.N == 0) return hipSuccess;
  CeEpilogue ce = {nullptr, nullptr, nullptr, 1, 1};
  gemm_kernel<true, false><<<gemm_workgroups(a.M, a.N), THREADS, LDS_BYTES, st>>>(a, ce);
  return hipGetLastError();
}

hipError_t launch_lmhead_ce(const CeArgs& c, hipStream_t st) {
  static bool ready = false;
  if (!ready) {
    hipError_t e = set_lds_attr((const void*)gemm_kernel<false, true>);
    if (e != hipSuccess) return e;
    ready = true;
  }
  GemmArgs a = {};
  a.x = c.x; a.w = c.w; a.M = c.M; a.N = c.V; a.K = c.K;
  CeEpilogue ce = {c.tok, c.part, c.tgt, c.S, c.n_slices};
  gemm_kernel<false, true><<<gemm_workgroups(c.M, c.V), THREADS, LDS_BYTES, st>>>(a, ce);
  return hipGetLastError();
}

}  // namespace qzo
