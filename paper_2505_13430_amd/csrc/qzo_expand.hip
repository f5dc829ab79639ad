// Expand-then-multiply: the weight formats whose reconstruction is a table lookup
// (the 16-bit-code codebook variant of Sec. 4.1, the 16-level normal-float format of
// Sec. 4.3) are first written out as one linear's perturbed bf16 matrix, which a plain
// bf16 GEMM then multiplies.  The lookup is done once per weight instead of once per
// weight and 256-token tile, and the GEMM loop carries no gather.  Both kernels are bound
// by HBM: about 2.3 bytes per weight (codes or nibbles in, bf16 out).
#include "qzo_device.hpp"
#include "qzo_kernels.hpp"

namespace qzo {

// Row p of the output holds source row gn(p): the identity, or for a fused-SwiGLU consumer
// the tile order of the GEMM (each 256-row tile = 4 x (32 gate rows, 32 up rows of the same
// features); N = 2F, F a multiple of 128).
__device__ __forceinline__ uint32_t expand_source_row(uint32_t p, uint32_t N, bool swiglu) {
  if (!swiglu) return p;
  const uint32_t tn = p >> 8, r = p & 255u;
  return ((r >> 5) & 1u) * (N >> 1) + tn * 128u + (r >> 6) * 32u + (r & 31u);
}

// Codebook variant: W[n, 8c .. 8c+7] = (c_n + sigma*eps*z_n) * codebook[code[n,c]][0..7],
// the product rounded once to bf16.  One wavefront per output row; the row's perturbed
// channel scale is one fp32 fma evaluated by every lane.
__global__ __launch_bounds__(256) void expand_codebook_kernel(const uint16_t* __restrict__ codes,
                                                              const uint4* __restrict__ cb,
                                                              const _Float16* __restrict__ c,
                                                              uint32_t N, uint32_t K, uint32_t row_base,
                                                              uint32_t seed_lo, uint32_t seed_hi,
                                                              float eps_signed, int swiglu,
                                                              uint4* __restrict__ out) {
  const uint32_t p = blockIdx.x * 4u + (threadIdx.x >> 6), lane = threadIdx.x & 63u;
  if (p >= N) return;
  const uint32_t gn = expand_source_row(p, N, swiglu != 0);
  const float ce = __builtin_fmaf(eps_signed, flat_normal(seed_lo, seed_hi, 1u, row_base + gn), (float)c[gn]);
  const uint32_t nc = K >> 3;
  const uint16_t* crow = codes + (uint64_t)gn * nc;
  uint4* orow = out + (uint64_t)p * nc;
  typedef _Float16 h2 __attribute__((ext_vector_type(2)));
  auto scaled = [&](const uint4 v) {
    const h2 a = __builtin_bit_cast(h2, v.x), b = __builtin_bit_cast(h2, v.y);
    const h2 d = __builtin_bit_cast(h2, v.z), e = __builtin_bit_cast(h2, v.w);
    return make_uint4(pack_bf16x2(ce * (float)a.x, ce * (float)a.y), pack_bf16x2(ce * (float)b.x, ce * (float)b.y),
                      pack_bf16x2(ce * (float)d.x, ce * (float)d.y), pack_bf16x2(ce * (float)e.x, ce * (float)e.y));
  };
  // four chunks per lane in flight: the codes first, then the four dependent gathers
  uint32_t kc = lane;
  for (; kc + 192u < nc; kc += 256u) {
    uint16_t code[4];
    uint4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) code[j] = crow[kc + 64u * j];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = cb[code[j]];
#pragma unroll
    for (int j = 0; j < 4; ++j) orow[kc + 64u * j] = scaled(v[j]);
  }
  for (; kc < nc; kc += 64u) orow[kc] = scaled(cb[crow[kc]]);
}

hipError_t launch_expand_codebook(const void* codes, const void* cb, const void* c_fp16, uint32_t N,
                                  uint32_t K, uint32_t row_base, uint32_t seed_lo, uint32_t seed_hi,
                                  float eps_signed, bool swiglu, void* out_bf16, hipStream_t st) {
  if (N == 0) return hipSuccess;
  expand_codebook_kernel<<<(N + 3) / 4, 256, 0, st>>>((const uint16_t*)codes, (const uint4*)cb,
                                                      (const _Float16*)c_fp16, N, K, row_base, seed_lo,
                                                      seed_hi, eps_signed, swiglu ? 1 : 0, (uint4*)out_bf16);
  return hipGetLastError();
}

}  // namespace qzo
