// Expand-then-multiply: the weight formats whose reconstruction is a table lookup
// (the 16-bit-code codebook variant of Sec. 4.1, the 16-level normal-float format of
// Sec. 4.3) are first written out as one linear's perturbed bf16 matrix, which a plain
// bf16 GEMM then multiplies.  The lookup is done once per weight instead of once per
// weight and 256-token tile, and the GEMM loop carries no gather.  Both kernels are bound
// by HBM: about 2.3 bytes per weight (codes or nibbles in, bf16 out).
#include "qzo_device.hpp"
#include "qzo_kernels.hpp"

namespace qzo {

// Row p of the output holds source row gn(p): the identity; for a fused-SwiGLU consumer the tile
// order of the GEMM (each 256-row tile = 4 x (32 gate rows, 32 up rows of the same features); N = 2F,
// F a multiple of 128); for a fused-RoPE consumer with heads of 128 features, within every 256 rows
// (two heads; N a multiple of 256) wavefront wn's 64 columns = features 32 (wn % 2) .. + 31 of head
// wn / 2 and the same features + 64.
__device__ __forceinline__ uint32_t expand_source_row(uint32_t p, uint32_t N, int order) {
  if (order == ROW_ORDER_NATURAL) return p;
  const uint32_t tn = p >> 8, r = p & 255u;
  if (order == ROW_ORDER_SWIGLU) return ((r >> 5) & 1u) * (N >> 1) + tn * 128u + (r >> 6) * 32u + (r & 31u);
  const uint32_t wn = r >> 6, j = (r >> 5) & 1u;
  return tn * 256u + (wn >> 1) * 128u + j * 64u + (wn & 1u) * 32u + (r & 31u);
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
  const uint32_t gn = expand_source_row(p, N, swiglu);
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
                                  float eps_signed, int swiglu, void* out_bf16, hipStream_t st) {
  if (N == 0) return hipSuccess;
  expand_codebook_kernel<<<(N + 3) / 4, 256, 0, st>>>((const uint16_t*)codes, (const uint4*)cb,
                                                      (const _Float16*)c_fp16, N, K, row_base, seed_lo,
                                                      seed_hi, eps_signed, swiglu, (uint4*)out_bf16);
  return hipGetLastError();
}

// ---- NormalFloat-4 blocks (Sec. 4.3's quantizer): W = (s + sigma*eps*z)[n, k/64] * level[u] ----
// The 16 levels of the published NormalFloat-4 code book (normal quantiles scaled to [-1, 1]).
__device__ const float NF4_LEVELS_DEV[16] = {
    -1.0f, -0.6961928009986877f, -0.5250730514526367f, -0.39491748809814453f,
    -0.28444138169288635f, -0.18477343022823334f, -0.09105003625154495f, 0.0f,
    0.07958029955625534f, 0.16093020141124725f, 0.24611230194568634f, 0.33791524171829224f,
    0.44070982933044434f, 0.5626170039176941f, 0.7229568362236023f, 1.0f};

// Perturbed block scales of one linear as fp32 [N, G]: s + (sigma*eps) z, one fma each.  A thread
// owns the eight scales of one Philox counter (row, 8 gb .. 8 gb + 7), as the update does.
__global__ __launch_bounds__(256) void perturbed_scales_kernel(const bf16_t* __restrict__ s, uint32_t N,
                                                               uint32_t G, uint32_t row_base,
                                                               uint32_t seed_lo, uint32_t seed_hi,
                                                               float eps_signed, float* __restrict__ se) {
  const uint32_t Gb = (G + 7u) >> 3;
  const uint64_t u = (uint64_t)blockIdx.x * 256u + threadIdx.x;
  if (u >= (uint64_t)N * Gb) return;
  const uint32_t row = (uint32_t)(u / Gb), gb = (uint32_t)(u - (uint64_t)row * Gb);
  float z[8];
  scale_normals8(seed_lo, seed_hi, 0u, row_base + row, gb, z);
  const uint32_t nv = min(8u, G - gb * 8u);
  const uint64_t base = (uint64_t)row * G + gb * 8u;
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if ((uint32_t)j < nv) se[base + j] = __builtin_fmaf(eps_signed, z[j], bf16_to_f32(s[base + j]));
}

// The same for every scale of a model in one launch, laid out like the scale arena (the update's
// plan: grid = (workgroups per layer, layers), a thread owns the eight scales of one counter).
__global__ __launch_bounds__(256) void perturbed_scales_all_kernel(const bf16_t* __restrict__ arena, UpdPlan plan,
                                                                   uint32_t seed_lo, uint32_t seed_hi,
                                                                   float eps_signed, float* __restrict__ se) {
  const uint32_t wg = blockIdx.x, layer = blockIdx.y;
  UpdSeg sg = plan.seg[0];
#pragma unroll
  for (int i = 1; i < 4; ++i)
    if ((uint32_t)i < plan.n_seg && wg >= plan.seg[i].first_wg) sg = plan.seg[i];
  const uint32_t Gb = (sg.G + 7u) >> 3;
  const uint32_t u = (wg - sg.first_wg) * 256u + threadIdx.x;
  if (u >= sg.rows * Gb) return;
  const uint32_t row = u / Gb, gb = u - row * Gb;
  float z[8];
  scale_normals8(seed_lo, seed_hi, 0u, layer * plan.rows_per_layer + sg.row_base + row, gb, z);
  const uint64_t base = (uint64_t)layer * plan.layer_stride + sg.off + (uint64_t)row * sg.G + gb * 8u;
  const uint32_t nv = min(8u, sg.G - gb * 8u);
  const bool fp16 = plan.fp16 != 0;
  if (nv == 8u && (sg.G & 1u) == 0u) {
    // a whole counter of a row that starts on a dword: one 16-byte load, two 16-byte stores
    // (4-byte aligned accesses: rows of 86 or 108 groups start on a dword only)
    struct a4_u32x4 { uint32_t x, y, z, w; } __attribute__((packed, aligned(4)));
    struct a4_f32x4 { float x, y, z, w; } __attribute__((packed, aligned(4)));
    const a4_u32x4 v = *reinterpret_cast<const a4_u32x4*>(arena + base);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    float o[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      o[2 * j] = __builtin_fmaf(eps_signed, z[2 * j], scale_to_f32(w[j] & 0xffffu, fp16));
      o[2 * j + 1] = __builtin_fmaf(eps_signed, z[2 * j + 1], scale_to_f32(w[j] >> 16, fp16));
    }
    a4_f32x4* dst = reinterpret_cast<a4_f32x4*>(se + base);
    dst[0] = a4_f32x4{o[0], o[1], o[2], o[3]};
    dst[1] = a4_f32x4{o[4], o[5], o[6], o[7]};
    return;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if ((uint32_t)j < nv)
      se[base + j] = __builtin_fmaf(eps_signed, z[j], scale_to_f32(arena[base + j], fp16));
}

// bf16 [N,K] from the indices and the perturbed scales: a thread turns one dword (eight
// indices, k = 8c .. 8c+7, lowest nibble first) into 16 bytes; the level table sits in LDS
// (16 words in 16 banks: any mix of indices is served without a conflict).
__global__ __launch_bounds__(256) void expand_nf4_kernel(const uint32_t* __restrict__ q,
                                                         const float* __restrict__ se, uint32_t N,
                                                         uint32_t K, int swiglu, uint4* __restrict__ out) {
  __shared__ float lut[16];
  if (threadIdx.x < 16) lut[threadIdx.x] = NF4_LEVELS_DEV[threadIdx.x];
  __syncthreads();
  const uint32_t p = blockIdx.x, nc = K >> 3, kc = blockIdx.y * 256u + threadIdx.x;
  if (kc >= nc) return;
  const uint32_t gn = expand_source_row(p, N, swiglu);
  const uint32_t w = q[(uint64_t)gn * nc + kc];
  const float sc = se[(uint64_t)gn * (K >> 6) + (kc >> 3)];
  uint32_t o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
    o[j] = pack_bf16x2(sc * lut[(w >> (8 * j)) & 15u], sc * lut[(w >> (8 * j + 4)) & 15u]);
  out[(uint64_t)p * nc + kc] = make_uint4(o[0], o[1], o[2], o[3]);
}

// int4 groups of 128 (Eq. 4-5): W = (s + sigma*eps*z)[n, k/128] * (u - zp), zp = 8 without a
// zero-point tensor.  u - zp is an exact small integer, so the one rounding is that of the product
// to bf16: the same bits as the weight tile of the fused GEMM.
// With activation reordering (g_idx, int32 [K]) column k belongs to group g_idx[k] instead of
// k / 128: scale and zero-point are then looked up per weight.
__global__ __launch_bounds__(256) void expand_int4_kernel(const uint32_t* __restrict__ q,
                                                          const float* __restrict__ se,
                                                          const uint8_t* __restrict__ zp,
                                                          const int32_t* __restrict__ g_idx, uint32_t N,
                                                          uint32_t K, int swiglu, uint4* __restrict__ out) {
  const uint32_t p = blockIdx.x, nc = K >> 3, kc = blockIdx.y * 256u + threadIdx.x;
  if (kc >= nc) return;
  const uint32_t gn = expand_source_row(p, N, swiglu);
  const uint32_t w = q[(uint64_t)gn * nc + kc];
  const uint64_t g0 = (uint64_t)gn * (K >> 7);
  uint32_t o[4];
  if (g_idx) {
    const int4 ga = reinterpret_cast<const int4*>(g_idx)[2 * kc], gb = reinterpret_cast<const int4*>(g_idx)[2 * kc + 1];
    const int g[8] = {ga.x, ga.y, ga.z, ga.w, gb.x, gb.y, gb.z, gb.w};
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint64_t gi = g0 + min((uint32_t)g[i], (K >> 7) - 1u);   // an index outside 0..G-1 is clamped
      v[i] = se[gi] * (float)((int)((w >> (4 * i)) & 15u) - (zp ? (int)zp[gi] : 8));
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = pack_bf16x2(v[2 * j], v[2 * j + 1]);
  } else {
    const uint64_t gi = g0 + (kc >> 4);
    const float sc = se[gi];
    const int z0 = zp ? (int)zp[gi] : 8;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      o[j] = pack_bf16x2(sc * (float)((int)((w >> (8 * j)) & 15u) - z0),
                         sc * (float)((int)((w >> (8 * j + 4)) & 15u) - z0));
  }
  out[(uint64_t)p * nc + kc] = make_uint4(o[0], o[1], o[2], o[3]);
}

hipError_t launch_expand_int4(const void* q, const void* s_bf16, const void* zp, const int32_t* g_idx,
                              uint32_t N, uint32_t K, uint32_t row_base, uint32_t seed_lo, uint32_t seed_hi, float eps_signed,
                              int swiglu, float* se_scratch, void* out_bf16, hipStream_t st) {
  if (N == 0) return hipSuccess;
  const uint32_t G = K >> 7, Gb = (G + 7u) >> 3;
  const uint64_t units = (uint64_t)N * Gb;
  perturbed_scales_kernel<<<(uint32_t)((units + 255) / 256), 256, 0, st>>>(
      (const bf16_t*)s_bf16, N, G, row_base, seed_lo, seed_hi, eps_signed, se_scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  expand_int4_kernel<<<dim3(N, ((K >> 3) + 255) / 256), 256, 0, st>>>(
      (const uint32_t*)q, se_scratch, (const uint8_t*)zp, g_idx, N, K, swiglu, (uint4*)out_bf16);
  return hipGetLastError();
}

hipError_t launch_perturbed_scales_all(const void* arena, const UpdPlan& plan, uint32_t seed_lo, uint32_t seed_hi,
                                       float eps_signed, float* se_all, hipStream_t st) {
  dim3 grid(plan.wgs_per_layer, plan.n_layers);
  if (grid.x == 0 || grid.y == 0) return hipSuccess;
  perturbed_scales_all_kernel<<<grid, 256, 0, st>>>((const bf16_t*)arena, plan, seed_lo, seed_hi, eps_signed, se_all);
  return hipGetLastError();
}

hipError_t launch_expand_int4_from(const void* q, const float* se, const void* zp, const int32_t* g_idx,
                                   uint32_t N, uint32_t K, int swiglu, void* out_bf16, hipStream_t st) {
  if (N == 0) return hipSuccess;
  expand_int4_kernel<<<dim3(N, ((K >> 3) + 255) / 256), 256, 0, st>>>(
      (const uint32_t*)q, se, (const uint8_t*)zp, g_idx, N, K, swiglu, (uint4*)out_bf16);
  return hipGetLastError();
}

hipError_t launch_expand_nf4_from(const void* q, const float* se, uint32_t N, uint32_t K, int swiglu,
                                  void* out_bf16, hipStream_t st) {
  if (N == 0) return hipSuccess;
  expand_nf4_kernel<<<dim3(N, ((K >> 3) + 255) / 256), 256, 0, st>>>((const uint32_t*)q, se, N, K, swiglu,
                                                                   (uint4*)out_bf16);
  return hipGetLastError();
}

hipError_t launch_expand_nf4(const void* q, const void* s_bf16, uint32_t N, uint32_t K, uint32_t row_base,
                             uint32_t seed_lo, uint32_t seed_hi, float eps_signed, int swiglu,
                             float* se_scratch, void* out_bf16, hipStream_t st) {
  if (N == 0) return hipSuccess;
  const uint32_t G = K >> 6, Gb = (G + 7u) >> 3;
  const uint64_t units = (uint64_t)N * Gb;
  perturbed_scales_kernel<<<(uint32_t)((units + 255) / 256), 256, 0, st>>>(
      (const bf16_t*)s_bf16, N, G, row_base, seed_lo, seed_hi, eps_signed, se_scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  expand_nf4_kernel<<<dim3(N, ((K >> 3) + 255) / 256), 256, 0, st>>>((const uint32_t*)q, se_scratch, N, K,
                                                                   swiglu, (uint4*)out_bf16);
  return hipGetLastError();
}

}  // namespace qzo
