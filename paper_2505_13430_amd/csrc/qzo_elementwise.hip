// Bandwidth-bound and scalar kernels of the QZO step for gfx950: the scale
// update of Algorithm 1, the SPSA scalar with directional-derivative clipping
// (Eq. 6), the RTN quantizer (Eq. 3), embedding, norms, RoPE, SwiGLU, the
// cross-entropy reduction, and the inspection kernels of the parity tests.
#include "qzo_device.hpp"
#include "qzo_kernels.hpp"

namespace qzo {

// ------------------------------------------------------------ update ------
// Delta_i <- max(Delta_i - eta*d'*z_i, 0) (Algorithm 1).  One thread owns the
// eight scales that share a Philox counter: (row, 8*gb .. 8*gb+7).  The arena
// is read and written once (4 B per scale); z costs no memory traffic.
// The kernel is bound by the vector ALU, not by memory: about 320 instructions per wavefront
// and counter, two thirds of them the four Box-Muller pairs (timing-only runs of this kernel:
// 45 us as is, 31 us with Philox but no Box-Muller, 30 us with no noise at all, at 50.6 M
// scales resident in the last-level cache).  Looking the angle factors of the pairs up in a
// 128 KB LDS table (one persistent workgroup per compute unit) was measured and is slower:
// 57 us, whatever the number of counters a thread interleaves.
struct u32x4_a4 { uint32_t x, y, z, w; } __attribute__((packed, aligned(4)));

// The eight scales of one Philox counter: where they are, how many of them exist, their noise row.
struct UpdUnit {
  bf16_t* p;          // null: no such counter (beyond the segment's last); 16-bit scales, bf16 or fp16
  uint32_t G, nv;     // groups per row of the segment; scales of this counter that exist (1 .. 8)
  uint32_t noise_row, gb;
};
__device__ __forceinline__ UpdUnit update_locate(bf16_t* __restrict__ arena, const UpdPlan& plan, uint32_t wg,
                                                 uint32_t layer, uint32_t tid) {
  UpdSeg sg = plan.seg[0];
#pragma unroll
  for (int i = 1; i < 4; ++i)
    if ((uint32_t)i < plan.n_seg && wg >= plan.seg[i].first_wg) sg = plan.seg[i];
  const uint32_t Gb = (sg.G + 7u) >> 3;
  const uint32_t u = (wg - sg.first_wg) * 256u + tid;
  UpdUnit r = {nullptr, sg.G, 0u, 0u, 0u};
  if (u >= sg.rows * Gb) return r;
  // row = u / Gb, gb = u % Gb for u < 2^24 (checked on the host)
  uint32_t row = (uint32_t)((float)u * __builtin_amdgcn_rcpf((float)Gb));
  int32_t gb = (int32_t)(u - __umul24(row, Gb));
  if (gb < 0) { row -= 1; gb += (int32_t)Gb; }
  else if (gb >= (int32_t)Gb) { row += 1; gb -= (int32_t)Gb; }
  r.p = arena + (uint64_t)layer * plan.layer_stride + sg.off + (uint64_t)row * sg.G + (uint32_t)gb * 8u;
  r.nv = min(8u, sg.G - (uint32_t)gb * 8u);
  r.noise_row = layer * plan.rows_per_layer + sg.row_base + row;
  r.gb = (uint32_t)gb;
  return r;
}
__device__ __forceinline__ void update_apply(const UpdUnit& un, float c, const float z[8], bool fp16) {
  if (!un.p) return;
  bf16_t* p = un.p;
  struct { uint32_t G; } sg = {un.G};
  const float nc = -c;
  const uint32_t nv = un.nv;
  if ((sg.G & 1u) == 0u && nv == 8u) {
    // rows start on a dword: one 16-byte access each way (16-byte aligned when G % 8 == 0)
    uint32_t in[4], out[4];
    if ((sg.G & 7u) == 0u) {
      const uint4 v = *reinterpret_cast<const uint4*>(p);
      in[0] = v.x; in[1] = v.y; in[2] = v.z; in[3] = v.w;
    } else {
      const u32x4_a4 v = *reinterpret_cast<const u32x4_a4*>(p);
      in[0] = v.x; in[1] = v.y; in[2] = v.z; in[3] = v.w;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float a = scale_to_f32(in[j] & 0xffffu, fp16), b = scale_to_f32(in[j] >> 16, fp16);
      a = fmaxf(__builtin_fmaf(nc, z[2 * j], a), 0.0f);
      b = fmaxf(__builtin_fmaf(nc, z[2 * j + 1], b), 0.0f);
      out[j] = pack_scale_x2(a, b, fp16);
    }
    if ((sg.G & 7u) == 0u) {
      *reinterpret_cast<uint4*>(p) = make_uint4(out[0], out[1], out[2], out[3]);
    } else {
      u32x4_a4 o = {out[0], out[1], out[2], out[3]};
      *reinterpret_cast<u32x4_a4*>(p) = o;
    }
  } else if ((sg.G & 1u) == 0u) {      // the last, partial block of a row: dword accesses
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (2u * j < nv) {
        uint32_t w = reinterpret_cast<const uint32_t*>(p)[j];
        float a = scale_to_f32(w & 0xffffu, fp16), b = scale_to_f32(w >> 16, fp16);
        a = fmaxf(__builtin_fmaf(nc, z[2 * j], a), 0.0f);
        b = fmaxf(__builtin_fmaf(nc, z[2 * j + 1], b), 0.0f);
        reinterpret_cast<uint32_t*>(p)[j] = pack_scale_x2(a, b, fp16);
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if ((uint32_t)j < nv) {
        float a = fmaxf(__builtin_fmaf(nc, z[j], scale_to_f32(p[j], fp16)), 0.0f);
        p[j] = (bf16_t)f32_to_scale(a, fp16);
      }
    }
  }
}

__global__ __launch_bounds__(256) void scale_update_kernel(bf16_t* __restrict__ arena, UpdPlan plan,
                                                           uint32_t seed_lo, uint32_t seed_hi,
                                                           float eta, float dclip_host,
                                                           const qzo_step_result* __restrict__ res) {
  float c;
  if (res) {
    if (res->status != 0) return;          // non-finite d: leave the scales alone
    c = eta * res->d_clipped;
  } else {
    c = eta * dclip_host;
  }
  const UpdUnit un = update_locate(arena, plan, blockIdx.x, blockIdx.y, threadIdx.x);
  if (!un.p) return;
  float z[8];
  scale_normals8(seed_lo, seed_hi, 0u, un.noise_row, un.gb, z);
  update_apply(un, c, z, plan.fp16 != 0);
}

hipError_t launch_scale_update(void* arena, const UpdPlan& plan, uint32_t seed_lo,
                               uint32_t seed_hi, float eta, float d_clipped,
                               const qzo_step_result* res, hipStream_t st) {
  dim3 grid(plan.wgs_per_layer, plan.n_layers);
  if (grid.x == 0 || grid.y == 0) return hipSuccess;
  scale_update_kernel<<<grid, 256, 0, st>>>((bf16_t*)arena, plan, seed_lo, seed_hi, eta, d_clipped,
                                            res);
  return hipGetLastError();
}

// Codebook variant: c_n <- max(c_n - eta*d'*z_n, 0) on fp16 per-channel scales.
__global__ void channel_update_kernel(_Float16* __restrict__ c, uint32_t n, uint32_t row_base,
                                      uint32_t seed_lo, uint32_t seed_hi, float eta, float dclip_host,
                                      const qzo_step_result* __restrict__ res) {
  float cs;
  if (res) {
    if (res->status != 0) return;
    cs = eta * res->d_clipped;
  } else {
    cs = eta * dclip_host;
  }
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float z = flat_normal(seed_lo, seed_hi, 1u, row_base + i);
  c[i] = (_Float16)fmaxf(__builtin_fmaf(-cs, z, (float)c[i]), 0.0f);
}
hipError_t launch_channel_update(void* c_fp16, uint32_t n, uint32_t row_base, uint32_t seed_lo,
                                 uint32_t seed_hi, float eta, float d_clipped,
                                 const qzo_step_result* res, hipStream_t st) {
  if (n == 0) return hipSuccess;
  channel_update_kernel<<<(n + 255) / 256, 256, 0, st>>>((_Float16*)c_fp16, n, row_base, seed_lo,
                                                         seed_hi, eta, d_clipped, res);
  return hipGetLastError();
}

// ---- joint SPSA on the un-quantized parameters (Sec. 3.2; the 2-bit setup of Sec. 4.1) ----
// theta_u is one flat fp32 master vector; entry i draws z_i from stream 2 at counter (i/8, 0)
// (eight consecutive entries share a Philox counter).  A thread owns eight entries.
//
// Perturbation: the model's 16-bit tensor that entry i belongs to receives
// round16(theta_i + sigma*eps*z_i) (one fp32 fma, one RNE to bf16 or fp16).  Tensors start at
// multiples of 8 entries; `segs` is sorted by first entry and searched per thread.
__global__ __launch_bounds__(256) void dense_perturb_kernel(const float* __restrict__ master,
                                                            const DenseSeg* __restrict__ segs,
                                                            uint32_t n_seg, uint64_t n8,
                                                            uint32_t seed_lo, uint32_t seed_hi,
                                                            float eps_signed) {
  const uint64_t t = (uint64_t)blockIdx.x * 256u + threadIdx.x;
  if (t >= n8) return;
  uint32_t lo = 0, hi = n_seg;            // last segment with first8 <= t
  while (hi - lo > 1) {
    const uint32_t mid = (lo + hi) >> 1;
    if (segs[mid].first8 <= t) lo = mid; else hi = mid;
  }
  const DenseSeg sg = segs[lo];
  float z[8];
  scale_normals8(seed_lo, seed_hi, 2u, (uint32_t)t, (uint32_t)(t >> 32), z);
  const float4 a = reinterpret_cast<const float4*>(master)[2 * t];
  const float4 b = reinterpret_cast<const float4*>(master)[2 * t + 1];
  const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
  uint32_t out[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float e0 = __builtin_fmaf(eps_signed, z[2 * j], v[2 * j]);
    const float e1 = __builtin_fmaf(eps_signed, z[2 * j + 1], v[2 * j + 1]);
    if (sg.fmt == 1) {
      const _Float16 h0 = (_Float16)e0, h1 = (_Float16)e1;
      out[j] = (uint32_t)__builtin_bit_cast(uint16_t, h0) | ((uint32_t)__builtin_bit_cast(uint16_t, h1) << 16);
    } else {
      out[j] = pack_bf16x2(e0, e1);
    }
  }
  reinterpret_cast<uint4*>(sg.out)[t - sg.first8] = make_uint4(out[0], out[1], out[2], out[3]);
}

hipError_t launch_dense_perturb(const float* master, const DenseSeg* segs_dev, uint32_t n_seg,
                                uint64_t n_dense, uint32_t seed_lo, uint32_t seed_hi, float eps_signed,
                                hipStream_t st) {
  const uint64_t n8 = n_dense / 8;
  if (n8 == 0) return hipSuccess;
  dense_perturb_kernel<<<(uint32_t)((n8 + 255) / 256), 256, 0, st>>>(master, segs_dev, n_seg, n8, seed_lo,
                                                                     seed_hi, eps_signed);
  return hipGetLastError();
}

// Update: theta_i <- theta_i - eta_u * d' * z_i (fp32, one fma, no clamp).
__global__ __launch_bounds__(256) void dense_update_kernel(float* __restrict__ master, uint64_t n8,
                                                           uint32_t seed_lo, uint32_t seed_hi, float eta,
                                                           float dclip_host,
                                                           const qzo_step_result* __restrict__ res) {
  float c;
  if (res) {
    if (res->status != 0) return;
    c = eta * res->d_clipped;
  } else {
    c = eta * dclip_host;
  }
  const uint64_t t = (uint64_t)blockIdx.x * 256u + threadIdx.x;
  if (t >= n8) return;
  float z[8];
  scale_normals8(seed_lo, seed_hi, 2u, (uint32_t)t, (uint32_t)(t >> 32), z);
  float4* p = reinterpret_cast<float4*>(master) + 2 * t;
  float4 a = p[0], b = p[1];
  const float nc = -c;
  a.x = __builtin_fmaf(nc, z[0], a.x); a.y = __builtin_fmaf(nc, z[1], a.y);
  a.z = __builtin_fmaf(nc, z[2], a.z); a.w = __builtin_fmaf(nc, z[3], a.w);
  b.x = __builtin_fmaf(nc, z[4], b.x); b.y = __builtin_fmaf(nc, z[5], b.y);
  b.z = __builtin_fmaf(nc, z[6], b.z); b.w = __builtin_fmaf(nc, z[7], b.w);
  p[0] = a;
  p[1] = b;
}

hipError_t launch_dense_update(float* master, uint64_t n_dense, uint32_t seed_lo, uint32_t seed_hi,
                               float eta, float d_clipped, const qzo_step_result* res, hipStream_t st) {
  const uint64_t n8 = n_dense / 8;
  if (n8 == 0) return hipSuccess;
  dense_update_kernel<<<(uint32_t)((n8 + 255) / 256), 256, 0, st>>>(master, n8, seed_lo, seed_hi, eta,
                                                                    d_clipped, res);
  return hipGetLastError();
}

// ------------------------------------------- SPSA scalar + DDC (Eq. 6) ----
__global__ void spsa_clip_kernel(const float* __restrict__ losses, float eps, float clip,
                                 qzo_step_result* __restrict__ res) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  float lp = losses[0], lm = losses[1];
  float d = (lp - lm) / (2.0f * eps);
  res->loss_plus = lp;
  res->loss_minus = lm;
  res->d = d;
  if (!isfinite(d)) {
    res->d_clipped = 0.0f;
    res->status = QZO_ERR_NONFINITE;
  } else {
    float dc = d > clip ? clip : (d < -clip ? -clip : d);
    res->d_clipped = dc;
    res->status = QZO_OK;
  }
  res->reserved[0] = res->reserved[1] = res->reserved[2] = 0u;
}
hipError_t launch_spsa_clip(const float* losses, float eps, float clip, qzo_step_result* res,
                            hipStream_t st) {
  spsa_clip_kernel<<<1, 64, 0, st>>>(losses, eps, clip, res);
  return hipGetLastError();
}

// ------------------------------------------------------ RTN (Eq. 3) -------
// One wavefront per group of 128 weights: absmax, Delta = bf16(absmax/7),
// wbar = clamp(rne(w/Delta), -8, 7), nibble = wbar + 8.
__global__ __launch_bounds__(256) void rtn_quantize_kernel(const float* __restrict__ w, uint32_t N,
                                                           uint32_t K, uint8_t* __restrict__ q,
                                                           bf16_t* __restrict__ s) {
  const uint32_t G = K >> 7;
  const uint64_t grp = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (grp >= (uint64_t)N * G) return;
  const uint32_t lane = threadIdx.x & 63;
  const uint64_t n = grp / G;
  const uint32_t g = (uint32_t)(grp - n * G);
  const float2 v = *reinterpret_cast<const float2*>(w + n * K + (uint64_t)g * 128 + lane * 2);
  float amax = wave_max(fmaxf(fabsf(v.x), fabsf(v.y)));
  float sc = bf16_to_f32(f32_to_bf16(amax / 7.0f));
  int q0 = 0, q1 = 0;
  if (sc > 0.0f) {
    q0 = (int)fminf(7.0f, fmaxf(-8.0f, rintf(v.x / sc)));
    q1 = (int)fminf(7.0f, fmaxf(-8.0f, rintf(v.y / sc)));
  }
  q[n * (K >> 1) + (uint64_t)g * 64 + lane] = (uint8_t)((q0 + 8) | ((q1 + 8) << 4));
  if (lane == 0) s[grp] = f32_to_bf16(sc);
}
hipError_t launch_rtn_quantize(const float* w, uint32_t N, uint32_t K, void* q, void* s,
                               hipStream_t st) {
  uint64_t groups = (uint64_t)N * (K >> 7);
  if (groups == 0) return hipSuccess;
  rtn_quantize_kernel<<<(uint32_t)((groups + 3) / 4), 256, 0, st>>>(w, N, K, (uint8_t*)q,
                                                                    (bf16_t*)s);
  return hipGetLastError();
}

// The same with a zero-point: the group's range [min(w, 0), max(w, 0)] on the 16 levels.
__global__ __launch_bounds__(256) void rtn_quantize_asym_kernel(const float* __restrict__ w, uint32_t N,
                                                                uint32_t K, bool s_fp16,
                                                                uint8_t* __restrict__ q,
                                                                uint8_t* __restrict__ zp,
                                                                bf16_t* __restrict__ s) {
  const uint32_t G = K >> 7;
  const uint64_t grp = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (grp >= (uint64_t)N * G) return;
  const uint32_t lane = threadIdx.x & 63;
  const uint64_t n = grp / G;
  const uint32_t g = (uint32_t)(grp - n * G);
  const float2 v = *reinterpret_cast<const float2*>(w + n * K + (uint64_t)g * 128 + lane * 2);
  const float hi = wave_max(fmaxf(fmaxf(v.x, v.y), 0.0f));
  const float lo = -wave_max(fmaxf(fmaxf(-v.x, -v.y), 0.0f));
  const uint32_t sbits = f32_to_scale((hi - lo) / 15.0f, s_fp16);
  const float sc = scale_to_f32(sbits, s_fp16);
  int z0 = 8, q0 = 8, q1 = 8;
  if (sc > 0.0f) {
    z0 = (int)fminf(15.0f, fmaxf(0.0f, rintf(-lo / sc)));
    q0 = (int)fminf(15.0f, fmaxf(0.0f, rintf(v.x / sc) + (float)z0));
    q1 = (int)fminf(15.0f, fmaxf(0.0f, rintf(v.y / sc) + (float)z0));
  }
  q[n * (K >> 1) + (uint64_t)g * 64 + lane] = (uint8_t)(q0 | (q1 << 4));
  if (lane == 0) {
    s[grp] = (bf16_t)sbits;
    zp[grp] = (uint8_t)z0;
  }
}
hipError_t launch_rtn_quantize_asym(const float* w, uint32_t N, uint32_t K, bool s_fp16, void* q, void* zp,
                                    void* s, hipStream_t st) {
  uint64_t groups = (uint64_t)N * (K >> 7);
  if (groups == 0) return hipSuccess;
  rtn_quantize_asym_kernel<<<(uint32_t)((groups + 3) / 4), 256, 0, st>>>(w, N, K, s_fp16, (uint8_t*)q,
                                                                         (uint8_t*)zp, (bf16_t*)s);
  return hipGetLastError();
}

// ------------------------------------------------------- inspection -------
__global__ void debug_normals_kernel(uint32_t seed_lo, uint32_t seed_hi, uint32_t stream_id,
                                     uint32_t row0, uint32_t n_rows, uint32_t G, float* out) {
  const uint32_t Gb = (G + 7) >> 3;
  const uint64_t u = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= (uint64_t)n_rows * Gb) return;
  const uint32_t r = (uint32_t)(u / Gb), gb = (uint32_t)(u % Gb);
  float z[8];
  scale_normals8(seed_lo, seed_hi, stream_id, row0 + r, gb, z);
  for (int j = 0; j < 8; ++j)
    if (gb * 8 + j < G) out[(uint64_t)r * G + gb * 8 + j] = z[j];
}
hipError_t launch_debug_normals(uint32_t seed_lo, uint32_t seed_hi, uint32_t stream_id,
                                uint32_t row0, uint32_t n_rows, uint32_t G, float* out,
                                hipStream_t st) {
  uint64_t units = (uint64_t)n_rows * ((G + 7) >> 3);
  if (units == 0) return hipSuccess;
  debug_normals_kernel<<<(uint32_t)((units + 255) / 256), 256, 0, st>>>(seed_lo, seed_hi, stream_id,
                                                                       row0, n_rows, G, out);
  return hipGetLastError();
}

__global__ void debug_philox_kernel(uint32_t seed_lo, uint32_t seed_hi, const uint32_t* ctr,
                                    uint32_t n, uint32_t* out) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  u32x4_t r = philox4x32_10(ctr[4 * i], ctr[4 * i + 1], ctr[4 * i + 2], ctr[4 * i + 3], seed_lo,
                          seed_hi);
  out[4 * i] = r.x; out[4 * i + 1] = r.y; out[4 * i + 2] = r.z; out[4 * i + 3] = r.w;
}
hipError_t launch_debug_philox(uint32_t seed_lo, uint32_t seed_hi, const uint32_t* ctr,
                               uint32_t n, uint32_t* out, hipStream_t st) {
  if (n == 0) return hipSuccess;
  debug_philox_kernel<<<(n + 255) / 256, 256, 0, st>>>(seed_lo, seed_hi, ctr, n, out);
  return hipGetLastError();
}

__global__ void debug_normal_pairs_kernel(const uint32_t* words, uint32_t n, float* out) {
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float a, b;
  normal_pair(words[i], a, b);
  out[2 * i] = a;
  out[2 * i + 1] = b;
}
hipError_t launch_debug_normal_pairs(const uint32_t* words, uint32_t n, float* out,
                                     hipStream_t st) {
  if (n == 0) return hipSuccess;
  debug_normal_pairs_kernel<<<(n + 255) / 256, 256, 0, st>>>(words, n, out);
  return hipGetLastError();
}

// bf16((s + sign*eps*z) * wbar) for every weight: thread = (n, 8 consecutive k).
// zp (nullable): one zero-point byte per (row, group); null = 8.
__global__ void debug_dequant_kernel(const uint8_t* __restrict__ q, const bf16_t* __restrict__ s,
                                     const uint8_t* __restrict__ zp, bool s_fp16,
                                     uint32_t row_base, uint32_t N, uint32_t K, uint32_t seed_lo,
                                     uint32_t seed_hi, float eps_signed, bf16_t* __restrict__ out) {
  const uint32_t cpr = K >> 3;
  const uint64_t u = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= (uint64_t)N * cpr) return;
  const uint32_t n = (uint32_t)(u / cpr), c = (uint32_t)(u % cpr);
  const uint32_t g = c >> 4, G = K >> 7;
  float z[8];
  scale_normals8(seed_lo, seed_hi, 0u, row_base + n, g >> 3, z);
  float zz = z[0];
#pragma unroll
  for (int j = 1; j < 8; ++j) zz = ((g & 7u) == (uint32_t)j) ? z[j] : zz;
  const float se = __builtin_fmaf(eps_signed, zz, scale_to_f32(s[(uint64_t)n * G + g], s_fp16));
  const uint32_t packed = *reinterpret_cast<const uint32_t*>(q + (uint64_t)n * (K >> 1) + c * 4);
  const int z0 = zp ? (int)zp[(uint64_t)n * G + g] : 8;
  uint32_t o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float a = se * (float)((int)((packed >> (8 * j)) & 15u) - z0);
    float b = se * (float)((int)((packed >> (8 * j + 4)) & 15u) - z0);
    o[j] = pack_bf16x2(a, b);
  }
  *reinterpret_cast<uint4*>(out + (uint64_t)n * K + c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}
hipError_t launch_debug_dequant(const void* q, const void* s, const void* zp, bool s_fp16, uint32_t row_base,
                                uint32_t N, uint32_t K, uint32_t seed_lo, uint32_t seed_hi, float eps_signed,
                                void* w_eff, hipStream_t st) {
  uint64_t units = (uint64_t)N * (K >> 3);
  if (units == 0) return hipSuccess;
  debug_dequant_kernel<<<(uint32_t)((units + 255) / 256), 256, 0, st>>>(
      (const uint8_t*)q, (const bf16_t*)s, (const uint8_t*)zp, s_fp16, row_base, N, K, seed_lo, seed_hi,
      eps_signed, (bf16_t*)w_eff);
  return hipGetLastError();
}

// Repack of an asymmetric 4-bit linear from the K-major checkpoint layout (qweight int32
// [K/8, N]: word (kk, n) = nibbles of k = 8 kk .. 8 kk + 7, lowest first; qzeros int32
// [G, N/8]: word (g, nn) = zero-points of n = 8 nn .. 8 nn + 7; scales fp16 [G, N]) into the
// library's row-major layout.  One thread per (n, 8 k): a dword of nibbles in k order is the
// source word itself; the first thread of a group also writes the zero-point and the scale.
__global__ void repack_kmajor_kernel(const uint32_t* __restrict__ qweight,
                                     const uint32_t* __restrict__ qzeros,
                                     const _Float16* __restrict__ scales, uint32_t N, uint32_t K,
                                     uint32_t zero_add, bool s_fp16, uint32_t* __restrict__ q_out,
                                     uint8_t* __restrict__ zp_out, bf16_t* __restrict__ s_out) {
  const uint32_t cpr = K >> 3, G = K >> 7;
  const uint64_t u = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= (uint64_t)N * cpr) return;
  // consecutive threads take consecutive n of one kk: coalesced reads of the K-major words
  const uint32_t kk = (uint32_t)(u / N), n = (uint32_t)(u % N);
  q_out[(uint64_t)n * cpr + kk] = qweight[(uint64_t)kk * N + n];
  if ((kk & 15u) == 0u) {
    const uint32_t g = kk >> 4;
    const uint32_t z = (qzeros[(uint64_t)g * (N >> 3) + (n >> 3)] >> (4 * (n & 7u))) & 15u;
    zp_out[(uint64_t)n * G + g] = (uint8_t)((z + zero_add) & 15u);
    s_out[(uint64_t)n * G + g] = (bf16_t)f32_to_scale((float)scales[(uint64_t)g * N + n], s_fp16);
  }
}
hipError_t launch_repack_kmajor(const void* qweight, const void* qzeros, const void* scales,
                                uint32_t N, uint32_t K, uint32_t zero_add, bool s_fp16, void* q_out,
                                void* zp_out, void* s_out, hipStream_t st) {
  const uint64_t units = (uint64_t)N * (K >> 3);
  if (units == 0) return hipSuccess;
  repack_kmajor_kernel<<<(uint32_t)((units + 255) / 256), 256, 0, st>>>(
      (const uint32_t*)qweight, (const uint32_t*)qzeros, (const _Float16*)scales, N, K, zero_add, s_fp16,
      (uint32_t*)q_out, (uint8_t*)zp_out, (bf16_t*)s_out);
  return hipGetLastError();
}

// -------------------------------------------------------- embedding -------
// Row m belongs to pass m / pass_stride and is row r = m % pass_stride of it: it embeds tok[r] at
// position r % S, or zeros when r >= tok_rows (rows that pad a pass to a whole number of GEMM tiles).
__global__ void embed_kernel(const int32_t* __restrict__ tok, uint32_t tok_rows, uint32_t pass_stride,
                             const bf16_t* __restrict__ te,
                             const bf16_t* __restrict__ pe, uint32_t M, uint32_t S, uint32_t d,
                             bf16_t* __restrict__ h) {
  const uint32_t cpr = d >> 3;
  const uint64_t u = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= (uint64_t)M * cpr) return;
  const uint32_t m = (uint32_t)(u / cpr), c = (uint32_t)(u % cpr), r = m % pass_stride;
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (r < tok_rows) {
    v = *reinterpret_cast<const uint4*>(te + (uint64_t)tok[r] * d + c * 8);
    if (pe) {
      uint4 p = *reinterpret_cast<const uint4*>(pe + (uint64_t)(r % S) * d + c * 8);
      uint32_t a[4] = {v.x, v.y, v.z, v.w}, b[4] = {p.x, p.y, p.z, p.w}, o[4];
#pragma unroll
      for (int j = 0; j < 4; ++j)
        o[j] = pack_bf16x2(__uint_as_float(a[j] << 16) + __uint_as_float(b[j] << 16),
                           __uint_as_float(a[j] & 0xffff0000u) + __uint_as_float(b[j] & 0xffff0000u));
      v = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
  *reinterpret_cast<uint4*>(h + (uint64_t)m * d + c * 8) = v;
}
hipError_t launch_embed(const int32_t* tok, uint32_t tok_rows, uint32_t pass_stride, const void* tok_emb,
                        const void* pos_emb, uint32_t M, uint32_t S, uint32_t d, void* h, hipStream_t st) {
  uint64_t units = (uint64_t)M * (d >> 3);
  embed_kernel<<<(uint32_t)((units + 255) / 256), 256, 0, st>>>(tok, tok_rows, pass_stride, (const bf16_t*)tok_emb,
                                                               (const bf16_t*)pos_emb, M, S, d,
                                                               (bf16_t*)h);
  return hipGetLastError();
}

// ------------------------------------------------------------ norms -------
// One workgroup per row; fp32 statistics, wavefront-shuffle reduction, fixed
// order across the four wavefronts.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// CACHED: the row fits four 16-byte chunks per thread and is read from memory once; else every
// pass over the row reads it again.
template <bool LAYERNORM, bool CACHED>
__global__ __launch_bounds__(256) void norm_kernel(const bf16_t* __restrict__ x,
                                                   const bf16_t* __restrict__ gain,
                                                   const bf16_t* __restrict__ bias, uint32_t d,
                                                   float eps, bf16_t* __restrict__ y,
                                                   float* __restrict__ xsum_t) {
  __shared__ float red[4];
  const bf16_t* xr = x + (uint64_t)blockIdx.x * d;
  bf16_t* yr = y + (uint64_t)blockIdx.x * d;
  const uint32_t cpr = d >> 3;
  constexpr int NC = 4;
  uint4 xv[NC];
  if (CACHED) {
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const uint32_t c = threadIdx.x + 256u * i;
      xv[i] = c < cpr ? *reinterpret_cast<const uint4*>(xr + c * 8) : make_uint4(0, 0, 0, 0);
    }
  }
  // chunk i of this thread (CACHED) or chunk c of the row
  auto chunk = [&](int i, uint32_t c) { return CACHED ? xv[i] : *reinterpret_cast<const uint4*>(xr + c * 8); };
  const uint32_t passes = CACHED ? NC : (cpr + 255) / 256;
  float mu = 0.0f;
  if (LAYERNORM) {
    float acc = 0.0f;
#pragma unroll
    for (uint32_t i = 0; i < passes; ++i) {
      const uint32_t c = threadIdx.x + 256u * i;
      if (c < cpr) {
        const uint4 v = chunk(i, c);
        const uint32_t a[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) acc += __uint_as_float(a[j] << 16) + __uint_as_float(a[j] & 0xffff0000u);
      }
    }
    mu = block_sum(acc, red) / (float)d;
  }
  float ss = 0.0f;
#pragma unroll
  for (uint32_t i = 0; i < passes; ++i) {
    const uint32_t c = threadIdx.x + 256u * i;
    if (c < cpr) {
      const uint4 v = chunk(i, c);
      const uint32_t a[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float lo = __uint_as_float(a[j] << 16) - mu, hi = __uint_as_float(a[j] & 0xffff0000u) - mu;
        ss = __builtin_fmaf(lo, lo, ss);
        ss = __builtin_fmaf(hi, hi, ss);
      }
    }
  }
  const float var = block_sum(ss, red) / (float)d;
  const float inv = 1.0f / sqrtf(var + eps);
#pragma unroll
  for (uint32_t i = 0; i < passes; ++i) {
    const uint32_t c = threadIdx.x + 256u * i;
    uint32_t o[4] = {0, 0, 0, 0};
    if (c < cpr) {
      const uint4 v = chunk(i, c);
      uint4 gq = *reinterpret_cast<const uint4*>(gain + c * 8);
      uint32_t a[4] = {v.x, v.y, v.z, v.w}, g[4] = {gq.x, gq.y, gq.z, gq.w}, b[4] = {0, 0, 0, 0};
      if (LAYERNORM) {
        uint4 bq = *reinterpret_cast<const uint4*>(bias + c * 8);
        b[0] = bq.x; b[1] = bq.y; b[2] = bq.z; b[3] = bq.w;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float lo = (__uint_as_float(a[j] << 16) - mu) * inv * __uint_as_float(g[j] << 16);
        float hi = (__uint_as_float(a[j] & 0xffff0000u) - mu) * inv * __uint_as_float(g[j] & 0xffff0000u);
        if (LAYERNORM) {
          lo += __uint_as_float(b[j] << 16);
          hi += __uint_as_float(b[j] & 0xffff0000u);
        }
        o[j] = pack_bf16x2(lo, hi);
      }
      *reinterpret_cast<uint4*>(yr + c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
    }
    if (xsum_t) {
      // block sums of the row's output for a few-token linear that reads it: the 16 chunks of 128 features
      // sit in 16 consecutive lanes (every lane takes part: lanes beyond the row add zero)
      float lo = 0.0f, hi = 0.0f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        lo += __uint_as_float(o[j] << 16);
        hi += __uint_as_float(o[j] & 0xffff0000u);
      }
      float sx = lo + hi;
      sx += __shfl_xor(sx, 1, 64); sx += __shfl_xor(sx, 2, 64);
      sx += __shfl_xor(sx, 4, 64); sx += __shfl_xor(sx, 8, 64);
      if (c < cpr && (c & 15u) == 0u) xsum_t[(uint64_t)(c >> 4) * gridDim.x + blockIdx.x] = sx;
    }
  }
}
hipError_t launch_rmsnorm(const void* x, const void* gain, uint32_t M, uint32_t d, float eps,
                          void* y, hipStream_t st, float* xsum_t) {
  if (d % 128) xsum_t = nullptr;
  if (d <= 8192)
    norm_kernel<false, true><<<M, 256, 0, st>>>((const bf16_t*)x, (const bf16_t*)gain, nullptr, d, eps, (bf16_t*)y,
                                                xsum_t);
  else
    norm_kernel<false, false><<<M, 256, 0, st>>>((const bf16_t*)x, (const bf16_t*)gain, nullptr, d, eps, (bf16_t*)y,
                                                 xsum_t);
  return hipGetLastError();
}
hipError_t launch_layernorm(const void* x, const void* gain, const void* bias, uint32_t M,
                            uint32_t d, float eps, void* y, hipStream_t st, float* xsum_t) {
  if (d % 128) xsum_t = nullptr;
  if (d <= 8192)
    norm_kernel<true, true><<<M, 256, 0, st>>>((const bf16_t*)x, (const bf16_t*)gain, (const bf16_t*)bias, d, eps,
                                               (bf16_t*)y, xsum_t);
  else
    norm_kernel<true, false><<<M, 256, 0, st>>>((const bf16_t*)x, (const bf16_t*)gain, (const bf16_t*)bias, d, eps,
                                                (bf16_t*)y, xsum_t);
  return hipGetLastError();
}

// ------------------------------------------------------------- RoPE -------
// table[t][i] = (cos, sin)(t * theta^(-2i/dh)), i < dh/2, evaluated in double.
__global__ void rope_table_kernel(float2* table, uint32_t max_seq, uint32_t half, double theta,
                                  double dh) {
  uint32_t u = blockIdx.x * blockDim.x + threadIdx.x;
  if (u >= max_seq * half) return;
  uint32_t t = u / half, i = u % half;
  double ang = (double)t * pow(theta, -2.0 * (double)i / dh);
  table[u] = make_float2((float)cos(ang), (float)sin(ang));
}
hipError_t launch_rope_table(float* table, uint32_t max_seq, uint32_t dh, float theta,
                             hipStream_t st) {
  uint32_t n = max_seq * (dh / 2);
  rope_table_kernel<<<(n + 255) / 256, 256, 0, st>>>((float2*)table, max_seq, dh / 2,
                                                     (double)theta, (double)dh);
  return hipGetLastError();
}
// rotate-half pairing (i, i+dh/2) on the q and k thirds of qkv [M, 3d], in place; row m is at
// position (m % pass_stride) % S.
__global__ void rope_kernel(bf16_t* __restrict__ qkv, const float2* __restrict__ table, uint32_t M,
                            uint32_t S, uint32_t pass_stride, uint32_t d, uint32_t n_heads) {
  const uint32_t dh = d / n_heads, half = dh >> 1, cph = half >> 3;   // 8-wide chunks per half head
  const uint64_t u = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const uint64_t per_row = (uint64_t)2 * n_heads * cph;
  if (u >= (uint64_t)M * per_row) return;
  const uint32_t m = (uint32_t)(u / per_row);
  uint32_t r = (uint32_t)(u % per_row);
  const uint32_t c = r % cph; r /= cph;
  const uint32_t h = r % n_heads, which = r / n_heads;
  bf16_t* p = qkv + (uint64_t)m * 3 * d + (uint64_t)which * d + h * dh + c * 8;
  const float2* tb = table + (uint64_t)((m % pass_stride) % S) * half + c * 8;
  uint4 va = *reinterpret_cast<const uint4*>(p), vb = *reinterpret_cast<const uint4*>(p + half);
  uint32_t a[4] = {va.x, va.y, va.z, va.w}, b[4] = {vb.x, vb.y, vb.z, vb.w}, oa[4], ob[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float2 t0 = tb[2 * j], t1 = tb[2 * j + 1];
    float a0 = __uint_as_float(a[j] << 16), a1 = __uint_as_float(a[j] & 0xffff0000u);
    float b0 = __uint_as_float(b[j] << 16), b1 = __uint_as_float(b[j] & 0xffff0000u);
    oa[j] = pack_bf16x2(a0 * t0.x - b0 * t0.y, a1 * t1.x - b1 * t1.y);
    ob[j] = pack_bf16x2(b0 * t0.x + a0 * t0.y, b1 * t1.x + a1 * t1.y);
  }
  *reinterpret_cast<uint4*>(p) = make_uint4(oa[0], oa[1], oa[2], oa[3]);
  *reinterpret_cast<uint4*>(p + half) = make_uint4(ob[0], ob[1], ob[2], ob[3]);
}
hipError_t launch_rope(void* qkv, const float* table, uint32_t M, uint32_t S, uint32_t pass_stride, uint32_t d,
                       uint32_t n_heads, hipStream_t st) {
  const uint32_t dh = d / n_heads;
  uint64_t units = (uint64_t)M * 2 * n_heads * (dh / 16);
  rope_kernel<<<(uint32_t)((units + 255) / 256), 256, 0, st>>>((bf16_t*)qkv, (const float2*)table,
                                                              M, S, pass_stride, d, n_heads);
  return hipGetLastError();
}

// --------------------------------------------- cross-entropy reduction ----
// part[m][slice] = (max, sum exp(l - max)) over the slice's columns.  One
// wavefront merges a row: lse - target logit; rows at the last position of a
// sequence predict nothing and contribute 0.
__global__ __launch_bounds__(256) void ce_rows_kernel(const float* __restrict__ part,
                                                      const float* __restrict__ tgt, uint32_t M,
                                                      uint32_t S, uint32_t n_slices,
                                                      float* __restrict__ rowloss) {
  const uint32_t m = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (m >= M) return;
  if (m % S == S - 1) {
    if (lane == 0) rowloss[m] = 0.0f;
    return;
  }
  const float2* p = reinterpret_cast<const float2*>(part) + (uint64_t)m * n_slices;
  float mx = -INFINITY;
  for (uint32_t i = lane; i < n_slices; i += 64) mx = fmaxf(mx, p[i].x);
  mx = wave_max(mx);
  float sum = 0.0f;
  for (uint32_t i = lane; i < n_slices; i += 64) {
    float2 v = p[i];
    if (v.y > 0.0f) sum += v.y * expf(v.x - mx);
  }
  sum = wave_sum(sum);
  if (lane == 0) rowloss[m] = (mx + logf(sum)) - tgt[m];
}
// Fixed-order sum of n floats in double by one workgroup; out = sum * scale.
__global__ __launch_bounds__(256) void sum_kernel(const float* __restrict__ v, uint32_t n,
                                                  double scale, float* __restrict__ out) {
  __shared__ double red[256];
  double acc = 0.0;
  for (uint32_t i = threadIdx.x; i < n; i += 256) acc += (double)v[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = (float)(red[0] * scale);
}
hipError_t launch_ce_reduce(const float* part, const float* tgt, uint32_t M, uint32_t S,
                            uint32_t n_slices, float* rowloss, float* loss_out, hipStream_t st) {
  ce_rows_kernel<<<(M + 3) / 4, 256, 0, st>>>(part, tgt, M, S, n_slices, rowloss);
  const uint32_t B = M / S;
  sum_kernel<<<1, 256, 0, st>>>(rowloss, M, 1.0 / ((double)B * (double)(S - 1)), loss_out);
  return hipGetLastError();
}
hipError_t launch_sum_partials(const float* partials, uint32_t n, float* out, hipStream_t st) {
  sum_kernel<<<1, 256, 0, st>>>(partials, n, 1.0, out);
  return hipGetLastError();
}

}  // namespace qzo
