// Causal self-attention softmax(Q K^T / sqrt(dh)) V for gfx950, bf16 MFMA with
// fp32 online softmax, head size 64 or 128.  Input is the fused projection
// output qkv [B*S, 3d] (q | k | v), output [B*S, d].
//
// A workgroup of four wavefronts serves 128 queries of one (batch, head); each
// wavefront owns 32 queries.  Scores are produced transposed (keys x queries)
// so that a lane owns one query: the softmax row reductions are in-register
// plus one cross-half shuffle, the probabilities are already in the B-operand
// layout of the second MFMA, and O^T = V^T P^T accumulates with a per-lane
// rescale.  K tiles (32 keys) sit row-major in LDS, V tiles transposed.
#include "qzo_device.hpp"
#include "qzo_kernels.hpp"

namespace qzo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int DH>
__global__ __launch_bounds__(256) void attention_kernel(const bf16_t* __restrict__ qkv, uint32_t S,
                                                        uint32_t n_heads, bf16_t* __restrict__ out) {
  constexpr int KT = DH / 16;        // k-steps of the score MFMA
  constexpr int DT = DH / 32;        // 32-wide slices of the head for the PV MFMA
  constexpr int CH = DH / 8;         // 16-byte chunks per K row
  constexpr int VT_STRIDE = 40;      // padded keys per V^T row (bf16 units)
  __shared__ __attribute__((aligned(16))) bf16_t Ks[32 * DH];
  __shared__ __attribute__((aligned(16))) bf16_t Vt[DH * VT_STRIDE];

  const uint32_t d = n_heads * DH, ld = 3 * d;
  const uint32_t b = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * 128;
  const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
  const uint32_t lrow = lane & 31u, lhalf = lane >> 5;
  const bf16_t* base = qkv + (uint64_t)b * S * ld + h * DH;
  const uint32_t qq = q0 + wave * 32 + lrow;            // this lane's query
  const uint32_t qc = min(qq, S - 1);

  bf16x8 qf[KT];
#pragma unroll
  for (int ks = 0; ks < KT; ++ks)
    qf[ks] = *reinterpret_cast<const bf16x8*>(base + (uint64_t)qc * ld + ks * 16 + lhalf * 8);

  floatx16 o[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;
  const float sc = 1.44269504088896f / sqrtf((float)DH);   // log2(e)/sqrt(dh)

  const uint32_t q_hi = min(q0 + 127u, S - 1);
  const uint32_t nkb = q_hi / 32 + 1;
  const uint32_t wave_q_hi = q0 + wave * 32 + 31;

  for (uint32_t kb = 0; kb < nkb; ++kb) {
    __syncthreads();
    // K tile: 32 rows x CH chunks, swizzled; V tile transposed.
    for (uint32_t c = t; c < 32u * CH; c += 256) {
      const uint32_t row = c / CH, ch = c % CH;
      const uint32_t key = min(kb * 32 + row, S - 1);
      const bf16_t* src = base + (uint64_t)key * ld + ch * 8;
      uint4 kv = *reinterpret_cast<const uint4*>(src + d);
      *reinterpret_cast<uint4*>(Ks + row * DH + ((ch ^ (row & 7u)) * 8)) = kv;
      uint4 vv = *reinterpret_cast<const uint4*>(src + 2 * d);
      const uint32_t w[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        Vt[(ch * 8 + 2 * j) * VT_STRIDE + row] = (bf16_t)(w[j] & 0xffffu);
        Vt[(ch * 8 + 2 * j + 1) * VT_STRIDE + row] = (bf16_t)(w[j] >> 16);
      }
    }
    __syncthreads();
    if (kb * 32 > wave_q_hi) continue;          // every key of the tile is in this wave's future

    // scores^T: rows = keys, cols = queries
    floatx16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.0f;
#pragma unroll
    for (int ks = 0; ks < KT; ++ks) {
      const uint32_t ch = ks * 2 + lhalf;
      bf16x8 kf = *reinterpret_cast<const bf16x8*>(Ks + lrow * DH + ((ch ^ (lrow & 7u)) * 8));
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s, 0, 0, 0);
    }
    float mx = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const uint32_t key = kb * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
      s[r] = key <= qq ? s[r] * sc : -INFINITY;
      mx = fmaxf(mx, s[r]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    float psum = 0.0f;
    float p[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      p[r] = __builtin_amdgcn_exp2f(s[r] - m_new);
      psum += p[r];
    }
    psum += __shfl_xor(psum, 32, 64);
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
    // P^T as the B operand: element e of k-step st is key 8(2 st + e/4) + 4 half + e%4,
    // i.e. score register 8 st + e.
#pragma unroll
    for (int st = 0; st < 2; ++st) {
      union { bf16x8 v; uint32_t u[4]; } pf;
#pragma unroll
      for (int e = 0; e < 4; ++e) pf.u[e] = pack_bf16x2(p[8 * st + 2 * e], p[8 * st + 2 * e + 1]);
#pragma unroll
      for (int i = 0; i < DT; ++i) {
        union { bf16x8 v; uint2 h[2]; } vf;
        const bf16_t* vr = Vt + (i * 32 + lrow) * VT_STRIDE + 16 * st + 4 * lhalf;
        vf.h[0] = *reinterpret_cast<const uint2*>(vr);
        vf.h[1] = *reinterpret_cast<const uint2*>(vr + 8);
        o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf.v, o[i], 0, 0, 0);
      }
    }
  }

  if (qq < S) {
    const float inv = 1.0f / l_run;
    bf16_t* dst = out + ((uint64_t)b * S + qq) * d + h * DH;
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 v;
        v.x = pack_bf16x2(o[i][4 * g] * inv, o[i][4 * g + 1] * inv);
        v.y = pack_bf16x2(o[i][4 * g + 2] * inv, o[i][4 * g + 3] * inv);
        *reinterpret_cast<uint2*>(dst + i * 32 + 8 * g + 4 * lhalf) = v;
      }
  }
}

hipError_t launch_attention(const void* qkv, uint32_t B, uint32_t S, uint32_t n_heads,
                            uint32_t dh, void* out, hipStream_t st) {
  dim3 grid((S + 127) / 128, n_heads, B);
  if (dh == 128)
    attention_kernel<128><<<grid, 256, 0, st>>>((const bf16_t*)qkv, S, n_heads, (bf16_t*)out);
  else if (dh == 64)
    attention_kernel<64><<<grid, 256, 0, st>>>((const bf16_t*)qkv, S, n_heads, (bf16_t*)out);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace qzo
