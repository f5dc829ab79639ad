// QZO CPU oracle -- TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, single-purpose C++ statement of what one step of Quantized
// Zeroth-order Optimization computes (paper Sec. 3.2, Eq. 3-6, Algorithm 1),
// used by the tests, the smoke check and the benchmark's cpu_baseline leg to
// judge the HIP path.  The product never calls it and it shares no code, no
// header and no table with the HIP sources: every constant below is typed
// here on its own.
//
// Precision: activations and every reduction are held in double.  The things
// the storage format fixes are done in that format: scales are bf16 values,
// the perturbed scale s + (sigma*eps)*z is one fp32 fma, the update is one
// fp32 fma followed by a round-to-nearest-even to bf16, and the normal
// variate z is an fp32 recipe made only of exact integer steps and fp32
// mul/add/fma so that any IEEE machine reproduces it bit for bit.  With
// act_bf16 != 0 the forward also rounds each activation tensor to bf16 where
// a 16-bit-activation implementation stores it (the "A16" of W4A16).
//
// No blocking, fusion or reordering: every function is the definition
// written out.  "#pragma omp parallel for" over independent output rows is
// the only concession to run time.
//
// Parity pins (tests/test_oracle_*.py): Philox published known answers,
// normal moments/accuracy against libm, RTN invariants, special-case GEMMs,
// closed-form SPSA on quadratic losses, brute-force finite differences on a
// tiny model, blocks against PyTorch CPU ops, the paper's Table 2 counts.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <cstdlib>
#include <map>
#include <vector>
#include <algorithm>

namespace {

// ---------------------------------------------------------------- bf16 ----
inline uint32_t f2u(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float u2f(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }

// Round-to-nearest-even of an fp32 value to the nearest bf16 value
// (returned as fp32).  NaN stays NaN.
inline float bf16_rne(float f) {
  uint32_t u = f2u(f);
  if ((u & 0x7f800000u) == 0x7f800000u && (u & 0x007fffffu)) return u2f(u | 0x00400000u);
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  return u2f(u);
}
// Round-to-nearest-even of an fp32 value to the nearest IEEE binary16 value
// (returned as fp32), subnormals and overflow to infinity included.
inline float fp16_rne(float f) {
  uint32_t u = f2u(f);
  uint32_t sign = u & 0x80000000u;
  uint32_t mag = u & 0x7fffffffu;
  if (mag >= 0x7f800000u) return f;                       // inf / nan
  if (mag >= 0x477ff000u) return u2f(sign | 0x7f800000u); // >= 65520 rounds to inf
  if (mag < 0x38800000u) {                                // below 2^-14: subnormal half, step 2^-24
    float a = u2f(mag);
    float r = (a + 0x1p-1f) - 0x1p-1f;                    // rounds a to a multiple of 2^-24 (RNE) exactly
    return u2f(sign | f2u(r));
  }
  uint32_t lsb = (mag >> 13) & 1u;
  mag += 0xfffu + lsb;
  mag &= 0xffffe000u;
  return u2f(sign | mag);
}
inline double round_act(double v, int act_bf16) {
  return act_bf16 ? (double)bf16_rne((float)v) : v;
}

// ------------------------------------------------------------- Philox ----
// Philox4x32 with 10 rounds (Salmon et al., "Parallel random numbers: as easy
// as 1, 2, 3", SC'11).  One round maps (c0,c1,c2,c3) to
// (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0)); the key is
// bumped by the Weyl constants after every round.
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53ull, M1 = 0xCD9E8D57ull;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    uint64_t p0 = M0 * (uint64_t)c0;
    uint64_t p1 = M1 * (uint64_t)c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// ------------------------------------------------- N(0,1) from 32 bits ----
// One 32-bit word gives one Box-Muller pair (z ~ N(0, I), paper Def. 3.1/3.3).
//   bits 31..16  h : u1 = (2h+1) / 2^17  in (0,1)
//   bit  15         : sign of the first variate
//   bit  14         : sign of the second variate
//   bits 13..0   k : first-quadrant angle phi = (k + 1/2) * (pi/2) / 2^14
// z0 = +-sqrt(-2 ln u1) cos(phi), z1 = +-sqrt(-2 ln u1) sin(phi).  Random
// signs on a first-quadrant angle give the same law as a full-circle angle.
// Everything is fp32 built from exact steps and mul/add/fma only:
//   -ln u1 = (17-E) ln2 + (1-m) Q(1-m),  2h+1 = m 2^E, m in [1/2,1)
//   sqrt(t) = t * y, y = 1/sqrt(t) by three Newton steps from an integer seed
//   with x = phi - pi/4 in (-pi/4, pi/4):  sqrt2 cos(phi) = cos x - sin x,
//   sqrt2 sin(phi) = cos x + sin x, and sqrt(-2 ln u1)/sqrt2 = sqrt(-ln u1).
void normal_pair(uint32_t w, float out[2]) {
  const float QL0 = 0x1.fffffap-1f, QL1 = 0x1.000586p-1f, QL2 = 0x1.53a4dcp-2f,
              QL3 = 0x1.18fbf0p-2f, QL4 = 0x1.a5d4cap-6f, QL5 = 0x1.a4912ap-1f,
              QL6 = -0x1.2245dap+0f, QL7 = 0x1.36ff60p+0f;
  const float LN2 = 0x1.62e430p-1f;
  const float ANG_STEP = 0x1.921fb6p-14f;   // (pi/2) / 2^14
  const float ANG_OFF = -0x1.92196cp-1f;    // half a step minus pi/4
  const float S0 = -0x1.555552p-3f, S1 = 0x1.110c2cp-7f, S2 = -0x1.9acab0p-13f;
  const float C0 = -0x1.000000p-1f, C1 = 0x1.55555ep-5f, C2 = -0x1.6c16a2p-10f,
              C3 = 0x1.9ca594p-16f;

  float a = (float)((w >> 15) | 1u);        // 2h+1, exact (< 2^17)
  int E;
  float m = std::frexp(a, &E);              // exact
  float f = 1.0f - m;                       // exact
  float q = QL7;
  q = std::fmaf(q, f, QL6); q = std::fmaf(q, f, QL5); q = std::fmaf(q, f, QL4);
  q = std::fmaf(q, f, QL3); q = std::fmaf(q, f, QL2); q = std::fmaf(q, f, QL1);
  q = std::fmaf(q, f, QL0);
  float fq = f * q;
  float t = std::fmaf((float)(17 - E), LN2, fq);          // -ln u1 > 0

  int32_t ti = (int32_t)f2u(t);
  float y = u2f((uint32_t)(0x5f3759df - (ti >> 1)));
  float ht = 0.5f * t;
  for (int it = 0; it < 3; ++it) {
    float hy = ht * y;
    float c = std::fmaf(-hy, y, 1.5f);
    y = y * c;
  }
  float r = t * y;                                        // sqrt(-ln u1)

  float x = std::fmaf((float)(w & 0x3fffu), ANG_STEP, ANG_OFF);
  float x2 = x * x;
  float sp = std::fmaf(x2, S2, S1);
  sp = std::fmaf(x2, sp, S0);
  float sx = std::fmaf(x2 * sp, x, x);                    // sin x
  float cp = std::fmaf(x2, C3, C2);
  cp = std::fmaf(x2, cp, C1);
  cp = std::fmaf(x2, cp, C0);
  float cx = std::fmaf(x2, cp, 1.0f);                     // cos x
  float z0 = r * (cx - sx);
  float z1 = r * (cx + sx);
  out[0] = u2f(f2u(z0) | ((w & 0x8000u) << 16));
  out[1] = u2f(f2u(z1) | ((w & 0x4000u) << 17));
}

// z for the scale of (row, group g) of a quantized linear; `row` is the
// row's index in the model-wide enumeration of quantized output rows.
// Counter = (row, g/8, stream, 0), key = seed; word (g%8)/2 of the block,
// variate g%2 of that word's pair.  The same seed regenerates the same z for
// the +eps pass, the -eps pass and the update (Algorithm 1: the generator is
// reset with seed s before each of them).
float scale_normal(uint64_t seed, uint32_t stream, uint32_t row, uint32_t g) {
  uint32_t ctr[4] = {row, g >> 3, stream, 0u};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t w[4];
  philox4x32_10(ctr, key, w);
  float pr[2];
  normal_pair(w[(g & 7u) >> 1], pr);
  return pr[g & 1u];
}

// z for entry i of a flat vector (per-output-channel scales of the codebook
// variant): counter = (i/8 low, i/8 high, stream, 0).
float flat_normal(uint64_t seed, uint32_t stream, uint64_t i) {
  uint64_t j = i >> 3;
  uint32_t ctr[4] = {(uint32_t)j, (uint32_t)(j >> 32), stream, 0u};
  uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  uint32_t w[4];
  philox4x32_10(ctr, key, w);
  float pr[2];
  normal_pair(w[(i & 7u) >> 1], pr);
  return pr[i & 1u];
}

inline int unpack_q(const uint8_t* qp, size_t K, size_t n, size_t k) {
  uint8_t b = qp[n * (K / 2) + k / 2];
  int u = (k & 1) ? (b >> 4) : (b & 15);
  return u - 8;
}

}  // namespace

extern "C" {

// ------------------------------------------------------------ RNG API ----
void orc_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  philox4x32_10(ctr, key, out);
}
void orc_normal_pair(uint32_t w, float* out) { normal_pair(w, out); }
void orc_normal_pairs(const uint32_t* w, uint64_t n, float* out) {
  for (uint64_t i = 0; i < n; ++i) normal_pair(w[i], out + 2 * i);
}
// out[r*G + g] = z(row0 + r, g)
void orc_scale_normals(uint64_t seed, uint32_t stream, uint32_t row0, uint32_t n_rows,
                       uint32_t G, float* out) {
  for (uint32_t r = 0; r < n_rows; ++r)
    for (uint32_t g = 0; g < G; ++g)
      out[(size_t)r * G + g] = scale_normal(seed, stream, row0 + r, g);
}
void orc_flat_normals(uint64_t seed, uint32_t stream, uint64_t first, uint64_t n, float* out) {
  for (uint64_t i = 0; i < n; ++i) out[i] = flat_normal(seed, stream, first + i);
}

float orc_bf16_rne(float f) { return bf16_rne(f); }
void orc_bf16_rne_array(float* x, uint64_t n) {
  for (uint64_t i = 0; i < n; ++i) x[i] = bf16_rne(x[i]);
}

// ------------------------------------------------ RTN quantization -------
// Eq. 3 with the paper's k-bit absmax scale, k = 4: for every row n and every
// group of `group` consecutive input features, Delta = absmax / 7 rounded to
// bf16 (its storage type), wbar = round-half-even(w / Delta) clamped to
// [-8,7].  A zero group gives Delta = 0, wbar = 0.  Stored nibble = wbar + 8,
// even k in the low nibble.
void orc_rtn_quantize(const float* w, uint64_t N, uint64_t K, uint32_t group,
                      uint8_t* qp, float* s) {
  uint64_t G = K / group;
  for (uint64_t n = 0; n < N; ++n) {
    for (uint64_t g = 0; g < G; ++g) {
      const float* wg = w + n * K + g * group;
      float amax = 0.f;
      for (uint32_t k = 0; k < group; ++k) amax = std::max(amax, std::fabs(wg[k]));
      float sc = bf16_rne(amax / 7.0f);
      s[n * G + g] = sc;
      for (uint32_t k = 0; k < group; ++k) {
        int qi = 0;
        if (sc > 0.f) {
          float r = std::nearbyintf(wg[k] / sc);   // default mode: ties to even
          qi = (int)std::min(7.0f, std::max(-8.0f, r));
        }
        uint64_t kk = g * group + k;
        uint8_t* b = qp + n * (K / 2) + kk / 2;
        uint8_t u = (uint8_t)(qi + 8);
        if (kk & 1) *b = (uint8_t)((*b & 0x0f) | (u << 4));
        else *b = (uint8_t)((*b & 0xf0) | u);
      }
    }
  }
}

// Asymmetric round-to-nearest groups (Eq. 3 with a zero-point): the range [min(w,0), max(w,0)]
// of a group is mapped on the 16 levels, s = round16((hi - lo) / 15), zp = rne(-lo / s) clamped to
// 0..15, u = clamp(rne(w / s) + zp, 0, 15); an all-zero group gives s = 0, zp = 8, u = 8.
// scale_fmt: the storage type of the scale, 0 = bf16, 1 = fp16 (what the 4-bit checkpoints of
// Sec. 4.1 hold).  g_idx (optional, int32 [K]): the group of every input column (activation
// reordering: the quantizer visits columns in an order of its own, so a group is any 128 columns,
// not 128 consecutive ones); null = k / group.
void orc_rtn_quantize_asym(const float* w, uint64_t N, uint64_t K, uint32_t group, int scale_fmt,
                           const int32_t* g_idx, uint8_t* qp, uint8_t* zp, float* s) {
  uint64_t G = K / group;
  auto grp = [&](uint64_t k) { return g_idx ? (uint64_t)g_idx[k] : k / group; };
  for (uint64_t n = 0; n < N; ++n) {
    std::vector<float> lo(G, 0.f), hi(G, 0.f);
    for (uint64_t k = 0; k < K; ++k) {
      const float v = w[n * K + k];
      lo[grp(k)] = std::min(lo[grp(k)], v);
      hi[grp(k)] = std::max(hi[grp(k)], v);
    }
    for (uint64_t g = 0; g < G; ++g) {
      const float raw = (hi[g] - lo[g]) / 15.0f;
      const float sc = scale_fmt == 1 ? fp16_rne(raw) : bf16_rne(raw);
      int z0 = 8;
      if (sc > 0.f) z0 = (int)std::min(15.0f, std::max(0.0f, std::nearbyintf(-lo[g] / sc)));
      s[n * G + g] = sc;
      zp[n * G + g] = (uint8_t)z0;
    }
    for (uint64_t k = 0; k < K; ++k) {
      const float sc = s[n * G + grp(k)];
      const int z0 = zp[n * G + grp(k)];
      int u = 8;
      if (sc > 0.f) u = (int)std::min(15.0f, std::max(0.0f, std::nearbyintf(w[n * K + k] / sc) + (float)z0));
      uint8_t* b = qp + n * (K / 2) + k / 2;
      if (k & 1) *b = (uint8_t)((*b & 0x0f) | (u << 4));
      else *b = (uint8_t)((*b & 0xf0) | u);
    }
  }
}

void orc_unpack_int4(const uint8_t* qp, uint64_t N, uint64_t K, int8_t* q) {
  for (uint64_t n = 0; n < N; ++n)
    for (uint64_t k = 0; k < K; ++k) q[n * K + k] = (int8_t)unpack_q(qp, K, n, k);
}

// ------------------------------------------- perturbed scales, Eq. 5 -----
// s_eff = s + (sigma*eps) * z as one fp32 fma; this is PERTURB_SCALES of
// Algorithm 1 evaluated functionally (the stored scale is never rewritten,
// which in exact arithmetic equals the +eps / -2eps / +eps sequence).
void orc_effective_scales(const float* s, uint32_t n_rows, uint32_t G, uint32_t row_base,
                          uint64_t seed, float eps_signed, double* out) {
  for (uint32_t r = 0; r < n_rows; ++r)
    for (uint32_t g = 0; g < G; ++g) {
      size_t i = (size_t)r * G + g;
      float z = scale_normal(seed, 0u, row_base + r, g);
      out[i] = (double)std::fmaf(eps_signed, z, s[i]);
    }
}

// Eq. 4 on the perturbed scale: W_eff[n,k] = s_eff[n, k/group] * wbar[n,k],
// the fp32 product, optionally viewed in bf16 (the bit-exact comparison point
// for unpack + indexing + perturbation).
void orc_dequant(const uint8_t* qp, const float* s, uint64_t N, uint64_t K, uint32_t group,
                 uint64_t seed, uint32_t row_base, float eps_signed, int to_bf16, float* w_eff) {
  uint64_t G = K / group;
  for (uint64_t n = 0; n < N; ++n)
    for (uint64_t k = 0; k < K; ++k) {
      uint64_t g = k / group;
      float z = scale_normal(seed, 0u, (uint32_t)(row_base + n), (uint32_t)g);
      float se = std::fmaf(eps_signed, z, s[n * G + g]);
      float v = se * (float)unpack_q(qp, K, n, k);
      w_eff[n * K + k] = to_bf16 ? bf16_rne(v) : v;
    }
}

// ---- asymmetric 4-bit groups (zero-points): the format of the 4-bit checkpoints the
// paper fine-tunes (Sec. 4.1: GPTQ, group 128).  W[n,k] = s[n,g] * (u[n,k] - zp[n,g]) with the
// stored nibble u in 0..15 and an integer zero-point zp in 0..15 per (row, group); Eq. 4-5 with
// wbar = u - zp.  zp = 8 is the symmetric format above.  With activation reordering the
// quantizer assigns input columns to groups in an order of its own: g_idx[k] (when given) is the
// group of column k instead of k / group; scales, zero-points and their noise stay per (row, group).
void orc_dequant_zp(const uint8_t* qp, const float* s, const uint8_t* zp, uint64_t N, uint64_t K,
                    uint32_t group, uint64_t seed, uint32_t row_base, float eps_signed, int to_bf16,
                    const int32_t* g_idx, float* w_eff) {
  uint64_t G = K / group;
  for (uint64_t n = 0; n < N; ++n)
    for (uint64_t k = 0; k < K; ++k) {
      uint64_t g = g_idx ? (uint64_t)g_idx[k] : k / group;
      float z = scale_normal(seed, 0u, (uint32_t)(row_base + n), (uint32_t)g);
      float se = std::fmaf(eps_signed, z, s[n * G + g]);
      int u = unpack_q(qp, K, n, k) + 8;                       // the stored nibble
      float v = se * (float)(u - (int)zp[n * G + g]);
      w_eff[n * K + k] = to_bf16 ? bf16_rne(v) : v;
    }
}
void orc_qlinear_zp(const double* x, uint64_t M, uint64_t K, const uint8_t* qp, const double* s_eff,
                    const uint8_t* zp, uint64_t N, uint32_t group, const float* bias,
                    const int32_t* g_idx, double* y) {
  uint64_t G = K / group;
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < (int64_t)N; ++n) {
    std::vector<double> wrow(K);
    for (uint64_t k = 0; k < K; ++k) {
      int u = unpack_q(qp, K, n, k) + 8;
      const uint64_t g = g_idx ? (uint64_t)g_idx[k] : k / group;
      wrow[k] = s_eff[n * G + g] * (double)(u - (int)zp[n * G + g]);
    }
    for (uint64_t m = 0; m < M; ++m) {
      double acc = 0.0;
      const double* xr = x + m * K;
      for (uint64_t k = 0; k < K; ++k) acc += xr[k] * wrow[k];
      y[m * N + n] = acc + (bias ? (double)bias[n] : 0.0);
    }
  }
}
// ---- 4-bit NormalFloat blocks (the quantizer of the text-to-image experiment, Sec. 4.3): a
// block of `block` (64) consecutive input features of a row shares one scale, the block's
// absmax; a weight is stored as the index u of the nearest of 16 fixed levels in [-1, 1]:
// W[n,k] = s[n, k/block] * level[u[n,k]], Eq. 4-5 with wbar = level[u].  The levels are the
// published NormalFloat-4 code book (Dettmers et al. 2023, App. E): the normal quantiles
// Phi^-1 at 8 evenly spaced probabilities from delta = 0.9677083 down to (not including) 1/2
// on the positive side, 7 on the negative side, and 0, divided by the largest.
const float NF4_LEVEL[16] = {
    -1.0f, -0.6961928009986877f, -0.5250730514526367f, -0.39491748809814453f,
    -0.28444138169288635f, -0.18477343022823334f, -0.09105003625154495f, 0.0f,
    0.07958029955625534f, 0.16093020141124725f, 0.24611230194568634f, 0.33791524171829224f,
    0.44070982933044434f, 0.5626170039176941f, 0.7229568362236023f, 1.0f};
void orc_nf4_levels(float* out) { for (int i = 0; i < 16; ++i) out[i] = NF4_LEVEL[i]; }

// s = bf16(absmax of the block) (the scale's storage type), u = index of the level nearest
// to w / s (the lower index on a tie); an all-zero block gives s = 0, u = 7 (level 0).
// Stored like the int4 format: two indices per byte, even k in the low nibble.
void orc_nf4_quantize(const float* w, uint64_t N, uint64_t K, uint32_t block, uint8_t* qp, float* s) {
  const uint64_t G = K / block;
  for (uint64_t n = 0; n < N; ++n)
    for (uint64_t g = 0; g < G; ++g) {
      float amax = 0.0f;
      for (uint32_t j = 0; j < block; ++j) amax = std::max(amax, std::fabs(w[n * K + g * block + j]));
      const float sc = bf16_rne(amax);
      s[n * G + g] = sc;
      for (uint32_t j = 0; j < block; ++j) {
        const uint64_t k = g * block + j;
        int u = 7;
        if (sc > 0.0f) {
          const double r = (double)w[n * K + k] / (double)sc;
          double best = 1e300;
          for (int i = 0; i < 16; ++i) {
            const double e = std::fabs(r - (double)NF4_LEVEL[i]);
            if (e < best) { best = e; u = i; }
          }
        }
        uint8_t& byte = qp[n * (K / 2) + k / 2];
        byte = (k & 1) ? (uint8_t)((byte & 0x0f) | (u << 4)) : (uint8_t)((byte & 0xf0) | u);
      }
    }
}
inline int nf4_index(const uint8_t* qp, uint64_t K, uint64_t n, uint64_t k) {
  const uint8_t b = qp[n * (K / 2) + k / 2];
  return (k & 1) ? (b >> 4) : (b & 0x0f);
}
// W_eff[n,k] = (s + sigma*eps*z)[n, k/block] * level[u[n,k]]: one fp32 fma, one fp32 product,
// optionally viewed in bf16.
void orc_dequant_nf4(const uint8_t* qp, const float* s, uint64_t N, uint64_t K, uint32_t block,
                     uint64_t seed, uint32_t row_base, float eps_signed, int to_bf16, float* w_eff) {
  const uint64_t G = K / block;
  for (uint64_t n = 0; n < N; ++n)
    for (uint64_t k = 0; k < K; ++k) {
      const uint64_t g = k / block;
      const float z = scale_normal(seed, 0u, (uint32_t)(row_base + n), (uint32_t)g);
      const float se = std::fmaf(eps_signed, z, s[n * G + g]);
      const float v = se * NF4_LEVEL[nf4_index(qp, K, n, k)];
      w_eff[n * K + k] = to_bf16 ? bf16_rne(v) : v;
    }
}
// Y[m,n] = sum_k X[m,k] * s_eff[n,k/block] * level[u[n,k]] (+ bias[n]).
void orc_qlinear_nf4(const double* x, uint64_t M, uint64_t K, const uint8_t* qp, const double* s_eff,
                     uint64_t N, uint32_t block, const float* bias, double* y) {
  const uint64_t G = K / block;
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < (int64_t)N; ++n) {
    std::vector<double> wrow(K);
    for (uint64_t k = 0; k < K; ++k)
      wrow[k] = s_eff[n * G + k / block] * (double)NF4_LEVEL[nf4_index(qp, K, n, k)];
    for (uint64_t m = 0; m < M; ++m) {
      double acc = 0.0;
      const double* xr = x + m * K;
      for (uint64_t k = 0; k < K; ++k) acc += xr[k] * wrow[k];
      y[m * N + n] = acc + (bias ? (double)bias[n] : 0.0);
    }
  }
}

// Repacking from the K-major checkpoint layout: qweight int32 [K/8, N], word (kk, n) holding
// the nibbles of k = 8 kk .. 8 kk + 7 of output n, lowest nibble first; qzeros int32 [G, N/8],
// word (g, nn) holding the zero-points of n = 8 nn .. 8 nn + 7; scales fp16 values [G, N].
// Out: nibbles [N, K/2] (low nibble = even k), zero-points [N, G] (stored value + zero_add,
// masked to 4 bits), scales [N, G] rounded to bf16.
void orc_repack_kmajor(const uint32_t* qweight, const uint32_t* qzeros, const float* scales_f16,
                       uint64_t N, uint64_t K, uint32_t group, uint32_t zero_add, uint8_t* qp,
                       uint8_t* zp, float* s_bf16) {
  uint64_t G = K / group;
  for (uint64_t n = 0; n < N; ++n) {
    for (uint64_t k = 0; k < K; k += 2) {
      uint32_t lo = (qweight[(k / 8) * N + n] >> (4 * (k % 8))) & 15u;
      uint32_t hi = (qweight[((k + 1) / 8) * N + n] >> (4 * ((k + 1) % 8))) & 15u;
      qp[n * (K / 2) + k / 2] = (uint8_t)(lo | (hi << 4));
    }
    for (uint64_t g = 0; g < G; ++g) {
      uint32_t z = (qzeros[g * (N / 8) + n / 8] >> (4 * (n % 8))) & 15u;
      zp[n * G + g] = (uint8_t)((z + zero_add) & 15u);
      s_bf16[n * G + g] = bf16_rne(scales_f16[g * N + n]);
    }
  }
}

// Y[m,n] = sum_k X[m,k] * s_eff[n,k/group] * wbar[n,k] (+ bias[n]).
void orc_qlinear(const double* x, uint64_t M, uint64_t K, const uint8_t* qp, const double* s_eff,
                 uint64_t N, uint32_t group, const float* bias, double* y) {
  uint64_t G = K / group;
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < (int64_t)N; ++n) {
    std::vector<double> wrow(K);
    for (uint64_t k = 0; k < K; ++k)
      wrow[k] = s_eff[n * G + k / group] * (double)unpack_q(qp, K, n, k);
    for (uint64_t m = 0; m < M; ++m) {
      double acc = 0.0;
      const double* xr = x + m * K;
      for (uint64_t k = 0; k < K; ++k) acc += xr[k] * wrow[k];
      y[m * N + n] = acc + (bias ? (double)bias[n] : 0.0);
    }
  }
}

// Plain dense Y = X W^T (+bias), W fp32 [N,K].
void orc_linear(const double* x, uint64_t M, uint64_t K, const float* w, uint64_t N,
                const float* bias, double* y) {
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < (int64_t)N; ++n)
    for (uint64_t m = 0; m < M; ++m) {
      double acc = 0.0;
      for (uint64_t k = 0; k < K; ++k) acc += x[m * K + k] * (double)w[n * K + k];
      y[m * N + n] = acc + (bias ? (double)bias[n] : 0.0);
    }
}

// sum over all entries of bf16_rne(y)^2 (the single-linear workload's loss).
double orc_sumsq_bf16(const double* y, uint64_t n) {
  double acc = 0.0;
  for (uint64_t i = 0; i < n; ++i) {
    double v = (double)bf16_rne((float)y[i]);
    acc += v * v;
  }
  return acc;
}

// ------------------------------------------------ transformer blocks -----
void orc_rmsnorm(const double* x, uint64_t M, uint64_t d, const float* gain, double eps, double* y) {
  for (uint64_t m = 0; m < M; ++m) {
    double ss = 0.0;
    for (uint64_t i = 0; i < d; ++i) ss += x[m * d + i] * x[m * d + i];
    double inv = 1.0 / std::sqrt(ss / (double)d + eps);
    for (uint64_t i = 0; i < d; ++i) y[m * d + i] = x[m * d + i] * inv * (double)gain[i];
  }
}

void orc_layernorm(const double* x, uint64_t M, uint64_t d, const float* gain, const float* bias,
                   double eps, double* y) {
  for (uint64_t m = 0; m < M; ++m) {
    double mu = 0.0;
    for (uint64_t i = 0; i < d; ++i) mu += x[m * d + i];
    mu /= (double)d;
    double var = 0.0;
    for (uint64_t i = 0; i < d; ++i) { double c = x[m * d + i] - mu; var += c * c; }
    var /= (double)d;
    double inv = 1.0 / std::sqrt(var + eps);
    for (uint64_t i = 0; i < d; ++i)
      y[m * d + i] = (x[m * d + i] - mu) * inv * (double)gain[i] + (double)bias[i];
  }
}

// Rotary embedding, rotate-half pairing (i, i+dh/2), angle = pos * theta^(-2i/dh).
// x: [B*S, row_stride] with n_heads heads of dh starting at column col0.
void orc_rope(double* x, uint64_t B, uint64_t S, uint64_t row_stride, uint64_t col0,
              uint64_t n_heads, uint64_t dh, double theta) {
  uint64_t half = dh / 2;
  for (uint64_t b = 0; b < B; ++b)
    for (uint64_t t = 0; t < S; ++t)
      for (uint64_t h = 0; h < n_heads; ++h) {
        double* v = x + (b * S + t) * row_stride + col0 + h * dh;
        for (uint64_t i = 0; i < half; ++i) {
          double ang = (double)t * std::pow(theta, -2.0 * (double)i / (double)dh);
          double c = std::cos(ang), sn = std::sin(ang);
          double a = v[i], bb = v[i + half];
          v[i] = a * c - bb * sn;
          v[i + half] = bb * c + a * sn;
        }
      }
}

// Causal softmax(Q K^T / sqrt(dh)) V.  qkv: [B*S, 3*d] rows = [q | k | v],
// each d = n_heads*dh wide.  out: [B*S, d].
void orc_attention(const double* qkv, uint64_t B, uint64_t S, uint64_t n_heads, uint64_t dh,
                   double* out) {
  uint64_t d = n_heads * dh, ld = 3 * d;
  double scale = 1.0 / std::sqrt((double)dh);
#pragma omp parallel for schedule(static) collapse(2)
  for (int64_t b = 0; b < (int64_t)B; ++b)
    for (int64_t h = 0; h < (int64_t)n_heads; ++h) {
      std::vector<double> p(S);
      for (uint64_t t = 0; t < S; ++t) {
        const double* q = qkv + (b * S + t) * ld + h * dh;
        double mx = -INFINITY;
        for (uint64_t u = 0; u <= t; ++u) {
          const double* k = qkv + (b * S + u) * ld + d + h * dh;
          double sc = 0.0;
          for (uint64_t i = 0; i < dh; ++i) sc += q[i] * k[i];
          p[u] = sc * scale;
          mx = std::max(mx, p[u]);
        }
        double den = 0.0;
        for (uint64_t u = 0; u <= t; ++u) { p[u] = std::exp(p[u] - mx); den += p[u]; }
        double* o = out + (b * S + t) * d + h * dh;
        for (uint64_t i = 0; i < dh; ++i) o[i] = 0.0;
        for (uint64_t u = 0; u <= t; ++u) {
          const double* v = qkv + (b * S + u) * ld + 2 * d + h * dh;
          double pw = p[u] / den;
          for (uint64_t i = 0; i < dh; ++i) o[i] += pw * v[i];
        }
      }
    }
}

// gu: [M, 2F] rows = [gate | up]; out[m,f] = silu(gate) * up.
void orc_swiglu(const double* gu, uint64_t M, uint64_t F, double* out) {
  for (uint64_t m = 0; m < M; ++m)
    for (uint64_t f = 0; f < F; ++f) {
      double g = gu[m * 2 * F + f], u = gu[m * 2 * F + F + f];
      out[m * F + f] = g / (1.0 + std::exp(-g)) * u;
    }
}

// Mean over the B*(S-1) positions t < S-1 of -log softmax(logits[b,t,:])[tok[b,t+1]].
double orc_next_token_ce(const double* logits, const int32_t* tok, uint64_t B, uint64_t S,
                         uint64_t V) {
  double total = 0.0;
  for (uint64_t b = 0; b < B; ++b)
    for (uint64_t t = 0; t + 1 < S; ++t) {
      const double* l = logits + (b * S + t) * V;
      double mx = l[0];
      for (uint64_t v = 1; v < V; ++v) mx = std::max(mx, l[v]);
      double den = 0.0;
      for (uint64_t v = 0; v < V; ++v) den += std::exp(l[v] - mx);
      total += (mx + std::log(den)) - l[tok[b * S + t + 1]];
    }
  return total / (double)(B * (S - 1));
}

// ------------------------------------------- codebook-quantized linear ----
// Codebook variant (the paper's 2-bit setting: one 16-bit code per 8 weights, one
// codebook of 65536 8-vectors per linear, a per-output-channel scale that Q-SPSA
// perturbs and updates): W[n,k] = c[n] * CB[idx[n,k/8]][k%8], so
// Y[m,n] = c_eff[n] * sum_k X[m,k] CB[idx[n,k/8]][k%8] (+ bias[n]).
float orc_fp16_rne(float f) { return fp16_rne(f); }
void orc_fp16_rne_array(float* x, uint64_t n) {
  for (uint64_t i = 0; i < n; ++i) x[i] = fp16_rne(x[i]);
}
void orc_codebook_linear(const double* x, uint64_t M, uint64_t K, const uint16_t* idx,
                         const float* cb, const double* c_eff, uint64_t N, const float* bias,
                         double* y) {
  const uint64_t KB = K / 8;
#pragma omp parallel for schedule(static)
  for (int64_t n = 0; n < (int64_t)N; ++n) {
    std::vector<double> wrow(K);
    for (uint64_t k = 0; k < K; ++k) wrow[k] = (double)cb[(uint64_t)idx[n * KB + k / 8] * 8 + (k & 7)];
    for (uint64_t m = 0; m < M; ++m) {
      double acc = 0.0;
      const double* xr = x + m * K;
      for (uint64_t k = 0; k < K; ++k) acc += xr[k] * wrow[k];
      y[m * N + n] = acc * c_eff[n] + (bias ? (double)bias[n] : 0.0);
    }
  }
}
// c_eff[n] = c[n] + (sigma*eps) * z(row_base + n) as one fp32 fma; z from the flat
// counter stream 1 (one Philox counter per 8 channels).
void orc_channel_effective_scales(const float* c, uint32_t n_rows, uint32_t row_base,
                                  uint64_t seed, float eps_signed, double* out) {
  for (uint32_t r = 0; r < n_rows; ++r)
    out[r] = (double)std::fmaf(eps_signed, flat_normal(seed, 1u, (uint64_t)row_base + r), c[r]);
}
// c_n <- max(c_n - eta*d'*z_n, 0), fp16 storage (Algorithm 1's update on channel scales).
void orc_update_channel_scales(float* c, uint32_t n_rows, uint32_t row_base, uint64_t seed,
                               float eta, float d_clipped) {
  const float cstep = eta * d_clipped;
  for (uint32_t r = 0; r < n_rows; ++r) {
    float z = flat_normal(seed, 1u, (uint64_t)row_base + r);
    c[r] = fp16_rne(std::max(std::fmaf(-cstep, z, c[r]), 0.0f));
  }
}

// ---- joint SPSA on the un-quantized parameters (Sec. 3.2: Q-SPSA on the scales may be combined
// with plain SPSA, Def. 3.1, on the parameters that were never quantized; Sec. 4.1 does so in the
// 2-bit runs).  These parameters form one flat fp32 master vector theta_u; entry i draws
// z_i = flat_normal(seed, stream 2, i), the same seed as the scales but a stream of its own.
// The model computes with 16-bit tensors, so a pass sees round16(theta_u + sigma*eps*z): one fp32
// fma, then one round-to-nearest-even to the tensor's storage format (0: bf16, 1: fp16).
void orc_dense_effective(const float* master, uint64_t first, uint64_t n, uint64_t seed,
                         float eps_signed, int fmt, float* out) {
  for (uint64_t i = 0; i < n; ++i) {
    float v = std::fmaf(eps_signed, flat_normal(seed, 2u, first + i), master[i]);
    out[i] = fmt == 1 ? fp16_rne(v) : bf16_rne(v);
  }
}
// theta_u <- theta_u - eta_u * d' * z (ZO-SGD with the SPSA estimate, Eq. 2 with the clipped
// scalar of Eq. 6; no clamp: these parameters may have either sign).  fp32 master: one fma.
void orc_dense_update(float* master, uint64_t first, uint64_t n, uint64_t seed, float eta,
                      float d_clipped) {
  const float cstep = eta * d_clipped;
  for (uint64_t i = 0; i < n; ++i)
    master[i] = std::fmaf(-cstep, flat_normal(seed, 2u, first + i), master[i]);
}

// ----------------------------------------------------- model forward -----
struct orc_config {
  uint32_t arch;        // 0 = Llama family (RMSNorm, RoPE, SwiGLU, no bias), 1 = OPT family
  uint32_t n_layers, d_model, n_heads, d_ffn, vocab, max_seq, group;
  double norm_eps, rope_theta;
  uint32_t quant;       // 0 = int4 + per-group scales, 1 = codebook + per-channel scales (Llama only),
                        // 2 = int4 with zero-points: every packed weight is followed by u8 [N, K/group]
                        // 3 = NormalFloat-4 indices + per-block scales (group = block = 64)
  uint32_t act_order;   // quant = 2 only: every zero-point tensor is followed by g_idx, int32 [K], the
                        // group of each input column (activation reordering of the Sec. 4.1 checkpoints)
};

// Tensor table, in this order (all fp32 arrays holding bf16 values unless noted):
//  Llama: tok_emb[V,d]; per layer { attn_norm[d], wqkv(u8 [3d,d/2]), wo(u8 [d,d/2]),
//         ffn_norm[d], wgu(u8 [2F,d/2], gate rows then up rows), wdown(u8 [d,F/2]) };
//         final_norm[d]; lm_head[V,d].
//  OPT:   tok_emb[V,d]; pos_emb[max_seq,d]; per layer { ln1_g[d], ln1_b[d], wqkv(u8), bqkv[3d],
//         wo(u8), bo[d], ln2_g[d], ln2_b[d], wfc1(u8 [F,d/2]), bfc1[F], wfc2(u8 [d,F/2]),
//         bfc2[d] }; lnf_g[d], lnf_b[d]; lm_head[V,d].
//  Llama, quant = 1: every quantized weight is two entries, the codes (u16 [N,K/8]) followed by
//         the codebook (fp32 holding fp16 values, [65536,8]); s_eff then holds one effective
//         scale per output row, per layer [3d][d][2F][d].
// s_eff: effective scales (double) in arena order: per layer [qkv: 3d x d/group]
// [o: d x d/group][gu or fc1: (2F or F) x d/group][down or fc2: d x F/group].
// Returns the loss L(Delta (.) theta_bar; B) of Algorithm 1.  Optional outputs
// (may be null): final hidden state after the last norm [M,d], logits [M,V].
double orc_forward_loss(const orc_config* c, const void* const* T, const double* s_eff,
                        const int32_t* tok, uint32_t B, uint32_t S, int act_bf16,
                        double* hidden_out, double* logits_out) {
  const uint64_t d = c->d_model, F = c->d_ffn, V = c->vocab, H = c->n_heads, dh = d / H;
  const uint64_t M = (uint64_t)B * S, Gd = d / c->group, GF = F / c->group;
  const bool llama = c->arch == 0;
  size_t ti = 0;
  const float* tok_emb = (const float*)T[ti++];
  const float* pos_emb = llama ? nullptr : (const float*)T[ti++];
  std::vector<double> h(M * d), a(M * d), qkv(M * 3 * d), att(M * d), lin(M * d);
  std::vector<double> ff(M * (llama ? 2 * F : F)), act(M * F);
  for (uint64_t b = 0; b < B; ++b)
    for (uint64_t t = 0; t < S; ++t) {
      uint64_t m = b * S + t;
      for (uint64_t i = 0; i < d; ++i) {
        double v = (double)tok_emb[(uint64_t)tok[m] * d + i];
        if (pos_emb) v = round_act(v + (double)pos_emb[t * d + i], act_bf16);
        h[m * d + i] = v;
      }
    }
  const double* se = s_eff;
  auto round_all = [&](std::vector<double>& x) {
    if (act_bf16) for (auto& v : x) v = (double)bf16_rne((float)v);
  };
  const bool asym = c->quant == 2;
  // a packed int4 weight and, in the asymmetric format, the zero-point tensor that follows it
  std::map<const uint8_t*, const int32_t*> group_index;     // of the weights that carry one
  auto take_w = [&](const uint8_t*& w, const uint8_t*& z) {
    w = (const uint8_t*)T[ti++];
    z = asym ? (const uint8_t*)T[ti++] : nullptr;
    if (asym && c->act_order) group_index[w] = (const int32_t*)T[ti++];
  };
  auto qlin = [&](const double* x, uint64_t K, const uint8_t* w, const uint8_t* z, const double* sc,
                  uint64_t N, const float* bias, double* y) {
    if (c->quant == 3) orc_qlinear_nf4(x, M, K, w, sc, N, c->group, bias, y);
    else if (z) orc_qlinear_zp(x, M, K, w, sc, z, N, c->group, bias,
                               group_index.count(w) ? group_index[w] : nullptr, y);
    else orc_qlinear(x, M, K, w, sc, N, c->group, bias, y);
  };
  for (uint32_t l = 0; l < c->n_layers; ++l) {
    if (llama && c->quant == 1) {
      const float* n1 = (const float*)T[ti++];
      const uint16_t* iqkv = (const uint16_t*)T[ti++]; const float* cqkv = (const float*)T[ti++];
      const uint16_t* io = (const uint16_t*)T[ti++]; const float* co = (const float*)T[ti++];
      const float* n2 = (const float*)T[ti++];
      const uint16_t* igu = (const uint16_t*)T[ti++]; const float* cgu = (const float*)T[ti++];
      const uint16_t* idn = (const uint16_t*)T[ti++]; const float* cdn = (const float*)T[ti++];
      orc_rmsnorm(h.data(), M, d, n1, c->norm_eps, a.data()); round_all(a);
      orc_codebook_linear(a.data(), M, d, iqkv, cqkv, se, 3 * d, nullptr, qkv.data()); se += 3 * d;
      round_all(qkv);
      orc_rope(qkv.data(), B, S, 3 * d, 0, H, dh, c->rope_theta);
      orc_rope(qkv.data(), B, S, 3 * d, d, H, dh, c->rope_theta);
      round_all(qkv);
      orc_attention(qkv.data(), B, S, H, dh, att.data()); round_all(att);
      orc_codebook_linear(att.data(), M, d, io, co, se, d, nullptr, lin.data()); se += d;
      for (uint64_t i = 0; i < M * d; ++i) h[i] = round_act(h[i] + lin[i], act_bf16);
      orc_rmsnorm(h.data(), M, d, n2, c->norm_eps, a.data()); round_all(a);
      orc_codebook_linear(a.data(), M, d, igu, cgu, se, 2 * F, nullptr, ff.data()); se += 2 * F;
      round_all(ff);
      orc_swiglu(ff.data(), M, F, act.data()); round_all(act);
      orc_codebook_linear(act.data(), M, F, idn, cdn, se, d, nullptr, lin.data()); se += d;
      for (uint64_t i = 0; i < M * d; ++i) h[i] = round_act(h[i] + lin[i], act_bf16);
    } else if (llama) {
      const uint8_t *wqkv, *zqkv, *wo, *zo, *wgu, *zgu, *wdn, *zdn;
      const float* n1 = (const float*)T[ti++];
      take_w(wqkv, zqkv);
      take_w(wo, zo);
      const float* n2 = (const float*)T[ti++];
      take_w(wgu, zgu);
      take_w(wdn, zdn);
      orc_rmsnorm(h.data(), M, d, n1, c->norm_eps, a.data()); round_all(a);
      qlin(a.data(), d, wqkv, zqkv, se, 3 * d, nullptr, qkv.data()); se += 3 * d * Gd;
      round_all(qkv);
      orc_rope(qkv.data(), B, S, 3 * d, 0, H, dh, c->rope_theta);
      orc_rope(qkv.data(), B, S, 3 * d, d, H, dh, c->rope_theta);
      round_all(qkv);
      orc_attention(qkv.data(), B, S, H, dh, att.data()); round_all(att);
      qlin(att.data(), d, wo, zo, se, d, nullptr, lin.data()); se += d * Gd;
      for (uint64_t i = 0; i < M * d; ++i) h[i] = round_act(h[i] + lin[i], act_bf16);
      orc_rmsnorm(h.data(), M, d, n2, c->norm_eps, a.data()); round_all(a);
      qlin(a.data(), d, wgu, zgu, se, 2 * F, nullptr, ff.data()); se += 2 * F * Gd;
      round_all(ff);
      orc_swiglu(ff.data(), M, F, act.data()); round_all(act);
      qlin(act.data(), F, wdn, zdn, se, d, nullptr, lin.data()); se += d * GF;
      for (uint64_t i = 0; i < M * d; ++i) h[i] = round_act(h[i] + lin[i], act_bf16);
    } else {
      const uint8_t *wqkv, *zqkv, *wo, *zo, *w1, *z1, *w2, *z2;
      const float* g1 = (const float*)T[ti++]; const float* b1 = (const float*)T[ti++];
      take_w(wqkv, zqkv); const float* bqkv = (const float*)T[ti++];
      take_w(wo, zo); const float* bo = (const float*)T[ti++];
      const float* g2 = (const float*)T[ti++]; const float* b2 = (const float*)T[ti++];
      take_w(w1, z1); const float* bf1 = (const float*)T[ti++];
      take_w(w2, z2); const float* bf2 = (const float*)T[ti++];
      orc_layernorm(h.data(), M, d, g1, b1, c->norm_eps, a.data()); round_all(a);
      qlin(a.data(), d, wqkv, zqkv, se, 3 * d, bqkv, qkv.data()); se += 3 * d * Gd;
      round_all(qkv);
      orc_attention(qkv.data(), B, S, H, dh, att.data()); round_all(att);
      qlin(att.data(), d, wo, zo, se, d, bo, lin.data()); se += d * Gd;
      for (uint64_t i = 0; i < M * d; ++i) h[i] = round_act(h[i] + lin[i], act_bf16);
      orc_layernorm(h.data(), M, d, g2, b2, c->norm_eps, a.data()); round_all(a);
      qlin(a.data(), d, w1, z1, se, F, bf1, ff.data()); se += F * Gd;
      for (uint64_t i = 0; i < M * F; ++i) act[i] = round_act(std::max(ff[i], 0.0), act_bf16);
      qlin(act.data(), F, w2, z2, se, d, bf2, lin.data()); se += d * GF;
      for (uint64_t i = 0; i < M * d; ++i) h[i] = round_act(h[i] + lin[i], act_bf16);
    }
  }
  if (llama) {
    const float* nf = (const float*)T[ti++];
    orc_rmsnorm(h.data(), M, d, nf, c->norm_eps, a.data());
  } else {
    const float* gf = (const float*)T[ti++]; const float* bf = (const float*)T[ti++];
    orc_layernorm(h.data(), M, d, gf, bf, c->norm_eps, a.data());
  }
  round_all(a);
  const float* lm = (const float*)T[ti++];
  std::vector<double> logits(M * V);
  orc_linear(a.data(), M, d, lm, V, nullptr, logits.data());
  if (hidden_out) std::memcpy(hidden_out, a.data(), sizeof(double) * M * d);
  if (logits_out) std::memcpy(logits_out, logits.data(), sizeof(double) * M * V);
  return orc_next_token_ce(logits.data(), tok, B, S, V);
}

// ------------------------------------- SPSA scalar, DDC, ZO-SGD update ---
// d = (l+ - l-) / (2 eps), fp32 (Algorithm 1; Eq. 5 without the trailing z).
float orc_spsa_d(float loss_plus, float loss_minus, float eps) {
  return (loss_plus - loss_minus) / (2.0f * eps);
}
// Eq. 6: d' = C if d > C, -C if d < -C, d otherwise.
float orc_clip(float d, float C) {
  if (d > C) return C;
  if (d < -C) return -C;
  return d;
}
// Delta_i <- max(Delta_i - eta*d'*z_i, 0) with z regenerated from the seed
// (Algorithm 1), in the scales' storage arithmetic: c = eta*d' (one fp32
// multiply), fp32 fma, clamp, round-to-nearest-even to the storage type
// (scale_fmt 0: bf16, 1: fp16).
void orc_update_scales(float* s, uint32_t n_rows, uint32_t G, uint32_t row_base, uint64_t seed,
                       float eta, float d_clipped, int scale_fmt) {
  float cstep = eta * d_clipped;
  for (uint32_t r = 0; r < n_rows; ++r)
    for (uint32_t g = 0; g < G; ++g) {
      size_t i = (size_t)r * G + g;
      float z = scale_normal(seed, 0u, row_base + r, g);
      float v = std::fmaf(-cstep, z, s[i]);
      s[i] = scale_fmt == 1 ? fp16_rne(std::max(v, 0.0f)) : bf16_rne(std::max(v, 0.0f));
    }
}

// Algorithm 1 as printed, on stored scales of arbitrary precision (double,
// no storage rounding): perturb +eps, -2eps, +eps in place.  Used only to
// check that the functional form above is the same computation.
void orc_perturb_in_place(double* s, uint32_t n_rows, uint32_t G, uint32_t row_base,
                          uint64_t seed, double eps) {
  for (uint32_t r = 0; r < n_rows; ++r)
    for (uint32_t g = 0; g < G; ++g)
      s[(size_t)r * G + g] += eps * (double)scale_normal(seed, 0u, row_base + r, g);
}

}  // extern "C"
