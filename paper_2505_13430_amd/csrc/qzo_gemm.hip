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
// by row pair so that 16 lanes of a fragment read hit all 64 banks), double
// buffered.  int4 weights are unpacked, scaled by the perturbed scale and
// rounded to bf16 once per workgroup while being written to LDS; the noise z is
// regenerated per row every eight groups from the Philox counter (row, g/8)
// and never touches memory.
//
// The weight tile is the MFMA's first operand and the activation tile its
// second, so a lane of the result owns one token and four consecutive output
// features per register group: stores are 8 bytes wide and the cross-entropy
// reductions run over a lane's own registers.
#include "qzo_gemm_tile.hpp"

namespace qzo {

uint32_t gemm_workgroups(uint32_t M, uint32_t N) {
  static uint32_t n_cu = 0;
  if (n_cu == 0) {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu < 8)
      cu = 256;
    n_cu = (uint32_t)cu & ~7u;
  }
  const uint32_t tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  return min(((tiles + 7) / 8) * 8, n_cu);
}

// Split-K of the int4 tile kernel: with fewer than half as many output tiles as compute units the K
// dimension is cut into slices of a multiple of 4 k-tiles (256 input features: whole groups, and an
// even first group so the noise pairs line up), enough of them to give every compute unit a slice.
uint32_t tile_ksplit(uint32_t M, uint32_t N, uint32_t K, uint32_t* kt_per) {
  const uint32_t tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN), nkt = K / BK;
  const uint32_t cus = gemm_workgroups(1u << 20, 1u << 20);            // compute units
  uint32_t ks = tiles ? cus / tiles : 1;
  ks = min(ks, nkt / 4u);
  if (ks < 2) { if (kt_per) *kt_per = nkt; return 1; }
  const uint32_t per = ((nkt + ks - 1) / ks + 3u) & ~3u;
  if (kt_per) *kt_per = per;
  return (nkt + per - 1) / per;
}
uint32_t tile_tail_cols(uint32_t M, uint32_t N, uint32_t K, uint32_t epi) {
  if (epi & (EPI_SWIGLU | EPI_ROPE | EPI_SUMSQ)) return 0;
  const uint32_t tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN, tiles = tm * tn;
  const uint32_t cus = gemm_workgroups(1u << 20, 1u << 20);
  if (tiles <= cus || tiles % cus == 0) return 0;
  uint32_t n1 = tn - 1;                              // feature tiles of the whole rounds
  while (n1 > 0 && (tm * n1) % cus != 0) --n1;
  if (n1 == 0) return 0;
  const uint32_t tail = tm * (tn - n1);
  // worth it when the tail can be cut into at least two K slices of at least 8 k-tiles
  if (tail * 2 > cus || tile_ksplit(M, N - n1 * BN, K, nullptr) < 2 || K / BK < 16) return 0;
  return n1 * BN;
}
uint64_t tile_split_ws_floats(uint32_t M, uint32_t N, uint32_t K) {
  const uint32_t ks = tile_ksplit(M, N, K, nullptr);
  if (ks > 1) return (uint64_t)ks * M * N;
  const uint32_t n1 = tile_tail_cols(M, N, K, 0);    // the epilogue is not known here: room for the plain case
  if (n1) return (uint64_t)tile_ksplit(M, N - n1, K, nullptr) * M * (N - n1);
  return 0;
}

// 8 nibbles of one dword -> 8 bf16 of (nibble-8)*se, in k order.  A byte holding
// a nibble u (0..15) read as an fp8 E4M3 pattern is exactly u * 2^-9, so one
// v_cvt_pk_f32_fp8 turns two nibbles into floats; fma(u 2^-9, 512 se, -8 se)
// is (u-8)*se with a single rounding, the same bits as se * float(u-8).
// With zero-points (ZP) the two parameters are the scale se and the negated zero-point:
// fma(u 2^-9, 512, -zp) is the integer u - zp exactly and its product with se is rounded
// once, the same bits as se * float(u - zp).
template <bool ZP = false>
__device__ __forceinline__ uint4 dequant8(uint32_t w, float se512, float m8se) {
  typedef float f2 __attribute__((ext_vector_type(2)));
  const uint32_t lo = w & 0x0f0f0f0fu, hi = (w >> 4) & 0x0f0f0f0fu;
  const f2 l01 = __builtin_amdgcn_cvt_pk_f32_fp8(lo, false);   // nibbles 0, 2
  const f2 l23 = __builtin_amdgcn_cvt_pk_f32_fp8(lo, true);    // nibbles 4, 6
  const f2 h01 = __builtin_amdgcn_cvt_pk_f32_fp8(hi, false);   // nibbles 1, 3
  const f2 h23 = __builtin_amdgcn_cvt_pk_f32_fp8(hi, true);    // nibbles 5, 7
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
  return make_uint4(pack_bf16x2(e0, e1), pack_bf16x2(e2, e3), pack_bf16x2(e4, e5),
                    pack_bf16x2(e6, e7));
}

// 8 fp16 values -> 8 bf16 (round-to-nearest-even), same order.
__device__ __forceinline__ uint4 half8_to_bf16(uint32_t __attribute__((ext_vector_type(4))) h) {
  typedef _Float16 h2 __attribute__((ext_vector_type(2)));
  const h2 p0 = __builtin_bit_cast(h2, (uint32_t)h.x), p1 = __builtin_bit_cast(h2, (uint32_t)h.y);
  const h2 p2 = __builtin_bit_cast(h2, (uint32_t)h.z), p3 = __builtin_bit_cast(h2, (uint32_t)h.w);
  return make_uint4(pack_bf16x2((float)p0.x, (float)p0.y), pack_bf16x2((float)p1.x, (float)p1.y),
                    pack_bf16x2((float)p2.x, (float)p2.y), pack_bf16x2((float)p3.x, (float)p3.y));
}

struct CeEpilogue {
  const int32_t* tok;
  float* part;
  float* tgt;
  uint32_t S, n_slices, tok_rows;
};

// NWN = wavefronts along N (2 along M): 4 -> 512 threads, each wavefront 128x64;
// 2 -> 256 threads (one wavefront per SIMD, twice the registers), each 128x128.
// QM = weight format: 0 int4 + per-group scales (perturbed in the weight tile), 1 plain bf16,
// 2 codebook (one 16-bit code per 8 weights into an fp16 [65536,8] codebook, gathered into the
// weight tile; the perturbed per-output-channel scale multiplies the accumulators).
// PIPE = how a k-tile's instructions are ordered: 0 left to the compiler, 1 one interleaved
// stream per wavefront with an explicit issue order, 2 alternating phases (see QZO_PP_TILE).
// ZP (int4 only) = asymmetric groups: a.zp holds one zero-point byte per (row, group).
template <int QM, bool CE, int NWN, int PIPE, bool ZP = false>
__global__ __launch_bounds__(128 * NWN, 1) void gemm_kernel(GemmArgs a, CeEpilogue ce) {
  static_assert(!ZP || QM == 0, "zero-points belong to the int4 format");
  constexpr bool W4 = QM == 0, CB = QM == 2, ROWMAP = W4 || CB;
  constexpr bool SCHED = PIPE == 1, PP = PIPE == 2;
  // PIPE == 3 (plain bf16 weights): both operand tiles go from memory straight into the LDS
  // (buffer loads with the lds modifier); no staging registers, no LDS store instructions
  constexpr bool DTL = PIPE == 3;
  static_assert(!DTL || QM == 1, "direct-to-LDS staging is written for plain bf16 weights");
  static_assert(!CB || NWN == 4, "codebook staging is written for 512 threads");
  static_assert(!PP || (NWN == 4 && W4), "the phase schedule is written for int4 weights, 512 threads");
  constexpr int THREADS = 128 * NWN;
  constexpr int TJ = 8 / NWN;                 // 32-wide feature tiles per wavefront
  constexpr int NA = 2048 / THREADS;          // 16-byte chunks of a 256x64 bf16 tile per thread
  constexpr int RSTEP = THREADS / 8;          // rows between a thread's consecutive chunks
  constexpr int TPR = THREADS / 256;          // W4: threads per weight row
  constexpr int NBQ = 2 / TPR;                // W4: 16-byte loads (32 nibbles) per thread
  constexpr int NBC = 4 * NBQ;                // W4: bf16 chunks written per thread
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  // Split-K (int4 and plain bf16 weights; a.ksplit > 1): a workgroup's unit of work is one K slice of an output tile,
  // a.kt_per k-tiles (a multiple of 4, so slices start on an even group) from k-tile kt0 on; its
  // fp32 accumulators go to a.split_ws[slice][M][N] and a second kernel adds the slices.
  constexpr bool SPLITK = (W4 || QM == 1) && !CE;
  const uint32_t ksplit = SPLITK ? max(a.ksplit, 1u) : 1u;
  const uint32_t real_tiles_n = (a.N + BN - 1) / BN;
  TileWalk walk = tile_walk_init(a.M, a.N, ksplit);
  uint32_t tile_m, tile_n, kslice = 0, kt0 = 0;
  if (!tile_walk_get(walk, tile_m, tile_n)) return;
  if (SPLITK && ksplit > 1) { kslice = tile_n / real_tiles_n; tile_n -= kslice * real_tiles_n; kt0 = kslice * a.kt_per; }
  const uint32_t tiles_m = walk.tiles_m;
  const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
  const uint32_t wm = wave / NWN, wn = wave % NWN;
  const uint32_t K = a.K;

  // ---- global -> register staging ---------------------------------------
  // Operands are read with buffer loads: base address and size sit in scalar
  // registers, a lane contributes a 32-bit byte offset fixed for the whole output
  // tile, and the k advance is a scalar offset.
  // A (and dense B): 2048 16-byte chunks per tile, 4 per thread; 8 consecutive
  // threads cover one 128-byte row segment.
  // W4: thread = (row t/2, half t%2): 16 bytes = 32 nibbles = 4 chunks.
  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(a.x), 0, (int)((uint64_t)a.M * K * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(a.w), 0,
      (int)(W4 ? (uint64_t)a.N * (K >> 1) : (CB ? (uint64_t)a.N * (K >> 2) : (uint64_t)a.N * K * 2)),
      0x00020000);
  const __amdgpu_buffer_rsrc_t rcb = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(CB ? a.cb : a.x), 0, CB ? (65536 * 16) : 16, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(W4 ? a.s : a.x), 0, (int)(W4 ? (uint64_t)a.N * (K >> 7) * 2 : 16), 0x00020000);
  const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<void*>(ZP ? a.zp : a.x), 0, (int)(ZP ? (uint64_t)a.N * (K >> 7) : 16), 0x00020000);
  // Direct-to-LDS: a wavefront's load instruction fills 1 KB of LDS in lane order (8 rows of
  // 128 bytes), so the XOR swizzle is applied on the memory side: the lane that fills position
  // p of row r fetches chunk p ^ swizzle(r).
  typedef int i32x4 __attribute__((ext_vector_type(4)));
  const i32x4 rx4 = {(int)(uint32_t)(uintptr_t)a.x, (int)(uint32_t)((uintptr_t)a.x >> 32),
                     (int)((uint64_t)a.M * K * 2), 0x00020000};
  const i32x4 rw4 = {(int)(uint32_t)(uintptr_t)a.w, (int)(uint32_t)((uintptr_t)a.w >> 32),
                     (int)((uint64_t)a.N * K * 2), 0x00020000};
  const uint32_t lds_wave = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)lds +
                            __builtin_amdgcn_readfirstlane(wave) * 1024u;
  uint32_t xo[NA], wo[NA], so = 0, gn_w4 = 0;
  float eps_tile = a.eps_signed;      // stacked passes: token tiles from row a.flip_row on take -eps
  const uint32_t brow = t / TPR, bpart = t % TPR;
  // LDS offsets: rows t/8 + RSTEP i share their swizzle, so chunk i is a_lds + i * RSTEP rows.
  const uint32_t a_lds = lds_off(t >> 3, t & 7u);
  uint32_t b_lds[ROWMAP ? NBC : 1];
  if (ROWMAP) {
#pragma unroll
    for (int c = 0; c < NBC; ++c) b_lds[c] = lds_off(brow, bpart * NBC + c);
  }
// Operand offsets of output tile (TM, TN).
#define QZO_TILE_PTRS(TM, TN)                                                                \
  do {                                                                                       \
    _Pragma("unroll") for (int i = 0; i < NA; ++i) {                                         \
      const uint32_t row = (t >> 3) + RSTEP * i;                                             \
      const uint32_t c = DTL ? ((t & 7u) ^ ((row >> 1) & 7u)) : (t & 7u);                    \
      xo[i] = (min((TM) * BM + row, a.M - 1) * K + c * 8) * 2;                               \
      if (!ROWMAP) wo[i] = (min((TN) * BN + row, a.N - 1) * K + c * 8) * 2;                  \
    }                                                                                        \
    eps_tile = (a.flip_row && (TM) * BM >= a.flip_row) ? -a.eps_signed : a.eps_signed;       \
    if (ROWMAP) {                                                                            \
      /* fused SwiGLU: the tile's rows are 4 x (32 gate rows, 32 up rows of the same   */      \
      /* features), so a lane's two accumulators hold gate and up of one feature      */      \
      gn_w4 = (a.epi & EPI_SWIGLU)                                                           \
                  ? ((brow >> 5) & 1u) * (a.N >> 1) + (TN) * 128u + (brow >> 6) * 32u + (brow & 31u) \
                  : min((TN) * BN + brow, a.N - 1);                                          \
      wo[0] = W4 ? gn_w4 * (K >> 1) + bpart * 16 : gn_w4 * (K >> 2) + bpart * 8;             \
      so = gn_w4 * (K >> 7) * 2;                                                             \
    }                                                                                        \
    if (SPLITK && kt0) { /* this slice's first k-tile: 128 B of activations, 32 B of nibbles, half a group */ \
      _Pragma("unroll") for (int i = 0; i < NA; ++i) xo[i] += kt0 * (BK * 2);                \
      if (W4) {                                                                              \
        wo[0] += kt0 * (BK / 2);                                                             \
        so += (kt0 >> 1) * 2;                                                                \
      } else {                                                                               \
        _Pragma("unroll") for (int i = 0; i < NA; ++i) wo[i] += kt0 * (BK * 2);              \
      }                                                                                      \
    }                                                                                        \
  } while (0)
  QZO_TILE_PTRS(tile_m, tile_n);

  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 ra[NA], rb[W4 ? NBQ : NA];
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  u32x4 rbp[2];                      // phase schedule: weight quads of the next two tiles
  u32x2 rq = {0, 0};                 // codebook: the four codes of the next weight chunk
  uint32_t zw[4] = {0, 0, 0, 0};     // Philox words of the current 8 groups
  float z_odd = 0.0f;                // second variate of the current pair
  float se512 = 0.0f, m8se = 0.0f;
  bf16_t s_next = 0;
  uint8_t z_next = 8;

  // LDS: A stage 0 | A stage 1 | B stage 0 | B stage 1, 32 KB each.  The k-loop is
  // unrolled by two so the stage is a compile-time constant and every LDS address is
  // a loop-invariant register plus an immediate offset.
  unsigned char* const lds_a = lds;
  unsigned char* const lds_b = lds + 2 * TILE_BYTES;

// Loads of k-tile KT into registers (KT is clamped by the caller, so the loads
// are unconditional and are issued a whole k-tile ahead of their use).
#define QZO_CODES(KT) rq = __builtin_amdgcn_raw_buffer_load_b64(rw, (int)wo[0], (int)((KT) * 16), 0)
#define QZO_GLOAD_A(KT)                                                                      \
  do {                                                                                       \
    _Pragma("unroll") for (int i = 0; i < NA; ++i)                                           \
        ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)xo[i], (int)((KT) * (BK * 2)), 0); \
  } while (0)
#define QZO_GLOAD_B(KT)                                                                      \
  do {                                                                                       \
    if (W4) {                                                                                \
      _Pragma("unroll") for (int q = 0; q < NBQ; ++q) rb[q] = __builtin_amdgcn_raw_buffer_load_b128( \
          rw, (int)wo[0] + q * 16, (int)((KT) * (BK / 2)), 0);                               \
    } else if (CB) { /* gather the 8-vectors of the codes read one tile earlier */           \
      rb[0] = __builtin_amdgcn_raw_buffer_load_b128(rcb, (int)((rq.x & 0xffffu) << 4), 0, 0); \
      rb[1] = __builtin_amdgcn_raw_buffer_load_b128(rcb, (int)((rq.x >> 16) << 4), 0, 0);    \
      rb[2] = __builtin_amdgcn_raw_buffer_load_b128(rcb, (int)((rq.y & 0xffffu) << 4), 0, 0); \
      rb[3] = __builtin_amdgcn_raw_buffer_load_b128(rcb, (int)((rq.y >> 16) << 4), 0, 0);    \
      QZO_CODES(min((uint32_t)(KT) + 1u, (K / BK) - 1u));                                    \
    } else {                                                                                 \
      _Pragma("unroll") for (int i = 0; i < NA; ++i)                                         \
          rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rw, (int)wo[i], (int)((KT) * (BK * 2)), 0); \
    }                                                                                        \
  } while (0)
#define QZO_GLOAD(KT)                                                                        \
  do {                                                                                       \
    if (CB) {                                                                                \
      QZO_GLOAD_B(KT);                                                                       \
      QZO_GLOAD_A(KT);                                                                       \
    } else {                                                                                 \
      QZO_GLOAD_A(KT);                                                                       \
      QZO_GLOAD_B(KT);                                                                       \
    }                                                                                        \
  } while (0)

// Direct-to-LDS: k-tile KT of both operands into LDS stage STAGE.  M0 carries the LDS address of
// the wavefront's 1 KB; the hardware adds 16 bytes per lane.  The compiler does not see these
// LDS writes: every read of the stage is separated from them by an explicit vmcnt(0) and a barrier.
#define QZO_DTL16(RSRC, LDSADDR, VOFF, SOFF)                                                 \
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"                \
               : : "s"(LDSADDR), "v"(VOFF), "s"(RSRC), "s"(SOFF) : "memory", "m0")
#define QZO_DTL_PART(KT, STAGE, I0, I1)                                                      \
  do {                                                                                       \
    const uint32_t so_ = (uint32_t)(KT) * (BK * 2);                                          \
    _Pragma("unroll") for (int i = (I0); i < (I1); ++i) {                                    \
      QZO_DTL16(rx4, lds_wave + (uint32_t)((STAGE) * TILE_BYTES + i * RSTEP * 128), xo[i], so_); \
      QZO_DTL16(rw4, lds_wave + (uint32_t)((2 + (STAGE)) * TILE_BYTES + i * RSTEP * 128), wo[i], so_); \
    }                                                                                        \
  } while (0)
#define QZO_DTL(KT, STAGE) QZO_DTL_PART(KT, STAGE, 0, NA)
#define QZO_DTL_LANDED()                                                                     \
  do {                                                                                       \
    __builtin_amdgcn_s_waitcnt(0x0F70); /* vmcnt(0) */                                       \
    __syncthreads();                                                                         \
  } while (0)

// New perturbed scale for group G_ (every two k-tiles): s + (sigma*eps)*z as one
// fp32 fma.  One Philox counter (row, G_/8) serves 8 groups; its four words are
// kept and each word's Box-Muller pair is evaluated when its even group starts.
// The stored scale itself was requested a tile earlier (QZO_SCALE_PREFETCH), ahead
// of that tile's operand loads: memory returns in order, so a scale requested here
// would make the wavefront wait for every operand load issued before it.
#define QZO_SCALE_PREFETCH(G_)                                                               \
  do {                                                                                       \
    const uint32_t gp_ = min((uint32_t)(G_), (nkt >> 1) - 1u);                               \
    s_next = (bf16_t)__builtin_amdgcn_raw_buffer_load_b16(rs, (int)so, (int)(gp_ * 2u), 0);  \
    if (ZP) z_next = __builtin_amdgcn_raw_buffer_load_b8(rz, (int)(so >> 1), (int)gp_, 0);   \
  } while (0)
#define QZO_NEW_GROUP(G_)                                                                    \
  do {                                                                                       \
    const uint32_t g_ = (G_) + (kt0 >> 1);      /* group index within the row */             \
    if ((g_ & 7u) == 0u || (G_) == 0u) {        /* a slice may start inside a counter */     \
      const u32x4_t pw_ = philox4x32_10(a.row_base + gn_w4, g_ >> 3, 0u, 0u, a.seed_lo, a.seed_hi); \
      zw[0] = pw_.x; zw[1] = pw_.y; zw[2] = pw_.z; zw[3] = pw_.w;                            \
    }                                                                                        \
    float zz_ = z_odd;                                                                       \
    if ((g_ & 1u) == 0u) {                                                                   \
      const uint32_t p_ = (g_ & 7u) >> 1;                                                    \
      const uint32_t w_ = p_ == 0 ? zw[0] : (p_ == 1 ? zw[1] : (p_ == 2 ? zw[2] : zw[3]));   \
      normal_pair(w_, zz_, z_odd);                                                           \
    }                                                                                        \
    const float se_ = __builtin_fmaf(eps_tile, zz_, scale_to_f32(s_next, a.s_fp16 != 0));    \
    se512 = ZP ? se_ : 512.0f * se_;                  /* ZP: the scale itself          */    \
    m8se = ZP ? -(float)z_next : -8.0f * se_;         /* ZP: the negated zero-point    */    \
  } while (0)

// Registers -> LDS stage STAGE (compile-time); the int4 tile is unpacked, scaled
// by the perturbed scale and rounded to bf16 on the way.
#define QZO_LSTORE_A(STAGE)                                                                  \
  do {                                                                                       \
    _Pragma("unroll") for (int i = 0; i < NA; ++i) *reinterpret_cast<u32x4*>(                \
        lds_a + a_lds + (i * RSTEP * 128 + (STAGE) * TILE_BYTES)) = ra[i];                   \
  } while (0)
#define QZO_LSTORE_B(STAGE)                                                                  \
  do {                                                                                       \
    if (W4) {                                                                                \
      _Pragma("unroll") for (int q = 0; q < NBQ; ++q) {                                      \
        *reinterpret_cast<uint4*>(lds_b + b_lds[4 * q + 0] + (STAGE) * TILE_BYTES) = dequant8<ZP>(rb[q].x, se512, m8se); \
        *reinterpret_cast<uint4*>(lds_b + b_lds[4 * q + 1] + (STAGE) * TILE_BYTES) = dequant8<ZP>(rb[q].y, se512, m8se); \
        *reinterpret_cast<uint4*>(lds_b + b_lds[4 * q + 2] + (STAGE) * TILE_BYTES) = dequant8<ZP>(rb[q].z, se512, m8se); \
        *reinterpret_cast<uint4*>(lds_b + b_lds[4 * q + 3] + (STAGE) * TILE_BYTES) = dequant8<ZP>(rb[q].w, se512, m8se); \
      }                                                                                      \
    } else if (CB) {                                                                         \
      _Pragma("unroll") for (int q = 0; q < 4; ++q) *reinterpret_cast<uint4*>(               \
          lds_b + b_lds[q] + (STAGE) * TILE_BYTES) = half8_to_bf16(rb[q]);                   \
    } else {                                                                                 \
      _Pragma("unroll") for (int i = 0; i < NA; ++i) *reinterpret_cast<u32x4*>(              \
          lds_b + a_lds + (i * RSTEP * 128 + (STAGE) * TILE_BYTES)) = rb[i];                 \
    }                                                                                        \
  } while (0)
#define QZO_LSTORE(STAGE)                                                                    \
  do {                                                                                       \
    QZO_LSTORE_A(STAGE);                                                                     \
    QZO_LSTORE_B(STAGE);                                                                     \
  } while (0)

  // acc[i][j]: output features 32 j .. 32 j + 31 (rows of the MFMA result) by
  // tokens 32 i .. 32 i + 31 (columns) of the wavefront's sub-tile.
  floatx16 acc[4][TJ];
  // Direct-to-LDS plain kernel: the output stores are buffer stores that every lane issues (a lane
  // outside the matrix gets an offset beyond the buffer, which drops the store), so the number of
  // memory instructions a wavefront issues behind the next tile's first loads is known, and the
  // wait for those loads at the top of the next k-loop can leave that many instructions, the
  // stores, in flight: vmcnt counts in issue order.  Waiting for the stores as well would expose
  // the time the memory system needs to take in 128 KB from every CU at once.
  constexpr bool TRAIL = DTL && !CE && TJ == 2;
  uint32_t trail_stores = 0;                       // stores issued by the last epilogue: 0, 8 or 16
  const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(
      a.y, 0, (int)(a.ldy ? ((uint64_t)(a.M - 1) * a.ldy + a.N) * 2
                          : (uint64_t)a.M * ((a.epi & EPI_SWIGLU) ? (a.N >> 1) : a.N) * 2), 0x00020000);
  const uint32_t ldy = a.ldy ? a.ldy : a.N;        // row stride of y and resid (plain epilogue)
  const uint32_t frow = lane & 31u, fhalf = lane >> 5;
  // fragment addresses: row base + swizzled chunk of k-step ks (chunk 2 ks + half);
  // row tiles i / j and the stage are immediate offsets.
  const uint32_t fsw = (frow >> 1) & 7u;
  uint32_t fa_k[4], fb_k[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const uint32_t co = ((uint32_t)(ks * 2 + fhalf) ^ fsw) << 4;
    fa_k[ks] = (wm * 128 + frow) * 128u + co;
    fb_k[ks] = (wn * (32 * TJ) + frow) * 128u + co;
  }

  // Fragment sets alternate between two register buffers.  The MFMAs of a tile's
  // last k-step are issued only after the next barrier, behind the first fragment
  // reads of the following tile, so the matrix pipe stays fed across the barrier.
  bf16x8 fa_[2][4], fb_[2][TJ];
#define QZO_FRAGS(BUF, KS, STAGE)                                                            \
  do {                                                                                       \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) fa_[BUF][i] = *reinterpret_cast<const bf16x8*>( \
        lds_a + fa_k[KS] + (i * 32 * 128 + (STAGE) * TILE_BYTES));                           \
    _Pragma("unroll") for (int j = 0; j < TJ; ++j) fb_[BUF][j] = *reinterpret_cast<const bf16x8*>( \
        lds_b + fb_k[KS] + (j * 32 * 128 + (STAGE) * TILE_BYTES));                           \
  } while (0)
#define QZO_MFMAS(BUF)                                                                       \
  do {                                                                                       \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                            \
        _Pragma("unroll") for (int j = 0; j < TJ; ++j) acc[i][j] =                           \
            __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb_[BUF][j], fa_[BUF][i], acc[i][j], 0, 0, 0); \
  } while (0)
// One k-tile.  Source order: the four fragment loads, each a k-step ahead of the
// MFMAs that use it; the MFMAs; the conversion and LDS stores of the next tile;
// the global loads of the tile after that.  QZO_SCHED then fixes the issue order
// inside the block: every MFMA is followed by a few conversion VALU operations,
// the LDS stores are spread over the first three k-steps (they are several times
// slower than LDS loads, the LDS executes in order and the barrier must wait for
// them, so they may neither bunch up in front of the fragment loads nor sit at
// the end), and the global loads go behind the last k-step's MFMAs.
#define QZO_TILE(STAGE, HOLD, STORE_STAGE, NEXT_KT, PREF_G)                                  \
  do {                                                                                       \
    QZO_FRAGS(0, 0, STAGE);                                                                  \
    if (HOLD) QZO_MFMAS(1); /* k-step 3 of the previous tile */                              \
    QZO_FRAGS(1, 1, STAGE);                                                                  \
    QZO_MFMAS(0);                                                                            \
    QZO_FRAGS(0, 2, STAGE);                                                                  \
    QZO_MFMAS(1);                                                                            \
    QZO_FRAGS(1, 3, STAGE);                                                                  \
    if ((STORE_STAGE) >= 0) {                                                                \
      QZO_LSTORE((STORE_STAGE) & 1);                                                         \
      if (W4 && (int)(PREF_G) >= 0) QZO_SCALE_PREFETCH(PREF_G);                              \
      QZO_GLOAD(NEXT_KT);                                                                    \
    }                                                                                        \
    QZO_MFMAS(0);                                                                            \
    if (SCHED) {                                                                             \
      constexpr int MPK = 4 * TJ, RPK = 4 + TJ;                                              \
      __builtin_amdgcn_sched_group_barrier(0x100, RPK, 0);                                   \
      _Pragma("unroll") for (int g_ = (HOLD) ? 0 : 1; g_ < 3; ++g_) {                        \
        _Pragma("unroll") for (int m_ = 0; m_ < MPK; ++m_) {                                 \
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                 \
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);                                 \
          if ((g_ * MPK + m_) % 3 == 2) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   \
        }                                                                                    \
        __builtin_amdgcn_sched_group_barrier(0x100, RPK, 0);                                 \
      }                                                                                      \
      _Pragma("unroll") for (int m_ = 0; m_ < MPK; ++m_) {                                   \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                   \
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                   \
      }                                                                                      \
    }                                                                                        \
  } while (0)

// One k-tile with direct-to-LDS staging: fragments and MFMAs as above.  The other stage was
// read last in the tile before this one (every wavefront is past that tile's closing barrier),
// so it is refilled with tile LOAD_KT, the one after this (< 0: nothing left to load), while
// this tile computes: half of the loads before the first MFMA group and half before the second
// (a little faster than all eight at once; spreading them further leaves the last ones too
// little time to land).  The tile closes once those loads have landed in every wavefront.
#define QZO_TILE_D(STAGE, HOLD, LOAD_KT)                                                     \
  do {                                                                                       \
    /* the fences keep the source order: each k-step's fragment reads are issued before the */ \
    /* MFMAs of the k-step before it (the compiler would otherwise sink them to their use)  */ \
    QZO_FRAGS(0, 0, STAGE);                                                                  \
    if ((int)(LOAD_KT) >= 0) QZO_DTL_PART(LOAD_KT, 1 - (STAGE), 0, NA / 2);                  \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    if (HOLD) QZO_MFMAS(1);                                                                  \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    QZO_FRAGS(1, 1, STAGE);                                                                  \
    if ((int)(LOAD_KT) >= 0) QZO_DTL_PART(LOAD_KT, 1 - (STAGE), NA / 2, NA);                 \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    QZO_MFMAS(0);                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    QZO_FRAGS(0, 2, STAGE);                                                                  \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    QZO_MFMAS(1);                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    QZO_FRAGS(1, 3, STAGE);                                                                  \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    QZO_MFMAS(0);                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    QZO_DTL_LANDED();                                                                        \
  } while (0)

// Phase schedule (int4 weights).  Wavefronts w and w + 4 share a SIMD.  A k-tile is cut
// into two halves of two k-steps; for each half a wavefront runs a memory phase and then a
// matrix phase of sixteen MFMAs whose operands are all in registers.  Phases are separated
// by workgroup barriers and wavefronts 4..7 run one phase behind wavefronts 0..3, so on
// every SIMD one wavefront feeds the matrix pipe while the other uses the LDS and the
// vector ALU.  With t the current tile (LDS stage t & 1):
//   memory A: 12 fragment reads (k-steps 0,1); while they are served, convert dwords 0,1
//             of tile t+1's weight quad; store them and activation chunks 0,1 of tile t+1
//   matrix A: 16 MFMAs; request activation chunks 0,1 of tile t+2 (and a scale)
//   memory B: 12 fragment reads (k-steps 2,3); convert and store dwords 2,3 and chunks
//             2,3 of tile t+1; then, before an even tile t+2, the scale of its group
//   matrix B: 16 MFMAs; request chunks 2,3 of tile t+2 and the weight quad of tile t+3
// Stage hazards: tile t+1 is written to the other stage during tile t's first three
// phases, after the barrier that ends the last fragment read of tile t-1 and before the
// barrier that precedes the first read of tile t+1 by the other half of the wavefronts.
#define QZO_PHASE_SYNC()                                                                     \
  do {                                                                                       \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    __syncthreads();                                                                         \
    __builtin_amdgcn_sched_barrier(0);                                                       \
  } while (0)
#define QZO_PP_LOAD_B(KT, PAR)                                                               \
  rbp[PAR] = __builtin_amdgcn_raw_buffer_load_b128(rw, (int)wo[0], (int)((KT) * (BK / 2)), 0)
#define QZO_PP_LOAD_A(KT, I0)                                                                \
  do {                                                                                       \
    ra[I0] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)xo[I0], (int)((KT) * (BK * 2)), 0); \
    ra[(I0) + 1] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)xo[(I0) + 1], (int)((KT) * (BK * 2)), 0); \
  } while (0)
/* half H (0, 1) of the staging of one tile: two weight dwords and two activation chunks */ \

#define QZO_PP_STAGE_HALF(PAR, STAGE, H)                                                     \
  do {                                                                                       \
    const uint4 c0_ = dequant8<ZP>((H) ? rbp[PAR].z : rbp[PAR].x, se512, m8se);                  \
    const uint4 c1_ = dequant8<ZP>((H) ? rbp[PAR].w : rbp[PAR].y, se512, m8se);                  \
    *reinterpret_cast<uint4*>(lds_b + b_lds[2 * (H)] + (STAGE) * TILE_BYTES) = c0_;          \
    *reinterpret_cast<uint4*>(lds_b + b_lds[2 * (H) + 1] + (STAGE) * TILE_BYTES) = c1_;      \
    *reinterpret_cast<u32x4*>(lds_a + a_lds + ((2 * (H)) * RSTEP * 128 + (STAGE) * TILE_BYTES)) = ra[2 * (H)]; \
    *reinterpret_cast<u32x4*>(lds_a + a_lds + ((2 * (H) + 1) * RSTEP * 128 + (STAGE) * TILE_BYTES)) = ra[2 * (H) + 1]; \
  } while (0)
#define QZO_PP_MFMAS()                                                                       \
  do {                                                                                       \
    QZO_MFMAS(0);                                                                            \
    QZO_MFMAS(1);                                                                            \
  } while (0)
#define QZO_PP_TILE(STAGE, STORE_STAGE, NEXT_KT, NEXT_B_KT, NEW_G, PREF_G)                   \
  do {                                                                                       \
    QZO_FRAGS(0, 0, STAGE);                                                                  \
    QZO_FRAGS(1, 1, STAGE);                                                                  \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    if ((STORE_STAGE) >= 0) QZO_PP_STAGE_HALF((STORE_STAGE) & 1, (STORE_STAGE) & 1, 0);      \
    QZO_PHASE_SYNC();                                                                        \
    __builtin_amdgcn_s_setprio(1);                                                           \
    QZO_PP_MFMAS();                                                                          \
    if ((STORE_STAGE) >= 0) {                                                                \
      if ((int)(PREF_G) >= 0) QZO_SCALE_PREFETCH(PREF_G);                                    \
      QZO_PP_LOAD_A(NEXT_KT, 0);                                                             \
    }                                                                                        \
    __builtin_amdgcn_s_setprio(0);                                                           \
    QZO_PHASE_SYNC();                                                                        \
    QZO_FRAGS(0, 2, STAGE);                                                                  \
    QZO_FRAGS(1, 3, STAGE);                                                                  \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    if ((STORE_STAGE) >= 0) {                                                                \
      QZO_PP_STAGE_HALF((STORE_STAGE) & 1, (STORE_STAGE) & 1, 1);                            \
      if ((int)(NEW_G) >= 0) QZO_NEW_GROUP((uint32_t)(NEW_G));                               \
    }                                                                                        \
    QZO_PHASE_SYNC();                                                                        \
    __builtin_amdgcn_s_setprio(1);                                                           \
    QZO_PP_MFMAS();                                                                          \
    if ((STORE_STAGE) >= 0) {                                                                \
      QZO_PP_LOAD_A(NEXT_KT, 2);                                                             \
      QZO_PP_LOAD_B(NEXT_B_KT, (STORE_STAGE) & 1);                                           \
    }                                                                                        \
    __builtin_amdgcn_s_setprio(0);                                                           \
    QZO_PHASE_SYNC();                                                                        \
  } while (0)
  const bool late_group = PP && __builtin_amdgcn_readfirstlane(wave) >= 4u;

  // K is a multiple of 128, so the number of k-tiles is even.  Tile kt lives in
  // LDS stage kt & 1; during tile kt the registers loaded one tile earlier (tile
  // kt+1) go to the other stage and tile kt+2 is requested from memory.
  uint32_t nkt = (SPLITK && ksplit > 1) ? min(a.kt_per, K / BK - kt0) : K / BK, last = nkt - 1;
  if (CB) QZO_CODES(0u);
  if (PP) {
    QZO_GLOAD_A(0);
    QZO_PP_LOAD_B(0u, 0);
  } else if (DTL) {
    QZO_DTL(0u, 0);
    QZO_DTL(1u, 1);
  } else {
    QZO_GLOAD(0);
  }
  for (;;) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
  if (W4) {
    QZO_SCALE_PREFETCH(0u);
    QZO_NEW_GROUP(0u);
    QZO_SCALE_PREFETCH(1u);
  }
  if (PP) {
    QZO_PP_STAGE_HALF(0, 0, 0);
    QZO_PP_STAGE_HALF(0, 0, 1);
    QZO_GLOAD_A(1u);
    QZO_PP_LOAD_B(1u, 1);
    QZO_PP_LOAD_B(min(2u, last), 0);
  } else if (!DTL) {
    QZO_LSTORE(0);
    QZO_GLOAD(1u);
  }
  if (TRAIL && trail_stores == 16) {
    __builtin_amdgcn_s_waitcnt(0x4F70);   /* vmcnt(16) */
    __syncthreads();
  } else if (TRAIL && trail_stores == 8) {
    __builtin_amdgcn_s_waitcnt(0x0F78);   /* vmcnt(8) */
    __syncthreads();
  } else if (DTL) {
    QZO_DTL_LANDED();
  } else {
    __syncthreads();
  }
  if (PP) {
    if (late_group) QZO_PHASE_SYNC();
    /* tile t stores tile t+1, requests activations of t+2 and weights of t+3; an even   */
    /* tile ends its staging with the scale of the group that tile t+2 starts            */
    QZO_PP_TILE(0, 1, min(2u, last), min(3u, last), 1, -1);
    for (uint32_t kt = 1; kt + 1 < nkt; kt += 2) {
      QZO_PP_TILE(1, 0, min(kt + 2, last), min(kt + 3, last), -1, (kt + 3) >> 1);
      QZO_PP_TILE(0, 1, min(kt + 3, last), min(kt + 4, last), (kt + 3) >> 1, -1);
    }
    QZO_PP_TILE(1, -1, 0u, 0u, -1, -1);
    if (!late_group) QZO_PHASE_SYNC();
  } else if (DTL) {
    QZO_TILE_D(0, false, -1);                 /* tiles 0 and 1 were requested ahead of the loop */
    for (uint32_t kt = 1; kt + 1 < nkt; kt += 2) {
      QZO_TILE_D(1, true, (int)(kt + 1));
      QZO_TILE_D(0, true, kt + 2 <= last ? (int)(kt + 2) : -1);
    }
    QZO_TILE_D(1, true, -1);
    QZO_MFMAS(1);
  } else {
  QZO_TILE(0, false, 1, min(2u, last), -1);
  __syncthreads();
  for (uint32_t kt = 1; kt + 1 < nkt; kt += 2) {
    if (W4) QZO_NEW_GROUP((kt + 1) >> 1);
    QZO_TILE(1, true, 0, min(kt + 2, last), -1);
    __syncthreads();
    QZO_TILE(0, true, 1, min(kt + 3, last), (kt + 3) >> 1);
    __syncthreads();
  }
  QZO_TILE(1, true, -1, 0u, -1);
  QZO_MFMAS(1);
  }

  // The next tile's first loads are requested before this tile's results are
  // written, and the stores are not waited for: the epilogue's memory traffic
  // overlaps the next tile's main loop.
  const uint32_t m0 = tile_m * BM, n0 = tile_n * BN;
  const uint32_t done_m = tile_m, done_n = tile_n, done_slice = kslice;
  walk.slot += walk.stride;
  const bool more = tile_walk_get(walk, tile_m, tile_n);
  if (more) {
    if (SPLITK && ksplit > 1) {
      kslice = tile_n / real_tiles_n;
      tile_n -= kslice * real_tiles_n;
      kt0 = kslice * a.kt_per;
      nkt = min(a.kt_per, K / BK - kt0);
      last = nkt - 1;
    }
    QZO_TILE_PTRS(tile_m, tile_n);
    if (CB) QZO_CODES(0u);
    if (PP) {
      QZO_GLOAD_A(0);
      QZO_PP_LOAD_B(0u, 0);
    } else if (DTL) {       /* every wavefront is past the barrier that ends the last k-tile */
      QZO_DTL(0u, 0);
      QZO_DTL(1u, 1);
    } else {
      QZO_GLOAD(0);
    }
  }

  // ---- epilogue ----------------------------------------------------------
  // acc[i][j][4 b + c]: token m = 32 i + lane%32, feature n = 32 j + 8 b + 4 (lane/32) + c
  // of the wavefront's 128 (tokens) x 64 (features) sub-tile.
  const uint32_t n_wave = n0 + wn * (32 * TJ) + 4 * fhalf;
  // codebook: perturbed per-output-channel scales of the tile's 256 rows,
  // c + (sigma*eps) z(row id) as one fp32 fma, staged in LDS behind the tiles
  float* const lds_c = reinterpret_cast<float*>(lds + LDS_BYTES);
  if (CB) {
    if (t < 256u) {
      const uint32_t gn = (a.epi & EPI_SWIGLU)
                              ? ((t >> 5) & 1u) * (a.N >> 1) + done_n * 128u + (t >> 6) * 32u + (t & 31u)
                              : min(n0 + t, a.N - 1);
      const float c0 = (float)reinterpret_cast<const _Float16*>(a.s)[gn];
      lds_c[t] = __builtin_fmaf(a.eps_signed, flat_normal(a.seed_lo, a.seed_hi, 1u, a.row_base + gn), c0);
    }
    __syncthreads();
  }
  // A lane holds 4 consecutive features per register group and the lane 32 away the next 4.
  // Groups b and b+1 are exchanged between the two halves of the wavefront
  // (v_permlane32_swap), after which lanes 0..31 own features 8b..8b+7 and lanes 32..63
  // features 8(b+1)..8(b+1)+7 of their token: every access of the epilogue is 16 bytes.
#define QZO_STORE_OUT(PTR, V) (*reinterpret_cast<uint4*>(PTR) = (V))
// Default cache policy on purpose: non-temporal stores keep the output out of the L2 and are
// 20 % faster in a loop of this structure on synthetic addresses, but the whole step gets 1.8 %
// slower with them.
#define QZO_STORE_OUT_ALWAYS(BYTE_OFF, V)                                                    \
  __builtin_amdgcn_raw_buffer_store_b128(u32x4{(V).x, (V).y, (V).z, (V).w}, ry, (int)(BYTE_OFF), 0, 0)
#define QZO_SWAP8(LO, HI)                                                                    \
  do {                                                                                       \
    _Pragma("unroll") for (int c_ = 0; c_ < 4; ++c_) {                                       \
      const auto r_ = __builtin_amdgcn_permlane32_swap(__float_as_uint((LO)[c_]),            \
                                                       __float_as_uint((HI)[c_]), false, false); \
      (LO)[c_] = __uint_as_float(r_[0]);                                                     \
      (HI)[c_] = __uint_as_float(r_[1]);                                                     \
    }                                                                                        \
  } while (0)
  if (SPLITK && ksplit > 1) {
    trail_stores = 0;
    // split-K: this slice's fp32 sums, [slice][M][N]; the epilogue proper runs in the reduction
    float* part = a.split_ws + (uint64_t)done_slice * a.M * a.N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t m = m0 + wm * 128 + i * 32 + frow;
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int bp = 0; bp < 2; ++bp) {
          float v[2][4];
#pragma unroll
          for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int c = 0; c < 4; ++c) v[h][c] = acc[i][j][4 * (2 * bp + h) + c];
          QZO_SWAP8(v[0], v[1]);
          const uint32_t n = n0 + wn * (32 * TJ) + j * 32 + (2u * bp + fhalf) * 8u;
          if (m < a.M && n < a.N) {
            float4* dst = reinterpret_cast<float4*>(part + (uint64_t)m * a.N + n);
            dst[0] = make_float4(v[0][0], v[0][1], v[0][2], v[0][3]);
            dst[1] = make_float4(v[1][0], v[1][1], v[1][2], v[1][3]);
          }
        }
    }
  } else if (!CE && TJ == 2 && (a.epi & EPI_SWIGLU)) {
    // y[m, f] = silu(gate) * up, f = 128 tile_n + 32 wn + 8 b + 4 (lane/32) + c; y is [M, N/2]
    bf16_t* y = (bf16_t*)a.y;
    const uint32_t F = a.N >> 1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t m = m0 + wm * 128 + i * 32 + frow;
#pragma unroll
      for (int bp = 0; bp < 2; ++bp) {
        float v[2][4];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int b = 2 * bp + h;
            float g = acc[i][0][4 * b + c], up = acc[i][TJ - 1][4 * b + c];
            if (CB) {
              g *= lds_c[wn * 64 + b * 8 + 4 * fhalf + c];
              up *= lds_c[wn * 64 + 32 + b * 8 + 4 * fhalf + c];
            }
            v[h][c] = g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504f * g)) * up;
          }
        QZO_SWAP8(v[0], v[1]);
        const uint32_t f = done_n * 128u + wn * 32u + (2u * bp + fhalf) * 8u;
        uint4 out;
        out.x = pack_bf16x2(v[0][0], v[0][1]); out.y = pack_bf16x2(v[0][2], v[0][3]);
        out.z = pack_bf16x2(v[1][0], v[1][1]); out.w = pack_bf16x2(v[1][2], v[1][3]);
        if (TRAIL) QZO_STORE_OUT_ALWAYS(m < a.M ? (m * F + f) * 2u : 0x80000000u, out);
        else if (m < a.M) QZO_STORE_OUT(y + (uint64_t)m * F + f, out);
      }
    }
    trail_stores = TRAIL ? 8 : 0;
  } else if (!CE && TJ == 2 && !W4 && !CB && (a.epi & EPI_ROPE)) {
    // qkv [M, 3d] with the rotary embedding on its q and k thirds.  The wavefront's two 32-wide
    // feature tiles hold feature i and feature i + dh/2 of a head for the same token (heads of 64:
    // the natural order; heads of 128: the rows of W were written in ROW_ORDER_ROPE128), so a lane
    // rotates its own pairs: each output is first rounded to bf16 (the value a separate RoPE pass
    // would read), then (a cos - b sin, b cos + a sin) in fp32 at position m % rope_S, rounded again.
    const uint32_t half = a.rope_dh >> 1, d2 = (a.N / 3u) * 2u;
    const float2* table = reinterpret_cast<const float2*>(a.rope);
    // step u = 2 i + bp handles token 32 i + frow and the lane's 8 features (2 bp + fhalf) * 8 .. + 7 of the
    // first tile with their partners in the second; the (cos, sin) values of step u + 1 are requested
    // before step u is worked on, so that one memory latency is exposed per output tile, not eight
    const uint32_t na_base = half == 64u ? n0 + (wn >> 1) * 128u + (wn & 1u) * 32u : n0 + wn * 64u;
    const uint32_t idx_base = half == 64u ? (wn & 1u) * 32u : 0u;
    const bool rotate = na_base < d2;            // a wavefront's 64 columns lie within one third of qkv
    auto tb_of = [&](int u) {
      const uint32_t m = m0 + wm * 128 + (u >> 1) * 32 + frow;
      const uint32_t pos = min(m, a.M - 1) % a.rope_S;
      return reinterpret_cast<const float4*>(table + (uint64_t)pos * half + idx_base + (2u * (u & 1) + fhalf) * 8u);
    };
    float4 tn[4] = {};
    if (rotate) {
#pragma unroll
      for (int j = 0; j < 4; ++j) tn[j] = tb_of(0)[j];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = u >> 1, bp = u & 1;
      const uint32_t m = m0 + wm * 128 + i * 32 + frow;
      float4 t[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) t[j] = tn[j];
      if (rotate && u < 7) {
#pragma unroll
        for (int j = 0; j < 4; ++j) tn[j] = tb_of(u + 1)[j];
      }
      float va[2][4], vb[2][4];
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          va[h][c] = acc[i][0][4 * (2 * bp + h) + c];
          vb[h][c] = acc[i][1][4 * (2 * bp + h) + c];
        }
      QZO_SWAP8(va[0], va[1]);
      QZO_SWAP8(vb[0], vb[1]);
      const uint32_t na = na_base + (2u * bp + fhalf) * 8u;
      uint32_t oa[4], ob[4];
      oa[0] = pack_bf16x2(va[0][0], va[0][1]); oa[1] = pack_bf16x2(va[0][2], va[0][3]);
      oa[2] = pack_bf16x2(va[1][0], va[1][1]); oa[3] = pack_bf16x2(va[1][2], va[1][3]);
      ob[0] = pack_bf16x2(vb[0][0], vb[0][1]); ob[1] = pack_bf16x2(vb[0][2], vb[0][3]);
      ob[2] = pack_bf16x2(vb[1][0], vb[1][1]); ob[3] = pack_bf16x2(vb[1][2], vb[1][3]);
      if (rotate) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {                  // t[j]: (cos, sin) of pairs 2 j and 2 j + 1
          const float a0 = __uint_as_float(oa[j] << 16), a1 = __uint_as_float(oa[j] & 0xffff0000u);
          const float b0 = __uint_as_float(ob[j] << 16), b1 = __uint_as_float(ob[j] & 0xffff0000u);
          oa[j] = pack_bf16x2(a0 * t[j].x - b0 * t[j].y, a1 * t[j].z - b1 * t[j].w);
          ob[j] = pack_bf16x2(b0 * t[j].x + a0 * t[j].y, b1 * t[j].z + a1 * t[j].w);
        }
      }
      const bool inside = m < a.M && na < a.N;
      const uint32_t o = (m * a.N + na) * 2u;
      const uint4 outa = {oa[0], oa[1], oa[2], oa[3]}, outb = {ob[0], ob[1], ob[2], ob[3]};
      if (TRAIL) {
        QZO_STORE_OUT_ALWAYS(inside ? o : 0x80000000u, outa);
        QZO_STORE_OUT_ALWAYS(inside ? o + half * 2u : 0x80000000u, outb);
      } else if (inside) {
        QZO_STORE_OUT((bf16_t*)a.y + (uint64_t)m * a.N + na, outa);
        QZO_STORE_OUT((bf16_t*)a.y + (uint64_t)m * a.N + na + half, outb);
      }
    }
    trail_stores = TRAIL ? 16 : 0;
  } else if (!CE) {
    float ssq = 0.0f;
    const bf16_t* bias = (const bf16_t*)a.bias;
    const bf16_t* resid = (const bf16_t*)a.resid;
    bf16_t* y = (bf16_t*)a.y;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t m = m0 + wm * 128 + i * 32 + frow;
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int bp = 0; bp < 2; ++bp) {
          float v[2][4];
#pragma unroll
          for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              v[h][c] = acc[i][j][4 * (2 * bp + h) + c];
              if (CB) v[h][c] *= lds_c[wn * (32 * TJ) + j * 32 + (2 * bp + h) * 8 + 4 * fhalf + c];
            }
          QZO_SWAP8(v[0], v[1]);
          // 8 features n .. n+7 (N % 8 == 0)
          const uint32_t n = n0 + wn * (32 * TJ) + j * 32 + (2u * bp + fhalf) * 8u;
          const bool inside = m < a.M && n < a.N;
          uint4 out = {0u, 0u, 0u, 0u};
          const uint64_t o = (uint64_t)m * ldy + n;
          if (inside) {
            if (a.epi & EPI_BIAS) {
              const uint4 bb = *reinterpret_cast<const uint4*>(bias + n);
              v[0][0] += __uint_as_float(bb.x << 16); v[0][1] += __uint_as_float(bb.x & 0xffff0000u);
              v[0][2] += __uint_as_float(bb.y << 16); v[0][3] += __uint_as_float(bb.y & 0xffff0000u);
              v[1][0] += __uint_as_float(bb.z << 16); v[1][1] += __uint_as_float(bb.z & 0xffff0000u);
              v[1][2] += __uint_as_float(bb.w << 16); v[1][3] += __uint_as_float(bb.w & 0xffff0000u);
            }
            if (a.epi & EPI_RESIDUAL) {
              const uint4 rr = *reinterpret_cast<const uint4*>(resid + o);
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
            out.x = pack_bf16x2(v[0][0], v[0][1]); out.y = pack_bf16x2(v[0][2], v[0][3]);
            out.z = pack_bf16x2(v[1][0], v[1][1]); out.w = pack_bf16x2(v[1][2], v[1][3]);
            if (!TRAIL) QZO_STORE_OUT(y + o, out);
            if (a.epi & EPI_SUMSQ) {
              const uint32_t ow[4] = {out.x, out.y, out.z, out.w};
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const float q0 = __uint_as_float(ow[q] << 16), q1 = __uint_as_float(ow[q] & 0xffff0000u);
                ssq = __builtin_fmaf(q0, q0, ssq);
                ssq = __builtin_fmaf(q1, q1, ssq);
              }
            }
          }
          if (TRAIL) QZO_STORE_OUT_ALWAYS(inside ? (uint32_t)o * 2u : 0x80000000u, out);
        }
    }
    trail_stores = TRAIL ? 16 : 0;
    if (a.epi & EPI_SUMSQ) {
      // direct-to-LDS staging: the next tile's loads are already landing in the stages
      float* red = reinterpret_cast<float*>(lds + (DTL ? LDS_BYTES : 0));
      ssq = wave_sum(ssq);
      __syncthreads();
      if (lane == 0) red[wave] = ssq;
      __syncthreads();
      if (t == 0) {
        float s = 0.0f;
        for (int w = 0; w < THREADS / 64; ++w) s += red[w];
        a.partials[done_n * tiles_m + done_m] = s;
      }
      __syncthreads();   // the next tile's LDS stores must not overtake the read of red[]
    }
  } else {
    // Cross-entropy partials: for each token, (max, sum exp(l - max)) over this
    // wavefront's 64 vocabulary columns (32 in this lane's registers, 32 in the lane
    // 32 away), and the target logit where it falls here.
    const uint32_t slice = done_n * NWN + wn;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t m = m0 + wm * 128 + i * 32 + frow;
      const bool has_target = m < a.M && (m % ce.S) != ce.S - 1;
      const uint32_t target = has_target ? (uint32_t)ce.tok[(m % ce.tok_rows) + 1] : 0xffffffffu;
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const uint32_t n = n_wave + j * 32 + (r >> 2) * 8 + (r & 3);
          if (n < a.N) mx = fmaxf(mx, acc[i][j][r]);
          if (n == target) ce.tgt[m] = acc[i][j][r];
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      float sum = 0.0f;
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const uint32_t n = n_wave + j * 32 + (r >> 2) * 8 + (r & 3);
          if (n < a.N) sum += expf(acc[i][j][r] - mx);
        }
      sum += __shfl_xor(sum, 32, 64);
      if (m < a.M && fhalf == 0)
        reinterpret_cast<float2*>(ce.part)[(uint64_t)m * ce.n_slices + slice] = make_float2(mx, sum);
    }
  }
  if (!more) break;
  }   // tile loop
#undef QZO_SWAP8
#undef QZO_STORE_OUT
#undef QZO_STORE_OUT_ALWAYS
#undef QZO_TILE
#undef QZO_TILE_D
#undef QZO_DTL
#undef QZO_DTL_PART
#undef QZO_DTL16
#undef QZO_DTL_LANDED
#undef QZO_PP_TILE
#undef QZO_PP_LOAD_A
#undef QZO_PP_LOAD_B
#undef QZO_PP_STAGE_HALF
#undef QZO_PP_MFMAS
#undef QZO_PHASE_SYNC
#undef QZO_LSTORE_A
#undef QZO_LSTORE_B
#undef QZO_GLOAD_A
#undef QZO_GLOAD_B
#undef QZO_MFMAS
#undef QZO_FRAGS
#undef QZO_LSTORE
#undef QZO_NEW_GROUP
#undef QZO_SCALE_PREFETCH
#undef QZO_GLOAD
#undef QZO_CODES
#undef QZO_TILE_PTRS
}

static hipError_t set_lds_attr(const void* fn) {
  return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
}

// Launch configuration of the perturbed W4A16 GEMM.  Measured on MI355X at the
// Llama-2-7B layer shapes (M = 8192): 4 wavefronts along N (512 threads, two per
// SIMD) with the explicit issue order is the fastest; 2 along N (256 threads, one
// per SIMD, 128x128 per wavefront) is about 10 % slower.
constexpr int W4_NWN = 4;
constexpr int W4_PIPE = 2;

// Columns [n1, N) of a GEMM as a call of its own: weights, scales, zero-points, bias, output and residual
// advanced, the noise rows offset; y and resid keep the full matrix's row stride.
static GemmArgs column_block(const GemmArgs& a, uint32_t first, uint32_t count, int w_bits, bool codes_per_scale_group) {
  (void)codes_per_scale_group;
  GemmArgs s = a;
  const uint32_t ld = a.ldy ? a.ldy : a.N;
  s.N = count; s.ldy = ld;
  s.w = (const char*)a.w + (uint64_t)first * a.K * w_bits / 8;
  if (w_bits == 4) {
    if (a.s) s.s = (const char*)a.s + (uint64_t)first * (a.K >> 7) * 2;
    if (a.zp) s.zp = (const char*)a.zp + (uint64_t)first * (a.K >> 7);
    s.row_base = a.row_base + first;
  }
  if (a.bias) s.bias = (const char*)a.bias + (uint64_t)first * 2;
  s.y = (char*)a.y + (uint64_t)first * 2;
  if (a.resid) s.resid = (const char*)a.resid + (uint64_t)first * 2;
  return s;
}

hipError_t launch_w4a16_gemm(const GemmArgs& a0, hipStream_t st) {
  static bool ready = false;
  if (!ready) {
    hipError_t e = set_lds_attr((const void*)gemm_kernel<0, false, W4_NWN, W4_PIPE>);
    if (e == hipSuccess) e = set_lds_attr((const void*)gemm_kernel<0, false, W4_NWN, W4_PIPE, true>);
    if (e != hipSuccess) return e;
    ready = true;
  }
  if (a0.M == 0 || a0.N == 0) return hipSuccess;
  if (a0.M <= SKINNY_MAX_M && a0.skinny_ws) return launch_skinny_gemm(a0, a0.skinny_ws, st);
  GemmArgs a = a0;
  if (a0.dual) {
    // both passes of a step stacked: the second pass starts on a tile boundary and its tiles take -eps
    const uint32_t stride = a0.pass_stride ? a0.pass_stride : a0.M;
    if (stride % BM != 0 || stride < a0.M) return hipErrorInvalidValue;
    a.M = stride + a0.M; a.flip_row = stride; a.dual = 0;
  }
  // buffer loads address each operand with 32-bit byte offsets
  if ((uint64_t)a.M * a.K * 2 >= (1ull << 31) || (uint64_t)a.N * a.K / 2 >= (1ull << 31))
    return hipErrorInvalidValue;
  if (a.split_ws && !a.ldy) {
    // a little more than whole rounds of tiles: the whole rounds as they are, the rest cut along K
    const uint32_t n1 = tile_tail_cols(a.M, a.N, a.K, a.epi);
    if (n1) {
      GemmArgs h = column_block(a, 0, n1, 4, false), t = column_block(a, n1, a.N - n1, 4, false);
      h.split_ws = nullptr;
      hipError_t e = launch_w4a16_gemm(h, st);
      return e != hipSuccess ? e : launch_w4a16_gemm(t, st);
    }
  }
  CeEpilogue ce = {nullptr, nullptr, nullptr, 1, 1, 1};
  GemmArgs g = a;
  g.ksplit = 1;
  g.kt_per = a.K / BK;
  if (a.split_ws) g.ksplit = tile_ksplit(a.M, a.N, a.K, &g.kt_per);
  if (g.ksplit > 1) g.epi = 0;       // natural row order, fp32 partial sums; the reduction applies a.epi
  const uint32_t wgs = gemm_workgroups(a.M, ((a.N + BN - 1) / BN) * g.ksplit * BN);
  if (a.zp)
    gemm_kernel<0, false, W4_NWN, W4_PIPE, true><<<wgs, 128 * W4_NWN, LDS_BYTES, st>>>(g, ce);
  else
    gemm_kernel<0, false, W4_NWN, W4_PIPE><<<wgs, 128 * W4_NWN, LDS_BYTES, st>>>(g, ce);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || g.ksplit == 1) return e;
  return launch_partial_reduce(a, a.split_ws, g.ksplit, st);
}

hipError_t launch_codebook_gemm(const GemmArgs& a, hipStream_t st) {
  static bool ready = false;
  if (!ready) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_kernel<2, false, 4, 1>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES + 1024);
    if (e != hipSuccess) return e;
    ready = true;
  }
  if (a.M == 0 || a.N == 0) return hipSuccess;
  if ((uint64_t)a.M * a.K * 2 >= (1ull << 31) || (uint64_t)a.N * a.K / 4 >= (1ull << 31))
    return hipErrorInvalidValue;
  CeEpilogue ce = {nullptr, nullptr, nullptr, 1, 1, 1};
  gemm_kernel<2, false, 4, 1><<<gemm_workgroups(a.M, a.N), 512, LDS_BYTES + 1024, st>>>(a, ce);
  return hipGetLastError();
}

// Plain GEMM on a bf16 weight matrix [N,K] (the second stage of the expand-then-multiply
// paths): same tiling, no conversion in the loop.
hipError_t launch_bf16_gemm(const GemmArgs& a, int pipe, hipStream_t st) {
  static bool ready = false;
  if (!ready) {
    hipError_t e = set_lds_attr((const void*)gemm_kernel<1, false, 4, 0>);
    if (e == hipSuccess) e = set_lds_attr((const void*)gemm_kernel<1, false, 4, 1>);
    if (e == hipSuccess)     // + 1 KB: the sum-of-squares scratch sits behind the stages
      e = hipFuncSetAttribute((const void*)gemm_kernel<1, false, 4, 3>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES + 1024);
    if (e != hipSuccess) return e;
    ready = true;
  }
  if (a.M == 0 || a.N == 0) return hipSuccess;
  // buffer loads and stores address the operands and the output with 32-bit byte offsets
  if ((uint64_t)a.M * a.K * 2 >= (1ull << 31) || (uint64_t)a.N * a.K * 2 >= (1ull << 31) ||
      (uint64_t)a.M * (a.ldy ? a.ldy : a.N) * 2 >= (1ull << 31))
    return hipErrorInvalidValue;
  if (a.split_ws && !a.ldy && pipe == 2) {
    // a little more than whole rounds of tiles: the whole rounds as they are, the rest cut along K
    const uint32_t n1 = tile_tail_cols(a.M, a.N, a.K, a.epi);
    if (n1) {
      GemmArgs h = column_block(a, 0, n1, 16, false), t = column_block(a, n1, a.N - n1, 16, false);
      h.split_ws = nullptr;
      hipError_t e = launch_bf16_gemm(h, pipe, st);
      return e != hipSuccess ? e : launch_bf16_gemm(t, pipe, st);
    }
  }
  CeEpilogue ce = {nullptr, nullptr, nullptr, 1, 1, 1};
  GemmArgs g = a;
  g.ksplit = 1;
  g.kt_per = a.K / BK;
  if (a.split_ws) g.ksplit = tile_ksplit(a.M, a.N, a.K, &g.kt_per);   // too few tiles for the chip: split K
  if (g.ksplit > 1) g.epi = 0;       // natural row order, fp32 partial sums; the reduction applies a.epi
  // the model's route: with enough output tiles for the chip, the kernel with one wavefront per SIMD; not with
  // the fused SwiGLU, whose half-width output makes the 512-thread kernel's store burst cheap (measured inside
  // the 7B step: gate/up 1088 us with the 512-thread kernel, 1130 us with the other)
  if (pipe == 2 && g.ksplit == 1 && !(g.epi & EPI_SWIGLU)) return launch_bf16_gemm_wide(g, st);
  const uint32_t wgs = gemm_workgroups(a.M, ((a.N + BN - 1) / BN) * g.ksplit * BN);
  if (pipe == 2)         // K split over workgroups: both operand tiles straight from memory into the LDS, 512 threads
    gemm_kernel<1, false, 4, 3><<<wgs, 512, LDS_BYTES + 1024, st>>>(g, ce);
  else if (pipe == 1)    // staged through registers, explicit issue order
    gemm_kernel<1, false, 4, 1><<<wgs, 512, LDS_BYTES, st>>>(g, ce);
  else                   // staged through registers, compiler's order
    gemm_kernel<1, false, 4, 0><<<wgs, 512, LDS_BYTES, st>>>(g, ce);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || g.ksplit == 1) return e;
  return launch_partial_reduce(a, a.split_ws, g.ksplit, st);
}

hipError_t launch_lmhead_ce(const CeArgs& c, hipStream_t st) {
  static bool ready = false;
  if (!ready) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_kernel<1, true, 4, 3>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES + 1024);
    if (e != hipSuccess) return e;
    ready = true;
  }
  if ((uint64_t)c.M * c.K * 2 >= (1ull << 31) || (uint64_t)c.V * c.K * 2 >= (1ull << 31))
    return hipErrorInvalidValue;
  GemmArgs a = {};
  a.x = c.x; a.w = c.w; a.M = c.M; a.N = c.V; a.K = c.K;
  CeEpilogue ce = {c.tok, c.part, c.tgt, c.S, c.n_slices, c.tok_rows ? c.tok_rows : c.M};
  gemm_kernel<1, true, 4, 3><<<gemm_workgroups(c.M, c.V), 512, LDS_BYTES + 1024, st>>>(a, ce);
  return hipGetLastError();
}

// Matrix-pipe rate probe: every wavefront of a 512-thread workgroup per compute unit
// issues `iters` x 16 independent v_mfma_f32_32x32x16_bf16 on register operands (all zero,
// or pseudo-random bf16 values) and nothing else.  What it sustains is the ceiling that
// the board's clock and power management leave to any bf16 MFMA kernel.
__global__ __launch_bounds__(512, 1) void mfma_rate_kernel(float* sink, uint32_t iters, int random_operands) {
  floatx16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
  bf16x8 fa[4], fb[2];
  const uint32_t t = threadIdx.x;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t h = (t * 2654435761u + (uint32_t)(i * 8 + e) * 40503u) >> 20;          // 0 .. 4095
      fa[i][e] = (__bf16)(random_operands ? ((float)h - 2048.0f) * (1.0f / 1024.0f) : 0.0f);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint32_t h = (t * 2246822519u + (uint32_t)(j * 8 + e) * 668265263u) >> 20;
      fb[j][e] = (__bf16)(random_operands ? ((float)h - 2048.0f) * (1.0f / 131072.0f) : 0.0f);
    }
  }
  for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
    for (int rep = 0; rep < 2; ++rep)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i * 2 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i * 2 + j], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[blockIdx.x * 512u + t] = s;
}

hipError_t launch_mfma_rate(float* sink, uint32_t workgroups, uint32_t iters, int random_operands,
                            hipStream_t st) {
  mfma_rate_kernel<<<workgroups, 512, 0, st>>>(sink, iters, random_operands);
  return hipGetLastError();
}

}  // namespace qzo
