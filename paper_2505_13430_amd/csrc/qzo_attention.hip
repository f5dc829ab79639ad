// Causal self-attention softmax(Q K^T / sqrt(dh)) V for gfx950, bf16 MFMA with
// fp32 online softmax, head size 64 or 128.  Input is the fused projection
// output qkv [B*S, 3d] (q | k | v), output [B*S, d].
//
// A workgroup of four wavefronts serves 128 queries of one (batch, head); each
// wavefront owns 32 queries.  Scores are produced transposed (keys x queries)
// so that a lane owns one query: the softmax row reductions are in-register
// plus one cross-half shuffle, the probabilities are already in the B-operand
// layout of the second MFMA, and O^T = V^T P^T accumulates with a per-lane
// rescale.
//
// Keys are processed 64 at a time.  The K tile sits row-major in LDS (16-byte
// chunks XOR-swizzled by row).  The V tile sits row-major as well (keys x head dimension, 32-byte segments
// XOR-swizzled by row): the second MFMA needs, per lane, eight keys of one feature, and gets them from two
// transposing LDS reads (ds_read_b64_tr_b16: within 16 lanes, lane j supplies four consecutive features of
// key j/4, lane i receives feature i of keys 0..3), so V is loaded from memory in whole rows and lands in
// the LDS as it is.  Two LDS buffers, one barrier per tile.
#include "qzo_device.hpp"
#include "qzo_kernels.hpp"

namespace qzo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// ROPE: q and k arrive without the rotary embedding and get it here: the queries once in
// registers, the keys of a tile on their way from registers to the LDS (the table of (cos, sin)
// per position and pair is read when a tile is stored, not ahead: the variant is for short
// sequences, where the separate RoPE launch costs more than these few exposed latencies).
// A lane rounds nothing extra: the inputs are the bf16 values a separate pass would read, the
// rotation is the same fp32 arithmetic, rounded once to bf16.
__device__ __forceinline__ void rope_pair8(uint32_t (&a)[4], uint32_t (&b)[4], const float4* tb) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float4 t = tb[j];                          // (cos, sin) of pairs 2 j and 2 j + 1
    const float a0 = __uint_as_float(a[j] << 16), a1 = __uint_as_float(a[j] & 0xffff0000u);
    const float b0 = __uint_as_float(b[j] << 16), b1 = __uint_as_float(b[j] & 0xffff0000u);
    a[j] = pack_bf16x2(a0 * t.x - b0 * t.y, a1 * t.z - b1 * t.w);
    b[j] = pack_bf16x2(b0 * t.x + a0 * t.y, b1 * t.z + a1 * t.w);
  }
}

template <int DH, bool ROPE, bool LONG>
__global__ __launch_bounds__(256, 2) void attention_kernel(const bf16_t* __restrict__ qkv, uint32_t S,
                                                           uint32_t n_heads, bf16_t* __restrict__ out,
                                                           const float2* __restrict__ rope, uint32_t walk) {
  constexpr int KB = 64;             // keys per tile
  constexpr int KT = DH / 16;        // k-steps of the score MFMA
  constexpr int DT = DH / 32;        // 32-wide slices of the head for the PV MFMA
  constexpr int CH = DH / 8;         // 16-byte chunks per K row
  constexpr int NK = KB * CH / 256;  // K chunks per thread and tile (4 or 2)
  constexpr uint32_t SWZ = CH - 1;   // chunk swizzle mask: DH 128 -> row & 15, DH 64 -> (row >> 1) & 7
  // Without ROPE both tiles go from memory straight into the LDS (buffer loads with the lds modifier: a
  // wavefront's load fills 1 KB in lane order, so both swizzles are applied on the memory side); with ROPE
  // the keys pass through registers to be rotated and V takes the same way.
  constexpr bool DTL = !ROPE;
  constexpr int NI = KB * DH * 2 / 4096;   // direct loads per wavefront, tile and operand (4 or 2)
  // LDS: K tile, V tile of buffer 0, then of buffer 1 (buffer 1 first holds the workgroup's 128 queries, at the
  // end the four wavefronts' output rows pass through buffer 0 and 1)
  constexpr int TILE = KB * DH;            // elements of one K or V tile
  __shared__ __attribute__((aligned(1024))) bf16_t smem[4 * TILE];

  const uint32_t d = n_heads * DH, ld = 3 * d;
  // Workgroups are handed to the 8 XCDs round-robin in launch order, and each XCD has its own L2: the
  // query blocks of one (batch, head) are given to workgroups of one XCD, so that its K and V are
  // fetched into one L2 only; within that, heavy query blocks (late positions, many keys) come first.
  uint32_t bx = blockIdx.x, hb = blockIdx.y + gridDim.y * blockIdx.z;
  const uint32_t nhb = gridDim.y * gridDim.z;
  if ((nhb & 7u) == 0u) {
    const uint32_t L = blockIdx.x + gridDim.x * hb, slot = L >> 3;
    hb = (L & 7u) + 8u * (slot / gridDim.x);
    bx = slot % gridDim.x;
  }
  const uint32_t b = hb / gridDim.y, h = hb % gridDim.y;
  const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
  const uint32_t lrow = lane & 31u, lhalf = lane >> 5;
  const bf16_t* base = qkv + (uint64_t)b * S * ld + h * DH;
  auto swz = [](uint32_t row) { return DH == 128 ? (row & SWZ) : ((row >> 1) & SWZ); };
  // V rows are unpadded; their 32-byte segments are XOR-swizzled so that the 4 rows x 2 segments that half a
  // wavefront touches in one transposing read fall into 8 different 32-byte bank groups
  auto vsw = [](uint32_t row) { return DH == 128 ? 2u * (row & 3u) : 2u * ((row >> 1) & 1u); };

  const float sc = 1.44269504088896f / sqrtf((float)DH);   // log2(e)/sqrt(dh)

  // staging registers: K and V chunks (row c / CH, chunk c % CH of the tile, c = t + 256 i)
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 kreg[NK], vreg[NK];
  // (macros, not lambdas: arrays captured by reference would be kept in scratch memory)
  // K chunk i of this thread: (row, chunk) = (c / CH, c % CH) with c = t + 256 i; with ROPE a thread
  // takes pairs of chunks (ch, ch + CH/2) of one row, which hold the two halves of 8 rotation pairs
#define QZO_ATT_KROW(I) (ROPE ? (t + 256u * ((I) >> 1)) / (CH / 2) : (t + 256u * (I)) / CH)
#define QZO_ATT_KCH(I) (ROPE ? (t + 256u * ((I) >> 1)) % (CH / 2) + ((I) & 1) * (CH / 2) : (t + 256u * (I)) % CH)
#define QZO_ATT_GLOAD(KB_)                                                                   \
  do {                                                                                       \
    _Pragma("unroll") for (int i = 0; i < NK; ++i) {                                         \
      const uint32_t row = QZO_ATT_KROW(i), ch = QZO_ATT_KCH(i);                             \
      const uint32_t key = min((KB_) * KB + row, S - 1);                                     \
      kreg[i] = *reinterpret_cast<const u32x4*>(base + (uint64_t)key * ld + d + ch * 8);     \
    }                                                                                        \
    _Pragma("unroll") for (int i = 0; i < NK; ++i) {                                         \
      const uint32_t c = t + 256u * i;                                                       \
      const uint32_t key = min((KB_) * KB + c / CH, S - 1);                                  \
      vreg[i] = *reinterpret_cast<const u32x4*>(base + (uint64_t)key * ld + 2 * d + (c % CH) * 8); \
    }                                                                                        \
  } while (0)
#define QZO_ATT_LSTORE(BUF, KB_)                                                             \
  do {                                                                                       \
    if (ROPE) {                                                                              \
      _Pragma("unroll") for (int p = 0; p < NK / 2; ++p) {                                   \
        const uint32_t row = QZO_ATT_KROW(2 * p), ch = QZO_ATT_KCH(2 * p);                   \
        const uint32_t key = min((KB_) * KB + row, S - 1);                                   \
        uint32_t ka_[4] = {kreg[2 * p].x, kreg[2 * p].y, kreg[2 * p].z, kreg[2 * p].w};      \
        uint32_t kb_[4] = {kreg[2 * p + 1].x, kreg[2 * p + 1].y, kreg[2 * p + 1].z, kreg[2 * p + 1].w}; \
        rope_pair8(ka_, kb_, reinterpret_cast<const float4*>(rope + (uint64_t)key * (DH / 2) + ch * 8)); \
        kreg[2 * p] = u32x4{ka_[0], ka_[1], ka_[2], ka_[3]};                                 \
        kreg[2 * p + 1] = u32x4{kb_[0], kb_[1], kb_[2], kb_[3]};                             \
      }                                                                                      \
    }                                                                                        \
    _Pragma("unroll") for (int i = 0; i < NK; ++i) {                                         \
      const uint32_t row = QZO_ATT_KROW(i), ch = QZO_ATT_KCH(i);                             \
      *reinterpret_cast<u32x4*>((smem + (BUF) * 2 * TILE) + row * DH + ((ch ^ swz(row)) * 8)) = kreg[i];      \
    }                                                                                        \
    _Pragma("unroll") for (int i = 0; i < NK; ++i) {                                         \
      const uint32_t c = t + 256u * i;                                                       \
      const uint32_t row = c / CH, ch = c % CH;                                              \
      *reinterpret_cast<u32x4*>((smem + (BUF) * 2 * TILE + TILE) + row * DH + (((ch >> 1) ^ vsw(row)) * 16 + (ch & 1u) * 8)) = vreg[i]; \
    }                                                                                        \
  } while (0)
  // Direct loads: load n of wavefront w fills bytes (4 n + w) 1024 .. + 1023 of a tile, lane l its 16 bytes at
  // l 16: row and physical chunk follow, the logical chunk is the physical one un-swizzled.
  typedef int i32x4 __attribute__((ext_vector_type(4)));
  const uint64_t base_addr = (uint64_t)(uintptr_t)base;
  const uint64_t left = ((uint64_t)(gridDim.z - b) * S * ld - h * DH) * 2;      // bytes from base to the end of qkv
  const i32x4 rqkv = {(int)(uint32_t)base_addr, (int)(uint32_t)(base_addr >> 32),
                      (int)(uint32_t)(left < 0xffffffffull ? left : 0xffffffffull), 0x00020000};
  uint32_t d_row[DTL ? NI : 1], d_koff[DTL ? NI : 1], d_voff[DTL ? NI : 1];
  if (DTL) {
#pragma unroll
    for (int n = 0; n < NI; ++n) {
      const uint32_t byte = (4u * n + wave) * 1024u + lane * 16u;
      const uint32_t row = byte / (DH * 2), pc = (byte % (DH * 2)) / 16;
      d_row[n] = row;
      d_koff[n] = (d + (pc ^ swz(row)) * 8) * 2;
      d_voff[n] = (2 * d + (((pc >> 1) ^ vsw(row)) * 2 + (pc & 1u)) * 8) * 2;
    }
  }
  const uint32_t lds_k = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) bf16_t*)&smem[0] +
                         __builtin_amdgcn_readfirstlane(wave) * 1024u;
  const uint32_t lds_v = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) bf16_t*)&smem[TILE] +
                         __builtin_amdgcn_readfirstlane(wave) * 1024u;
#define QZO_ATT_DTL16(LDSADDR, VOFF)                                                         \
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"                 \
               : : "s"(LDSADDR), "v"(VOFF), "s"(rqkv) : "memory", "m0")
// load J of a tile: J < NI the K loads, then the V loads; BUF, KB_ may be run-time values.  ON (uniform)
// false: the offset is out of the buffer's range, the load fetches nothing and writes zeros to a buffer
// that nobody reads (no branch around the load: the score loop stays one block for the scheduler)
#define QZO_ATT_DTL_ONE(BUF, KB_, J, ON)                                                     \
  do {                                                                                       \
    const int n_ = (J) < NI ? (J) : (J) - NI;                                                \
    const uint32_t key = min((KB_) * KB + d_row[n_], S - 1);                                 \
    const uint32_t off_ = key * (ld * 2) + ((J) < NI ? d_koff[n_] : d_voff[n_]);             \
    QZO_ATT_DTL16(((J) < NI ? lds_k : lds_v) + (uint32_t)((BUF) * (4 * TILE) + n_ * 4096), (ON) ? off_ : 0xfffffff0u); \
  } while (0)
#define QZO_ATT_DTL(BUF, KB_)                                                                \
  do {                                                                                       \
    _Pragma("unroll") for (int j_ = 0; j_ < 2 * NI; ++j_) QZO_ATT_DTL_ONE(BUF, KB_, j_, true); \
  } while (0)
  // Registers (ROPE): tile kb is computed from LDS buffer kb & 1 while tile kb+1 goes from registers to the
  // other buffer and tile kb+2 is requested from memory.  Direct loads: tile kb+1 is requested into the
  // other buffer at the start of tile kb (every wavefront is past the barrier, so tile kb-1 has been read)
  // and has landed when each wavefront's own loads are back and the next barrier is passed.  One barrier
  // per tile either way.
  // walk != 0: the workgroups of a (batch, head) walk its query blocks themselves, late (heavy) blocks
  // first.  gridDim.x == 1: one workgroup takes them all.  gridDim.x == 2: two workgroups share them in
  // snake order (blocks n-1 | n-2, n-3 | n-4, n-5 | ... from the heavy end: equal work for 4 blocks);
  // the launch-index remap above puts the two on one XCD in neighbouring slots, they start together
  // and ask for the same K and V tiles at about the same time, so the second one's loads hit the L2
  // (the kernel is bound by what crosses from memory into the L2s, not by its arithmetic).
  // walk == 0: a workgroup serves the one query block its launch index names.
  const uint32_t nqb = (S + 127) / 128;
  constexpr bool via_lds = LONG;               // more than one query block per head
  const bool walk_ = LONG && walk != 0u;
  const uint32_t n_it = walk_ ? nqb : 1u;
  for (uint32_t it = 0; it < n_it; ++it) {
  if (walk_ && gridDim.x == 2u && (((it + 1u) >> 1) & 1u) != bx) continue;
  const uint32_t q0 = (walk_ ? nqb - 1 - it : gridDim.x - 1 - bx) * 128;
  const uint32_t qq = q0 + wave * 32 + lrow;            // this lane's query
  const uint32_t qc = min(qq, S - 1);
  bf16x8 qf[KT];
  floatx16 o[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;
  const uint32_t q_hi = min(q0 + 127u, S - 1);
  const uint32_t nkb = q_hi / KB + 1;
  const uint32_t wave_q_hi = q0 + wave * 32 + 31;

  // Long sequences: the 128 queries come in whole rows as well: direct loads put them (K's layout and swizzle,
  // 128 rows) where buffer 1 will be; every wavefront then reads its fragments (a lane: its query, k-step ks,
  // half) from there.  Short sequences (one or a few tiles per workgroup) cannot afford the two barriers this
  // takes: there a lane reads its query's fragments from memory.
  if (via_lds) {
    constexpr int NQ = 128 * DH * 2 / 4096;      // loads per wavefront
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      const uint32_t byte = (4u * n + wave) * 1024u + lane * 16u;
      const uint32_t row = byte / (DH * 2), pc = (byte % (DH * 2)) / 16;
      const uint32_t q = min(q0 + row, S - 1);
      QZO_ATT_DTL16(lds_k + (uint32_t)(4 * TILE + n * 4096), q * (ld * 2) + ((pc ^ swz(row)) * 8) * 2);
    }
  } else {
#pragma unroll
    for (int ks = 0; ks < KT; ++ks)
      qf[ks] = *reinterpret_cast<const bf16x8*>(base + (uint64_t)qc * ld + ks * 16 + lhalf * 8);
  }
  if (DTL) {
    QZO_ATT_DTL(0, 0u);
  } else {
    QZO_ATT_GLOAD(0u);
  }
  if (via_lds) {
    __builtin_amdgcn_s_waitcnt(0x0F70);         // vmcnt(0): this wavefront's part of the queries (and of tile 0)
    __syncthreads();
    const bf16_t* Qs = smem + 2 * TILE;
    const uint32_t row = wave * 32 + lrow;
#pragma unroll
    for (int ks = 0; ks < KT; ++ks)
      qf[ks] = *reinterpret_cast<const bf16x8*>(Qs + row * DH + (((uint32_t)(ks * 2) + lhalf) ^ swz(row)) * 8);
  }
  if (ROPE) {
    // k-step ks < KT/2 holds features ks*16 + 8 lhalf .. + 7 of the head, k-step ks + KT/2 the same + DH/2
#pragma unroll
    for (int ks = 0; ks < KT / 2; ++ks) {
      union { bf16x8 v; uint32_t u[4]; } qa, qb;
      qa.v = qf[ks]; qb.v = qf[ks + KT / 2];
      rope_pair8(qa.u, qb.u, reinterpret_cast<const float4*>(rope + (uint64_t)qc * (DH / 2) + ks * 16 + lhalf * 8));
      qf[ks] = qa.v; qf[ks + KT / 2] = qb.v;
    }
  }

  if (!DTL) {
    QZO_ATT_LSTORE(0, 0u);
    if (nkb > 1) QZO_ATT_GLOAD(1u);
  } else if (!via_lds) {
    __builtin_amdgcn_s_waitcnt(0x0F70);         // vmcnt(0): this wavefront's part of tile 0
  }
  __syncthreads();                              // tile 0 is complete (and the queries have been read: buffer 1 is free)

  for (uint32_t kb = 0; kb < nkb; ++kb) {
    if (kb > 0) {                               // tile kb is complete, tile kb-1 has been read
      if (DTL) __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
    }
    // direct loads of tile kb+1: one per k-step of the score MFMAs below (a wavefront whose tile is wholly
    // in its future issues them here)
    const bool dtl_next = DTL && kb + 1 < nkb;
    const uint32_t nbuf = (kb + 1) & 1u;
    if (kb + 1 < nkb) {
      if (DTL) {
        if (kb * KB > wave_q_hi) QZO_ATT_DTL(nbuf, kb + 1);
      } else {
        if (kb & 1u) QZO_ATT_LSTORE(0, kb + 1); else QZO_ATT_LSTORE(1, kb + 1);
        if (kb + 2 < nkb) QZO_ATT_GLOAD(kb + 2);
      }
    }
    const bf16_t* Ks = smem + (kb & 1u) * 2 * TILE;
    const bf16_t* Vs = Ks + TILE;
    if (kb * KB > wave_q_hi) continue;          // every key of the tile is in this wave's future
    const bool two = kb * KB + 32 <= wave_q_hi; // the tile's second half holds visible keys

    // scores^T: rows = keys, cols = queries; sub-tile u covers keys 32 u .. 32 u + 31.
    // The two sub-tiles are independent accumulators and alternate in the matrix pipe.
    floatx16 s[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[u][r] = 0.0f;
    if (two) {
#pragma unroll
      for (int ks = 0; ks < KT; ++ks) {
        const uint32_t ch = ks * 2 + lhalf;
        const bf16x8 k0 = *reinterpret_cast<const bf16x8*>(Ks + lrow * DH + ((ch ^ swz(lrow)) * 8));
        const bf16x8 k1 = *reinterpret_cast<const bf16x8*>(Ks + (32 + lrow) * DH + ((ch ^ swz(32 + lrow)) * 8));
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[ks], s[0], 0, 0, 0);
        s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, qf[ks], s[1], 0, 0, 0);
        if (DTL && ks < 2 * NI) QZO_ATT_DTL_ONE(nbuf, kb + 1, ks, dtl_next);
      }
      // issue order: six fragment reads ahead, then one pair of reads per pair of MFMAs
      __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
      for (int ks = 0; ks < KT; ++ks) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        if (ks < KT - 3) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < KT; ++ks) {
        const uint32_t ch = ks * 2 + lhalf;
        const bf16x8 k0 = *reinterpret_cast<const bf16x8*>(Ks + lrow * DH + ((ch ^ swz(lrow)) * 8));
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[ks], s[0], 0, 0, 0);
        if (DTL && ks < 2 * NI) QZO_ATT_DTL_ONE(nbuf, kb + 1, ks, dtl_next);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int ks = 0; ks < KT; ++ks) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (ks < KT - 4) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
    }
    // running maximum in raw score units; the 1/sqrt(dh) log2(e) factor is folded into the
    // exponent: p = exp2(s * sc - m * sc).  Only tiles that touch the diagonal need the mask.
    if (kb * KB + (KB - 1) > q0 + wave * 32) {
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const uint32_t key = kb * KB + u * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
          s[u][r] = key <= qq ? s[u][r] : -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[u][r]);
    {   // both halves of the wavefront: lane l and lane l ^ 32 hold the two halves of a query's keys
      const auto r_ = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
      mx = fmaxf(__uint_as_float(r_[0]), __uint_as_float(r_[1]));
    }
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);
    const float nm = -m_new * sc;
    float psum = 0.0f;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[u][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[u][r], sc, nm));
        psum += s[u][r];
      }
    {
      const auto r_ = __builtin_amdgcn_permlane32_swap(__float_as_uint(psum), __float_as_uint(psum), false, false);
      psum = __uint_as_float(r_[0]) + __uint_as_float(r_[1]);
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {   // some lane's maximum moved
#pragma unroll
      for (int i = 0; i < DT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
    }
    // P^T as the B operand: element e of k-step st (16 keys) is key 8 (e/4) + 4 half + e%4 of
    // that group, i.e. score register 8 (st & 1) + e of sub-tile st / 2.  The V operand of the same
    // k-step: a lane's feature is 32 i + lane % 32, its keys come from two transposing reads (keys
    // 16 st + 4 half + 0..3 and the same + 8), for which lane j of each 16 supplies features
    // 4 (j % 4) .. + 3 of its 16-feature block at key + j / 4.
    // (rows 16 st + 4 half + j / 4 (+ 8): the swizzle depends on j / 4 only; segment 2 i + (lane / 16) % 2)
    const uint32_t v_r = (lane & 15u) >> 2;
    const uint32_t v_src = (4 * lhalf + v_r) * DH + ((lane >> 4) & 1u) * 16 + (lane & 3u) * 4;
    const uint32_t v_x = vsw(v_r);
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      if (st < 2 || two) {
        union { bf16x8 v; uint32_t u[4]; } pf;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          pf.u[e] = pack_bf16x2(s[st >> 1][8 * (st & 1) + 2 * e], s[st >> 1][8 * (st & 1) + 2 * e + 1]);
#pragma unroll
        for (int i = 0; i < DT; ++i) {
          typedef short short4v __attribute__((ext_vector_type(4)));
          typedef __attribute__((address_space(3))) short4v* lds_s4;
          union { bf16x8 v; short4v h[2]; } vf;
          const bf16_t* src = Vs + v_src + (16 * st) * DH + ((2u * i) ^ v_x) * 16;
          vf.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(src));
          vf.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(src + 8 * DH));
          o[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf.v, o[i], 0, 0, 0);
        }
      }
    }
  }

  // Output: a lane holds one query's features in 4-feature pieces.  Long sequences: each wavefront passes its
  // 32 rows through the LDS (rows padded by 16 bytes) so that they leave in whole rows, 16 bytes per lane;
  // short sequences store the pieces as they are.
  if (DTL) __builtin_amdgcn_s_waitcnt(0x0F70);   // the last tile's (empty) direct loads have written their zeros
  const float inv = 1.0f / l_run;
  if (via_lds) {
    __syncthreads();                             // every wavefront is done with the tiles
    constexpr int OS = DH + 8;                   // padded output row (elements)
    bf16_t* Os = smem + wave * (32 * OS);
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 v;
        v.x = pack_bf16x2(o[i][4 * g] * inv, o[i][4 * g + 1] * inv);
        v.y = pack_bf16x2(o[i][4 * g + 2] * inv, o[i][4 * g + 3] * inv);
        *reinterpret_cast<uint2*>(Os + lrow * OS + i * 32 + 8 * g + 4 * lhalf) = v;
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    constexpr int LPR = DH / 8;                  // lanes per row
    constexpr int RPI = 64 / LPR;                // rows per store instruction
#pragma unroll
    for (int j = 0; j < 32 / RPI; ++j) {
      const uint32_t row = j * RPI + lane / LPR, ch = lane % LPR;
      const uint32_t q = q0 + wave * 32 + row;
      const uint4 v = *reinterpret_cast<const uint4*>(Os + row * OS + ch * 8);
      if (q < S) *reinterpret_cast<uint4*>(out + ((uint64_t)b * S + q) * d + h * DH + ch * 8) = v;
    }
  } else if (qq < S) {
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
  if (it + 1 < n_it) __syncthreads();            // the output rows have been read: the LDS is free for the next block
  }   // query blocks
}

#undef QZO_ATT_KROW
#undef QZO_ATT_KCH
#undef QZO_ATT_GLOAD
#undef QZO_ATT_LSTORE
#undef QZO_ATT_DTL
#undef QZO_ATT_DTL_ONE
#undef QZO_ATT_DTL16

// rope (nullable): (cos, sin) of [S positions][dh/2 pairs]; with it q and k are rotated on the fly.
hipError_t launch_attention(const void* qkv, uint32_t B, uint32_t S, uint32_t n_heads,
                            uint32_t dh, void* out, const float* rope, hipStream_t st) {
  // the direct loads address qkv with 32-bit byte offsets and use an offset near 2^32 as "out of range"
  if ((uint64_t)B * S * 3 * n_heads * dh * 2 >= (1ull << 31)) return hipErrorInvalidValue;
  // The (batch, head) pairs alone fill the chip twice over (two workgroups fit a CU): their workgroups walk
  // the query blocks, two workgroups per pair from three query blocks on, else one.
  static int n_cu = 0;
  if (n_cu == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0)
      n_cu = 256;
  }
  const bool lng = S > 128 && !rope;           // more than one query block per head: the long-sequence paths
  const bool per_head = (uint64_t)n_heads * B >= 2ull * (uint64_t)n_cu && lng;
  const bool pair = per_head && S > 256;
  const uint32_t walk = per_head ? 1u : 0u;
  dim3 grid(pair ? 2 : (per_head ? 1 : (S + 127) / 128), n_heads, B);
  const float2* tb = (const float2*)rope;
  if (dh == 128 && rope)
    attention_kernel<128, true, false><<<grid, 256, 0, st>>>((const bf16_t*)qkv, S, n_heads, (bf16_t*)out, tb, walk);
  else if (dh == 128 && lng)
    attention_kernel<128, false, true><<<grid, 256, 0, st>>>((const bf16_t*)qkv, S, n_heads, (bf16_t*)out, tb, walk);
  else if (dh == 128)
    attention_kernel<128, false, false><<<grid, 256, 0, st>>>((const bf16_t*)qkv, S, n_heads, (bf16_t*)out, tb, walk);
  else if (dh == 64 && rope)
    attention_kernel<64, true, false><<<grid, 256, 0, st>>>((const bf16_t*)qkv, S, n_heads, (bf16_t*)out, tb, walk);
  else if (dh == 64 && lng)
    attention_kernel<64, false, true><<<grid, 256, 0, st>>>((const bf16_t*)qkv, S, n_heads, (bf16_t*)out, tb, walk);
  else if (dh == 64)
    attention_kernel<64, false, false><<<grid, 256, 0, st>>>((const bf16_t*)qkv, S, n_heads, (bf16_t*)out, tb, walk);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace qzo
