// Geometry shared by the tile GEMM kernels: the 256 x 256 x 64 workgroup tile, its LDS layout and the
// XCD-aware walk of persistent workgroups over the output tiles.
#pragma once
#include "qzo_device.hpp"
#include "qzo_kernels.hpp"

namespace qzo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int TILE_BYTES = BM * BK * 2;            // 32 KB per operand per stage
constexpr int LDS_BYTES = 4 * TILE_BYTES;          // A0 A1 B0 B1

// Persistent workgroups: the grid is one workgroup per compute unit (or fewer when
// there are fewer tiles) and every workgroup walks a list of output tiles.
// Hardware deals consecutive workgroup ids to the eight XCDs in turn; each XCD
// gets one contiguous eighth of a tile order in which groups of WALK_M M-tiles sweep
// the N-tiles, and its workgroups take consecutive entries of that eighth, so the
// tiles in flight on one XCD share a few A and B row-panels in that XCD's L2.
// M-tiles per group of the walk.  With 32 tiles resident per XCD, groups of 4 (or 2) minimise
// the bytes streamed from HBM (activation panel re-read 6 times, int4 panel 8 times).
constexpr uint32_t WALK_M = 4;
struct TileWalk {
  uint32_t tiles_m, tiles_n, total, per, xcd, slot, stride;
};
// With K slices (split-K) the walk runs over feature-tiles x slices: entry tn of the walk is feature
// tile tn % real_tiles_n, slice tn / real_tiles_n.
__device__ __forceinline__ TileWalk tile_walk_init(uint32_t M, uint32_t N, uint32_t ksplit = 1) {
  TileWalk w;
  w.tiles_m = (M + BM - 1) / BM;
  w.tiles_n = ((N + BN - 1) / BN) * ksplit;
  w.total = w.tiles_m * w.tiles_n;
  w.per = (w.total + 7) >> 3;
  w.xcd = blockIdx.x & 7u;
  w.slot = blockIdx.x >> 3;
  w.stride = gridDim.x >> 3;
  return w;
}
// Tile of the walk's current slot; false when the walk is over.
__device__ __forceinline__ bool tile_walk_get(const TileWalk& w, uint32_t& tm, uint32_t& tn) {
  if (w.slot >= w.per) return false;
  const uint32_t id = w.xcd * w.per + w.slot;
  if (id >= w.total) return false;
  const uint32_t width = WALK_M * w.tiles_n;
  const uint32_t group = id / width;
  const uint32_t first = group * WALK_M;
  const uint32_t gsz = min(w.tiles_m - first, WALK_M);
  const uint32_t in = id - group * width;
  tm = first + in % gsz;
  tn = in / gsz;
  return true;
}

__device__ __forceinline__ uint32_t lds_off(uint32_t row, uint32_t chunk) {
  return row * 128u + ((chunk ^ ((row >> 1) & 7u)) << 4);
}

}  // namespace qzo
