// Geometry of the packed layouts (see include/spqr.h for the normative text).
// Shared by the host packer, the validators and the kernels of this library.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__) || defined(__HIP__)
#define SPQR_HD __attribute__((host)) __attribute__((device)) inline __attribute__((always_inline))
#else
#define SPQR_HD inline
#endif

namespace spqr {

constexpr int kBlockTiles = 64;   // tiles per interleave block = lanes per wavefront

// Statistic layouts (values of spqr_matrix_t::layout_version).
constexpr int kBilevel = 1;       // 3-bit codes per group, (s_s, z_s, s_z, z_z) per tile
constexpr int kRoundZero = 2;     // the zero code is the zero-point; (s_s, z_s) per tile
constexpr int kStats16 = 3;       // binary16 (s, z) per group, nothing per tile

struct Geometry {
  int32_t m, n, w_bits, beta1, beta2, axis;
  int32_t tile_rows, tile_cols;   // (beta2, beta1) for axis 0, (beta1, beta2) for axis 1
  int32_t ntr, ntc;               // tile grid
  int32_t kw;                     // 16-byte code words per tile
  int32_t sd;                     // statistic dwords per tile (incl. the second-level dwords)
  int32_t swf, sr;                // full statistic words, remaining dwords
  int32_t tile_bytes;
  int32_t layout;                 // kBilevel, kRoundZero, kStats16
};

// Returns 0 or a negative spqr_status value (-2 shape, -3 param).
SPQR_HD int make_geometry(int32_t layout, int32_t m, int32_t n, int32_t w_bits, int32_t s_bits, int32_t z_bits,
                          int32_t beta1, int32_t beta2, int32_t axis, Geometry* g) {
  if (layout != kBilevel && layout != kRoundZero && layout != kStats16) return -3;
  if (w_bits != 3 && w_bits != 4) return -3;
  if (layout == kStats16 ? (s_bits != 16 || z_bits != 16) : (s_bits != 3 || z_bits != 3)) return -3;
  if (axis != 0 && axis != 1) return -3;
  if (beta1 < 1 || beta2 < 16 || beta1 > 4096 || beta2 > 4096) return -3;
  if (beta2 % 16 != 0) return -3;
  if (((int64_t)beta1 * beta2 * w_bits) % 128 != 0) return -3;
  int32_t tr = axis == 0 ? beta2 : beta1;
  int32_t tc = axis == 0 ? beta1 : beta2;
  if (tc % 2 != 0) return -3;
  if (m <= 0 || n <= 0 || n > 65536) return -2;
  if (m % tr != 0 || n % tc != 0) return -2;
  g->m = m; g->n = n; g->w_bits = w_bits; g->beta1 = beta1; g->beta2 = beta2; g->axis = axis;
  g->tile_rows = tr; g->tile_cols = tc;
  g->ntr = m / tr; g->ntc = n / tc;
  g->kw = (int32_t)(((int64_t)tr * tc * w_bits) / 128);
  g->layout = layout;
  g->sd = layout == kStats16 ? beta2 : 3 * beta2 / 16 + (layout == kRoundZero ? 1 : 2);
  g->swf = g->sd / 4; g->sr = g->sd % 4;
  g->tile_bytes = 16 * g->kw + 4 * g->sd;
  return 0;
}

// Where the 3-bit / 4-bit pair number q lives inside a tile's dword array.
// For the split pair of a 3-bit triple (q % 16 == 15) `split` is set and
// `dword` is the first dword of the triple.
struct PairLoc { int32_t dword; int32_t shift; bool split; };

SPQR_HD PairLoc pair_loc(int32_t w_bits, int32_t q) {
  PairLoc p;
  if (w_bits == 4) {
    p.dword = q >> 2; p.shift = 4 * (q & 3); p.split = false;
  } else {
    int32_t t = q >> 4, e = q & 15;
    if (e < 15) { p.dword = 3 * t + e / 5; p.shift = 3 * (e % 5); p.split = false; }
    else        { p.dword = 3 * t;         p.shift = 15;          p.split = true;  }
  }
  return p;
}

// Byte offset, inside the packed buffer, of dword `d` of the code area of tile
// (tile_row, tile_col).
SPQR_HD int64_t code_dword_offset(const Geometry& g, int32_t tile_row, int32_t tile_col, int32_t d) {
  int32_t blk = tile_col / kBlockTiles, l = tile_col % kBlockTiles;
  int32_t L = g.ntc - blk * kBlockTiles; if (L > kBlockTiles) L = kBlockTiles;
  int64_t base = ((int64_t)tile_row * g.ntc + (int64_t)blk * kBlockTiles) * g.tile_bytes;
  return base + ((int64_t)(d >> 2) * L + l) * 16 + (d & 3) * 4;
}

// Byte offset of statistic dword `d` (0 <= d < sd) of tile (tile_row, tile_col).
SPQR_HD int64_t stat_dword_offset(const Geometry& g, int32_t tile_row, int32_t tile_col, int32_t d) {
  int32_t blk = tile_col / kBlockTiles, l = tile_col % kBlockTiles;
  int32_t L = g.ntc - blk * kBlockTiles; if (L > kBlockTiles) L = kBlockTiles;
  int64_t base = ((int64_t)tile_row * g.ntc + (int64_t)blk * kBlockTiles) * g.tile_bytes
               + (int64_t)16 * g.kw * L;
  if (d < 4 * g.swf) return base + ((int64_t)(d >> 2) * L + l) * 16 + (d & 3) * 4;
  return base + (int64_t)16 * g.swf * L + ((int64_t)(d - 4 * g.swf) * L + l) * 4;
}

}  // namespace spqr
