// Host-side packer and size model of the packed layouts.  No GPU calls.
#include <algorithm>
#include <atomic>
#include <cstring>
#include <thread>
#include <vector>

#include "../../include/spqr.h"
#include "spqr_layout.h"

using spqr::Geometry;

extern "C" int64_t spqr_packed_bytes(int32_t m, int32_t n, int32_t w_bits, int32_t s_bits,
                                     int32_t z_bits, int32_t beta1, int32_t beta2,
                                     int32_t group_axis) {
  return spqr_packed_bytes_layout(SPQR_LAYOUT_V1, m, n, w_bits, s_bits, z_bits, beta1, beta2, group_axis);
}

extern "C" int64_t spqr_packed_bytes_layout(int32_t layout_version, int32_t m, int32_t n, int32_t w_bits,
                                            int32_t s_bits, int32_t z_bits, int32_t beta1, int32_t beta2,
                                            int32_t group_axis) {
  Geometry g;
  int rc = spqr::make_geometry(layout_version, m, n, w_bits, s_bits, z_bits, beta1, beta2, group_axis, &g);
  if (rc) return rc;
  return (int64_t)g.ntr * g.ntc * g.tile_bytes;
}

namespace {

// Store one pair (lo, hi) of `bits`-bit codes as pair number q of dword array d.
inline void put_pair(uint32_t* d, int bits, int q, uint32_t lo, uint32_t hi) {
  spqr::PairLoc p = spqr::pair_loc(bits, q);
  if (!p.split) {
    d[p.dword] |= (lo << p.shift) | (hi << (p.shift + 16));
  } else {
    for (int i = 0; i < 3; ++i)
      d[p.dword + i] |= (((lo >> i) & 1u) << 15) | (((hi >> i) & 1u) << 31);
  }
}

}  // namespace

extern "C" int spqr_pack_host(int32_t m, int32_t n, int32_t w_bits, int32_t s_bits, int32_t z_bits,
                              int32_t beta1, int32_t beta2, int32_t group_axis,
                              const uint8_t* Q, const uint8_t* s_q, const uint8_t* z_q,
                              const uint16_t* s_s, const uint16_t* z_s,
                              const uint16_t* s_z, const uint16_t* z_z,
                              void* packed_out, int64_t packed_bytes) {
  return spqr_pack_host_layout(SPQR_LAYOUT_V1, m, n, w_bits, s_bits, z_bits, beta1, beta2, group_axis, Q, s_q, z_q,
                               s_s, z_s, s_z, z_z, packed_out, packed_bytes);
}

extern "C" int spqr_pack_host_layout(int32_t layout_version, int32_t m, int32_t n, int32_t w_bits,
                                     int32_t s_bits, int32_t z_bits, int32_t beta1, int32_t beta2,
                                     int32_t group_axis, const uint8_t* Q, const void* s_first,
                                     const void* z_first, const uint16_t* s_s, const uint16_t* z_s,
                                     const uint16_t* s_z, const uint16_t* z_z, void* packed_out,
                                     int64_t packed_bytes) {
  Geometry g;
  int rc = spqr::make_geometry(layout_version, m, n, w_bits, s_bits, z_bits, beta1, beta2, group_axis, &g);
  if (rc) return rc;
  const bool codes = g.layout != spqr::kStats16;     // first-level statistics are 3-bit codes
  if (!Q || !s_first || !z_first || !packed_out) return SPQR_ERR_NULL;
  if (codes && (!s_s || !z_s)) return SPQR_ERR_NULL;
  if (g.layout == spqr::kBilevel && (!s_z || !z_z)) return SPQR_ERR_NULL;
  if (packed_bytes != (int64_t)g.ntr * g.ntc * g.tile_bytes) return SPQR_ERR_SIZE;
  const uint8_t* s_q = static_cast<const uint8_t*>(s_first);
  const uint8_t* z_q = static_cast<const uint8_t*>(z_first);
  const uint16_t* s16 = static_cast<const uint16_t*>(s_first);
  const uint16_t* z16 = static_cast<const uint16_t*>(z_first);

  uint8_t* out = static_cast<uint8_t*>(packed_out);
  const int cd = 4 * g.kw;                 // code dwords per tile
  const int ppr = g.tile_cols / 2;         // pairs per tile row
  const uint32_t wmax = 1u << w_bits;
  const int64_t gcols = group_axis == 0 ? n / beta1 : n;   // row stride of s_q / z_q
  std::atomic<int> bad{0};

  auto work = [&](int tr_begin, int tr_end) {
    std::vector<uint32_t> code(cd), stat(g.sd);
    for (int tr = tr_begin; tr < tr_end; ++tr) {
      for (int tc = 0; tc < g.ntc; ++tc) {
        std::fill(code.begin(), code.end(), 0u);
        std::fill(stat.begin(), stat.end(), 0u);
        const int64_t r0 = (int64_t)tr * g.tile_rows, c0 = (int64_t)tc * g.tile_cols;
        for (int r = 0; r < g.tile_rows; ++r) {
          const uint8_t* row = Q + (r0 + r) * n + c0;
          for (int p = 0; p < ppr; ++p) {
            uint32_t lo = row[2 * p], hi = row[2 * p + 1];
            if (lo >= wmax || hi >= wmax) { bad.store(1); lo &= wmax - 1; hi &= wmax - 1; }
            put_pair(code.data(), w_bits, r * ppr + p, lo, hi);
          }
        }
        const int64_t t = (int64_t)tr * g.ntc + tc;
        auto group_index = [&](int gi) -> int64_t {
          return group_axis == 0 ? (r0 + gi) * gcols + tc            // group = row of the tile
                                 : (int64_t)tr * gcols + c0 + gi;    // group = column of the tile
        };
        if (codes) {
          // statistic codes of the beta2 groups of this tile: s_q[0..beta2), z_q[0..beta2)
          for (int which = 0; which < 2; ++which) {
            const uint8_t* src = which == 0 ? s_q : z_q;
            for (int gq = 0; gq < beta2 / 2; ++gq) {
              uint32_t v[2];
              for (int h = 0; h < 2; ++h) {
                v[h] = src[group_index(2 * gq + h)];
                if (v[h] >= 8u) { bad.store(1); v[h] &= 7u; }
              }
              put_pair(stat.data(), 3, which * (beta2 / 2) + gq, v[0], v[1]);
            }
          }
          const int nc = 3 * beta2 / 16;
          stat[nc] = (uint32_t)s_s[t] | ((uint32_t)z_s[t] << 16);
          if (g.layout == spqr::kBilevel) stat[nc + 1] = (uint32_t)s_z[t] | ((uint32_t)z_z[t] << 16);
        } else {
          for (int gi = 0; gi < beta2; ++gi)
            stat[gi] = (uint32_t)s16[group_index(gi)] | ((uint32_t)z16[group_index(gi)] << 16);
        }
        for (int d = 0; d < cd; ++d)
          std::memcpy(out + spqr::code_dword_offset(g, tr, tc, d), &code[d], 4);
        for (int d = 0; d < g.sd; ++d)
          std::memcpy(out + spqr::stat_dword_offset(g, tr, tc, d), &stat[d], 4);
      }
    }
  };

  unsigned hw = std::thread::hardware_concurrency();
  int nthreads = (int)std::max(1u, std::min(hw ? hw : 1u, 16u));
  nthreads = std::min(nthreads, g.ntr);
  if ((int64_t)m * n < (1 << 20)) nthreads = 1;
  if (nthreads == 1) {
    work(0, g.ntr);
  } else {
    std::vector<std::thread> th;
    int per = (g.ntr + nthreads - 1) / nthreads;
    for (int i = 0; i < nthreads; ++i) {
      int a = i * per, b = std::min(g.ntr, a + per);
      if (a < b) th.emplace_back(work, a, b);
    }
    for (auto& t : th) t.join();
  }
  return bad.load() ? SPQR_ERR_PARAM : SPQR_OK;
}

extern "C" const char* spqr_strerror(int status) {
  switch (status) {
    case SPQR_OK:            return "ok";
    case SPQR_ERR_NULL:      return "required pointer is NULL";
    case SPQR_ERR_SHAPE:     return "matrix shape is not a positive multiple of the tile or n > 65536";
    case SPQR_ERR_PARAM:     return "unsupported bit width, group size, axis or layout version";
    case SPQR_ERR_SIZE:      return "buffer size does not match the format's closed form";
    case SPQR_ERR_ALIGN:     return "buffer is misaligned";
    case SPQR_ERR_CSR:       return "outlier CSR arrays are not a valid sorted row-major set";
    case SPQR_ERR_NONFINITE: return "non-finite 16-bit statistic or outlier value";
    case SPQR_ERR_BATCH:     return "batch size out of range";
    case SPQR_ERR_HIP:       return "HIP runtime call or kernel launch failed";
    case SPQR_ERR_DTYPE:     return "unknown output dtype or selector";
    case SPQR_ERR_WORKSPACE: return "workspace smaller than spqr_workspace_bytes() says, or beyond the static scratch";
    default:                 return "unknown status";
  }
}

extern "C" int32_t spqr_version(void) { return (1 << 16) | SPQR_LAYOUT_STATS16; }
