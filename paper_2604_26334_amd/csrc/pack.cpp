// Host packer: logical (scales, codes) rows -> the private device layout.
//
// Physical layout of one row-tile (16 rows, full K), chosen so that one 64-lane wavefront
// reads it as a contiguous stream of 16-byte loads and so that a lane's 4 dwords are,
// unchanged, the A operands of four 16x16x32 fp16 MFMA steps:
//   lane = c*16 + i  (i = row in tile, c = 0..3)
//   super-block sb (128 k) = 64 lanes x 16 B; lane (i, c) holds block b = 4*sb + c of row i,
//     dword kk (0..3) = the 8 weights k = 32*b + 8*kk + t, t = 0..7,
//     weight t sits in nibble position (t >> 1) + 4 * (t & 1), so the masks 0x000F000F /
//     0x00F000F0 on the dword (and on dword >> 8) pull out the pairs (t0,t1) (t2,t3) (t4,t5) (t6,t7)
//   scale group g (8 super-blocks): its nibble super-blocks, then 64 lanes x 16 B of scales,
//     lane (i, c) half s = scale of block 4*(8g+s)+c of row i (0 past the end of the row)
#include <algorithm>
#include <cstring>

#include "ps_internal.h"

namespace ps {

void pack_tile(const MatGeom &g, const uint16_t *scales, const uint8_t *codes,
               uint32_t logical_tile, uint8_t *dst) {
    const uint32_t K = g.K, nb = K / 32;
    const size_t row0 = (size_t)logical_tile * kTileRows;
    for (uint32_t grp = 0; grp < g.ngroups; ++grp) {
        const uint32_t nsb_g = std::min(kGroupSb, g.nsb - grp * kGroupSb);
        uint8_t *gbase = dst + (size_t)grp * (kGroupSb + 1) * kSbBytes;
        for (uint32_t s = 0; s < nsb_g; ++s) {
            const uint32_t sb = grp * kGroupSb + s;
            uint32_t *out = reinterpret_cast<uint32_t *>(gbase + (size_t)s * kSbBytes);
            for (uint32_t lane = 0; lane < 64; ++lane) {
                const uint32_t i = lane & 15, c = lane >> 4;
                const uint8_t *q = codes + (row0 + i) * K + (size_t)(4 * sb + c) * 32;
                for (uint32_t kk = 0; kk < 4; ++kk) {
                    uint32_t v = 0;
                    for (uint32_t t = 0; t < 8; ++t)
                        v |= (uint32_t)(q[8 * kk + t] & 15u) << (4 * ((t >> 1) + 4 * (t & 1)));
                    out[lane * 4 + kk] = v;
                }
            }
        }
        uint16_t *sc = reinterpret_cast<uint16_t *>(gbase + (size_t)nsb_g * kSbBytes);
        for (uint32_t lane = 0; lane < 64; ++lane) {
            const uint32_t i = lane & 15, c = lane >> 4;
            for (uint32_t s = 0; s < kGroupSb; ++s) {
                const uint32_t b = 4 * (grp * kGroupSb + s) + c;
                sc[lane * 8 + s] = (s < nsb_g) ? scales[(row0 + i) * nb + b] : (uint16_t)0;
            }
        }
    }
}

}  // namespace ps

extern "C" int32_t ps_pack_matrix(const uint16_t *scales, const uint8_t *codes, uint32_t rows, uint32_t K,
                                  uint8_t *out) {
    if (!scales || !codes || !out || K == 0 || K % ps::kSuperK || K > 16384 || rows == 0 || rows % ps::kTileRows) {
        ps::set_error("ps_pack_matrix: need K %% 128 == 0, K <= 16384, rows %% 16 == 0");
        return PS_E_ARG;
    }
    const ps::MatGeom g = ps::make_geom(rows, K, false);
    for (uint32_t t = 0; t < g.ntiles; ++t) ps::pack_tile(g, scales, codes, t, out + (uint64_t)t * g.tile_bytes);
    return PS_OK;
}
