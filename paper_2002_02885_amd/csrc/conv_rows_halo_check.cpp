// Host-side walk of the address rules of the halo form of the stride-1 convolution forward pass and
// input gradient (conv_rows_halo.h) against the definition of the operation: for one tile, every global
// load the kernel's threads issue for a channel block must lie inside the images the tile's descriptor
// covers, and every 16-byte fragment a lane reads from LDS for (pixel block, tap, reduction step) must hold
// exactly the source pixel and channels the definition pairs with the lane's output pixel, or zeros where
// that pixel lies in the padding ring.  Used by pack_plan_check; nothing here touches a device.
#include "conv_rows_halo.h"

#include <string>
#include <vector>

namespace packk {
namespace {

template <int ESZ, int TN>
std::string walk_rows_tile(const GemmProb& p, const TileRef& tr, bool dx, long long a_bytes, long long* loads, long long* frag_reads) {
    typedef RowsCfg<ESZ, 4, 1, TN> Cfg;
    constexpr int BM = Cfg::BM, V = Cfg::VE;
    if (!rows_halo_supported<Cfg>(p, dx)) return "the problem does not fit the form its launch was given";
    const RowsGeom g = rows_geom<BM>(p, dx);
    int b0, y0;
    rows_tile_origin<BM>(p, g, tr.tm, b0, y0);
    const long long img_bytes = (long long)g.SH * g.SW * g.SC * ESZ, desc_size = g.nimg * img_bytes;
    if (b0 < 0 || (long long)b0 * img_bytes + desc_size > a_bytes) return "the tile's images are not inside the operand";
    const int ncb = g.SC / Cfg::CB;
    // what each 16-byte slot of the LDS halo block holds after a channel block has been staged: the byte offset
    // (inside the descriptor, channel block 0) it was loaded from, -1 for zeros, -2 if nothing wrote it
    std::vector<long long> lds((size_t)Cfg::MAXP * 8, -2);
    for (int tid = 0; tid < 256; ++tid)
        for (int i = 0; i < Cfg::NLD; ++i) {
            const int v = tid + 256 * i;
            if (v >= Cfg::MAXP * 8) continue;   // (the kernel skips the store)
            const unsigned off = rows_vec_offset<Cfg, ESZ>(g, y0, v);
            const int at = rows_lds_offset<Cfg>(v);
            if (at % 16 || at / Cfg::PIXB >= Cfg::MAXP || at % Cfg::PIXB + 16 > 128) return "a halo vector is stored outside the LDS block";
            long long& cell = lds[(size_t)(at / Cfg::PIXB) * 8 + (at % Cfg::PIXB) / 16];
            if (cell != -2) return "two halo vectors go to one LDS slot";
            if (off == ROWS_POISON) { cell = -1; continue; }
            if ((long long)off + (long long)(ncb - 1) * 128 + 16 > desc_size) return "a halo load leaves the tile's images";
            cell = off;
            ++*loads;
        }
    for (int wm = 0; wm < 4; ++wm)
        for (int a = 0; a < 2; ++a)
            for (int lane = 0; lane < 64; ++lane) {
                const int m = wm * 64 + a * 32 + (lane & 31), half = lane >> 5;
                const int r = tr.tm * BM + m;
                const int b = r / (g.SH * g.SW), y = (r / g.SW) % g.SH, x = r % g.SW;
                for (int tap = 0; tap < 9; ++tap) {
                    const int u = tap / 3, v = tap % 3;
                    const int sy = dx ? y + 1 - u : y + u - 1, sx = dx ? x + 1 - v : x + v - 1;
                    for (int kk = 0; kk < Cfg::CB; kk += 2 * V) {
                        const int byte = (rows_slot(g, m) + rows_tap_slots(g, u, v)) * Cfg::PIXB + half * 16 + kk * ESZ;
                        const int slot = byte / Cfg::PIXB, within = byte % Cfg::PIXB;
                        if (byte < 0 || slot >= Cfg::MAXP || within + 16 > 128) return "a fragment read leaves the halo block";
                        const long long have = lds[(size_t)slot * 8 + within / 16];
                        if (have == -2) return "a fragment read meets an LDS slot nothing wrote";
                        const bool inside = sy >= 0 && sy < g.SH && sx >= 0 && sx < g.SW;
                        const long long want = inside ? ((((long long)(b - b0) * g.SH + sy) * g.SW + sx) * g.SC + kk + half * V) * ESZ : -1;
                        if (have != want) return "a fragment read meets the wrong source pixel or channels";
                        ++*frag_reads;
                    }
                }
            }
    return std::string();
}

}  // namespace

// One tile of a rows-halo launch; bf16 / narrow (32 output columns per tile) select the instantiation, dx the
// direction.  a_bytes: size of the gathered operand.  Returns an empty string or what is wrong.
std::string conv_rows_halo_walk(bool bf16, bool narrow, bool dx, const GemmProb& p, const TileRef& tr, long long a_bytes,
                                long long* loads, long long* frag_reads) {
    if (bf16) return narrow ? walk_rows_tile<2, 1>(p, tr, dx, a_bytes, loads, frag_reads) : walk_rows_tile<2, 2>(p, tr, dx, a_bytes, loads, frag_reads);
    return narrow ? walk_rows_tile<4, 1>(p, tr, dx, a_bytes, loads, frag_reads) : walk_rows_tile<4, 2>(p, tr, dx, a_bytes, loads, frag_reads);
}

}  // namespace packk
