// Address rules of the halo form of a stride-1 3x3 convolution whose rows are pixels:
//     forward         Z[b, i, j, o]  = sum over taps (u, v), channels c of In[b, i + u - 1, j + v - 1, c] * W[o, (u, v), c]
//     input gradient  dX[b, y, x, c] = sum over taps (u, v), channels o of dZ[b, y + 1 - u, x + 1 - v, o] * Wt[c, (u, v), o]
// (zero padding 1; the forward and backward passes of a packed member's convolution layer).
//
// One workgroup owns BM consecutive pixels (whole image rows of one image, or whole images) x BN output
// columns.  The gathered operand is walked in blocks of CB channels (128 bytes per pixel); per block the
// workgroup stages, once, every source pixel its pixels' nine taps can reach (the "halo": the tile's rows
// plus one row above and below, one column left and right, the padding ring as zeros) in LDS, pixel by
// pixel as they lie in memory.  The nine taps' operand tiles are nine shifted views of that block, so a
// source pixel is fetched once per channel block instead of once per tap.
//
// Everything here is plain integer arithmetic usable on the host and on the device, so that the rules the
// kernel addresses memory by can be walked on the CPU against the definition above.
#pragma once
#include "pack_internal.h"

#ifndef __HIPCC__
#define PACK_HD
#else
#define PACK_HD __host__ __device__
#endif

// PACK_HALO_PLANT (0 in every build of the library): a CPU test compiles the host-side walk with one rule
// deliberately wrong, to show that the walk notices.
#ifndef PACK_HALO_PLANT
#define PACK_HALO_PLANT 0
#endif

namespace packk {

constexpr unsigned ROWS_POISON = 0x80000000u;   // byte offset of a vector that does not exist (beyond any descriptor)

// Compile-time shape.  ESZ: bytes per element; WM x WN: grid of the four wavefronts; a wave owns 64 pixels x
// 32 * TN columns.
template <int ESZ, int WM, int WN, int TN_>
struct RowsCfg {
    static_assert(WM * WN == 4, "256 threads");
    static constexpr int TN = TN_, ESZ_ = ESZ;
    static constexpr int BM = 64 * WM, BN = 32 * TN_ * WN;
    static constexpr int CB = 128 / ESZ;                  // channels per block: 128 bytes of a pixel
    static constexpr int VE = 16 / ESZ;                   // elements per 16-byte vector
    static constexpr int MAXP = (BM == 256) ? 400 : 264;  // halo pixels that fit (the planner checks a problem against it)
    static constexpr int PIXB = 144;                      // bytes from a pixel to the next in LDS: 128 + 16, so that the
                                                          // 16-byte reads of consecutive pixels fall into different banks
    static constexpr int NLD = (MAXP * 8 + 255) / 256;    // halo vectors a thread loads per channel block
    static constexpr int HALO_BYTES = MAXP * PIXB;
};

// Run-time shape of one problem's tiles.  The "source" is the gathered operand: the layer's input (forward)
// or the gradient of its output (input gradient); at stride 1 both have the extent of the result.
struct RowsGeom {
    int SH, SW, SC;     // source rows, columns, channels
    int rows, nimg;     // a tile covers nimg images x rows rows each (nimg = 1 unless an image is smaller than a tile)
    int HWD, blk, NP;   // halo columns, halo pixels per image of the tile, halo pixels in all
    int span;           // reduction indices per tap (= SC)
    int lgW, lgPer, lgImg;   // base-2 logarithms of SW, of rows * SW and of SH * SW (all powers of two)
    unsigned mHWD, mblk;   // n / HWD = (n * mHWD) >> 20 and n / blk = (n * mblk) >> 20 for every n the kernel divides (n * d < 2^20)
    bool dx;            // input gradient: taps displace the other way
};
PACK_HD inline int rows_div(int n, unsigned magic) { return (int)(((unsigned)n * magic) >> 20); }

template <int BM>
PACK_HD inline RowsGeom rows_geom(const GemmProb& p, bool dx) {
    RowsGeom g;
    g.dx = dx;
    g.SH = p.H; g.SW = p.W; g.SC = dx ? p.Cout : p.Cin;
    const int img = p.H * p.W;
    g.nimg = img >= BM ? 1 : BM / img;
    g.rows = img >= BM ? BM / p.W : p.H;
    g.HWD = p.W + 2;
    g.blk = (g.rows + 2) * g.HWD;
    g.NP = g.nimg * g.blk;
    g.span = g.SC;
    g.lgW = 31 - __builtin_clz((unsigned)g.SW);
    g.lgPer = 31 - __builtin_clz((unsigned)(g.rows * g.SW));
    g.lgImg = 31 - __builtin_clz((unsigned)(g.SH * g.SW));
    g.mHWD = ((1u << 20) + (unsigned)g.HWD - 1) / (unsigned)g.HWD;
    g.mblk = ((1u << 20) + (unsigned)g.blk - 1) / (unsigned)g.blk;
    return g;
}

// Whether a problem can take this form; everything the kernel assumes is listed here and nowhere else.
// (Alignment of the operands for 16-byte loads is the caller's F_VEC_A / F_VEC_B.)
template <class Cfg>
PACK_HD inline bool rows_halo_supported(const GemmProb& p, bool dx) {
    if (p.stride != 1 || (p.flags & F_ROWMAP)) return false;
    if (p.Ho != p.H || p.Wo != p.W) return false;
    const int sc = dx ? p.Cout : p.Cin;
    if (sc % Cfg::CB) return false;
    if (p.Kd != 9 * sc || p.ksplit < p.Kd) return false;
    if (p.Kd < 512 && Cfg::BN > 32) return false;                      // (measured: a reduction that short is no faster here than on the staged tiles)
    if (p.W < 4 || (p.W & (p.W - 1)) || (p.H & (p.H - 1))) return false;                    // rows and pixels are found by shifts
    const int img = p.H * p.W;
    if (img >= Cfg::BM ? (Cfg::BM % p.W || img % Cfg::BM) : (Cfg::BM % img)) return false;
    if (p.R % Cfg::BM) return false;                                   // no ragged last tile
    const RowsGeom g = rows_geom<Cfg::BM>(p, dx);
    if (g.NP > Cfg::MAXP) return false;
    if ((long long)Cfg::NLD * 256 / 8 * g.blk >= (1 << 20)) return false;                   // range of the multiply-shift divisions
    if ((double)(g.nimg + 1) * img * sc * Cfg::ESZ_ >= 1.0e9) return false;   // offsets inside a tile's images stay far from the poison value
    return true;
}

// first image and first row (within it) of tile tm
template <int BM>
PACK_HD inline void rows_tile_origin(const GemmProb& p, const RowsGeom& g, int tm, int& b0, int& y0) {
    const int px0 = tm * BM;
    b0 = px0 >> g.lgImg;
    y0 = (px0 & ((1 << g.lgImg) - 1)) >> g.lgW;
}

// Halo vector v of a tile (v = pixel slot * 8 + part; slot = image of the tile * blk + halo row * HWD + halo
// column): byte offset from the first element of image b0, channel block 0, or ROWS_POISON for a pixel of
// the padding ring or a vector beyond the halo.  The channel block adds cb * 128 bytes.
template <class Cfg, int ESZ>
PACK_HD inline unsigned rows_vec_offset(const RowsGeom& g, int y0, int v) {
    const int slot = v >> 3, part = v & 7;
    if (slot >= g.NP) return ROWS_POISON;
    const int ii = rows_div(slot, g.mblk), rem = slot - ii * g.blk;
    const int hr = rows_div(rem, g.mHWD), hc = rem - hr * g.HWD;
    const int y = y0 + hr - 1, x = hc - 1 + (PACK_HALO_PLANT == 6);
    if (y < 0 || y >= g.SH || x < 0 || x >= g.SW) return ROWS_POISON;
    return (unsigned)((((ii * g.SH + y) * g.SW + x) * g.SC) * ESZ + part * 16);
}
// where halo vector v goes in the LDS halo block
template <class Cfg>
PACK_HD inline int rows_lds_offset(int v) { return (v >> 3) * Cfg::PIXB + (v & 7) * 16; }

// LDS pixel slot of the halo pixel at displacement (-1, -1) from pixel m of the tile (m in [0, BM))
PACK_HD inline int rows_slot(const RowsGeom& g, int m) {
    const int ii = m >> g.lgPer, rem = m & ((1 << g.lgPer) - 1);
    return ii * g.blk + (rem >> g.lgW) * g.HWD + (rem & (g.SW - 1));
}
// slots from there to the pixel tap (u, v) reads
PACK_HD inline int rows_tap_slots(const RowsGeom& g, int u, int v) {
    return (g.dx && PACK_HALO_PLANT != 5) ? (2 - u) * g.HWD + (2 - v) : u * g.HWD + v;
}

}  // namespace packk
