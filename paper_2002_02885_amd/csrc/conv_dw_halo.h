// Address rules of the halo form of the convolution weight gradient
//     dW[o, (u, v), c] = sum over output pixels (b, i, j) of dZ[b, i, j, o] * In[b, s*i + u - 1, s*j + v - 1, c]
// (the backward pass of a packed member's 3x3 convolution, zero padding 1, stride s = 1 or 2).
//
// One workgroup owns CO_T output channels x CI_T input channels x all nine taps and walks the output
// pixels of its split in chunks of CH consecutive pixels (whole image rows).  Per chunk it stages, once,
// the rows of the input the chunk's nine taps can reach (the "halo": rows s*i0 - 1 .. s*(i0 + rows - 1) + 1,
// columns -1 .. s*(Wo - 1) + 1, the padding ring included as zeros) and the chunk's dZ rows in LDS, pixel
// by pixel as they lie in memory (channels contiguous); the nine taps' operand tiles are then nine shifted
// views of the same LDS block, so an input pixel is fetched once per chunk instead of once per tap.
//
// Everything here is plain integer arithmetic usable on the host and on the device, so that the rules the
// kernel addresses memory by can be walked on the CPU against the definition above (conv_dw_halo_check).
#pragma once
#include "pack_internal.h"

#ifndef __HIPCC__
#define PACK_HD
#else
#define PACK_HD __host__ __device__
#endif

// PACK_HALO_PLANT (0 in every build of the library): a CPU test compiles the host-side walk with one rule
// deliberately wrong, to show that the walk notices (tests/test_plan_check_host.py).
#ifndef PACK_HALO_PLANT
#define PACK_HALO_PLANT 0
#endif

namespace packk {

constexpr unsigned HALO_POISON = 0x80000000u;   // byte offset of a vector that does not exist (beyond any image)

// Compile-time shape of one kernel instantiation.  ESZ: bytes per element (2 = bfloat16, 4 = float);
// WM x WN: grid of wavefronts, each owning a 32 x 32 block of (output channel, input channel); TG: the nine
// taps of a block are dealt over TG waves (1: one wave holds all nine; 2: taps 0-4 and taps 5-8; 3: one tap row each), i.e.
// TG waves per SIMD, which hide each other's waits.
template <int ESZ, int WM, int WN, int STRIDE, int TG_ = 1>
struct HaloCfg {
    static constexpr int S = STRIDE, TG = TG_;
    static constexpr int NT = 64 * WM * WN * TG;         // threads per workgroup
    static constexpr int CH = (ESZ == 2) ? 64 : 32;      // output pixels per chunk (the reduction runs in ascending chunks of this many)
    static constexpr int CO_T = 32 * WM, CI_T = 32 * WN;
    static constexpr int VE = 16 / ESZ;                  // elements per 16-byte vector
    static constexpr int VPP_A = CO_T / VE, VPP_B = CI_T / VE;   // vectors per pixel of the dZ / input block
    static constexpr int NLA = (CH * VPP_A + NT - 1) / NT;   // dZ vectors a thread loads per chunk (threads beyond the block load none)
    static constexpr int NLD = (((STRIDE == 1) ? 7 : 11) + TG - 1) / TG;   // halo vectors a thread loads per chunk (upper bound; the planner checks it)
    static constexpr int MAX_SLOTS = NLD * NT / VPP_B;   // halo pixels that fit those loads
    // bytes from one pixel to the next in LDS: the channels plus padding chosen so that the 32 lanes that a
    // transposing read serves together (four consecutive output pixels, i.e. halo pixels S apart, 64 bytes of
    // each) fall into four different 64-byte windows of the 256 bytes the banks span: S * PIXB = 64 or 192 (mod 256)
    static constexpr int PIXB_A = CO_T * ESZ + ((ESZ == 2) ? 64 : 0);
    static constexpr int PIXB_B = CI_T * ESZ + ((ESZ == 2) ? ((STRIDE == 1) ? (WN == 2 ? 64 : 0) : 32) : 0);
    static constexpr int HALO_BYTES = MAX_SLOTS * PIXB_B, DZ_BYTES = CH * PIXB_A;
    static constexpr int LDS_BYTES = 2 * (HALO_BYTES + DZ_BYTES);   // two buffers of each
};

// Run-time shape of one problem.
struct HaloGeom {
    int S, H, W, Cin, Cout, Ho, Wo, lgWo;
    int rows;        // output rows per chunk
    int NR, HWD;     // halo rows and columns per chunk
    int img_px;      // output pixels per image
    int row_bytes;   // bytes of one input row (W * Cin elements)
    long long img_bytes;   // bytes of one input image
};

template <int ESZ, int CH>
PACK_HD inline HaloGeom halo_geom(const GemmProb& p) {
    HaloGeom g;
    g.S = p.stride; g.H = p.H; g.W = p.W; g.Cin = p.Cin; g.Cout = p.Cout; g.Ho = p.Ho; g.Wo = p.Wo;
    g.lgWo = 0;
    while ((1 << g.lgWo) < p.Wo) ++g.lgWo;
    g.rows = CH / p.Wo;
    g.NR = p.stride * (g.rows - 1) + 3;
    g.HWD = p.stride * (p.Wo - 1) + 3;
    g.img_px = p.Ho * p.Wo;
    g.row_bytes = p.W * p.Cin * ESZ;
    g.img_bytes = (long long)p.H * g.row_bytes;
    return g;
}

// Whether a problem can take the halo form built as Cfg; everything the kernel assumes is listed here and
// nowhere else.  (Operand alignment for 16-byte loads is the caller's F_VEC_A / F_VEC_B.)
template <class Cfg, int ESZ>
PACK_HD inline bool halo_supported(const GemmProb& p) {
    if (p.stride != Cfg::S || p.Cin % Cfg::CI_T || p.Cout % Cfg::CO_T) return false;
    if (p.Wo < 8 || p.Wo > Cfg::CH || (p.Wo & (p.Wo - 1))) return false;          // chunks are whole rows; eight pixels of a row per fragment
    if ((p.Ho * p.Wo) % Cfg::CH) return false;                                      // a chunk never straddles two images
    if (p.Ho != (p.H - 1) / p.stride + 1 || p.Wo != (p.W - 1) / p.stride + 1) return false;
    if (p.Kd % Cfg::CH || p.ksplit % Cfg::CH) return false;                         // splits are whole chunks
    const HaloGeom g = halo_geom<ESZ, Cfg::CH>(p);
    if (g.NR * g.HWD > Cfg::MAX_SLOTS) return false;
    if (g.img_bytes + 2ll * g.row_bytes >= 0x40000000ll) return false;              // offsets inside an image stay far from the poison value
    if ((double)p.Kd * p.Cout * ESZ >= 2.0e9) return false;                         // dZ is addressed with 32-bit byte offsets
    return true;
}

// Where a chunk lies: its image and its first output pixel inside that image.  The kernel finds it once per
// tile and then steps from chunk to chunk (a chunk never straddles two images), without a division per chunk.
struct HaloCursor {
    int img, pix;
};
PACK_HD inline HaloCursor halo_cursor(const HaloGeom& g, int k0) {
    HaloCursor c;
    c.img = k0 / g.img_px;
    c.pix = k0 - c.img * g.img_px;
    return c;
}
PACK_HD inline void halo_cursor_advance(const HaloGeom& g, int chunk, HaloCursor& c) {
    c.pix += chunk;
    if (c.pix >= g.img_px) {
        c.pix -= g.img_px;
        ++c.img;
    }
}

// ---- global -> LDS ---------------------------------------------------------------------------------
// Halo vector number v of a chunk (v = pixel slot * VPP_B + part; slot = halo row * HWD + halo column):
// its byte offset from the first element of halo row 0, image column 0, channel c0 of the image the chunk
// lies in, or HALO_POISON for a column of the padding ring or a vector beyond the halo.  The chunk's own
// part, halo_row_offset, is added to it; rows above or below the image then leave the image's byte range
// (below zero, which wraps to the top of the unsigned range, or beyond its end) and read as zeros.
template <class Cfg, int ESZ>
PACK_HD inline unsigned halo_vec_offset(const HaloGeom& g, int c0, int v) {
    const int slot = v / Cfg::VPP_B, part = v % Cfg::VPP_B;
    if (slot >= g.NR * g.HWD) return HALO_POISON;
    const int ry = slot / g.HWD, x = slot % g.HWD - 1;
    if (x < 0 || (x >= g.W && PACK_HALO_PLANT != 3)) return HALO_POISON;
    return (unsigned)(ry * g.row_bytes + (x * g.Cin + c0) * ESZ + part * 16);
}
// bytes from the image's first row to halo row 0 of the chunk whose first output row is i0 (negative for i0 = 0)
PACK_HD inline int halo_row_offset(const HaloGeom& g, int i0) { return (g.S * i0 - 1 + (PACK_HALO_PLANT == 1)) * g.row_bytes; }
// where halo vector v goes in the LDS halo block
template <class Cfg>
PACK_HD inline int halo_lds_offset(int v) { return (v / Cfg::VPP_B) * Cfg::PIXB_B + (v % Cfg::VPP_B) * 16; }
// dZ vector v of a chunk (v = pixel * VPP_A + part): byte offset from the chunk's first pixel, channel o0
template <class Cfg, int ESZ>
PACK_HD inline unsigned dz_vec_offset(const HaloGeom& g, int o0, int v) {
    if (v >= Cfg::CH * Cfg::VPP_A) return HALO_POISON;
    return (unsigned)(((v / Cfg::VPP_A) * g.Cout + o0) * ESZ + (v % Cfg::VPP_A) * 16);
}
template <class Cfg>
PACK_HD inline int dz_lds_offset(int v) { return (v / Cfg::VPP_A) * Cfg::PIXB_A + (v % Cfg::VPP_A) * 16; }

// ---- LDS -> matrix-instruction operands ---------------------------------------------------------------
// LDS pixel slot of the input pixel that tap (0, 0) pairs with output pixel q of the chunk (q in [0, CH));
// tap (u, v) reads halo_tap_slots(u, v) slots further on.
PACK_HD inline int halo_slot(const HaloGeom& g, int q) { return ((q >> g.lgWo) * g.S) * g.HWD + (q & (g.Wo - 1)) * (PACK_HALO_PLANT == 4 ? 1 : g.S); }
PACK_HD inline int halo_tap_slots(const HaloGeom& g, int u, int v) { return u * g.HWD + v; }

// bfloat16, matrix instruction 32x32x16: a lane holds eight consecutive reduction indices (pixels) of one
// row (channel) of its operand, lanes 0-31 the first eight of a step of sixteen, lanes 32-63 the second
// eight.  They come from two transposing 8-byte LDS reads: in each group of sixteen lanes, lane s supplies
// the address of four consecutive channels of pixel (s / 4) of four consecutive pixels, and receives those
// four pixels of channel s of the group's sixteen channels.
// frag_pixel: first of the four pixels (relative to the chunk) lane `lane` addresses in read `r` (0 or 1) of step kk;
// frag_channel: first of the four channels it addresses, relative to the wave's 32-channel block.
PACK_HD inline int frag_pixel_bf16(int lane, int kk, int r) { return kk * 16 + (lane >> 5) * 8 + r * 4 + ((lane & 15) >> 2); }
PACK_HD inline int frag_channel_bf16(int lane) { return (((lane >> 4) & 1) ^ (PACK_HALO_PLANT == 2)) * 16 + (lane & 3) * 4; }
// what the lane ends up holding after the two reads: element e (0..7) is pixel, channel
PACK_HD inline int frag_holds_pixel_bf16(int lane, int kk, int e) { return kk * 16 + (lane >> 5) * 8 + e; }
PACK_HD inline int frag_holds_channel(int lane) { return lane & 31; }

// float, matrix instruction 32x32x2: a lane holds ONE reduction index of one row: lanes 0-31 pixel A,
// lanes 32-63 pixel B of the step.  Eight pixels are consumed by four instructions that pair pixel j with
// pixel j + 4 (j = 0..3), the pairing and order of the staged-tile form of the same product.
PACK_HD inline int frag_pixel_f32(int lane, int k8, int j) { return k8 * 8 + j + (lane >> 5) * 4; }

// taps of tap group tg: first tap and number of taps
template <int TG> PACK_HD constexpr int tap_first(int tg) { return TG == 1 ? 0 : TG == 2 ? (tg == 0 ? 0 : 5) : 3 * tg; }
template <int TG> PACK_HD constexpr int tap_count(int tg) { return TG == 1 ? 9 : TG == 2 ? (tg == 0 ? 5 : 4) : 3; }

}  // namespace packk
