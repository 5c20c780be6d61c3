// Host-side walk of the halo weight-gradient kernel's address rules (conv_dw_halo.h) against the
// definition of the product.  No GPU is involved: the kernel's data movement is replayed symbolically.
//
// For one tile the walk follows the kernel step by step: per chunk, every thread's loads (descriptor,
// byte offset, range check as the hardware applies it to a raw buffer) are resolved to "element number
// of the input tensor" or "zero" and written to a model of the LDS block; then every lane's fragment
// reads (the transposing 8-byte reads for bfloat16, the 4-byte reads for float) are resolved through that
// model, and what the lane would hold in slot e of its matrix-instruction operand is compared with what the
// definition  dW[o,(u,v),c] = sum_(b,i,j) dZ[b,i,j,o] * In[b, s*i+u-1, s*j+v-1, c]  says belongs there.
// It also checks that no load that the range check lets through leaves its tensor, that a load the kernel
// means to suppress is indeed out of range, and that the tiles of a problem write every element of the
// gradient (or of each partial) exactly once.
#include "conv_dw_halo.h"

#include <cstdint>
#include <string>
#include <vector>

namespace packk {

namespace {

struct Walk {
    std::string err;
    long long loads = 0, frag_reads = 0;
    bool fail(const std::string& m) {
        if (err.empty()) err = m;
        return false;
    }
};

constexpr long long ZERO = -1;      // symbolic value: the load returned zeros
constexpr long long UNSET = -2;     // LDS position never written

template <int ESZ, int WM, int WN, int STRIDE, int TG = 1>
bool walk_tile(const GemmProb& p, const TileRef& tr, long long a_bytes, long long b_bytes, bool every_chunk, Walk& w) {
    typedef HaloCfg<ESZ, WM, WN, STRIDE, TG> Cfg;
    constexpr int NT = Cfg::NT, CH = Cfg::CH, VE = Cfg::VE;
    if (!halo_supported<Cfg, ESZ>(p)) return w.fail("problem does not satisfy halo_supported");
    const HaloGeom g = halo_geom<ESZ, CH>(p);
    const int o0 = tr.tm * Cfg::CO_T, c0 = tr.tn * Cfg::CI_T;
    if (o0 + Cfg::CO_T > p.Cout || c0 + Cfg::CI_T > p.Cin) return w.fail("tile beyond the channel extents");
    const int kbeg = tr.ks * p.ksplit;
    const int kend = std::min(p.Kd, kbeg + p.ksplit);
    if (kbeg >= kend || (kend - kbeg) % CH) return w.fail("split is not a whole number of chunks");
    const int nk = (kend - kbeg) / CH;
    const int nvec = g.NR * g.HWD * Cfg::VPP_B;
    if (nvec > Cfg::NLD * NT) return w.fail("halo does not fit the loads a thread issues");
    if (nvec * 16 / Cfg::VPP_B / 16 * Cfg::PIXB_B > Cfg::HALO_BYTES) return w.fail("halo does not fit its LDS block");

    // symbolic LDS: one entry per element position of the halo block and of the dZ block
    std::vector<long long> halo((size_t)Cfg::HALO_BYTES / ESZ), dz((size_t)Cfg::DZ_BYTES / ESZ);
    HaloCursor cur = halo_cursor(g, kbeg);     // the kernel's way from chunk to chunk
    for (int t = 0; t < nk + 3; ++t) {        // the kernel prefetches up to three chunks beyond the reduction
        const bool live = t < nk;
        const int k0 = kbeg + t * CH;
        const int img = live ? k0 / g.img_px : 0;
        const int i0 = live ? ((k0 - img * g.img_px) >> g.lgWo) : 0;
        if (live && (cur.img != img || (cur.pix >> g.lgWo) != i0 || (cur.pix & (g.Wo - 1)))) return w.fail("the chunk cursor is not where the chunk lies");
        halo_cursor_advance(g, CH, cur);
        if (live && (k0 % g.img_px) + CH > g.img_px) return w.fail("chunk straddles two images");
        const unsigned records = live ? (unsigned)g.img_bytes : 0u;
        const unsigned roff = (unsigned)halo_row_offset(g, i0);
        const bool first = t == 0 || ((k0 % g.img_px) == 0), last = t + 1 >= nk || ((k0 + CH) % g.img_px) == 0;
        const bool frags = live && (every_chunk || first || last || t == 1);
        if (frags) {
            std::fill(halo.begin(), halo.end(), UNSET);
            std::fill(dz.begin(), dz.end(), UNSET);
        }
        for (int tid = 0; tid < NT; ++tid) {
            for (int i = 0; i < Cfg::NLD; ++i) {
                const int v = tid + NT * i;
                const unsigned off = halo_vec_offset<Cfg, ESZ>(g, c0, v) + roff;    // 32-bit wrap, as on the device
                const bool in_range = records != 0 && (unsigned long long)off + 16 <= records;
                ++w.loads;
                long long elem = ZERO;
                if (in_range) {
                    const long long byte = (long long)img * g.img_bytes + off;
                    if (byte < 0 || byte + 16 > b_bytes) return w.fail("halo load leaves the input tensor");
                    elem = byte / ESZ;
                }
                // what belongs at this LDS position: halo pixel (ry, rx) of the chunk
                if (v < nvec && live) {
                    const int slot = v / Cfg::VPP_B, part = v % Cfg::VPP_B;
                    const int y = g.S * i0 - 1 + slot / g.HWD, xx = slot % g.HWD - 1;
                    long long want = ZERO;
                    if (y >= 0 && y < g.H && xx >= 0 && xx < g.W)
                        want = (((long long)img * g.H + y) * g.W + xx) * g.Cin + c0 + part * VE;
                    if (elem != want) return w.fail("halo load fetches the wrong element (or a padding position is not zero)");
                    if (frags) {
                        const int lo = halo_lds_offset<Cfg>(v);
                        if (lo < 0 || lo + 16 > Cfg::HALO_BYTES) return w.fail("halo store leaves its LDS block");
                        for (int e = 0; e < VE; ++e) halo[(size_t)lo / ESZ + e] = elem == ZERO ? ZERO : elem + e;
                    }
                } else if (in_range && !live) {
                    return w.fail("a prefetch beyond the reduction touches memory");
                } else if (v >= nvec && in_range) {
                    return w.fail("a load slot beyond the halo touches memory");
                }
            }
            for (int j = 0; j < Cfg::NLA; ++j) {
                const int v = tid + NT * j;
                const unsigned off = dz_vec_offset<Cfg, ESZ>(g, o0, v);
                const unsigned soff = live ? (unsigned)k0 * (unsigned)(g.Cout * ESZ) : 0u;
                ++w.loads;
                if (!live) continue;                                   // empty descriptor: nothing is read
                if (v >= CH * Cfg::VPP_A) {                            // a thread beyond the block: its load must be cut off
                    if (off < 0x80000000u) return w.fail("a dZ load slot beyond the block touches memory");
                    continue;
                }
                if (off >= 0x80000000u) return w.fail("dZ offset beyond the descriptor");
                const long long byte = (long long)soff + off;
                if (byte + 16 > a_bytes) return w.fail("dZ load leaves the output-gradient tensor");
                const int q = v / Cfg::VPP_A, part = v % Cfg::VPP_A;
                const long long want = (long long)(k0 + q) * g.Cout + o0 + part * VE;
                if (byte / ESZ != want) return w.fail("dZ load fetches the wrong element");
                if (frags) {
                    const int lo = dz_lds_offset<Cfg>(v);
                    if (lo < 0 || lo + 16 > Cfg::DZ_BYTES) return w.fail("dZ store leaves its LDS block");
                    for (int e = 0; e < VE; ++e) dz[(size_t)lo / ESZ + e] = want + e;
                }
            }
        }
        if (!frags) continue;
        // fragment reads of every wave
        auto in_def = [&](int q, int u, int v, int c) -> long long {      // In[b, s*i+u-1, s*j+v-1, c] of output pixel q of the chunk
            const int pix = (k0 % g.img_px) + q, i = pix >> g.lgWo, j = pix & (g.Wo - 1);
            const int y = g.S * i + u - 1, xx = g.S * j + v - 1;
            if (y < 0 || y >= g.H || xx < 0 || xx >= g.W) return ZERO;
            return (((long long)img * g.H + y) * g.W + xx) * g.Cin + c;
        };
        std::vector<int> tap_owners(9, 0);            // every tap of every channel block belongs to exactly one wave
        for (int wave_id = 0; wave_id < WM * WN * TG; ++wave_id) {
            const int tg = wave_id / (WM * WN), wave = wave_id % (WM * WN);
            const int wm = wave / WN, wn = wave % WN;
            const int tap0 = tap_first<TG>(tg), ntap = tap_count<TG>(tg);
            for (int t = tap0; t < tap0 + ntap; ++t) ++tap_owners[t];
            for (int lane = 0; lane < 64; ++lane) {
                if (ESZ == 2) {
                    for (int kk = 0; kk < 4; ++kk)
                        for (int r = 0; r < 2; ++r)
                            for (int e = 0; e < 4; ++e) {
                                // transposing read: value e of group-lane l comes from the datum addressed by
                                // group-lane 4 * e + l / 4, element l % 4 of its four
                                const int l = lane & 15, src = (lane & ~15) | (4 * e + l / 4);
                                const int hold_q = frag_holds_pixel_bf16(lane, kk, r * 4 + e), hold_ch = frag_holds_channel(lane);
                                {   // operand A: dZ
                                    const int byte = frag_pixel_bf16(src, kk, r) * Cfg::PIXB_A + (wm * 32 + frag_channel_bf16(src)) * 2 + 2 * (l % 4);
                                    if (byte < 0 || byte + 2 > Cfg::DZ_BYTES) return w.fail("dZ fragment read leaves its LDS block");
                                    const long long want = (long long)(k0 + hold_q) * g.Cout + o0 + wm * 32 + hold_ch;
                                    if (dz[(size_t)byte / 2] != want) return w.fail("dZ fragment holds the wrong element");
                                    ++w.frag_reads;
                                }
                                for (int tap = tap0; tap < tap0 + ntap; ++tap) {
                                    const int u = tap / 3, v = tap % 3;
                                    {
                                        const int slot = halo_slot(g, frag_pixel_bf16(src, kk, 0)) + r * 4 * STRIDE + halo_tap_slots(g, u, v);
                                        const int byte = slot * Cfg::PIXB_B + (wn * 32 + frag_channel_bf16(src)) * 2 + 2 * (l % 4);
                                        if (byte < 0 || byte + 2 > Cfg::HALO_BYTES) return w.fail("input fragment read leaves its LDS block");
                                        const long long want = in_def(hold_q, u, v, c0 + wn * 32 + hold_ch);
                                        if (halo[(size_t)byte / 2] != want) return w.fail("input fragment holds the wrong element");
                                        ++w.frag_reads;
                                    }
                                }
                            }
                } else {
                    for (int k8 = 0; k8 < CH / 8; ++k8)
                        for (int j = 0; j < 4; ++j) {
                            const int q = frag_pixel_f32(lane, k8, j), ch = lane & 31;
                            const int abyte = q * Cfg::PIXB_A + (wm * 32 + ch) * 4;
                            if (abyte < 0 || abyte + 4 > Cfg::DZ_BYTES) return w.fail("dZ fragment read leaves its LDS block");
                            if (dz[(size_t)abyte / 4] != (long long)(k0 + q) * g.Cout + o0 + wm * 32 + ch) return w.fail("dZ fragment holds the wrong element");
                            ++w.frag_reads;
                            for (int tap = tap0; tap < tap0 + ntap; ++tap) {
                                const int u = tap / 3, v = tap % 3;
                                {
                                    const int byte = (halo_slot(g, q) + halo_tap_slots(g, u, v)) * Cfg::PIXB_B + (wn * 32 + ch) * 4;
                                    if (byte < 0 || byte + 4 > Cfg::HALO_BYTES) return w.fail("input fragment read leaves its LDS block");
                                    if (halo[(size_t)byte / 4] != in_def(q, u, v, c0 + wn * 32 + ch)) return w.fail("input fragment holds the wrong element");
                                    ++w.frag_reads;
                                }
                            }
                        }
                }
            }
        }
        for (int t = 0; t < 9; ++t)
            if (tap_owners[t] != WM * WN) return w.fail("a tap is not owned by exactly one wave per channel block");
    }
    return true;
}

}  // namespace

// Walks tile `tr` of problem `p` (operand tensors of a_bytes / b_bytes bytes); wide: 64 input channels per
// tile, else 32.  every_chunk = false replays the fragment reads only for the first, second and last chunk
// of the split and for the chunks at the top and bottom of an image (the loads of every chunk are always
// checked).  Returns "" or what went wrong.
std::string conv_dw_halo_walk(bool bf16, bool wide, const GemmProb& p, const TileRef& tr, long long a_bytes, long long b_bytes,
                              bool every_chunk, long long* loads, long long* frag_reads) {
    Walk w;
    const bool s1 = p.stride == 1;
    if (wide) {
        if (bf16) s1 ? walk_tile<2, 2, 2, 1, 2>(p, tr, a_bytes, b_bytes, every_chunk, w) : walk_tile<2, 2, 2, 2, 2>(p, tr, a_bytes, b_bytes, every_chunk, w);
        else s1 ? walk_tile<4, 2, 2, 1>(p, tr, a_bytes, b_bytes, every_chunk, w) : walk_tile<4, 2, 2, 2>(p, tr, a_bytes, b_bytes, every_chunk, w);
    } else if (!s1) {
        w.fail("there is no 32-channel form at stride 2");
    } else if (bf16) {
        walk_tile<2, 2, 1, 1>(p, tr, a_bytes, b_bytes, every_chunk, w);
    } else {
        walk_tile<4, 2, 1, 1>(p, tr, a_bytes, b_bytes, every_chunk, w);
    }
    if (loads) *loads += w.loads;
    if (frag_reads) *frag_reads += w.frag_reads;
    return w.err;
}

}  // namespace packk
