// Address rules of the grouped matrix products of the packed training step: which element of an operand a
// (row, reduction index) pair names in each of the six modes (off_a / off_b, the definition the scalar
// kernels load by), the geometry of an operand tile in LDS, and the fetchers of the aligned kernels, which
// turn those rules into one 32-bit byte offset per load and thread plus a wave-uniform offset per chunk.
//
// Included by the kernels (pack_kernels.hip) and, with PACK_FETCH_ON_HOST defined, by the host-side walk
// (gemm_fetch_check.cpp), which runs these same fetchers thread by thread on the CPU, with the buffer load
// replaced by a recorder, and compares every load with the definition.  In that build the includer supplies the
// few device facilities used here: PACK_TID (the thread index), pack_uniform, make_rsrc, buf_load16, the vector
// types and ET<T>.
#pragma once
#include "pack_internal.h"

// PACK_HALO_PLANT (0 in every build of the library): a CPU test compiles the host-side walk with one rule
// deliberately wrong, to show that the walk notices.
#ifndef PACK_HALO_PLANT
#define PACK_HALO_PLANT 0
#endif

#ifdef PACK_FETCH_ON_HOST
#define PACK_DEV inline
#else
#include "pack_device.h"
#define PACK_DEV __device__ __forceinline__
#define PACK_TID ((int)threadIdx.x)
namespace packk {
// a value that is the same in every lane of a wave, handed over in a scalar register
__device__ __forceinline__ int pack_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
}  // namespace packk
#endif

namespace packk {
// Buffer descriptor over the 2 GB window that starts margin_bytes before `base` (raw buffer, range checked).
PACK_DEV i32x4_t make_rsrc(const void* base, long long margin_bytes) {
    const unsigned long long a = (unsigned long long)base - (unsigned long long)margin_bytes;
    i32x4_t r;
    r.x = pack_uniform((int)(unsigned)a);
    r.y = pack_uniform((int)(unsigned)(a >> 32));   // stride 0: raw buffer
    r.z = (int)BUF_RECORDS;
    r.w = 0x00020000;                               // 32-bit data format
    return r;
}


// F_ROWMAP problems (one parity class of a stride-2 input gradient): the tap that reduction
// block `tc` of the class stands for, and the pixel an output row stands for
PACK_DEV int class_tap(const GemmProb& p, int tc) {
    const int ntx = p.cls_px ? 1 : 2;
    const int iu = tc / ntx, iv = tc - iu * ntx;
    const int u = p.cls_py ? 1 : 2 * iu, v = p.cls_px ? 1 : 2 * iv;
    return u * 3 + v;
}
// row index of a problem whose rows are pixels -> (image, pixel row, pixel column); shifts when the
// extents are powers of two (uniform branch), divisions otherwise
PACK_DEV void decode_row(const GemmProb& p, int r, int& b, int& i, int& j) {
    if (p.lg_row_hw >= 0) {
        b = r >> p.lg_row_hw;
        const int rem = r & (p.row_hw - 1);
        i = rem >> p.lg_row_w;
        j = rem & (p.row_w - 1);
    } else {
        b = r / p.row_hw;
        const int rem = r - b * p.row_hw;
        i = rem / p.row_w;
        j = rem - i * p.row_w;
    }
}
PACK_DEV void class_pixel(const GemmProb& p, int r, int& b, int& y, int& x) {
    int yc, xc;
    decode_row(p, r, b, yc, xc);
    y = 2 * yc + 1 - p.cls_py;
    x = 2 * xc + 1 - p.cls_px;
}
// element offset of output row `row` (times the leading dimension) for the epilogue
PACK_DEV size_t out_row_base(const GemmProb& p, int row) {
    if (p.flags & F_ROWMAP) {
        int b, y, x;
        class_pixel(p, row, b, y, x);
        return ((size_t)(b * p.H + y) * p.W + x) * p.ldc;
    }
    return (size_t)row * p.ldc;
}

// ------------------------------------------------------------------------------------------------
// operand address rules: element (row, k) of operand A / B for each mode.  Each rule returns
// whether the element exists (otherwise it reads as zero) and its element offset from the
// operand's base; the offset is forced to 0 for missing elements so that the caller can always
// issue the load (branch-free, so that many loads stay in flight) and discard the value.
// ------------------------------------------------------------------------------------------------
template <int MODE>
PACK_DEV bool off_a(const GemmProb& p, int r, int k, size_t& off) {
    bool ok = (r < p.R) && (k < p.Kd);
    size_t o;
    if constexpr (MODE == LIN_FWD || MODE == LIN_DX) {
        o = (size_t)r * p.lda + k;
    } else if constexpr (MODE == LIN_DW || MODE == CONV_DW) {
        o = (size_t)k * p.lda + r;
    } else if constexpr (MODE == CONV_FWD) {
        const int hw = p.Ho * p.Wo;
        const int b = r / hw, rem = r - b * hw;
        const int i = rem / p.Wo, j = rem - i * p.Wo;
        const int tap = k / p.Cin, c = k - tap * p.Cin;
        const int u = tap / 3, v = tap - 3 * u;
        const int y = p.stride * i + u - 1, x = p.stride * j + v - 1;
        ok = ok && ((unsigned)y < (unsigned)p.H) && ((unsigned)x < (unsigned)p.W);
        o = ((size_t)(b * p.H + y) * p.W + x) * p.Cin + c;
    } else {  // CONV_DX: row = input pixel (b, y, x), k = (tap, o)
        const int hw = p.H * p.W;
        const int b = r / hw, rem = r - b * hw;
        const int y = rem / p.W, x = rem - y * p.W;
        const int tap = k / p.Cout, oc = k - tap * p.Cout;
        const int u = tap / 3, v = tap - 3 * u;
        int ty = y + 1 - u, tx = x + 1 - v;
        ok = ok && (ty >= 0) && (tx >= 0);
        if (p.stride == 2) {
            ok = ok && (((ty | tx) & 1) == 0);
            ty >>= 1;
            tx >>= 1;
        }
        ok = ok && (ty < p.Ho) && (tx < p.Wo);
        o = ((size_t)(b * p.Ho + ty) * p.Wo + tx) * p.Cout + oc;
    }
    off = ok ? o : (size_t)0;
    return ok;
}

template <int MODE>
PACK_DEV bool off_b(const GemmProb& p, int q, int k, size_t& off) {
    bool ok = (q < p.Q) && (k < p.Kd);
    size_t o;
    if constexpr (MODE == LIN_FWD || MODE == CONV_FWD) {
        o = (size_t)q * p.ldb + k;
    } else if constexpr (MODE == LIN_DX || MODE == LIN_DW) {
        o = (size_t)k * p.ldb + q;
    } else if constexpr (MODE == CONV_DX) {
        // q = input channel c, k = (tap, o); the operand is the per-step transposed copy of the
        // weights, [Cin][9][Cout], so the reduction is contiguous (ldb = 9 * Cout)
        int kk = k;
        if (p.flags & F_ROWMAP) {
            const int tc = k / p.Cout;
            kk = class_tap(p, tc) * p.Cout + (k - tc * p.Cout);
        }
        o = (size_t)q * p.ldb + kk;
    } else {  // CONV_DW: q = (tap, c), k = output pixel (b, i, j)
        const int tap = q / p.Cin, c = q - tap * p.Cin;
        const int u = tap / 3, v = tap - 3 * u;
        const int hw = p.Ho * p.Wo;
        const int b = k / hw, rem = k - b * hw;
        const int i = rem / p.Wo, j = rem - i * p.Wo;
        const int y = p.stride * i + u - 1, x = p.stride * j + v - 1;
        ok = ok && ((unsigned)y < (unsigned)p.H) && ((unsigned)x < (unsigned)p.W);
        o = ((size_t)(b * p.H + y) * p.W + x) * p.Cin + c;
    }
    off = ok ? o : (size_t)0;
    return ok;
}

// Which operands are contiguous along the reduction (KC) and which along their row index (RC).
template <int MODE> struct OperandLayout {
    static constexpr bool A_KC = (MODE == LIN_FWD || MODE == LIN_DX || MODE == CONV_FWD || MODE == CONV_DX);
    static constexpr bool B_KC = (MODE == LIN_FWD || MODE == CONV_FWD || MODE == CONV_DX);
};

// ------------------------------------------------------------------------------------------------
// grouped MFMA GEMM
// ------------------------------------------------------------------------------------------------
// LDS tile of one operand: BR rows x BK reduction indices, each row padded by 16 bytes so that
// the 16-byte fragment reads of 16 consecutive rows fall into 64 different banks.
template <typename T, int BR, int BK_>
struct TileGeom {
    static constexpr int V = ET<T>::V;
    static constexpr int BK = BK_;
    static constexpr int LDS_LD = BK + V;
    static constexpr int VPR = BK / V;                 // KC: 16-byte vectors per row
    static constexpr int NVEC = BR * BK / V;           // 16-byte vectors per tile
    static constexpr int KC_SLOTS = (NVEC + 255) / 256;// vectors per thread
    static constexpr int RPV = BR / V;                 // row-vectors per reduction index
    // RC operands are moved as blocks of 4 reduction indices x V rows (four vectors per block).
    // Block b: kq_lo = b % 16 (fastest, so that the transposed LDS stores of neighbouring lanes
    // fall into different banks), rv = (b / 16) % RPV, kq_hi = b / (16 * RPV).
    static constexpr int RC_BLOCKS = NVEC / 4;
    static constexpr int RC_PER_THREAD = (RC_BLOCKS + 255) / 256;
    static constexpr int NREG = (KC_SLOTS > 4 * RC_PER_THREAD) ? KC_SLOTS : 4 * RC_PER_THREAD;
    static_assert(BK % 64 == 0 || sizeof(T) == 4, "bf16 tiles hold multiples of 64 reduction indices");
    static_assert(BK % (16 * 4) == 0 || BK % 32 == 0, "reduction extent");
};

// number of load_vec() calls fetch_tile<..., VEC = true> makes per thread and chunk
template <int MODE, typename T, bool IS_A, int BR, int BK>
struct LoadsPerChunk {
    typedef TileGeom<T, BR, BK> G;
    static constexpr bool KC = IS_A ? OperandLayout<MODE>::A_KC : OperandLayout<MODE>::B_KC;
    static constexpr int value = KC ? G::KC_SLOTS : 4 * G::RC_PER_THREAD;
};

template <typename G>
PACK_DEV void rc_block_coords(int b, int& kq, int& rv) {
    constexpr int KQ_LO = (G::BK / 4 < 16) ? G::BK / 4 : 16;
    const int lo = b % KQ_LO;
    const int rest = b / KQ_LO;
    rv = rest % G::RPV;
    kq = (rest / G::RPV) * KQ_LO + lo;
}

// the element-by-element gather of the kernels for unaligned shapes (device only)
template <int MODE, typename T, bool IS_A, int BR, int BK, bool VEC>
PACK_DEV void fetch_tile(const GemmProb& p, int row0, int k0, int kend, u32x4_t (&regs)[TileGeom<T, BR, BK>::NREG]);

// ------------------------------------------------------------------------------------------------
// Operand fetch of the aligned kernels: raw buffer loads.  Each operand gets a buffer descriptor
// (base address, 2 GB of records); a thread keeps one 32-bit byte offset per load that is fixed
// for the whole tile, the part that changes per chunk is wave-uniform and travels in the scalar
// offset of the instruction, and an element that does not exist is addressed beyond the records,
// which the hardware answers with zeros without touching memory.  So a load costs no vector
// arithmetic at all unless its validity changes from chunk to chunk (border taps of the gathered
// convolution operands, a reduction that ends inside a chunk).  The planner only marks a problem
// as aligned when every operand spans less than 2 GB, so that offset + scalar offset never wraps.
// The loads are assembly statements for the same reason as before: their completion is awaited
// by hand (wait_stage), not by the compiler.
// ------------------------------------------------------------------------------------------------
// Per-thread operand fetcher of one tile.  VEC kernels use the buffer form above: everything that
// depends on the thread's rows (pixel coordinates, border validity of the nine taps) is decoded
// ONCE per tile into the per-load offsets; it relies on the alignment the planner checks before
// it marks a convolution problem as vectorisable: a chunk of BK reduction indices never straddles
// a tap (forward: Cin % BK == 0, input gradient: Cout % BK == 0) or an image (weight gradient:
// Ho*Wo % BK == 0 with Wo a power of two).  The scalar kernels recompute addresses from (row, k)
// for every element (fetch_tile).
template <int MODE, typename T, bool IS_A, int BR, int BK, bool VEC>
struct Fetcher {
    typedef TileGeom<T, BR, BK> G;
    static constexpr bool KC = IS_A ? OperandLayout<MODE>::A_KC : OperandLayout<MODE>::B_KC;
    static constexpr bool BUF = VEC;
    static constexpr bool GATHER_KC = BUF && IS_A && (MODE == CONV_FWD || MODE == CONV_DX);
    static constexpr bool WEIGHT_KC = BUF && !IS_A && (MODE == CONV_DX || MODE == CONV_FWD);
    static constexpr bool GATHER_RC = BUF && !IS_A && MODE == CONV_DW;
    static constexpr bool PLAIN_KC = BUF && KC && !GATHER_KC && !WEIGHT_KC;
    static constexpr bool PLAIN_RC = BUF && !KC && !GATHER_RC;
    static constexpr int NL = KC ? G::KC_SLOTS : 4 * G::RC_PER_THREAD;   // loads per thread and chunk
    static constexpr int NB = KC ? G::KC_SLOTS : G::RC_PER_THREAD;       // rows (KC) or blocks (RC) per thread
    static constexpr int ESZ = (int)sizeof(T);

    int row0;
    i32x4_t rsrc;
    unsigned voff[BUF ? NL : 1];    // byte offset of each load, BUF_POISON when the row does not exist
    unsigned mask[BUF ? NB : 1];    // GATHER_KC: bit t = tap t reads inside the image
    int kpos[BUF ? NB : 1];         // PLAIN_KC: first reduction index of the slot; RC forms: 4 * kq
    int du[GATHER_RC ? NB : 1], dv[GATHER_RC ? NB : 1];   // GATHER_RC: tap offsets u - 1, v - 1

    PACK_DEV void init(const GemmProb& p, int row0_) {
        row0 = row0_;
        const int tid = PACK_TID;
        const void* src = IS_A ? p.A : p.B;
        if constexpr (GATHER_KC) {
            // margin: the first tap of a border pixel lies one row and one pixel before the tensor
            const int pw = (MODE == CONV_FWD) ? p.W : p.Wo, pc = (MODE == CONV_FWD) ? p.Cin : p.Cout;
            const int margin = (pw + 1) * pc;
            rsrc = make_rsrc(src, (long long)margin * ESZ);
#pragma unroll
            for (int s = 0; s < NB; ++s) {
                const int vid = tid + 256 * s;
                const int r = row0 + vid / G::VPR;
                const int kv = (vid % G::VPR) * G::V;
                const bool live = (vid < G::NVEC) && (r < p.R);
                unsigned m = 0;
                // tap (u, v) is inside the image iff row condition u and column condition v hold:
                // three bits each, combined into the nine-bit mask
                unsigned rb = 0, cb = 0;
                int base;
                if constexpr (MODE == CONV_FWD) {
                    int b, i, j;
                    decode_row(p, r, b, i, j);
                    const int y0 = p.stride * i - 1, x0 = p.stride * j - 1;
                    base = ((b * p.H + y0) * p.W + x0 + (PACK_HALO_PLANT == 7)) * p.Cin + kv;
#pragma unroll
                    for (int t = 0; t < 3; ++t) {
                        if ((unsigned)(y0 + t) < (unsigned)p.H) rb |= 1u << t;
                        if ((unsigned)(x0 + t) < (unsigned)p.W) cb |= 1u << t;
                    }
                } else {   // CONV_DX: rows are input pixels, the gather reads dz; the thread's
                           // offset is that of the LAST tap (2, 2) (or the class's last), so that
                           // the per-chunk part is never negative
                    int b, y, x;
                    if (p.flags & F_ROWMAP) class_pixel(p, r, b, y, x);
                    else decode_row(p, r, b, y, x);
                    const int yy = y + 1, xx = x + 1;
                    const int sh = (p.stride == 2) ? 1 : 0;
                    const int um = (p.flags & F_ROWMAP) ? (p.cls_py ? 1 : 2) : 2;
                    const int vm = (p.flags & F_ROWMAP) ? (p.cls_px ? 1 : 2) : 2;
                    base = ((b * p.Ho + ((yy - um) >> sh)) * p.Wo + ((xx - vm) >> sh)) * p.Cout + kv;
#pragma unroll
                    for (int t = 0; t < 3; ++t) {
                        const int ty = yy - t, tx = xx - t;
                        if (ty >= 0 && !(ty & sh) && (ty >> sh) < p.Ho) rb |= 1u << t;
                        if (tx >= 0 && !(tx & sh) && (tx >> sh) < p.Wo) cb |= 1u << t;
                    }
                }
                m = ((rb & 1u) ? cb : 0u) | ((rb & 2u) ? cb << 3 : 0u) | ((rb & 4u) ? cb << 6 : 0u);
                mask[s] = live ? m : 0u;
                voff[s] = (unsigned)(base + margin) * ESZ;
            }
        } else if constexpr (WEIGHT_KC || PLAIN_KC) {
            rsrc = make_rsrc(src, 0);
            const int ld = IS_A ? p.lda : p.ldb;
            const int rows = IS_A ? p.R : p.Q;
#pragma unroll
            for (int s = 0; s < NB; ++s) {
                const int vid = tid + 256 * s;
                const int r = row0 + vid / G::VPR;
                kpos[s] = (vid % G::VPR) * G::V;
                const bool live = (vid < G::NVEC) && (r < rows);
                voff[s] = (live || PACK_HALO_PLANT == 8) ? (unsigned)(r * ld + kpos[s]) * ESZ : BUF_POISON;
            }
        } else if constexpr (PLAIN_RC) {
            rsrc = make_rsrc(src, 0);
            const int ld = IS_A ? p.lda : p.ldb;
            const int rows = IS_A ? p.R : p.Q;
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int b = tid + 256 * j;
                int kq, rv;
                rc_block_coords<G>(b, kq, rv);
                const int r = row0 + rv * G::V;
                kpos[j] = kq * 4;
                const bool live = (b < G::RC_BLOCKS) && (r < rows);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    voff[4 * j + e] = live ? (unsigned)((kq * 4 + e) * ld + r) * ESZ : BUF_POISON;
            }
        } else if constexpr (GATHER_RC) {
            const int margin = (p.W + 1) * p.Cin;
            rsrc = make_rsrc(src, (long long)margin * ESZ);
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int b = tid + 256 * j;
                int kq, rv;
                rc_block_coords<G>(b, kq, rv);
                const int q = row0 + rv * G::V;
                const int tap = q / p.Cin, c = q - tap * p.Cin;
                du[j] = tap / 3 - 1;
                dv[j] = tap % 3 - 1;
                kpos[j] = kq * 4;
                const bool live = (b < G::RC_BLOCKS) && (q < p.Q);
                // fixed part: channel and tap displacement; the pixel part is added per chunk
                voff[4 * j] = live ? (unsigned)((du[j] * p.W + dv[j]) * p.Cin + c + margin) * ESZ : BUF_POISON;
            }
        }
    }

    PACK_DEV void fetch(const GemmProb& p, int k0, int kend, u32x4_t (&regs)[G::NREG]) const {
        if constexpr (GATHER_KC) {
            // the whole chunk lies in one tap: its offset is the same for every thread
            const int span = (MODE == CONV_FWD) ? p.Cin : p.Cout;
            const int tc = k0 / span, c0 = k0 - tc * span;
            int tap, toff;
            if constexpr (MODE == CONV_FWD) {
                tap = tc;
                const int u = tap / 3, v = tap - 3 * u;
                toff = (u * p.W + v) * p.Cin + c0;
            } else {
                const bool cls = (p.flags & F_ROWMAP) != 0;
                tap = cls ? class_tap(p, tc) : tc;
                const int u = tap / 3, v = tap - 3 * u;
                const int sh = (p.stride == 2) ? 1 : 0;
                const int um = cls ? (p.cls_py ? 1 : 2) : 2, vm = cls ? (p.cls_px ? 1 : 2) : 2;
                toff = (((um - u) >> sh) * p.Wo + ((vm - v) >> sh)) * p.Cout + c0;
            }
            i32x4_t r = rsrc;
            r.z = pack_uniform((k0 < kend) ? (int)BUF_RECORDS : 0);   // a chunk beyond the reduction reads zeros
            const unsigned soff = (unsigned)toff * ESZ;
#pragma unroll
            for (int s = 0; s < NB; ++s) {
                const unsigned o = ((mask[s] >> tap) & 1u) ? voff[s] : BUF_POISON;
                regs[s] = buf_load16(r, o, soff);
            }
        } else if constexpr (WEIGHT_KC) {
            // forward: W[Cout][9*Cin], the chunk starts at k0; input gradient: transposed weights
            // [Cin][9][Cout], the chunk lies in one tap (class problems skip taps)
            int koff = k0;
            if constexpr (MODE == CONV_DX) {
                if (p.flags & F_ROWMAP) {
                    const int tc = k0 / p.Cout;
                    koff = class_tap(p, tc) * p.Cout + (k0 - tc * p.Cout);
                }
            }
            i32x4_t r = rsrc;
            r.z = pack_uniform((k0 < kend) ? (int)BUF_RECORDS : 0);
            const unsigned soff = (unsigned)koff * ESZ;
#pragma unroll
            for (int s = 0; s < NB; ++s) regs[s] = buf_load16(r, voff[s], soff);
        } else if constexpr (PLAIN_KC) {
            const int rem = kend - k0;   // reduction indices left; the last chunk may end inside
            const unsigned soff = (unsigned)max(k0, 0) * ESZ;
#pragma unroll
            for (int s = 0; s < NB; ++s) {
                const unsigned o = (kpos[s] < rem) ? voff[s] : BUF_POISON;
                regs[s] = buf_load16(rsrc, o, soff);
            }
        } else if constexpr (PLAIN_RC) {
            const int ld = IS_A ? p.lda : p.ldb;
            const int rem = kend - k0;
            i32x4_t r = rsrc;
            r.z = pack_uniform((rem > 0) ? (int)BUF_RECORDS : 0);
            const unsigned soff = (rem > 0) ? (unsigned)k0 * (unsigned)ld * ESZ : 0u;
#pragma unroll
            for (int j = 0; j < NB; ++j) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const unsigned o = (kpos[j] + e < rem) ? voff[4 * j + e] : BUF_POISON;
                    regs[4 * j + e] = buf_load16(r, o, soff);
                }
            }
        } else if constexpr (GATHER_RC) {
            // reduction index = output pixel; the chunk lies inside one image, and the four
            // pixels of a block lie in one image row (Wo is a power of two >= 4)
            const int hw = p.Ho * p.Wo;
            const int img = k0 / hw, p0 = k0 - img * hw;
            const int lw = 31 - __builtin_clz(p.Wo);
            i32x4_t r = rsrc;
            r.z = pack_uniform((k0 < kend) ? (int)BUF_RECORDS : 0);
            const unsigned soff = (k0 < kend) ? (unsigned)(img * p.H * p.W * p.Cin) * ESZ : 0u;
            const int xstep = p.stride * p.Cin * ESZ;
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int pidx = p0 + kpos[j];
                const int i = pidx >> lw, jx = pidx & (p.Wo - 1);
                const int yb = p.stride * i, xb = p.stride * jx;
                const bool rowok = (voff[4 * j] != BUF_POISON) && ((unsigned)(yb + du[j]) < (unsigned)p.H);
                const unsigned pix = voff[4 * j] + (unsigned)((yb * p.W + xb) * p.Cin) * ESZ;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool ok = rowok && ((unsigned)(xb + e * p.stride + dv[j]) < (unsigned)p.W);
                    regs[4 * j + e] = buf_load16(r, ok ? pix + e * xstep : BUF_POISON, soff);
                }
            }
        } else {
            fetch_tile<MODE, T, IS_A, BR, BK, VEC>(p, row0, k0, kend, regs);
        }
    }
};

}  // namespace packk
