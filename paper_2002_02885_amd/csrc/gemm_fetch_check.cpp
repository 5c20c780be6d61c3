// Host-side walk of the fetchers of the aligned staged-tile kernels (gemm_fetch.h).  The fetchers
// themselves are compiled here for the CPU: the thread index is a variable, the buffer load a recorder.  For
// one tile, every thread's loads of every chunk (the prefetches beyond the reduction included) are run and
// each recorded load is compared with the definition of the product's operands (off_a / off_b): a load of
// elements that exist must be inside the descriptor's window and name exactly those elements; a load of
// elements that do not exist (padding, rows or reduction indices beyond the problem, chunks beyond the
// reduction) must be one the range check cuts off by construction, i.e. carry the poison offset or an empty
// descriptor.  Used by pack_plan_check; nothing here touches a device.
#define PACK_FETCH_ON_HOST
#include "pack_internal.h"

#include <string>
#include <vector>

namespace packk {
namespace {
struct LoadRec {
    unsigned long long base;
    unsigned records, voff, soff;
};
thread_local int g_tid = 0;
thread_local std::vector<LoadRec>* g_log = nullptr;
}  // namespace

#define PACK_TID (::packk::g_tid)
inline int pack_uniform(int v) { return v; }
inline u32x4_t buf_load16(const i32x4_t rsrc, unsigned voff, unsigned soff) {
    g_log->push_back(LoadRec{(unsigned long long)(unsigned)rsrc.x | ((unsigned long long)(unsigned)rsrc.y << 32), (unsigned)rsrc.z, voff, soff});
    return u32x4_t{0u, 0u, 0u, 0u};
}
template <typename T> struct ET;
template <> struct ET<float> { static constexpr int V = 4, BK = 32; };
template <> struct ET<bf16_t> { static constexpr int V = 8, BK = 64; };
}  // namespace packk

#include "gemm_fetch.h"

namespace packk {
namespace {

struct Span {   // lowest and one past the highest byte address the real loads of an operand touched
    unsigned long long lo = ~0ull, hi = 0;
};

// The element (row r, reduction index k) of an operand by the definition of the product: off_a / off_b, and for
// the parity classes of a stride-2 input gradient (rows = the pixels of one class, reduction = the taps that
// reach the class, which only the aligned kernels run) the same rule written out for a class:
// dX[b, y, x, c] sums dZ[b, (y + 1 - u) / 2, (x + 1 - v) / 2, o] over the taps (u, v) for which both are whole.
template <int MODE, bool IS_A>
bool element(const GemmProb& p, int r, int k, size_t& off) {
    if constexpr (MODE == CONV_DX && IS_A) {
        if (p.flags & F_ROWMAP) {
            off = 0;
            if (r >= p.R || k >= p.Kd) return false;
            int b, y, x;
            class_pixel(p, r, b, y, x);
            const int tc = k / p.Cout, oc = k - tc * p.Cout;
            const int tap = class_tap(p, tc), u = tap / 3, v = tap % 3;
            const int ty = y + 1 - u, tx = x + 1 - v;
            if (ty < 0 || tx < 0 || ((ty | tx) & 1) || ty / 2 >= p.Ho || tx / 2 >= p.Wo) return false;
            off = ((size_t)(b * p.Ho + ty / 2) * p.Wo + tx / 2) * p.Cout + oc;
            return true;
        }
    }
    return IS_A ? off_a<MODE>(p, r, k, off) : off_b<MODE>(p, r, k, off);
}

template <int MODE, typename T, bool IS_A, int BR, int BK>
std::string check_loads(const GemmProb& p, const std::vector<LoadRec>& log, int tid, int row0, int k0, int kend, Span& span, long long* loads) {
    typedef TileGeom<T, BR, BK> G;
    constexpr bool KC = IS_A ? OperandLayout<MODE>::A_KC : OperandLayout<MODE>::B_KC;
    constexpr int V = G::V, ESZ = (int)sizeof(T);
    if ((int)log.size() != LoadsPerChunk<MODE, T, IS_A, BR, BK>::value) return "a thread issues another number of loads than the waits count";
    const unsigned long long operand = (unsigned long long)(IS_A ? p.A : p.B);
    for (size_t n = 0; n < log.size(); ++n) {
        // the V elements load n stands for (what stash_tile stores it as)
        int r[8], k[8];
        bool slot = true;
        if (KC) {
            const int vid = tid + 256 * (int)n;
            slot = vid < G::NVEC;
            for (int e = 0; e < V; ++e) { r[e] = row0 + vid / G::VPR; k[e] = k0 + (vid % G::VPR) * V + e; }
        } else {
            const int b = tid + 256 * (int)(n / 4);
            int kq, rv;
            rc_block_coords<G>(b, kq, rv);
            slot = b < G::RC_BLOCKS;
            for (int e = 0; e < V; ++e) { r[e] = row0 + rv * V + e; k[e] = k0 + kq * 4 + (int)(n % 4); }
        }
        // Elements a load may cover although the product does not use them, provided its first element exists:
        // rows beyond the problem (their results are never stored) and, in dense operands whose rows are padded
        // to whole vectors (the gradient of the logits), the padding between the last reduction index and the
        // leading dimension, which is zero in memory and meets cut-off elements of the other operand.
        const int rows = IS_A ? p.R : p.Q;
        const bool dense = MODE == LIN_FWD || MODE == LIN_DX || MODE == LIN_DW;
        const int ld = IS_A ? p.lda : p.ldb;
        bool any = false, all = true, first_ok = false;
        size_t first = 0;
        for (int e = 0; e < V; ++e) {
            size_t off = 0;
            bool ok = slot && k[e] < kend && element<MODE, IS_A>(p, r[e], k[e], off);
            if (e == 0) { first = off; first_ok = ok; }
            if (ok && off != first + (size_t)e) return "the elements of one 16-byte load are not contiguous in memory";
            const bool spare = first_ok && slot && ((!KC && r[e] >= rows) || (KC && dense && k[e] >= p.Kd && k[e] < ld));
            any = any || ok;
            all = all && (ok || spare);
        }
        if (any && !all) return "a 16-byte load straddles the edge of its operand";
        const LoadRec& L = log[n];
        const bool cut_off = L.voff >= BUF_POISON || L.records == 0;
        if (!any) {
            if (!cut_off) return "a load of elements that do not exist is not cut off by construction";
            continue;
        }
        if (cut_off) return "a load of elements that exist is cut off";
        if ((unsigned long long)L.voff + L.soff + 16 > L.records) return "a load of elements that exist leaves the descriptor's window";
        const unsigned long long addr = L.base + L.voff + L.soff;
        if (addr != operand + (unsigned long long)first * ESZ) return "a load names other elements than the definition";
        if (addr % 16) return "a 16-byte load is not aligned";
        span.lo = addr < span.lo ? addr : span.lo;
        span.hi = addr + 16 > span.hi ? addr + 16 : span.hi;
        ++*loads;
    }
    return std::string();
}

template <int MODE, typename T, int BM, int BN>
std::string walk_tile(const GemmProb& p, const TileRef& tr, Span& sa, Span& sb, long long* loads) {
    constexpr int BK = ET<T>::BK;
    typedef TileGeom<T, BM, BK> GA;
    typedef TileGeom<T, BN, BK> GB;
    const int row0 = tr.tm * BM, col0 = tr.tn * BN;
    const int kbeg = tr.ks * p.ksplit, kend = p.Kd < kbeg + p.ksplit ? p.Kd : kbeg + p.ksplit;
    if (row0 < 0 || row0 >= p.R || col0 < 0 || col0 >= p.Q || kbeg < 0 || kbeg >= p.Kd) return "the tile lies outside its problem";
    const int nk = (kend - kbeg + BK - 1) / BK;
    std::vector<LoadRec> log;
    g_log = &log;
    for (int tid = 0; tid < 256; ++tid) {
        g_tid = tid;
        Fetcher<MODE, T, true, BM, BK, true> fa;
        Fetcher<MODE, T, false, BN, BK, true> fb;
        fa.init(p, row0);
        fb.init(p, col0);
        u32x4_t ra[GA::NREG], rb[GB::NREG];
        for (int c = 0; c < nk + 4; ++c) {   // the pipeline requests up to four chunks beyond the reduction
            const int k0 = kbeg + c * BK;
            log.clear();
            fa.fetch(p, k0, kend, ra);
            std::string err = check_loads<MODE, T, true, BM, BK>(p, log, tid, row0, k0, kend, sa, loads);
            if (!err.empty()) return "operand A, thread " + std::to_string(tid) + ", chunk " + std::to_string(c) + ": " + err;
            log.clear();
            fb.fetch(p, k0, kend, rb);
            err = check_loads<MODE, T, false, BN, BK>(p, log, tid, col0, k0, kend, sb, loads);
            if (!err.empty()) return "operand B, thread " + std::to_string(tid) + ", chunk " + std::to_string(c) + ": " + err;
        }
    }
    g_log = nullptr;
    return std::string();
}

template <int MODE, typename T>
std::string walk_shape(int bm, int bn, const GemmProb& p, const TileRef& tr, Span& sa, Span& sb, long long* loads) {
    if (bm == 128 && bn == 128) return walk_tile<MODE, T, 128, 128>(p, tr, sa, sb, loads);
    if (bm == 128 && bn == 64) return walk_tile<MODE, T, 128, 64>(p, tr, sa, sb, loads);
    if (bm == 64 && bn == 64) return walk_tile<MODE, T, 64, 64>(p, tr, sa, sb, loads);
    return "no aligned kernel has this tile shape";
}

template <typename T>
std::string walk_mode(int mode, int bm, int bn, const GemmProb& p, const TileRef& tr, Span& sa, Span& sb, long long* loads) {
    switch (mode) {
        case LIN_FWD: return walk_shape<LIN_FWD, T>(bm, bn, p, tr, sa, sb, loads);
        case LIN_DX: return walk_shape<LIN_DX, T>(bm, bn, p, tr, sa, sb, loads);
        case LIN_DW: return walk_shape<LIN_DW, T>(bm, bn, p, tr, sa, sb, loads);
        case CONV_FWD: return walk_shape<CONV_FWD, T>(bm, bn, p, tr, sa, sb, loads);
        case CONV_DX: return walk_shape<CONV_DX, T>(bm, bn, p, tr, sa, sb, loads);
        case CONV_DW: return walk_shape<CONV_DW, T>(bm, bn, p, tr, sa, sb, loads);
        default: return "unknown mode";
    }
}

}  // namespace

// One tile of a launch on the aligned staged-tile kernels (tile shape bm x bn).  On success a_lo .. b_hi hold
// the range of addresses the tile's real loads of each operand touched (lo > hi: none), for the caller to hold
// against its allocations.  Returns an empty string or what is wrong.
std::string gemm_fetch_walk(bool bf16, int mode, int bm, int bn, const GemmProb& p, const TileRef& tr, unsigned long long* a_lo,
                            unsigned long long* a_hi, unsigned long long* b_lo, unsigned long long* b_hi, long long* loads) {
    Span sa, sb;
    const std::string err = bf16 ? walk_mode<bf16_t>(mode, bm, bn, p, tr, sa, sb, loads) : walk_mode<float>(mode, bm, bn, p, tr, sa, sb, loads);
    *a_lo = sa.lo; *a_hi = sa.hi; *b_lo = sb.lo; *b_hi = sb.hi;
    return err;
}

}  // namespace packk
