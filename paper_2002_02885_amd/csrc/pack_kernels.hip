// gfx950 (CDNA4) kernels of the packed training step.
//
// The paper describes `pack` at graph level (Section 2.2, 3.1, 3.4) and leaves the execution to a
// framework; its closing section names a custom execution platform with ragged-array support as
// open work.  These kernels are that platform for one GPU: every launch processes a LIST of
// problems (one per packed member and layer), so K members cost one launch sequence, and members
// of different widths, depths and batch sizes (Section 3.2) sit side by side in one grid.
//
// Matrix products run on the matrix cores (MFMA 32x32 tiles, 64-lane wavefronts), operands staged
// through LDS with rows laid out reduction-contiguous so that every fragment read is one
// 16-byte access.  The SGD update of plain-SGD packs is applied in the epilogue of the
// weight-gradient products; a classifier head with few classes (last layer, loss, its input
// gradient) is one kernel.  Everything else (pooling, shortcuts, optimisers with state, batch
// assembly) is bandwidth work written as coalesced streaming kernels.  All reductions have a
// fixed order: results are bit-reproducible and a member's result does not depend on which
// other members share the pack (the isolation guarantee of Section 2.2).
#include "pack_internal.h"
#include "pack_device.h"
#include "conv_rows_halo.h"
#include "gemm_fetch.h"

#include <type_traits>
#include <utility>

namespace packk {
// Workgroup barrier for LDS hand-over only: waits for this wave's outstanding LDS operations, not for its
// global loads (__syncthreads waits for those too, which would put every round trip requested before the
// barrier in front of it).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

typedef const __attribute__((address_space(1))) u32x4_t* gvec_ptr;
typedef const __attribute__((address_space(1))) unsigned short* gu16_ptr;
typedef const __attribute__((address_space(1))) float* gf32_ptr;

// One 16-byte vector of operand A or B at (r, k), zero where the element does not exist.  The
// load is unconditional: a missing element is fetched from the problem's block of zeros, so
// nothing has to look at the loaded value until it is stored to LDS and the load can stay in
// flight across the multiplication of earlier chunks.
// The load is written as an assembly statement on purpose: the compiler does not count it as
// outstanding memory traffic, so it inserts no wait for it (left to itself it drains every
// outstanding load once per unrolled group of chunks, which serialises the pipeline).  The
// matching wait is wait_stage() below; loads of one type return in issue order, so "at most N
// newer loads outstanding" implies that a stage issued before those N has landed.
// `live` = false (a thread with no element of the tile) still issues the load, from the zeros
// block: every wave must issue the same number of loads per chunk for the count to be right.
template <int MODE, typename T, bool IS_A>
__device__ __forceinline__ u32x4_t load_vec(const GemmProb& p, int r, int k, int kend, bool live = true) {
    size_t off;
    bool ok = IS_A ? off_a<MODE>(p, r, k, off) : off_b<MODE>(p, r, k, off);
    ok = ok && (k < kend) && live;
    const T* base = (const T*)(IS_A ? p.A : p.B);
    const void* ptr = ok ? (const void*)(base + off) : p.zeros;
    u32x4_t v;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(ptr) : "memory");
    return v;
}

// gathers V scalars into one 16-byte register group (slow path for unaligned shapes)
template <int MODE, typename T, bool IS_A, bool KC>
__device__ __forceinline__ u32x4_t fetch_scalars(const GemmProb& p, int r, int k, int kend) {
    constexpr int V = ET<T>::V;
    const T* base = (const T*)(IS_A ? p.A : p.B);
    T tmp[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        const int rr = KC ? r : r + e;
        const int kk = KC ? k + e : k;
        size_t off;
        bool ok = IS_A ? off_a<MODE>(p, rr, kk, off) : off_b<MODE>(p, rr, kk, off);
        ok = ok && (kk < kend);
        const void* ptr = ok ? (const void*)(base + off) : p.zeros;
        if constexpr (sizeof(T) == 4) tmp[e] = *(gf32_ptr)ptr;
        else tmp[e] = *(gu16_ptr)ptr;
    }
    u32x4_t val;
    if constexpr (sizeof(T) == 4) {
        val.x = __float_as_uint(tmp[0]); val.y = __float_as_uint(tmp[1]);
        val.z = __float_as_uint(tmp[2]); val.w = __float_as_uint(tmp[3]);
    } else {
        val.x = (unsigned)tmp[0] | ((unsigned)tmp[1] << 16);
        val.y = (unsigned)tmp[2] | ((unsigned)tmp[3] << 16);
        val.z = (unsigned)tmp[4] | ((unsigned)tmp[5] << 16);
        val.w = (unsigned)tmp[6] | ((unsigned)tmp[7] << 16);
    }
    return val;
}

// Global -> registers.  KC operands: each thread takes 16-byte vectors along the reduction.
// RC operands (contiguous along the row index): with `vec`, each thread takes blocks of 4
// reduction indices x V rows as four 16-byte vectors each.
template <int MODE, typename T, bool IS_A, int BR, int BK, bool VEC>
__device__ __forceinline__ void fetch_tile(const GemmProb& p, int row0, int k0, int kend,
                                           u32x4_t (&regs)[TileGeom<T, BR, BK>::NREG]) {
    constexpr bool vec = VEC;
    typedef TileGeom<T, BR, BK> G;
    constexpr bool KC = IS_A ? OperandLayout<MODE>::A_KC : OperandLayout<MODE>::B_KC;
    const int tid = threadIdx.x;
    if constexpr (KC) {
#pragma unroll
        for (int s = 0; s < G::KC_SLOTS; ++s) {
            const int vid = tid + 256 * s;
            const int r = row0 + vid / G::VPR;
            const int k = k0 + (vid % G::VPR) * G::V;
            if (vec) {
                regs[s] = load_vec<MODE, T, IS_A>(p, r, k, kend, vid < G::NVEC);
            } else {
                if (G::NVEC % 256 != 0 && vid >= G::NVEC) break;
                regs[s] = fetch_scalars<MODE, T, IS_A, true>(p, r, k, kend);
            }
        }
    } else {
        if (vec) {
#pragma unroll
            for (int j = 0; j < G::RC_PER_THREAD; ++j) {
                const int b = tid + 256 * j;
                int kq, rv;
                rc_block_coords<G>(b, kq, rv);
                const int r = row0 + rv * G::V;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    regs[4 * j + e] = load_vec<MODE, T, IS_A>(p, r, k0 + kq * 4 + e, kend, b < G::RC_BLOCKS);
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < G::KC_SLOTS; ++s) {
                const int vid = tid + 256 * s;
                if (G::NVEC % 256 != 0 && vid >= G::NVEC) break;
                const int k = k0 + vid / G::RPV;
                const int r = row0 + (vid % G::RPV) * G::V;
                regs[s] = fetch_scalars<MODE, T, IS_A, false>(p, r, k, kend);
            }
        }
    }
}

// Registers -> LDS, always as rows with the reduction index contiguous.
template <int MODE, typename T, bool IS_A, int BR, int BK, bool VEC>
__device__ __forceinline__ void stash_tile(T* __restrict__ Sbase,
                                           const u32x4_t (&regs)[TileGeom<T, BR, BK>::NREG]) {
    constexpr bool vec = VEC;
    typedef TileGeom<T, BR, BK> G;
    constexpr bool KC = IS_A ? OperandLayout<MODE>::A_KC : OperandLayout<MODE>::B_KC;
    T(*S)[G::LDS_LD] = reinterpret_cast<T(*)[G::LDS_LD]>(Sbase);
    const int tid = threadIdx.x;
    if constexpr (KC) {
#pragma unroll
        for (int s = 0; s < G::KC_SLOTS; ++s) {
            const int vid = tid + 256 * s;
            if (G::NVEC % 256 != 0 && vid >= G::NVEC) break;
            *reinterpret_cast<u32x4_t*>(&S[vid / G::VPR][(vid % G::VPR) * G::V]) = regs[s];
        }
    } else if (vec) {
#pragma unroll
        for (int j = 0; j < G::RC_PER_THREAD; ++j) {
            const int b = tid + 256 * j;
            if (G::RC_BLOCKS % 256 != 0 && b >= G::RC_BLOCKS) break;
            int kq, rv;
            rc_block_coords<G>(b, kq, rv);
            const u32x4_t r0 = regs[4 * j], r1 = regs[4 * j + 1], r2 = regs[4 * j + 2], r3 = regs[4 * j + 3];
            if constexpr (sizeof(T) == 4) {
                // 4x4 transpose is a renaming of registers: row i gets component i of each vector
                *reinterpret_cast<u32x4_t*>(&S[rv * 4 + 0][kq * 4]) = u32x4_t{r0.x, r1.x, r2.x, r3.x};
                *reinterpret_cast<u32x4_t*>(&S[rv * 4 + 1][kq * 4]) = u32x4_t{r0.y, r1.y, r2.y, r3.y};
                *reinterpret_cast<u32x4_t*>(&S[rv * 4 + 2][kq * 4]) = u32x4_t{r0.z, r1.z, r2.z, r3.z};
                *reinterpret_cast<u32x4_t*>(&S[rv * 4 + 3][kq * 4]) = u32x4_t{r0.w, r1.w, r2.w, r3.w};
            } else {
                // 4 (reduction) x 8 (rows) block of 16-bit values: row i collects element i of
                // each of the four vectors into 8 bytes
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const unsigned a0 = r0[d], a1 = r1[d], a2 = r2[d], a3 = r3[d];
                    uint2 even, odd;
                    even.x = (a0 & 0xffffu) | (a1 << 16);
                    even.y = (a2 & 0xffffu) | (a3 << 16);
                    odd.x = (a0 >> 16) | (a1 & 0xffff0000u);
                    odd.y = (a2 >> 16) | (a3 & 0xffff0000u);
                    *reinterpret_cast<uint2*>(&S[rv * 8 + 2 * d][kq * 4]) = even;
                    *reinterpret_cast<uint2*>(&S[rv * 8 + 2 * d + 1][kq * 4]) = odd;
                }
            }
        }
    } else {
#pragma unroll
        for (int s = 0; s < G::KC_SLOTS; ++s) {
            const int vid = tid + 256 * s;
            if (G::NVEC % 256 != 0 && vid >= G::NVEC) break;
            const int kk = vid / G::RPV, r = (vid % G::RPV) * G::V;
            const u32x4_t v = regs[s];
            if constexpr (sizeof(T) == 4) {
                S[r + 0][kk] = __uint_as_float(v.x);
                S[r + 1][kk] = __uint_as_float(v.y);
                S[r + 2][kk] = __uint_as_float(v.z);
                S[r + 3][kk] = __uint_as_float(v.w);
            } else {
                S[r + 0][kk] = (T)(v.x & 0xffffu); S[r + 1][kk] = (T)(v.x >> 16);
                S[r + 2][kk] = (T)(v.y & 0xffffu); S[r + 3][kk] = (T)(v.y >> 16);
                S[r + 4][kk] = (T)(v.z & 0xffffu); S[r + 5][kk] = (T)(v.z >> 16);
                S[r + 6][kk] = (T)(v.w & 0xffffu); S[r + 7][kk] = (T)(v.w >> 16);
            }
        }
    }
}

// One workgroup (4 waves, 2 x 2) computes a BM x BN tile of one problem.  Every output element is
// the sum over the reduction in ascending order, sixteen (bf16) or two (fp32) indices per MFMA,
// whatever BM, BN and the LDS chunk BK are, so the choice of tile shape never changes a result bit.
// BKM scales the LDS chunk: skinny problems (few rows, long reduction) are bound by the latency
// of one global round trip per chunk, so they take chunks four times as long.
// issues one assembly load of 16 bytes from `ptr` (see load_vec for why it is assembly)
__device__ __forceinline__ u32x4_t asm_load16(const void* ptr) {
    u32x4_t v;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(ptr) : "memory");
    return v;
}

template <int... Is, typename F>
__device__ __forceinline__ void for_each_stage(std::integer_sequence<int, Is...>, F&& f) {
    (f(std::integral_constant<int, Is>{}), ...);
}

template <int BM, int BN, int BKM, bool VEC>
struct StageCount {   // register stages of prefetch per tile shape (bounded by the register file): 2, 3, 4 from the largest tile down
    static constexpr int value = (BKM > 1 || !VEC) ? 2 : ((BM * BN >= 128 * 128) ? 2 : ((BM * BN >= 128 * 64) ? 3 : 4));
};

__device__ __forceinline__ void update_one(const GemmProb& p, size_t off, float g, float lr) {
    const float w = sgd_apply(p.upd_w[off], g, lr);
    p.upd_w[off] = w;
    if (p.upd_shadow) ((bf16_t*)p.upd_shadow)[off] = ET<bf16_t>::from_f(w);
}

// Gradient that reaches output row `row` of an input-gradient problem through the block's shortcut
// (element offset into p.sc of column 0), or -1 if none does.  Identity: same pixel.  Subsampling
// shortcut: only pixels with even coordinates, from the pixel at half the coordinates; a problem
// that covers one parity class of pixels (F_ROWMAP) carries the flag only for the even-even class,
// whose rows are already numbered by the halved coordinates.
__device__ __forceinline__ long long shortcut_row(const GemmProb& p, int row) {
    if (p.flags & F_SC_ID) return (long long)out_row_base(p, row);
    int b, i, j;
    decode_row(p, row, b, i, j);
    if (!(p.flags & F_ROWMAP)) {
        if ((i | j) & 1) return -1;
        i >>= 1;
        j >>= 1;
    }
    return ((long long)(b * p.scH + i) * p.scW + j) * p.scC;
}

// LEAN (aligned operands, reductions only a few chunks long): one register stage and one LDS buffer
// instead of several.  A tile of such a product spends most of its life in its prologue and
// epilogue, so what counts is how many tiles a compute unit can hold at once, not the depth of one
// tile's pipeline.  Two forms: 128 x 128 weight gradients, whose epilogue stages the accumulators in
// two halves (three workgroups per compute unit), and 128 x 64 forward products / input gradients,
// whose LDS block is sized for the epilogue's staging tile (four workgroups per compute unit).
// Both multiply the same chunks in the same order as the regular kernels: the bits are the same.
//
// Bytes of the workgroup's LDS block: the operand buffers (two of each, one in the lean forms); the
// lean forward / input-gradient form, whose epilogue stages the whole fp32 tile, takes the larger of
// that and the staging tile.
template <typename T, int BM, int BN, int BK, bool LEAN, bool IS_DW>
struct LdsBytes {
    static constexpr size_t operands = (size_t)(LEAN ? 1 : 2) * (BM * TileGeom<T, BM, BK>::LDS_LD + BN * TileGeom<T, BN, BK>::LDS_LD) * sizeof(T);
    static constexpr size_t staging = (size_t)BM * (BN + 8) * 4;
    static constexpr size_t value = (LEAN && !IS_DW && staging > operands) ? staging : operands;
};

// The tail of a forward or input-gradient tile, shared by the staged-tile and the halo kernels.  The
// accumulators lie in LDS as fp32 (`stage`, BM rows of SLD floats), so that global memory is touched with
// 16-byte vectors along rows: bias, residual / mask source and previous value are read and the result is
// written as full vectors.  256 threads; bias_v: the forward bias of the thread's eight columns (vector form).
// MAXB: rows whose global reads are requested together (one round trip per batch).  `staged()` is called
// once, before the first read of `stage`: a caller that fills `stage` there (barrier, writes, barrier) has the
// first batch's round trip run under that instead of after it.
struct NoHook { __device__ __forceinline__ void operator()() const {} };
template <int MODE, typename T, int BM, int BN, int MAXB = 4, class Hook = NoHook>
__device__ __forceinline__ void finish_tile(const GemmProb& p, const int row0, const int col0, float (*stage)[BN + 8],
                                            const float (&bias_v)[8], const bool vec_out, Hook staged = Hook()) {
    constexpr bool IS_DW = false;   // (weight-gradient tiles have a tail of their own)
    constexpr bool IS_FWD = (MODE == LIN_FWD || MODE == CONV_FWD);
    const bool out_f32 = IS_FWD && (p.flags & F_OUT_F32);
    // element-wise tail of one output element; `v` comes from the staging tile
    auto finish = [&](float v, int row, int col, size_t off) -> float {
        if constexpr (IS_FWD) {
            v += p.bias[col];
            if (p.flags & F_RES_ID) v += ET<T>::to_f(((const T*)p.aux)[off]);
            if (p.flags & F_RES_DOWN) {
                if (col < p.resC) {
                    int bb, i, j;
                    decode_row(p, row, bb, i, j);
                    v += ET<T>::to_f(((const T*)p.aux)[((size_t)(bb * p.resH + 2 * i) * p.resW + 2 * j) * p.resC + col]);
                }
            }
            if (p.flags & F_RELU) v = fmaxf(v, 0.f);
            else if (p.act > ACT_RELU) v = act_apply(p.act, v);
        } else if constexpr (!IS_DW) {
            if (p.flags & (F_SC_ID | F_SC_DOWN)) {
                const long long so = shortcut_row(p, row);
                if (so >= 0) v += ET<T>::to_f(((const T*)p.sc)[so + col]);
            }
            if (p.flags & F_MASK) {
                const float a = ET<T>::to_f(((const T*)p.aux)[off]);
                if (p.mask_act == ACT_RELU) { if (!(a > 0.f)) v = 0.f; }
                else v *= act_deriv(p.mask_act, a);
            }
            if (p.flags & F_ACCUM) v += ET<T>::to_f(((const T*)p.C)[off]);
        }
        return v;
    };
    float* const cf = (float*)p.C;

    // vector form: 8 consecutive columns per thread (two 16-byte LDS reads); needs aligned rows.
    // A thread keeps its column group for all its rows.  What the tail reads from global memory
    // (shortcut source, mask source, previous value) is requested for a batch of rows before any
    // of it is used, so a batch costs one round trip instead of one per row.
    if (vec_out) {
        constexpr int GROUPS = BN / 8, NIT = BM * GROUPS / 256, RSTEP = 256 / GROUPS;
        constexpr int BATCH = (NIT < MAXB) ? NIT : MAXB;
        static_assert(256 % GROUPS == 0 && NIT % BATCH == 0, "tile shape");
        const int lc = (threadIdx.x % GROUPS) * 8, lr0 = threadIdx.x / GROUPS;
        const int col = col0 + lc;
        const bool full = col + 8 <= p.Q;
        typedef typename std::conditional<sizeof(T) == 2, u32x4_t, f32x4_t>::type ev_t;   // 8 bf16 or 4 floats
        constexpr int EV = (sizeof(T) == 2) ? 1 : 2;   // vectors per 8 elements
        const bool col_ok = col < p.Q;   // (a thread beyond the last column still walks the loop: `staged` may hold barriers)
        // Whole tiles of the plain cases (shortcut and residual at the same pixel, ReLU or no activation, output in
        // the pack's type): one offset per row serves every tensor the tail touches (the first row's plus a multiple
        // of one stride, or the row's pixel for the parity classes of a stride-2 input gradient) and the flags are
        // looked at once per tile instead of once per row.  The arithmetic per element is that of the general form
        // below, operation for operation.
        bool plain = !(p.flags & (F_RES_DOWN | F_SC_DOWN | F_GENERAL_TAIL)) && !out_f32 && row0 + BM <= p.R && col0 + BN <= p.Q;
        if constexpr (IS_FWD) plain = plain && ((p.flags & F_RELU) || !(p.act > ACT_RELU));
        else plain = plain && (!(p.flags & F_MASK) || p.mask_act == ACT_RELU);
        if (plain) {
            const bool by_pixel = (p.flags & F_ROWMAP) != 0;
            const size_t base = (size_t)(row0 + lr0) * p.ldc + col, step = (size_t)RSTEP * p.ldc;
            const T* ap = nullptr;
            const T* op = nullptr;
            bool relu = false, add_sc = false, mask = false, accum = false;
            if constexpr (IS_FWD) {
                if (p.flags & F_RES_ID) ap = (const T*)p.aux;
                relu = (p.flags & F_RELU) != 0;
            } else {
                mask = (p.flags & F_MASK) != 0;
                accum = (p.flags & F_ACCUM) != 0;
                add_sc = (p.flags & F_SC_ID) != 0;
                if (mask) ap = (const T*)p.aux;
                if (accum) op = (const T*)p.C;
                if (add_sc) op = (const T*)p.sc;   // never together with F_ACCUM
            }
            T* const out = (T*)p.C;
#pragma unroll 1
            for (int n0 = 0; n0 < NIT; n0 += BATCH) {
                ev_t auxv[BATCH][EV], oldv[BATCH][EV];
                size_t offn[BATCH];
#pragma unroll
                for (int n = 0; n < BATCH; ++n)
                    offn[n] = by_pixel ? out_row_base(p, row0 + lr0 + (n0 + n) * RSTEP) + col : base + (size_t)(n0 + n) * step;
                if (ap) {
#pragma unroll
                    for (int n = 0; n < BATCH; ++n)
#pragma unroll
                        for (int h = 0; h < EV; ++h) auxv[n][h] = *reinterpret_cast<const ev_t*>(ap + offn[n] + h * 4);
                } else {
#pragma unroll
                    for (int n = 0; n < BATCH; ++n)
#pragma unroll
                        for (int h = 0; h < EV; ++h) {
                            if constexpr (sizeof(T) == 2) auxv[n][h] = u32x4_t{0u, 0u, 0u, 0u};
                            else auxv[n][h] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                        }
                }
                if (op) {
#pragma unroll
                    for (int n = 0; n < BATCH; ++n)
#pragma unroll
                        for (int h = 0; h < EV; ++h) oldv[n][h] = *reinterpret_cast<const ev_t*>(op + offn[n] + h * 4);
                } else {
#pragma unroll
                    for (int n = 0; n < BATCH; ++n)
#pragma unroll
                        for (int h = 0; h < EV; ++h) {
                            if constexpr (sizeof(T) == 2) oldv[n][h] = u32x4_t{0u, 0u, 0u, 0u};
                            else oldv[n][h] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                        }
                }
                if (n0 == 0) staged();
#pragma unroll
                for (int n = 0; n < BATCH; ++n) {
                    const int lr = lr0 + (n0 + n) * RSTEP;
                    float v[8], ax[8], old[8];
                    {
                        const f32x4_t s0 = *reinterpret_cast<const f32x4_t*>(&stage[lr][lc]);
                        const f32x4_t s1 = *reinterpret_cast<const f32x4_t*>(&stage[lr][lc + 4]);
                        v[0] = s0.x; v[1] = s0.y; v[2] = s0.z; v[3] = s0.w;
                        v[4] = s1.x; v[5] = s1.y; v[6] = s1.z; v[7] = s1.w;
                    }
                    if constexpr (sizeof(T) == 2) {
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            ax[2 * d] = __uint_as_float(auxv[n][0][d] << 16); ax[2 * d + 1] = __uint_as_float(auxv[n][0][d] & 0xffff0000u);
                            old[2 * d] = __uint_as_float(oldv[n][0][d] << 16); old[2 * d + 1] = __uint_as_float(oldv[n][0][d] & 0xffff0000u);
                        }
                    } else {
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            ax[d] = auxv[n][0][d]; ax[4 + d] = auxv[n][EV - 1][d];
                            old[d] = oldv[n][0][d]; old[4 + d] = oldv[n][EV - 1][d];
                        }
                    }
                    if constexpr (IS_FWD) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = (v[e] + bias_v[e]) + ax[e];
                        if (relu) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
                        }
                    } else {
                        if (add_sc) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] += old[e];
                        }
                        if (mask) {
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (!(ax[e] > 0.f)) v[e] = 0.f;
                        }
                        if (accum) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] += old[e];
                        }
                    }
                    T* const o = out + offn[n];
                    if constexpr (sizeof(T) == 2) {
                        u32x4_t w;
#pragma unroll
                        for (int d = 0; d < 4; ++d) w[d] = pack2bf(v[2 * d], v[2 * d + 1]);
                        *reinterpret_cast<u32x4_t*>(o) = w;
                    } else {
                        *reinterpret_cast<f32x4_t*>(o) = f32x4_t{v[0], v[1], v[2], v[3]};
                        *reinterpret_cast<f32x4_t*>(o + 4) = f32x4_t{v[4], v[5], v[6], v[7]};
                    }
                }
            }
            return;
        }
        {
#pragma unroll 1
            for (int n0 = 0; n0 < NIT; n0 += BATCH) {
                size_t off[BATCH];
                bool live[BATCH];
                ev_t auxv[BATCH][EV], oldv[BATCH][EV];
#pragma unroll
                for (int n = 0; n < BATCH; ++n) {
                    const int row = row0 + lr0 + (n0 + n) * RSTEP;
                    live[n] = col_ok && row < p.R;
                    off[n] = out_row_base(p, live[n] ? row : row0) + col;
                    const T* ap = nullptr;
                    const T* op = nullptr;
                    if (live[n] && full) {
                        if constexpr (IS_FWD) {
                            if (p.flags & F_RES_ID) {
                                ap = (const T*)p.aux + off[n];
                            } else if ((p.flags & F_RES_DOWN) && col < p.resC) {
                                int bb, i, j;
                                decode_row(p, row, bb, i, j);
                                ap = (const T*)p.aux + ((size_t)(bb * p.resH + 2 * i) * p.resW + 2 * j) * p.resC + col;
                            }
                        } else if constexpr (!IS_DW) {
                            if (p.flags & F_MASK) ap = (const T*)p.aux + off[n];
                            if (p.flags & F_ACCUM) op = (const T*)p.C + off[n];
                            if (p.flags & (F_SC_ID | F_SC_DOWN)) {   // never together with F_ACCUM
                                const long long so = shortcut_row(p, row);
                                if (so >= 0) op = (const T*)p.sc + so + col;
                            }
                        }
                    }
#pragma unroll
                    for (int h = 0; h < EV; ++h) {
                        // absent source: zeros for the shortcut and the previous value, ones for the mask
                        const float fill = (!IS_FWD && !IS_DW) ? 1.f : 0.f;
                        ev_t fz;
                        if constexpr (sizeof(T) == 2) fz = u32x4_t{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
                        else fz = f32x4_t{fill, fill, fill, fill};
                        if constexpr (sizeof(T) == 2) { if (IS_FWD) fz = u32x4_t{0u, 0u, 0u, 0u}; }
                        auxv[n][h] = ap ? *reinterpret_cast<const ev_t*>(ap + h * 4) : fz;
                        ev_t oz;
                        if constexpr (sizeof(T) == 2) oz = u32x4_t{0u, 0u, 0u, 0u};
                        else oz = f32x4_t{0.f, 0.f, 0.f, 0.f};
                        oldv[n][h] = op ? *reinterpret_cast<const ev_t*>(op + h * 4) : oz;
                    }
                }
                if (n0 == 0) staged();
#pragma unroll
                for (int n = 0; n < BATCH; ++n) {
                    if (!live[n]) continue;
                    const int lr = lr0 + (n0 + n) * RSTEP;
                    const int row = row0 + lr;
                    float v[8];
                    {
                        const f32x4_t s0 = *reinterpret_cast<const f32x4_t*>(&stage[lr][lc]);
                        const f32x4_t s1 = *reinterpret_cast<const f32x4_t*>(&stage[lr][lc + 4]);
                        v[0] = s0.x; v[1] = s0.y; v[2] = s0.z; v[3] = s0.w;
                        v[4] = s1.x; v[5] = s1.y; v[6] = s1.z; v[7] = s1.w;
                    }
                    if (!full) {   // ragged right edge: element by element
                        for (int e = 0; e < 8 && col + e < p.Q; ++e) {
                            const float r = finish(v[e], row, col + e, off[n] + e);
                            if (out_f32) cf[off[n] + e] = r;
                            else ((T*)p.C)[off[n] + e] = ET<T>::from_f(r);
                        }
                        continue;
                    }
                    float ax[8], old[8];
                    if constexpr (sizeof(T) == 2) {
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            ax[2 * d] = __uint_as_float(auxv[n][0][d] << 16); ax[2 * d + 1] = __uint_as_float(auxv[n][0][d] & 0xffff0000u);
                            old[2 * d] = __uint_as_float(oldv[n][0][d] << 16); old[2 * d + 1] = __uint_as_float(oldv[n][0][d] & 0xffff0000u);
                        }
                    } else {
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            ax[d] = auxv[n][0][d]; ax[4 + d] = auxv[n][EV - 1][d];
                            old[d] = oldv[n][0][d]; old[4 + d] = oldv[n][EV - 1][d];
                        }
                    }
                    if constexpr (IS_FWD) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = (v[e] + bias_v[e]) + ax[e];
                        if (p.flags & F_RELU) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
                        } else if (p.act > ACT_RELU) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] = act_apply(p.act, v[e]);
                        }
                    } else if constexpr (!IS_DW) {
                        const bool accum = (p.flags & F_ACCUM) != 0;
                        if (p.flags & (F_SC_ID | F_SC_DOWN)) {   // the shortcut's share joins before the mask
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] += old[e];
                        }
                        if (!(p.flags & F_MASK) || p.mask_act == ACT_RELU) {   // absent mask source reads as ones
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (!(ax[e] > 0.f)) v[e] = 0.f;
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[e] *= act_deriv(p.mask_act, ax[e]);
                        }
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (accum) v[e] += old[e];
                    }
                    if (out_f32) {
                        *reinterpret_cast<f32x4_t*>(cf + off[n]) = f32x4_t{v[0], v[1], v[2], v[3]};
                        *reinterpret_cast<f32x4_t*>(cf + off[n] + 4) = f32x4_t{v[4], v[5], v[6], v[7]};
                    } else if constexpr (sizeof(T) == 2) {
                        u32x4_t o;
#pragma unroll
                        for (int d = 0; d < 4; ++d) o[d] = pack2bf(v[2 * d], v[2 * d + 1]);
                        *reinterpret_cast<u32x4_t*>((T*)p.C + off[n]) = o;
                    } else {
                        *reinterpret_cast<f32x4_t*>((float*)p.C + off[n]) = f32x4_t{v[0], v[1], v[2], v[3]};
                        *reinterpret_cast<f32x4_t*>((float*)p.C + off[n] + 4) = f32x4_t{v[4], v[5], v[6], v[7]};
                    }
                }
            }
        }
    } else {
        staged();
        for (int idx = threadIdx.x; idx < BM * BN; idx += 256) {
            const int lr = idx / BN, lc = idx % BN;
            const int row = row0 + lr, col = col0 + lc;
            if (row >= p.R || col >= p.Q) continue;
            const size_t off = out_row_base(p, row) + col;
            const float r = finish(stage[lr][lc], row, col, off);
            if (out_f32) cf[off] = r;
            else ((T*)p.C)[off] = ET<T>::from_f(r);
        }
    }
}

template <int MODE, typename T, int BM, int BN, int BKM, bool VEC, bool LEAN = false>
__device__ __forceinline__ void gemm_body(const GemmProb& p, const TileRef& tr, T* __restrict__ As_, T* __restrict__ Bs_, float lrk) {
    constexpr int V = ET<T>::V, BK = ET<T>::BK * BKM;
    typedef TileGeom<T, BM, BK> GA;
    typedef TileGeom<T, BN, BK> GB;
    constexpr int TM = BM / 64, TN = BN / 64;   // 32x32 MFMA blocks per wave in each direction
    constexpr bool IS_DW = (MODE == LIN_DW || MODE == CONV_DW);
    // Two LDS buffers (one barrier per chunk) and ST register stages: the global loads of chunk
    // i + ST are issued when chunk i starts to be multiplied, so ST - 1 round trips to memory are
    // in flight per workgroup; a skinny layer has too few workgroups per compute unit to hide that
    // latency by occupancy alone.
    constexpr int ST = LEAN ? 1 : StageCount<BM, BN, BKM, VEC>::value;
    static_assert(!LEAN || (VEC && BM == 128 && (IS_DW ? BN == 128 : BN == 64)), "lean form: aligned operands, 128x128 weight gradients or 128x64 forward / input gradients");
    T(*As)[BM][GA::LDS_LD] = reinterpret_cast<T(*)[BM][GA::LDS_LD]>(As_);
    T(*Bs)[BN][GB::LDS_LD] = reinterpret_cast<T(*)[BN][GB::LDS_LD]>(Bs_);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int row0 = tr.tm * BM, col0 = tr.tn * BN;
    const int kbeg = tr.ks * p.ksplit;
    const int kend = min(p.Kd, kbeg + p.ksplit);
    const int nk = (kend - kbeg + BK - 1) / BK;
    const bool do_bias_grad = IS_DW && tr.tn == 0 && p.dbias != nullptr;

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;
    float bias_grad = 0.f;

    u32x4_t ra[ST][GA::NREG], rb[ST][GB::NREG];
    Fetcher<MODE, T, true, BM, BK, VEC> fa;
    Fetcher<MODE, T, false, BN, BK, VEC> fb;
    fa.init(p, row0);
    fb.init(p, col0);
    // the epilogue's vector form, decided now so that the forward bias of the thread's eight
    // columns is requested before the main loop instead of at its end
    const bool vec_out = (p.ldc % 8 == 0) && (!(p.flags & F_RES_DOWN) || (p.resC % 8 == 0));
    float bias_v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if constexpr (MODE == LIN_FWD || MODE == CONV_FWD) {
        const int bcol = col0 + (int)(threadIdx.x % (BN / 8)) * 8;
        if (vec_out && bcol + 8 <= p.Q) {
            const f32x4_t b0 = *reinterpret_cast<const f32x4_t*>(p.bias + bcol);
            const f32x4_t b1 = *reinterpret_cast<const f32x4_t*>(p.bias + bcol + 4);
            bias_v[0] = b0.x; bias_v[1] = b0.y; bias_v[2] = b0.z; bias_v[3] = b0.w;
            bias_v[4] = b1.x; bias_v[5] = b1.y; bias_v[6] = b1.z; bias_v[7] = b1.w;
        }
    }
    // Weight-gradient tiles with the fused update: a thread owns four consecutive columns (one
    // 16-byte vector of fp32 weights) in DW_NIT rows, requested when the main loop ends.  (Requesting
    // some ahead of the operands measured slower: loads return in order, and the operands, which
    // come from L2, then queue behind weights that come from HBM.)
    constexpr int DW_G = BN / 4, DW_NIT = BM * DW_G / 256, DW_RSTEP = 256 / DW_G;
    const int dw_lc = (threadIdx.x % DW_G) * 4, dw_lr0 = threadIdx.x / DW_G;
    const bool dw_full = vec_out && (col0 + dw_lc + 4 <= p.Q);
    const bool upd = IS_DW && (p.flags & F_UPDATE);
    const bool keep_g = !upd || (p.flags & F_KEEP_G);
    f32x4_t dw_w[IS_DW ? DW_NIT : 1];
    constexpr int LOADS = LoadsPerChunk<MODE, T, true, BM, BK>::value + LoadsPerChunk<MODE, T, false, BN, BK>::value;
    constexpr bool ASM_WAITS = VEC;
    if constexpr (LEAN) {
        // chunk it: wait for its operands, store them to the one LDS buffer (after everybody has
        // finished reading the previous chunk from it), request chunk it + 1 into the same
        // registers, multiply
        fa.fetch(p, kbeg, kend, ra[0]);
        fb.fetch(p, kbeg, kend, rb[0]);
        for (int it = 0; it < nk; ++it) {
            wait_stage<0>(ra[0]);
            wait_stage<0>(rb[0]);
            lds_barrier();
            stash_tile<MODE, T, true, BM, BK, VEC>(&As[0][0][0], ra[0]);
            stash_tile<MODE, T, false, BN, BK, VEC>(&Bs[0][0][0], rb[0]);
            __builtin_amdgcn_sched_barrier(0);
            fa.fetch(p, kbeg + (it + 1) * BK, kend, ra[0]);   // beyond the reduction: zeros, no memory access
            fb.fetch(p, kbeg + (it + 1) * BK, kend, rb[0]);
            __builtin_amdgcn_sched_barrier(0);
            lds_barrier();
            T(*Ab)[GA::LDS_LD] = As[0];
            T(*Bb)[GB::LDS_LD] = Bs[0];
            if (do_bias_grad && threadIdx.x < BM) {
#pragma unroll
                for (int kk = 0; kk < BK; kk += V) {
                    const u32x4_t v = *reinterpret_cast<const u32x4_t*>(&Ab[threadIdx.x][kk]);
                    if constexpr (sizeof(T) == 4) {
                        bias_grad += __uint_as_float(v.x); bias_grad += __uint_as_float(v.y);
                        bias_grad += __uint_as_float(v.z); bias_grad += __uint_as_float(v.w);
                    } else {
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            bias_grad += __uint_as_float(v[d] << 16);
                            bias_grad += __uint_as_float(v[d] & 0xffff0000u);
                        }
                    }
                }
            }
#pragma unroll
            for (int kk = 0; kk < BK; kk += 2 * V) {
                u32x4_t fra[TM], frb[TN];
#pragma unroll
                for (int a = 0; a < TM; ++a)
                    fra[a] = *reinterpret_cast<const u32x4_t*>(&Ab[wm * (BM / 2) + a * 32 + (lane & 31)][kk + (lane >> 5) * V]);
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    frb[b] = *reinterpret_cast<const u32x4_t*>(&Bb[wn * (BN / 2) + b * 32 + (lane & 31)][kk + (lane >> 5) * V]);
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int b = 0; b < TN; ++b) {
                        if constexpr (sizeof(T) == 2) {
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(bf16x8_t, fra[a]), __builtin_bit_cast(bf16x8_t, frb[b]), acc[a][b], 0, 0, 0);
                        } else {
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fra[a].x), __uint_as_float(frb[b].x), acc[a][b], 0, 0, 0);
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fra[a].y), __uint_as_float(frb[b].y), acc[a][b], 0, 0, 0);
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fra[a].z), __uint_as_float(frb[b].z), acc[a][b], 0, 0, 0);
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fra[a].w), __uint_as_float(frb[b].w), acc[a][b], 0, 0, 0);
                        }
                    }
            }
        }
        // the request beyond the last chunk still targets the stage registers
        wait_stage<0>(ra[0]);
        wait_stage<0>(rb[0]);
    } else {
#pragma unroll
    for (int s = 0; s < ST; ++s) {
        // always issued: a chunk beyond the reduction reads the block of zeros.  Keeping the
        // loads unconditional keeps the loop body free of branches.
        fa.fetch(p, kbeg + s * BK, kend, ra[s]);
        fb.fetch(p, kbeg + s * BK, kend, rb[s]);
        __builtin_amdgcn_sched_barrier(0);   // keep the stages' loads in issue order
    }
    // chunk 0 goes to LDS buffer 0 ahead of the loop
    if constexpr (ASM_WAITS) {
        wait_stage<(ST - 1) * LOADS>(ra[0]);
        wait_stage<(ST - 1) * LOADS>(rb[0]);
    }
    stash_tile<MODE, T, true, BM, BK, VEC>(&As[0][0][0], ra[0]);
    stash_tile<MODE, T, false, BN, BK, VEC>(&Bs[0][0][0], rb[0]);
    // One chunk `it` (register stage s = it % ST, LDS buffer par = it & 1, both static in the
    // unrolled body).  At its barrier chunk `it` is complete in buffer par (stored during the
    // previous chunk) and nobody reads buffer par ^ 1 any more.  Then, in this order:
    //   - stage s, emptied by the previous chunk, is refilled with the loads of chunk it + ST;
    //   - the first MFMA step of chunk `it` is issued from buffer par;
    //   - chunk it + 1 (stage s + 1, with ST - 1 newer stages in flight behind it) is stored to
    //     buffer par ^ 1 while those MFMAs run: the wait for global memory and the LDS store
    //     latency hide under the multiplication instead of standing between two barriers;
    //   - the remaining MFMA steps.
    auto chunk = [&](auto S, auto PAR, const int it) {
        constexpr int s = decltype(S)::value;
        constexpr int par = decltype(PAR)::value;
        constexpr int sn = (s + 1) % ST;
        lds_barrier();
        fa.fetch(p, kbeg + (it + ST) * BK, kend, ra[s]);
        fb.fetch(p, kbeg + (it + ST) * BK, kend, rb[s]);
        __builtin_amdgcn_sched_barrier(0);
        T(*Ab)[GA::LDS_LD] = As[par];
        T(*Bb)[GB::LDS_LD] = Bs[par];
        if constexpr (IS_DW) {
            // bias gradient = sum of dz over the reduction: rows of the A tile, summed in order
            if (do_bias_grad && threadIdx.x < BM) {
#pragma unroll
                for (int kk = 0; kk < BK; kk += V) {
                    const u32x4_t v = *reinterpret_cast<const u32x4_t*>(&Ab[threadIdx.x][kk]);
                    if constexpr (sizeof(T) == 4) {
                        bias_grad += __uint_as_float(v.x); bias_grad += __uint_as_float(v.y);
                        bias_grad += __uint_as_float(v.z); bias_grad += __uint_as_float(v.w);
                    } else {
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            bias_grad += __uint_as_float(v[d] << 16);
                            bias_grad += __uint_as_float(v[d] & 0xffff0000u);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2 * V) {
            u32x4_t fa[TM], fb[TN];
#pragma unroll
            for (int a = 0; a < TM; ++a)
                fa[a] = *reinterpret_cast<const u32x4_t*>(&Ab[wm * (BM / 2) + a * 32 + (lane & 31)][kk + (lane >> 5) * V]);
#pragma unroll
            for (int b = 0; b < TN; ++b)
                fb[b] = *reinterpret_cast<const u32x4_t*>(&Bb[wn * (BN / 2) + b * 32 + (lane & 31)][kk + (lane >> 5) * V]);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b) {
                    if constexpr (sizeof(T) == 2) {
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8_t, fa[a]), __builtin_bit_cast(bf16x8_t, fb[b]), acc[a][b], 0, 0, 0);
                    } else {
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fa[a].x), __uint_as_float(fb[b].x), acc[a][b], 0, 0, 0);
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fa[a].y), __uint_as_float(fb[b].y), acc[a][b], 0, 0, 0);
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fa[a].z), __uint_as_float(fb[b].z), acc[a][b], 0, 0, 0);
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fa[a].w), __uint_as_float(fb[b].w), acc[a][b], 0, 0, 0);
                    }
                }
            if (kk == 0) {
                if constexpr (ASM_WAITS) {
                    wait_stage<(ST - 1) * LOADS>(ra[sn]);
                    wait_stage<(ST - 1) * LOADS>(rb[sn]);
                }
                stash_tile<MODE, T, true, BM, BK, VEC>(&As[par ^ 1][0][0], ra[sn]);
                stash_tile<MODE, T, false, BN, BK, VEC>(&Bs[par ^ 1][0][0], rb[sn]);
            }
        }
    };
    using std::integral_constant;
    // Chunks run in groups of G (a multiple of the stage count and of the two LDS buffers), so
    // that stage and buffer of every chunk in the unrolled body are compile-time constants and
    // the body is free of branches.  Every chunk prefetches, also the last ones, whose prefetch
    // lies beyond the reduction and reads the block of zeros.
    constexpr int G = (ST % 2 == 0) ? ST : 2 * ST;
    int it0 = 0;
    for (; it0 + G <= nk; it0 += G)
        for_each_stage(std::make_integer_sequence<int, G>{}, [&](auto J) {
            constexpr int j = decltype(J)::value;
            chunk(integral_constant<int, j % ST>{}, integral_constant<int, j & 1>{}, it0 + j);
        });
    // (the remaining chunks as nested conditions: chunk j + 1 only after chunk j, so that no path through
    // the code skips a chunk and runs a later one with the stages out of step)
    auto rest = [&](auto self, auto J) -> void {
        constexpr int j = decltype(J)::value;
        if constexpr (j < G - 1) {
            if (it0 + j < nk) {
                chunk(integral_constant<int, j % ST>{}, integral_constant<int, j & 1>{}, it0 + j);
                self(self, integral_constant<int, j + 1>{});
            }
        }
    };
    rest(rest, integral_constant<int, 0>{});
    if constexpr (VEC) {
        // The last chunks prefetched beyond the reduction (reads of the zeros block).
        // Those loads are invisible to the compiler and still target the stage registers, which
        // it would otherwise reuse for the epilogue at once: drain them, with every stage
        // register as an operand of the wait so that none of them counts as free before it.
#pragma unroll
        for (int s = 0; s < ST; ++s) {
            wait_stage<0>(ra[s]);
            wait_stage<0>(rb[s]);
        }
    }
    }   // !LEAN

    // fused update (F_UPDATE): W <- W - lr dW is applied where the gradient is produced, so the
    // gradient is neither written nor read back by a separate update launch
    if constexpr (IS_DW) {
        if (do_bias_grad && threadIdx.x < BM && row0 + (int)threadIdx.x < p.R) {
            const int r = row0 + threadIdx.x;
            if (keep_g) p.dbias[(size_t)tr.ks * p.R + r] = bias_grad;
            if (upd) p.upd_b[r] = sgd_apply(p.upd_b[r], bias_grad, lrk);
        }
    }

    // ---- epilogue ----
    // Accumulators go through LDS (as fp32) so that global memory is touched with 16-byte
    // vectors along rows: the bias, the residual / mask source and the previous value are read
    // and the result is written as full vectors instead of one element per lane.
    // Accumulator register e of a 32x32 block holds row 8*(e/4) + 4*(lane/32) + e%4, column lane%32.
    constexpr int SLD = BN + 8;   // 4 rows apart = 32 banks apart: the two half-waves do not collide
    // the lean weight-gradient form has one operand buffer: room for half the tile at a time; the lean
    // forward / input-gradient form sizes its LDS block for the whole staging tile (LeanLds below)
    constexpr int HALVES = (LEAN && IS_DW) ? 2 : 1;
    static_assert((size_t)(BM / HALVES) * SLD * 4 <= LdsBytes<T, BM, BN, BK, LEAN, IS_DW>::value, "staging tile must fit");
    float(*stage)[SLD] = reinterpret_cast<float(*)[SLD]>(As_);
    // the weights of the tile: their round trip runs under the staging of the accumulators
    if constexpr (IS_DW) {
        if (upd && dw_full) {
#pragma unroll
            for (int n = 0; n < DW_NIT; ++n) {
                const int row = row0 + dw_lr0 + n * DW_RSTEP;
                if (row < p.R) dw_w[n] = *reinterpret_cast<const f32x4_t*>(p.upd_w + (size_t)row * p.ldc + col0 + dw_lc);
            }
        }
    }
    if constexpr (LEAN && IS_DW) {
        // two passes: the waves that own the upper (then the lower) half of the rows stage their
        // accumulators, then all threads apply that half
        float* const gf = (float*)p.C + (size_t)tr.ks * p.split_stride;
        const int col = col0 + dw_lc;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            lds_barrier();   // operand tiles (half 0) or the previous half's staging no longer read
            if (wm == half) {
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            stage[a * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3)][wn * (BN / 2) + b * 32 + (lane & 31)] = acc[a][b][e];
            }
            lds_barrier();
            if (vec_out) {
                if (col < p.Q) {
#pragma unroll
                    for (int n = half * (DW_NIT / 2); n < (half + 1) * (DW_NIT / 2); ++n) {
                        const int lr = dw_lr0 + n * DW_RSTEP, row = row0 + lr;   // lr in [half * BM/2, (half + 1) * BM/2)
                        if (row >= p.R) continue;
                        const size_t off = (size_t)row * p.ldc + col;
                        const f32x4_t g = *reinterpret_cast<const f32x4_t*>(&stage[lr - half * (BM / 2)][dw_lc]);
                        if (!dw_full) {
                            for (int e = 0; e < 4 && col + e < p.Q; ++e) {
                                if (upd) update_one(p, off + e, g[e], lrk);
                                if (keep_g) gf[off + e] = g[e];
                            }
                            continue;
                        }
                        if (upd) {
                            f32x4_t w;
#pragma unroll
                            for (int e = 0; e < 4; ++e) w[e] = sgd_apply(dw_w[n][e], g[e], lrk);
                            *reinterpret_cast<f32x4_t*>(p.upd_w + off) = w;
                            if (p.upd_shadow) {
                                typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;
                                *reinterpret_cast<u32x2_t*>((bf16_t*)p.upd_shadow + off) = u32x2_t{pack2bf(w[0], w[1]), pack2bf(w[2], w[3])};
                            }
                        }
                        if (keep_g) *reinterpret_cast<f32x4_t*>(gf + off) = g;
                    }
                }
            } else {
                for (int idx = threadIdx.x; idx < (BM / 2) * BN; idx += 256) {
                    const int lr = idx / BN, lc = idx % BN;
                    const int row = row0 + half * (BM / 2) + lr, c2 = col0 + lc;
                    if (row >= p.R || c2 >= p.Q) continue;
                    const size_t off = (size_t)row * p.ldc + c2;
                    if (upd) update_one(p, off, stage[lr][lc], lrk);
                    if (keep_g) gf[off] = stage[lr][lc];
                }
            }
        }
        return;
    }
    auto fill_stage = [&]() {
        lds_barrier();   // every wave is done with the operand tiles
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    stage[wm * (BM / 2) + a * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3)][wn * (BN / 2) + b * 32 + (lane & 31)] = acc[a][b][e];
        lds_barrier();
    };
    if constexpr (IS_DW) fill_stage();

    if constexpr (IS_DW) {
        float* const gf = (float*)p.C + (size_t)tr.ks * p.split_stride;
        if (vec_out) {
            const int col = col0 + dw_lc;
            if (col < p.Q) {
#pragma unroll
                for (int n = 0; n < DW_NIT; ++n) {
                    const int lr = dw_lr0 + n * DW_RSTEP, row = row0 + lr;
                    if (row >= p.R) continue;
                    const size_t off = (size_t)row * p.ldc + col;
                    const f32x4_t g = *reinterpret_cast<const f32x4_t*>(&stage[lr][dw_lc]);
                    if (!dw_full) {   // ragged right edge: element by element
                        for (int e = 0; e < 4 && col + e < p.Q; ++e) {
                            if (upd) update_one(p, off + e, g[e], lrk);
                            if (keep_g) gf[off + e] = g[e];
                        }
                        continue;
                    }
                    if (upd) {
                        f32x4_t w;
#pragma unroll
                        for (int e = 0; e < 4; ++e) w[e] = sgd_apply(dw_w[n][e], g[e], lrk);
                        *reinterpret_cast<f32x4_t*>(p.upd_w + off) = w;
                        if (p.upd_shadow) {
                            typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;
                            *reinterpret_cast<u32x2_t*>((bf16_t*)p.upd_shadow + off) = u32x2_t{pack2bf(w[0], w[1]), pack2bf(w[2], w[3])};
                        }
                    }
                    if (keep_g) *reinterpret_cast<f32x4_t*>(gf + off) = g;
                }
            }
        } else {
            for (int idx = threadIdx.x; idx < BM * BN; idx += 256) {
                const int lr = idx / BN, lc = idx % BN;
                const int row = row0 + lr, col = col0 + lc;
                if (row >= p.R || col >= p.Q) continue;
                const size_t off = (size_t)row * p.ldc + col;
                if (upd) update_one(p, off, stage[lr][lc], lrk);
                if (keep_g) gf[off] = stage[lr][lc];
            }
        }
        return;
    }

    // forward / input gradient: what the tail reads from global memory is requested first, the accumulators are
    // staged while that round trip runs
    if constexpr (!IS_DW) finish_tile<MODE, T, BM, BN>(p, row0, col0, stage, bias_v, vec_out, fill_stage);
}

// ------------------------------------------------------------------------------------------------
// Halo form of the stride-1 convolution forward pass and input gradient (address rules: conv_rows_halo.h).
//
// The staged-tile form gathers the pixel operand again for every tap: nine times the tile's pixels cross
// the L2 -> LDS path per block of channels, and those launches run at the rate the L2 delivers, not the
// matrix cores'.  Here the pixels a tile's nine taps can reach lie in LDS once per block of channels, as
// they lie in memory, and a tap is a shift of the fragment reads' pixel slot.  The weight operand is
// staged per (channel block, tap) exactly as in the staged-tile form (same fetcher, two LDS buffers, two
// register stages, one barrier per tap).  The reduction runs channel block by channel block and tap by tap
// inside a block; with a single channel block that is the staged-tile form's order, and the bits are the same.
// ------------------------------------------------------------------------------------------------
template <int MODE, typename T, int WM, int WN, int TN>
__global__ __launch_bounds__(256, 2) void conv_rows_halo_kernel(const GemmProb* __restrict__ probs, const TileRef* __restrict__ tiles,
                                                               const void* __restrict__ x) {
    static_assert(MODE == CONV_FWD || MODE == CONV_DX, "rows are pixels");
    constexpr int ESZ = (int)sizeof(T);
    typedef RowsCfg<ESZ, WM, WN, TN> Cfg;
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::CB, V = ET<T>::V, TM = 2, NLD = Cfg::NLD, PIXB = Cfg::PIXB;
    static_assert(BK == ET<T>::BK, "a channel block is one chunk of the weight operand");
    typedef TileGeom<T, BN, BK> GB;
    constexpr size_t B_BYTES = (size_t)BN * GB::LDS_LD * ESZ, OPERANDS = Cfg::HALO_BYTES + 2 * B_BYTES, STAGING = (size_t)BM * (BN + 8) * 4;
    constexpr size_t LDS_BYTES = OPERANDS > STAGING ? OPERANDS : STAGING;
    static_assert(2 * LDS_BYTES <= 160 * 1024, "two workgroups per compute unit");
    static_assert(GB::LDS_LD * ESZ == PIXB, "both operands: 128 bytes of reduction indices per row plus 16");
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];

    const TileRef tr = tiles[blockIdx.x];
    if (tr.prob < 0) return;
    GemmProb p = probs[tr.prob];
    const void* const xin = (const char*)x + p.x_off;
    if (p.flags & F_A_INPUT) p.A = xin;
    if (p.flags & F_AUX_INPUT) p.aux = xin;

    const RowsGeom g = rows_geom<BM>(p, MODE == CONV_DX);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int row0 = tr.tm * BM, col0 = tr.tn * BN;
    const int ncb = g.SC / BK, nq = 9 * ncb;

    char* const halo = lds;
    T(*Bs)[BN][GB::LDS_LD] = reinterpret_cast<T(*)[BN][GB::LDS_LD]>(lds + Cfg::HALO_BYTES);

    // the pixel operand: a descriptor over the images of this tile, so that nothing outside them can be read
    int b0, y0;
    rows_tile_origin<BM>(p, g, tr.tm, b0, y0);
    const long long img_bytes = (long long)g.SH * g.SW * g.SC * ESZ;
    i32x4_t rs;
    {
        const unsigned long long base = (unsigned long long)p.A + (unsigned long long)b0 * (unsigned long long)img_bytes;
        rs.x = __builtin_amdgcn_readfirstlane((int)(unsigned)base);
        rs.y = __builtin_amdgcn_readfirstlane((int)(unsigned)(base >> 32));
        rs.z = __builtin_amdgcn_readfirstlane((int)(g.nimg * img_bytes));
        rs.w = 0x00020000;
    }
    unsigned hv[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) hv[i] = rows_vec_offset<Cfg, ESZ>(g, y0, tid + 256 * i);
    // channel block cb of the halo: global -> registers, and (once at most NEWER younger loads are outstanding) -> LDS
    u32x4_t rh[NLD];
    auto request_halo = [&](int cb) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) rh[i] = buf_load16(rs, hv[i], (unsigned)(cb * 128));
    };
    auto stash_halo = [&](auto NEWER) {
        wait_loads<decltype(NEWER)::value>();
        pin_regs(rh);
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            if (Cfg::MAXP * 8 % 256 == 0 || tid + 256 * i < Cfg::MAXP * 8)
                *reinterpret_cast<u32x4_t*>(halo + rows_lds_offset<Cfg>(tid + 256 * i)) = rh[i];
    };
    request_halo(0);   // first of all: its round trip runs under the rest of the set-up
    __builtin_amdgcn_sched_barrier(0);

    // the weight operand, as in the staged-tile form
    Fetcher<MODE, T, false, BN, BK, true> fb;
    fb.init(p, col0);
    constexpr int LOADS_B = LoadsPerChunk<MODE, T, false, BN, BK>::value;
    u32x4_t rb[2][GB::NREG];
    auto k_of = [&](int q) { const int cb = q / 9, tap = q - 9 * cb; return tap * g.span + cb * BK; };

    const bool vec_out = (p.ldc % 8 == 0) && (!(p.flags & F_RES_DOWN) || (p.resC % 8 == 0));
    float bias_v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if constexpr (MODE == CONV_FWD) {
        const int bcol = col0 + (tid % (BN / 8)) * 8;
        if (vec_out && bcol + 8 <= p.Q) {
            const f32x4_t b0v = *reinterpret_cast<const f32x4_t*>(p.bias + bcol);
            const f32x4_t b1v = *reinterpret_cast<const f32x4_t*>(p.bias + bcol + 4);
            bias_v[0] = b0v.x; bias_v[1] = b0v.y; bias_v[2] = b0v.z; bias_v[3] = b0v.w;
            bias_v[4] = b1v.x; bias_v[5] = b1v.y; bias_v[6] = b1v.z; bias_v[7] = b1v.w;
        }
    }

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

    // byte offset of the lane's fragment of block a inside the halo, at tap displacement (-1, -1)
    int a_off[TM];
#pragma unroll
    for (int a = 0; a < TM; ++a) a_off[a] = rows_slot(g, wm * 64 + a * 32 + (lane & 31)) * PIXB + (lane >> 5) * 16;

    fb.fetch(p, k_of(0), p.Kd, rb[0]);
    __builtin_amdgcn_sched_barrier(0);
    fb.fetch(p, k_of(1), p.Kd, rb[1]);
    __builtin_amdgcn_sched_barrier(0);
    stash_halo(std::integral_constant<int, 2 * LOADS_B>{});
    wait_stage<LOADS_B>(rb[0]);
    stash_tile<MODE, T, false, BN, BK, true>(&Bs[0][0][0], rb[0]);

    // step q = (channel block, tap); weight tile q in buffer q & 1, register stage q & 1
    auto step = [&](auto PAR, const int q) {
        constexpr int par = decltype(PAR)::value;
        const int cb = q / 9, tap = q - 9 * cb;
        lds_barrier();                              // tile q (and the halo) complete; nobody reads buffer par ^ 1 any more
        fb.fetch(p, (q + 2 < nq) ? k_of(q + 2) : p.Kd, p.Kd, rb[par]);   // beyond the reduction: zeros, no memory access
        __builtin_amdgcn_sched_barrier(0);
        const int u = tap / 3, v = tap - 3 * u;
        const char* const hp = halo + rows_tap_slots(g, u, v) * PIXB;
        T(*Bb)[GB::LDS_LD] = Bs[par];
        // The fragments of reduction step s + 1 are requested before the matrix instructions of step s are issued
        // (two sets of fragment registers; scheduling barriers keep that order), so that a wave's LDS latency
        // runs under its own matrix instructions.
        constexpr int STEPS = BK / (2 * V);
        u32x4_t fa[2][TM], fbv[2][TN];
        auto read_step = [&](auto S) {
            constexpr int st = decltype(S)::value, kk = st * 2 * V;
#pragma unroll
            for (int a = 0; a < TM; ++a) fa[st & 1][a] = *reinterpret_cast<const u32x4_t*>(hp + a_off[a] + kk * ESZ);
#pragma unroll
            for (int b = 0; b < TN; ++b)
                fbv[st & 1][b] = *reinterpret_cast<const u32x4_t*>(&Bb[wn * (TN * 32) + b * 32 + (lane & 31)][kk + (lane >> 5) * V]);
        };
        read_step(std::integral_constant<int, 0>{});
        for_each_stage(std::make_integer_sequence<int, STEPS>{}, [&](auto S) {
            constexpr int st = decltype(S)::value;
            if constexpr (st + 1 < STEPS) read_step(std::integral_constant<int, st + 1>{});
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b) {
                    const u32x4_t va = fa[st & 1][a], vb = fbv[st & 1][b];
                    if constexpr (ESZ == 2) {
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, va), __builtin_bit_cast(bf16x8_t, vb), acc[a][b], 0, 0, 0);
                    } else {
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(va.x), __uint_as_float(vb.x), acc[a][b], 0, 0, 0);
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(va.y), __uint_as_float(vb.y), acc[a][b], 0, 0, 0);
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(va.z), __uint_as_float(vb.z), acc[a][b], 0, 0, 0);
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(va.w), __uint_as_float(vb.w), acc[a][b], 0, 0, 0);
                    }
                }
            if constexpr (st == 0) {
                wait_stage<LOADS_B>(rb[par ^ 1]);
                stash_tile<MODE, T, false, BN, BK, true>(&Bs[par ^ 1][0][0], rb[par ^ 1]);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        if (tap == 8 && cb + 1 < ncb) {               // the next channel block replaces the halo once everybody has left it
            lds_barrier();
            request_halo(cb + 1);
            stash_halo(std::integral_constant<int, 0>{});
        }
    };
    using std::integral_constant;
    int q = 0;
    for (; q + 2 <= nq; q += 2) {
        step(integral_constant<int, 0>{}, q);
        step(integral_constant<int, 1>{}, q + 1);
    }
    if (q < nq) step(integral_constant<int, 0>{}, q);
    // the requests beyond the last tap still target the stage registers
    wait_stage<0>(rb[0]);
    wait_stage<0>(rb[1]);

    // The tail shared with the staged-tile form.  What it reads from global memory is requested for all of a
    // thread's rows at once, and the accumulators go to LDS (as fp32) while that round trip runs.
    float(*stage)[BN + 8] = reinterpret_cast<float(*)[BN + 8]>(lds);
    auto fill_stage = [&]() {
        lds_barrier();   // every wave is done with the operand blocks
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    stage[wm * 64 + a * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3)][wn * (TN * 32) + b * 32 + (lane & 31)] = acc[a][b][e];
        lds_barrier();
    };
    finish_tile<MODE, T, BM, BN, 8>(p, row0, col0, stage, bias_v, vec_out, fill_stage);
}

// weight-gradient kernels also take the step's learning rates (by value), the others nothing
struct NoLr {};
template <int MODE>
using LrArg = typename std::conditional<MODE == LIN_DW || MODE == CONV_DW, LrTable, NoLr>::type;

// VEC = true: every problem of the launch has both operands aligned for 16-byte loads (the planner
// sorts problems into launches by that); VEC = false: the element-by-element gather for any shape.
// They are separate kernels because the gather needs many more registers, which would halve the
// occupancy of the aligned path if both lived in one kernel.
template <int MODE, typename T, int BM, int BN, int BKM, bool VEC, bool LEAN = false>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmProb* __restrict__ probs,
                                                   const TileRef* __restrict__ tiles,
                                                   const void* __restrict__ x, char* __restrict__ ws, LrArg<MODE> lr) {
    constexpr int BK = ET<T>::BK * BKM;
    const TileRef tr = tiles[blockIdx.x];
    if (tr.prob < 0) return;
    GemmProb p = probs[tr.prob];
    // the shared input batch (Section 3.4) arrives per step; every member's first layer reads it
    // (x_off is 0 then; it is the member's own block when the members train on different data)
    const void* const xin = (const char*)x + p.x_off;
    if (p.flags & F_A_INPUT) p.A = xin;
    if (p.flags & F_B_INPUT) p.B = xin;
    if (p.flags & F_AUX_INPUT) p.aux = xin;
    if constexpr (MODE == LIN_DW || MODE == CONV_DW) {
        if (p.flags & F_WS) {   // partial sums of a split reduction go to the workspace this launch was given
            p.C = ws + (size_t)p.C;
            p.dbias = (float*)(ws + (size_t)p.dbias);
        }
    }
    // one block: operand tiles A (two buffers) then B (two buffers); the epilogue reuses it
    constexpr int NBUF = LEAN ? 1 : 2;
    __shared__ __attribute__((aligned(16))) T lds[LdsBytes<T, BM, BN, BK, LEAN, (MODE == LIN_DW || MODE == CONV_DW)>::value / sizeof(T)];
    T* const As = lds;
    T* const Bs = lds + NBUF * BM * TileGeom<T, BM, BK>::LDS_LD;
    float lrk = 0.f;
    if constexpr (MODE == LIN_DW || MODE == CONV_DW) lrk = lr.lr[p.member];
    gemm_body<MODE, T, BM, BN, BKM, VEC, LEAN>(p, tr, As, Bs, lrk);
}

template <int MODE, typename T>
static void launch_gemm_tile(int tile_cfg, const GemmProb* probs, const TileRef* tiles, int n, const void* x, char* ws, const LrTable& lr, hipStream_t st) {
    LrArg<MODE> la;
    if constexpr (MODE == LIN_DW || MODE == CONV_DW) la = lr;
    switch (tile_cfg) {
        case 0: hipLaunchKernelGGL((gemm_kernel<MODE, T, 128, 128, 1, true>), dim3(n), dim3(256), 0, st, probs, tiles, x, ws, la); break;
        case 1: hipLaunchKernelGGL((gemm_kernel<MODE, T, 128, 64, 1, true>), dim3(n), dim3(256), 0, st, probs, tiles, x, ws, la); break;
        case 2: hipLaunchKernelGGL((gemm_kernel<MODE, T, 64, 64, 1, true>), dim3(n), dim3(256), 0, st, probs, tiles, x, ws, la); break;
        case GEMM_CFG_LEAN:
            if constexpr (MODE == LIN_DW || MODE == CONV_DW)
                hipLaunchKernelGGL((gemm_kernel<MODE, T, 128, 128, 1, true, true>), dim3(n), dim3(256), 0, st, probs, tiles, x, ws, la);
            break;
        case GEMM_CFG_LEAN64:
            if constexpr (!(MODE == LIN_DW || MODE == CONV_DW))
                hipLaunchKernelGGL((gemm_kernel<MODE, T, 128, 64, 1, true, true>), dim3(n), dim3(256), 0, st, probs, tiles, x, ws, la);
            break;
        default: hipLaunchKernelGGL((gemm_kernel<MODE, T, 64, 64, 1, false>), dim3(n), dim3(256), 0, st, probs, tiles, x, ws, la); break;
    }
}

template <int MODE>
static hipError_t launch_gemm_mode(bool bf16, int tile_cfg, const GemmProb* probs, const TileRef* tiles, int n, const void* x, char* ws, const LrTable& lr, hipStream_t st) {
    if (bf16) launch_gemm_tile<MODE, bf16_t>(tile_cfg, probs, tiles, n, x, ws, lr, st);
    else launch_gemm_tile<MODE, float>(tile_cfg, probs, tiles, n, x, ws, lr, st);
    return hipGetLastError();
}

template <int MODE, typename T>
static void launch_rows_halo(int tile_cfg, const GemmProb* probs, const TileRef* tiles, int n, const void* x, hipStream_t st) {
    if (tile_cfg == GEMM_CFG_ROWS64) hipLaunchKernelGGL((conv_rows_halo_kernel<MODE, T, 4, 1, 2>), dim3(n), dim3(256), 0, st, probs, tiles, x);
    else hipLaunchKernelGGL((conv_rows_halo_kernel<MODE, T, 4, 1, 1>), dim3(n), dim3(256), 0, st, probs, tiles, x);
}

int conv_rows_halo_cfg(bool bf16, int mode, const GemmProb& p) {
    if (mode != CONV_FWD && mode != CONV_DX) return -1;
    const bool dx = mode == CONV_DX;
    if (p.flags & (F_A_INPUT | F_B_INPUT)) return -1;
    const bool narrow = p.Q <= 32;
    const bool ok = bf16 ? (narrow ? rows_halo_supported<RowsCfg<2, 4, 1, 1>>(p, dx) : rows_halo_supported<RowsCfg<2, 4, 1, 2>>(p, dx))
                         : (narrow ? rows_halo_supported<RowsCfg<4, 4, 1, 1>>(p, dx) : rows_halo_supported<RowsCfg<4, 4, 1, 2>>(p, dx));
    if (!ok) return -1;
    return narrow ? GEMM_CFG_ROWS32 : GEMM_CFG_ROWS64;
}

hipError_t launch_gemm(int mode, bool bf16, int tile_cfg, const GemmProb* probs, const TileRef* tiles, int n, const void* x, char* ws, const LrTable& lr, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (is_rows_cfg(tile_cfg)) {
        if (mode == CONV_FWD) { if (bf16) launch_rows_halo<CONV_FWD, bf16_t>(tile_cfg, probs, tiles, n, x, st); else launch_rows_halo<CONV_FWD, float>(tile_cfg, probs, tiles, n, x, st); }
        else if (mode == CONV_DX) { if (bf16) launch_rows_halo<CONV_DX, bf16_t>(tile_cfg, probs, tiles, n, x, st); else launch_rows_halo<CONV_DX, float>(tile_cfg, probs, tiles, n, x, st); }
        else return hipErrorInvalidValue;
        return hipGetLastError();
    }
    if (mode == CONV_DW && is_halo_cfg(tile_cfg)) return launch_conv_dw_halo(bf16, tile_cfg, probs, tiles, n, x, ws, lr, st);
    switch (mode) {
        case LIN_FWD: return launch_gemm_mode<LIN_FWD>(bf16, tile_cfg, probs, tiles, n, x, ws, lr, st);
        case LIN_DX: return launch_gemm_mode<LIN_DX>(bf16, tile_cfg, probs, tiles, n, x, ws, lr, st);
        case LIN_DW: return launch_gemm_mode<LIN_DW>(bf16, tile_cfg, probs, tiles, n, x, ws, lr, st);
        case CONV_FWD: return launch_gemm_mode<CONV_FWD>(bf16, tile_cfg, probs, tiles, n, x, ws, lr, st);
        case CONV_DX: return launch_gemm_mode<CONV_DX>(bf16, tile_cfg, probs, tiles, n, x, ws, lr, st);
        case CONV_DW: return launch_gemm_mode<CONV_DW>(bf16, tile_cfg, probs, tiles, n, x, ws, lr, st);
        default: return hipErrorInvalidValue;
    }
}

// out[e] = sum over S partials, in order
__global__ __launch_bounds__(256) void reduce_kernel(const ReduceProb* __restrict__ probs, const int2* __restrict__ map,
                                                     const char* __restrict__ ws, LrTable lr) {
    const int2 m = map[blockIdx.x];
    ReduceProb p = probs[m.x];
    p.in = (const float*)(ws + (size_t)p.in);   // the partial sums lie in the workspace this launch was given
    const float lrk = p.upd_w ? lr.lr[p.member] : 0.f;
    // A thread owns four elements.  Partials are added in split order; the loads of eight splits of
    // all four elements (32 loads) are issued before their adds, so that the strided reads overlap
    // instead of paying one round trip each.
    const int e0 = m.y * 1024 + threadIdx.x;
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < p.S; k0 += 8) {
        float v[4][8];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                v[i][j] = (k0 + j < p.S && e0 + i * 256 < p.n) ? p.in[(size_t)(k0 + j) * p.stride + e0 + i * 256] : 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) s[i] += v[i][j];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = e0 + i * 256;
        if (e < p.n) {
            if (p.upd_w) {   // fused update: the summed gradient goes straight into the weights
                const float w = sgd_apply(p.upd_w[e], s[i], lrk);
                p.upd_w[e] = w;
                if (p.upd_shadow) ((bf16_t*)p.upd_shadow)[e] = ET<bf16_t>::from_f(w);
            }
            if (!p.upd_w || p.keep_g) p.out[e] = s[i];
        }
    }
}

hipError_t launch_reduce(const ReduceProb* probs, const int2* map, int n, const char* ws, const LrTable& lr, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(reduce_kernel, dim3(n), dim3(256), 0, st, probs, map, ws, lr);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// softmax cross-entropy, its gradient, and the argmax: one workgroup per member
// ------------------------------------------------------------------------------------------------
constexpr int CE_WAVES = 16;   // wavefronts per workgroup
constexpr int CE_PER_LANE = 4;  // classes a lane keeps in registers (fast path: C <= 4 * lanes per row)

// One workgroup per member.  A row is handled by a group of `lpr` lanes (a power of two, at
// least min(C, 64)), so a wavefront handles 64 / lpr rows at once and the logits of a row are
// read from memory exactly once, into registers.  Row maximum (lowest index among equals), sum
// of exponentials and argmax are combined by a fixed butterfly inside the group; each group
// adds its rows' losses in row order and the groups' sums are added in a fixed order, so the
// loss is reproducible bit for bit and depends on nothing but the member's own rows.
template <typename T>
__global__ __launch_bounds__(64 * CE_WAVES) void ce_kernel(const CeProb* __restrict__ probs,
                                                            const int32_t* __restrict__ labels,
                                                            int* __restrict__ err_flag) {
    const CeProb p = probs[blockIdx.x];
    int lpr = 1;
    while (lpr < 64 && lpr < p.C) lpr <<= 1;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int rpw = 64 / lpr, sub = lane / lpr, sl = lane - sub * lpr;
    const int rows_per_pass = CE_WAVES * rpw;
    const float inv_rows = 1.f / (float)p.rows;
    const bool in_regs = p.C <= CE_PER_LANE * lpr;
    float group_loss = 0.f;
    for (int row0 = 0; row0 < p.rows; row0 += rows_per_pass) {
        const int row = row0 + wave * rpw + sub;
        const bool active = row < p.rows;
        const float* z = p.logits + (size_t)(active ? row : 0) * p.ld;
        const int y = active ? labels[p.label_off + row] : 0;
        float zv[CE_PER_LANE];
        float mx = -INFINITY;
        int arg = 0x7fffffff;
        if (in_regs) {
#pragma unroll
            for (int i = 0; i < CE_PER_LANE; ++i) {
                const int c = sl + i * lpr;
                zv[i] = (c < p.C) ? z[c] : -INFINITY;
            }
#pragma unroll
            for (int i = 0; i < CE_PER_LANE; ++i)
                if (zv[i] > mx) { mx = zv[i]; arg = sl + i * lpr; }   // ascending class index
        } else {
            for (int c = sl; c < p.C; c += lpr) {
                const float v = z[c];
                if (v > mx) { mx = v; arg = c; }
            }
        }
        for (int m = lpr >> 1; m > 0; m >>= 1) {
            const float om = __shfl_xor(mx, m, 64);
            const int oa = __shfl_xor(arg, m, 64);
            if (om > mx || (om == mx && oa < arg)) { mx = om; arg = oa; }
        }
        float ev[CE_PER_LANE];
        float s = 0.f;
        if (in_regs) {
#pragma unroll
            for (int i = 0; i < CE_PER_LANE; ++i) {
                ev[i] = (sl + i * lpr < p.C) ? expf(zv[i] - mx) : 0.f;
                s += ev[i];
            }
        } else {
            for (int c = sl; c < p.C; c += lpr) s += expf(z[c] - mx);
        }
        for (int m = lpr >> 1; m > 0; m >>= 1) s += __shfl_xor(s, m, 64);
        const bool ok = (y >= 0 && y < p.C);
        if (active && !ok && sl == 0) atomicOr(err_flag, 1);
        // the logit of the label: held by lane y % lpr of the group, slot y / lpr
        float zy = 0.f;
        if (in_regs) {
            const int yy = ok ? y : 0;
            float cand = zv[0];
#pragma unroll
            for (int i = 1; i < CE_PER_LANE; ++i)
                if (yy / lpr == i) cand = zv[i];
            zy = __shfl(cand, sub * lpr + (yy & (lpr - 1)), 64);
        } else if (ok && active) {
            zy = z[y];
        }
        if (active && ok) group_loss += (mx + logf(s)) - zy;
        const float inv_s = 1.f / s;
        T* d = (T*)p.dlogits + (size_t)(active ? row : 0) * p.ldd;
        if (active) {
            if (in_regs) {
#pragma unroll
                for (int i = 0; i < CE_PER_LANE; ++i) {
                    const int c = sl + i * lpr;
                    if (c < p.C) {
                        const float g = ok ? (ev[i] * inv_s - (c == y ? 1.f : 0.f)) * inv_rows : 0.f;
                        d[c] = ET<T>::from_f(g);
                    }
                }
            } else {
                for (int c = sl; c < p.C; c += lpr) {
                    const float g = ok ? (expf(z[c] - mx) * inv_s - (c == y ? 1.f : 0.f)) * inv_rows : 0.f;
                    d[c] = ET<T>::from_f(g);
                }
            }
            if (sl == 0) p.pred[row] = arg;
        }
    }
    // groups of one wave by a fixed butterfly over the group index, then the waves in order
    float wsum = (sl == 0) ? group_loss : 0.f;
    for (int m = 32; m >= lpr; m >>= 1) wsum += __shfl_xor(wsum, m, 64);
    __shared__ float part[CE_WAVES];
    if (lane == 0) part[wave] = wsum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int w = 0; w < CE_WAVES; ++w) t += part[w];
        *p.loss = t * inv_rows;
    }
}

hipError_t launch_ce(bool bf16, const CeProb* probs, int K, const int32_t* labels, int* err_flag, hipStream_t st) {
    if (bf16) hipLaunchKernelGGL(ce_kernel<bf16_t>, dim3(K), dim3(64 * CE_WAVES), 0, st, probs, labels, err_flag);
    else hipLaunchKernelGGL(ce_kernel<float>, dim3(K), dim3(64 * CE_WAVES), 0, st, probs, labels, err_flag);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Classifier head in one kernel (few classes): logits = h W^T + b, softmax cross-entropy with its
// gradient and the argmax, and the gradient wrt h.  With ten classes the three matrix products
// around the loss are a few MFLOP each and cost a launch apiece at the dispatch floor; here a
// block takes HEAD_ROWS rows of one member, eight lanes share a row (each a 16-byte slice of every
// 128 bytes of it) and keep the C partial sums in registers.  Every sum has a fixed order: a
// lane's slices in ascending k, the eight lanes by a butterfly, rows of a block in row order,
// blocks of a member in block order (by a small kernel when the loss is read), classes ascending
// in the input gradient.  Rounding points are those of the separate kernels: dlogits is rounded
// to the pack dtype before it is multiplied with the weights.
// ------------------------------------------------------------------------------------------------
template <typename T, int MAXC>
__global__ __launch_bounds__(256) void head_kernel(const HeadProb* __restrict__ probs, const int2* __restrict__ map,
                                                   const int32_t* __restrict__ labels, int* __restrict__ err_flag) {
    constexpr int V = ET<T>::V;
    constexpr int LPR = 256 / HEAD_ROWS;   // lanes that share a row
    constexpr int KCH = 128 * V;           // reduction indices per pass (the weights of a pass sit in LDS)
    constexpr int NV = KCH / (LPR * V);    // 16-byte vectors of a row a lane handles per pass
    typedef typename std::conditional<sizeof(T) == 2, u32x4_t, f32x4_t>::type vec_t;
    __shared__ __attribute__((aligned(16))) T Ws[MAXC][KCH];
    __shared__ float row_losses[HEAD_ROWS];
    const int2 mb = map[blockIdx.x];
    const HeadProb p = probs[mb.x];
    const int kl = threadIdx.x % LPR, lr = threadIdx.x / LPR;
    const int row = mb.y * HEAD_ROWS + lr;
    const bool active = row < p.rows;
    const T* hrow = (const T*)p.h + (size_t)(active ? row : 0) * p.Kd;
    const int nch = (p.Kd + KCH - 1) / KCH;
    auto unpack = [](const vec_t& v, float (&f)[V]) {
        if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int d = 0; d < 4; ++d) { f[2 * d] = __uint_as_float(v[d] << 16); f[2 * d + 1] = __uint_as_float(v[d] & 0xffff0000u); }
        } else {
#pragma unroll
            for (int d = 0; d < 4; ++d) f[d] = v[d];
        }
    };
    vec_t zero_v;
#pragma unroll
    for (int d = 0; d < 4; ++d) zero_v[d] = 0;
    vec_t hv[NV];
    // all of a pass's loads are requested before any is used: the lane's slices of its row ...
    auto load_h = [&](int ch) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int k = ch * KCH + (j * LPR + kl) * V;
            hv[j] = (active && k < p.Kd) ? *reinterpret_cast<const vec_t*>(hrow + k) : zero_v;
        }
    };
    // ... and the block's share of the weights of the pass, which go to LDS
    auto stage_w = [&](int ch) {
        constexpr int VPR = KCH / V;   // vectors per class row of the pass
        for (int i0 = 0; i0 < MAXC * VPR; i0 += 4 * 256) {
            vec_t wv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = i0 + u * 256 + threadIdx.x;
                const int c = idx / VPR, k = ch * KCH + (idx % VPR) * V;
                wv[u] = (c < p.C && k < p.Kd) ? *reinterpret_cast<const vec_t*>((const T*)p.W + (size_t)c * p.Kd + k) : zero_v;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = i0 + u * 256 + threadIdx.x;
                if (idx < MAXC * VPR) *reinterpret_cast<vec_t*>(&Ws[idx / VPR][(idx % VPR) * V]) = wv[u];
            }
        }
    };

    // ---- logits ----
    float acc[MAXC];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) acc[c] = 0.f;
    for (int ch = 0; ch < nch; ++ch) {
        if (ch > 0) __syncthreads();   // the previous pass's weights are no longer read
        load_h(ch);
        stage_w(ch);
        __syncthreads();
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            float hf[V];
            unpack(hv[j], hf);
            // all MAXC rows, without a branch on the class count (rows beyond it hold zeros), so
            // that the LDS reads of a slice are requested together
            vec_t wv[MAXC];
#pragma unroll
            for (int c = 0; c < MAXC; ++c) wv[c] = *reinterpret_cast<const vec_t*>(&Ws[c][(j * LPR + kl) * V]);
            __builtin_amdgcn_sched_barrier(0);   // keep the sixteen LDS reads together, ahead of their use
#pragma unroll
            for (int c = 0; c < MAXC; ++c) {
                float wf[V];
                unpack(wv[c], wf);
#pragma unroll
                for (int e = 0; e < V; ++e) acc[c] = __builtin_fmaf(hf[e], wf[e], acc[c]);
            }
        }
    }
#pragma unroll
    for (int c = 0; c < MAXC; ++c)
#pragma unroll
        for (int m = 1; m < LPR; m <<= 1) acc[c] += __shfl_xor(acc[c], m, 64);

    // ---- softmax cross-entropy of the row (every lane of the row's group computes the same) ----
    const int y = active ? labels[p.label_off + row] : 0;
    const bool ok = (y >= 0 && y < p.C);
    if (active && !ok && kl == 0) atomicOr(err_flag, 1);
    float mx = -INFINITY, zy = 0.f;
    int arg = 0;
    float bias[MAXC];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) bias[c] = p.bias[c < p.C ? c : 0];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        acc[c] = (c < p.C) ? acc[c] + bias[c] : -INFINITY;
        if (acc[c] > mx) { mx = acc[c]; arg = c; }   // ascending class index: lowest among equals
        if (c == y) zy = acc[c];
    }
    float ssum = 0.f;
    float dz[MAXC];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        dz[c] = expf(acc[c] - mx);   // exp(-inf) = 0 beyond the class count
        ssum += dz[c];
    }
    const float inv_rows = 1.f / (float)p.rows, inv_s = 1.f / ssum;
    const float row_loss = (active && ok) ? (mx + logf(ssum)) - zy : 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const float g = (ok && c < p.C) ? (dz[c] * inv_s - (c == y ? 1.f : 0.f)) * inv_rows : 0.f;
        dz[c] = ET<T>::to_f(ET<T>::from_f(g));   // as stored: the input gradient multiplies the rounded value
    }
    if (active && kl == 0) {
        float* zr = p.logits + (size_t)row * p.C;
        T* dr = (T*)p.dlogits + (size_t)row * p.ldd;
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            if (c < p.C) {
                zr[c] = acc[c];
                dr[c] = ET<T>::from_f(dz[c]);
            }
        }
        p.pred[row] = arg;
    }
    if (kl == 0) row_losses[lr] = row_loss;

    // ---- gradient wrt h: dh[r, k] = act'(h[r, k]) * sum_c dz[r, c] W[c, k] ----
    T* drow = (T*)p.dh + (size_t)(active ? row : 0) * p.Kd;
    for (int ch = 0; ch < (p.dh ? nch : 0); ++ch) {
        if (nch > 1) {   // a single pass still has its weights in LDS and its slices of h in registers
            __syncthreads();
            load_h(ch);
            stage_w(ch);
            __syncthreads();
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int k = ch * KCH + (j * LPR + kl) * V;
            float o[V];
#pragma unroll
            for (int e = 0; e < V; ++e) o[e] = 0.f;
            vec_t wv[MAXC];
#pragma unroll
            for (int c = 0; c < MAXC; ++c) wv[c] = *reinterpret_cast<const vec_t*>(&Ws[c][(j * LPR + kl) * V]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < MAXC; ++c) {   // dz is zero beyond the class count
                float wf[V];
                unpack(wv[c], wf);
#pragma unroll
                for (int e = 0; e < V; ++e) o[e] = __builtin_fmaf(dz[c], wf[e], o[e]);
            }
            if (p.mask_act != ACT_NONE) {
                float hf[V];
                unpack(hv[j], hf);
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    if (p.mask_act == ACT_RELU) { if (!(hf[e] > 0.f)) o[e] = 0.f; }
                    else o[e] *= act_deriv(p.mask_act, hf[e]);
                }
            }
            vec_t out;
            if constexpr (sizeof(T) == 2) {
#pragma unroll
                for (int d = 0; d < 4; ++d) out[d] = pack2bf(o[2 * d], o[2 * d + 1]);
            } else {
#pragma unroll
                for (int d = 0; d < 4; ++d) out[d] = o[d];
            }
            if (active && k < p.Kd) *reinterpret_cast<vec_t*>(drow + k) = out;
        }
    }

    // ---- the block's share of the member's loss: its rows in row order ----
    // (the blocks' sums are added in block order by head_loss_kernel when the loss is read)
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int r = 0; r < HEAD_ROWS; ++r) t += row_losses[r];
        p.partial[mb.y] = t;
    }
}

// loss of each member with a fused head = (sum of its blocks' sums, in block order) / rows
__global__ __launch_bounds__(256) void head_loss_kernel(const HeadProb* __restrict__ probs) {
    const HeadProb p = probs[blockIdx.x];
    __shared__ float block_sums[256];
    float total = 0.f;
    for (int b0 = 0; b0 < p.nblk; b0 += 256) {
        const int b = b0 + threadIdx.x;
        block_sums[threadIdx.x] = (b < p.nblk) ? p.partial[b] : 0.f;
        __syncthreads();
        if (threadIdx.x == 0)
            for (int i = 0; i < 256 && b0 + i < p.nblk; ++i) total += block_sums[i];
        __syncthreads();
    }
    if (threadIdx.x == 0) *p.loss = total * (1.f / (float)p.rows);
}

hipError_t launch_head_loss(const HeadProb* probs, int n_members, hipStream_t st) {
    if (n_members <= 0) return hipSuccess;
    hipLaunchKernelGGL(head_loss_kernel, dim3(n_members), dim3(256), 0, st, probs);
    return hipGetLastError();
}

template <typename T>
static void launch_head_t(int max_c, const HeadProb* probs, const int2* map, int n, const int32_t* labels, int* err_flag, hipStream_t st) {
    // instantiated for a few class counts: the kernel's arithmetic grows with the count it is built for
    if (max_c <= 4) hipLaunchKernelGGL((head_kernel<T, 4>), dim3(n), dim3(256), 0, st, probs, map, labels, err_flag);
    else if (max_c <= 10) hipLaunchKernelGGL((head_kernel<T, 10>), dim3(n), dim3(256), 0, st, probs, map, labels, err_flag);
    else hipLaunchKernelGGL((head_kernel<T, HEAD_MAX_C>), dim3(n), dim3(256), 0, st, probs, map, labels, err_flag);
}

hipError_t launch_head(bool bf16, int max_c, const HeadProb* probs, const int2* map, int n, const int32_t* labels, int* err_flag, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (max_c > HEAD_MAX_C) return hipErrorInvalidValue;
    if (bf16) launch_head_t<bf16_t>(max_c, probs, map, n, labels, err_flag, st);
    else launch_head_t<float>(max_c, probs, map, n, labels, err_flag, st);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// global average pool
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gap_fwd_kernel(const GapProb* __restrict__ probs, const int2* __restrict__ map) {
    const int2 m = map[blockIdx.x];
    const GapProb p = probs[m.x];
    const int e = m.y * 256 + threadIdx.x;   // output element (n, c)
    if (e >= p.n * p.c) return;
    const int n = e / p.c, c = e - n * p.c;
    const T* in = (const T*)p.in + (size_t)n * p.hw * p.c + c;
    // pixels are added in order; eight loads are issued before their adds so that they overlap
    float s = 0.f;
    for (int i0 = 0; i0 < p.hw; i0 += 8) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (i0 + j < p.hw) ? ET<T>::to_f(in[(size_t)(i0 + j) * p.c]) : 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) s += v[j];
    }
    ((T*)p.out)[e] = ET<T>::from_f(s / (float)p.hw);
}

template <typename T>
__global__ __launch_bounds__(256) void gap_bwd_kernel(const GapProb* __restrict__ probs, const int2* __restrict__ map) {
    const int2 m = map[blockIdx.x];
    const GapProb p = probs[m.x];
    const long long total = (long long)p.n * p.hw * p.c;
    const float inv = 1.f / (float)p.hw;
#pragma unroll
    for (int i = 0; i < ELEMWISE_PER_BLOCK / 256; ++i) {
        const long long e = (long long)m.y * ELEMWISE_PER_BLOCK + i * 256 + threadIdx.x;
        if (e >= total) break;
        const int c = (int)(e % p.c);
        const int n = (int)(e / ((long long)p.hw * p.c));
        float g = ET<T>::to_f(((const T*)p.dz_out)[(size_t)n * p.c + c]) * inv;
        if (p.mask == ACT_RELU) { if (!(ET<T>::to_f(((const T*)p.in)[e]) > 0.f)) g = 0.f; }
        else if (p.mask) g *= act_deriv(p.mask, ET<T>::to_f(((const T*)p.in)[e]));
        if (p.accum) g += ET<T>::to_f(((const T*)p.dz_in)[e]);
        ((T*)p.dz_in)[e] = ET<T>::from_f(g);
    }
}

hipError_t launch_gap(bool bf16, bool backward, const GapProb* probs, const int2* map, int n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (!backward) {
        if (bf16) hipLaunchKernelGGL(gap_fwd_kernel<bf16_t>, dim3(n), dim3(256), 0, st, probs, map);
        else hipLaunchKernelGGL(gap_fwd_kernel<float>, dim3(n), dim3(256), 0, st, probs, map);
    } else {
        if (bf16) hipLaunchKernelGGL(gap_bwd_kernel<bf16_t>, dim3(n), dim3(256), 0, st, probs, map);
        else hipLaunchKernelGGL(gap_bwd_kernel<float>, dim3(n), dim3(256), 0, st, probs, map);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// backward of the residual shortcut
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void shortcut_bwd_kernel(const ShortcutProb* __restrict__ probs, const int2* __restrict__ map) {
    const int2 m = map[blockIdx.x];
    const ShortcutProb p = probs[m.x];
    const long long total = (long long)p.n * p.H * p.W * p.C;
    constexpr int V = ET<T>::V;
    if (p.C % V == 0 && p.Co % V == 0) {
        // 16-byte vectors: V consecutive channels of one pixel
        for (int vi = threadIdx.x; vi < ELEMWISE_PER_BLOCK / V; vi += 256) {
        const long long e = ((long long)m.y * (ELEMWISE_PER_BLOCK / V) + vi) * V;
        if (e >= total) break;
        u32x4_t g = {0u, 0u, 0u, 0u};
        if (!p.down) {
            g = *reinterpret_cast<const u32x4_t*>((const T*)p.dz_out + e);
        } else {
            const int c = (int)(e % p.C);
            long long t = e / p.C;
            const int x = (int)(t % p.W);
            t /= p.W;
            const int y = (int)(t % p.H);
            const int n = (int)(t / p.H);
            if (((x | y) & 1) == 0 && (y >> 1) < p.Ho && (x >> 1) < p.Wo)
                g = *reinterpret_cast<const u32x4_t*>((const T*)p.dz_out + ((size_t)(n * p.Ho + (y >> 1)) * p.Wo + (x >> 1)) * p.Co + c);
        }
        T gv[V], sv[V], ov[V];
        __builtin_memcpy(gv, &g, 16);
        if (p.mask) { const u32x4_t t = *reinterpret_cast<const u32x4_t*>((const T*)p.src + e); __builtin_memcpy(sv, &t, 16); }
        if (p.accum) { const u32x4_t t = *reinterpret_cast<const u32x4_t*>((const T*)p.dz_src + e); __builtin_memcpy(ov, &t, 16); }
        T out[V];
#pragma unroll
        for (int i = 0; i < V; ++i) {
            float v = ET<T>::to_f(gv[i]);
            if (p.mask == ACT_RELU) { if (!(ET<T>::to_f(sv[i]) > 0.f)) v = 0.f; }
            else if (p.mask) v *= act_deriv(p.mask, ET<T>::to_f(sv[i]));
            if (p.accum) v += ET<T>::to_f(ov[i]);
            out[i] = ET<T>::from_f(v);
        }
        u32x4_t o;
        __builtin_memcpy(&o, out, 16);
        *reinterpret_cast<u32x4_t*>((T*)p.dz_src + e) = o;
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < ELEMWISE_PER_BLOCK / 256; ++i) {
        const long long e = (long long)m.y * ELEMWISE_PER_BLOCK + i * 256 + threadIdx.x;
        if (e >= total) break;
        float g;
        if (!p.down) {
            g = ET<T>::to_f(((const T*)p.dz_out)[e]);
        } else {
            const int c = (int)(e % p.C);
            long long t = e / p.C;
            const int x = (int)(t % p.W);
            t /= p.W;
            const int y = (int)(t % p.H);
            const int n = (int)(t / p.H);
            g = 0.f;
            if (((x | y) & 1) == 0 && (y >> 1) < p.Ho && (x >> 1) < p.Wo)
                g = ET<T>::to_f(((const T*)p.dz_out)[((size_t)(n * p.Ho + (y >> 1)) * p.Wo + (x >> 1)) * p.Co + c]);
        }
        if (p.mask == ACT_RELU) { if (!(ET<T>::to_f(((const T*)p.src)[e]) > 0.f)) g = 0.f; }
        else if (p.mask) g *= act_deriv(p.mask, ET<T>::to_f(((const T*)p.src)[e]));
        if (p.accum) g += ET<T>::to_f(((const T*)p.dz_src)[e]);
        ((T*)p.dz_src)[e] = ET<T>::from_f(g);
    }
}

hipError_t launch_shortcut_bwd(bool bf16, const ShortcutProb* probs, const int2* map, int n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (bf16) hipLaunchKernelGGL(shortcut_bwd_kernel<bf16_t>, dim3(n), dim3(256), 0, st, probs, map);
    else hipLaunchKernelGGL(shortcut_bwd_kernel<float>, dim3(n), dim3(256), 0, st, probs, map);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// SGD with one learning rate per member: W <- W - lr_k dW over the whole parameter arena.
// Streams 12 bytes per parameter (fp32 packs) or 14 (bf16 packs: also refreshes the bf16 copy).
// ------------------------------------------------------------------------------------------------
template <bool SHADOW>
__global__ __launch_bounds__(256) void sgd_kernel(float* __restrict__ w, const float* __restrict__ g,
                                                  bf16_t* __restrict__ shadow, long long n,
                                                  const long long* __restrict__ seg_end, int K, LrTable lr) {
    __shared__ float s_lr[256];
    __shared__ long long s_end[256];
    for (int i = threadIdx.x; i < K; i += 256) {
        s_lr[i] = lr.lr[i];
        s_end[i] = seg_end[i];
    }
    __syncthreads();
    const long long base = (long long)blockIdx.x * SGD_PER_BLOCK;
    // member that owns the first parameter of this block (segments are sorted)
    int lo = 0, hi = K - 1;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (s_end[mid] > base) hi = mid; else lo = mid + 1;
    }
    constexpr int IT = SGD_PER_BLOCK / 1024;
    f32x4_t wv[IT], gv[IT];
    long long idx[IT];
#pragma unroll
    for (int i = 0; i < IT; ++i) {
        idx[i] = base + i * 1024 + threadIdx.x * 4;
        if (idx[i] < n) {
            wv[i] = *reinterpret_cast<const f32x4_t*>(w + idx[i]);
            gv[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(g + idx[i]));
        }
    }
    int mdl = lo;
#pragma unroll
    for (int i = 0; i < IT; ++i) {
        if (idx[i] < n) {
            while (mdl < K - 1 && idx[i] >= s_end[mdl]) ++mdl;
            const float r = s_lr[mdl];
            f32x4_t o;
            o.x = sgd_apply(wv[i].x, gv[i].x, r);
            o.y = sgd_apply(wv[i].y, gv[i].y, r);
            o.z = sgd_apply(wv[i].z, gv[i].z, r);
            o.w = sgd_apply(wv[i].w, gv[i].w, r);
            // streaming stores: nothing re-reads these lines before they leave the caches
            __builtin_nontemporal_store(o, reinterpret_cast<f32x4_t*>(w + idx[i]));
            if constexpr (SHADOW) {
                typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;
                __builtin_nontemporal_store(u32x2_t{pack2bf(o.x, o.y), pack2bf(o.z, o.w)}, reinterpret_cast<u32x2_t*>(shadow + idx[i]));
            }
        }
    }
}

hipError_t launch_sgd(float* master, const float* grad, void* shadow, long long n, const long long* seg_end,
                      int K, const LrTable& lr, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    const int blocks = (int)((n + SGD_PER_BLOCK - 1) / SGD_PER_BLOCK);
    if (shadow) hipLaunchKernelGGL(sgd_kernel<true>, dim3(blocks), dim3(256), 0, st, master, grad, (bf16_t*)shadow, n, seg_end, K, lr);
    else hipLaunchKernelGGL(sgd_kernel<false>, dim3(blocks), dim3(256), 0, st, master, grad, (bf16_t*)nullptr, n, seg_end, K, lr);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// The other optimisers of the paper's search space (Table 3), each member with its own kind,
// hyper-parameters and state (Section 2.2 keeps the optimiser state with the model it belongs to):
//   momentum  acc <- mu*acc + g;  W <- W - lr*acc
//   adagrad   acc <- acc + g*g;   W <- W - lr*g/sqrt(acc)
//   adam      m <- b1*m + (1-b1)*g;  v <- b2*v + (1-b2)*g*g;  W <- W - lr*(m*c1)/(sqrt(v*c2) + eps),
//             c1 = 1/(1-b1^t), c2 = 1/(1-b2^t) for step number t (computed on the host in double)
// `m` holds the momentum / Adagrad accumulator or Adam's first moment, `v` Adam's second moment.
// Streams 20-22 bytes per parameter for momentum and Adagrad, 28-30 for Adam.  Packs whose members
// all use plain SGD never launch this kernel.
// ------------------------------------------------------------------------------------------------
enum OptKind { OPT_SGD = 0, OPT_MOMENTUM = 1, OPT_ADAGRAD = 2, OPT_ADAM = 3 };

template <bool SHADOW>
__global__ __launch_bounds__(256) void opt_kernel(float* __restrict__ w, const float* __restrict__ g,
                                                  bf16_t* __restrict__ shadow, float* __restrict__ ms,
                                                  float* __restrict__ vs, long long n,
                                                  const long long* __restrict__ seg_end,
                                                  const OptStatic* __restrict__ params, int K, OptTable tab) {
    __shared__ float s_lr[256], s_c1[256], s_c2[256];
    __shared__ long long s_end[256];
    __shared__ OptStatic s_par[256];
    for (int i = threadIdx.x; i < K; i += 256) {
        s_lr[i] = tab.lr[i];
        s_c1[i] = tab.c1[i];
        s_c2[i] = tab.c2[i];
        s_end[i] = seg_end[i];
        s_par[i] = params[i];
    }
    __syncthreads();
    const long long base = (long long)blockIdx.x * SGD_PER_BLOCK;
    int lo = 0, hi = K - 1;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (s_end[mid] > base) hi = mid; else lo = mid + 1;
    }
    int mdl = lo;
    constexpr int IT = SGD_PER_BLOCK / 1024;
    // all loads of the block's vectors are requested before any arithmetic
    long long idx[IT];
    int mem[IT];
    f32x4_t wv[IT], gv[IT], av[IT], bv[IT];
#pragma unroll
    for (int i = 0; i < IT; ++i) {
        idx[i] = base + i * 1024 + threadIdx.x * 4;
        if (idx[i] < n) {
            while (mdl < K - 1 && idx[i] >= s_end[mdl]) ++mdl;
            mem[i] = mdl;
            const int kind = s_par[mdl].kind;
            wv[i] = *reinterpret_cast<const f32x4_t*>(w + idx[i]);
            gv[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(g + idx[i]));
            if (kind != OPT_SGD) av[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(ms + idx[i]));
            if (kind == OPT_ADAM) bv[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(vs + idx[i]));
        }
    }
#pragma unroll
    for (int i = 0; i < IT; ++i) {
        if (idx[i] >= n) continue;
        const OptStatic o = s_par[mem[i]];
        const float lr = s_lr[mem[i]];
        f32x4_t wo = wv[i], a = av[i], b = bv[i];
        const f32x4_t gg = gv[i];
        if (o.kind == OPT_SGD) {
#pragma unroll
            for (int e = 0; e < 4; ++e) wo[e] = sgd_apply(wo[e], gg[e], lr);
        } else if (o.kind == OPT_MOMENTUM) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                a[e] = o.mu * a[e] + gg[e];
                wo[e] = wo[e] - lr * a[e];
            }
            __builtin_nontemporal_store(a, reinterpret_cast<f32x4_t*>(ms + idx[i]));
        } else if (o.kind == OPT_ADAGRAD) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                a[e] = a[e] + gg[e] * gg[e];
                wo[e] = wo[e] - lr * (gg[e] / sqrtf(a[e]));
            }
            __builtin_nontemporal_store(a, reinterpret_cast<f32x4_t*>(ms + idx[i]));
        } else {
            const float c1 = s_c1[mem[i]], c2 = s_c2[mem[i]];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                a[e] = o.beta1 * a[e] + (1.f - o.beta1) * gg[e];
                b[e] = o.beta2 * b[e] + (1.f - o.beta2) * (gg[e] * gg[e]);
                wo[e] = wo[e] - lr * ((a[e] * c1) / (sqrtf(b[e] * c2) + o.eps));
            }
            __builtin_nontemporal_store(a, reinterpret_cast<f32x4_t*>(ms + idx[i]));
            __builtin_nontemporal_store(b, reinterpret_cast<f32x4_t*>(vs + idx[i]));
        }
        __builtin_nontemporal_store(wo, reinterpret_cast<f32x4_t*>(w + idx[i]));
        if constexpr (SHADOW) {
            typedef __attribute__((ext_vector_type(2))) unsigned int u32x2_t;
            __builtin_nontemporal_store(u32x2_t{pack2bf(wo.x, wo.y), pack2bf(wo.z, wo.w)}, reinterpret_cast<u32x2_t*>(shadow + idx[i]));
        }
    }
}

hipError_t launch_opt(float* master, const float* grad, void* shadow, float* m, float* v, long long n,
                      const long long* seg_end, const OptStatic* params, int K, const OptTable& tab, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    const int blocks = (int)((n + SGD_PER_BLOCK - 1) / SGD_PER_BLOCK);
    if (shadow) hipLaunchKernelGGL(opt_kernel<true>, dim3(blocks), dim3(256), 0, st, master, grad, (bf16_t*)shadow, m, v, n, seg_end, params, K, tab);
    else hipLaunchKernelGGL(opt_kernel<false>, dim3(blocks), dim3(256), 0, st, master, grad, (bf16_t*)nullptr, m, v, n, seg_end, params, K, tab);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Shared-input loader for packs whose first layer is a convolution over few channels (paper
// Section 3.4: the members read ONE input).  The nine shifted views of the batch are written
// once per step as a dense matrix xcol[(b,i,j), tap*C + c] (zero for taps outside the image and
// for the padding columns up to Kp); every member's first convolution and its weight gradient
// are then plain aligned matrix products over that one buffer, instead of each member gathering
// 3-channel pixels element by element.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void im2col_kernel(Im2colProb p, const T* __restrict__ x) {
    constexpr int V = ET<T>::V;
    const int groups = p.Kp / V;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long rows = (long long)p.B * p.Ho * p.Wo;
    if (idx >= rows * groups) return;
    const int g = (int)(idx % groups);
    const long long r = idx / groups;
    const int hw = p.Ho * p.Wo;
    const int b = (int)(r / hw), rem = (int)(r - (long long)b * hw);
    const int i = rem / p.Wo, j = rem - i * p.Wo;
    T vals[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        const int k = g * V + e;
        const int tap = k / p.C, c = k - tap * p.C;
        const int y = p.stride * i + tap / 3 - 1, xx = p.stride * j + tap % 3 - 1;
        T v = (T)0;
        if (tap < 9 && (unsigned)y < (unsigned)p.H && (unsigned)xx < (unsigned)p.W)
            v = x[((size_t)(b * p.H + y) * p.W + xx) * p.C + c];
        vals[e] = v;
    }
    u32x4_t o;
    __builtin_memcpy(&o, vals, 16);
    *reinterpret_cast<u32x4_t*>((T*)p.out + (size_t)r * p.Kp + g * V) = o;
}

hipError_t launch_im2col(bool bf16, const Im2colProb& p, const void* x_dev, hipStream_t st) {
    const long long items = (long long)p.B * p.Ho * p.Wo * (p.Kp / (bf16 ? 8 : 4));
    const int blocks = (int)((items + 255) / 256);
    if (blocks <= 0) return hipSuccess;
    if (bf16) hipLaunchKernelGGL(im2col_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, p, (const bf16_t*)x_dev);
    else hipLaunchKernelGGL(im2col_kernel<float>, dim3(blocks), dim3(256), 0, st, p, (const float*)x_dev);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Per-tap transpose of convolution weights, once per step: [Cout][9][Cin] -> [Cin][9][Cout].
// The input gradient of a convolution is itself a convolution of dz with these transposed
// weights; with the copy both of its operands are contiguous along the reduction, like the
// forward pass.  One block moves a 64 x 64 (Cout x Cin) tile of one tap through LDS.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void wtranspose_kernel(const TransposeProb* __restrict__ probs, const int2* __restrict__ map) {
    __shared__ T tile[64][64 + 4 / sizeof(T)];
    const int2 pb = map[blockIdx.x];
    const TransposeProb p = probs[pb.x];
    const int tap = pb.y % 9, rest = pb.y / 9;
    const int ci0 = (rest % p.tiles_ci) * 64, co0 = (rest / p.tiles_ci) * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const T* __restrict__ src = (const T*)p.src;
    T* __restrict__ dst = (T*)p.dst;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int co = co0 + ty + 4 * i, ci = ci0 + tx;
        if (co < p.Cout && ci < p.Cin) tile[ty + 4 * i][tx] = src[((size_t)co * 9 + tap) * p.Cin + ci];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int ci = ci0 + ty + 4 * i, co = co0 + tx;
        if (co < p.Cout && ci < p.Cin) dst[((size_t)ci * 9 + tap) * p.Cout + co] = tile[tx][ty + 4 * i];
    }
}

hipError_t launch_wtranspose(bool bf16, const TransposeProb* probs_dev, const int2* map_dev, int n_blocks, hipStream_t st) {
    if (n_blocks <= 0) return hipSuccess;
    if (bf16) hipLaunchKernelGGL(wtranspose_kernel<bf16_t>, dim3(n_blocks), dim3(256), 0, st, probs_dev, map_dev);
    else hipLaunchKernelGGL(wtranspose_kernel<float>, dim3(n_blocks), dim3(256), 0, st, probs_dev, map_dev);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void cast_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst, long long n) {
    const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= n) return;
    const f32x4_t v = *reinterpret_cast<const f32x4_t*>(src + i);
    uint2 pk;
    pk.x = pack2bf(v.x, v.y);
    pk.y = pack2bf(v.z, v.w);
    *reinterpret_cast<uint2*>(dst + i) = pk;
}

hipError_t launch_cast_bf16(const float* src, void* dst, long long n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    const int blocks = (int)((n / 4 + 255) / 256);
    hipLaunchKernelGGL(cast_bf16_kernel, dim3(blocks), dim3(256), 0, st, src, (bf16_t*)dst, n);
    return hipGetLastError();
}

// Batch assembly for epochs in which the shared batch is cut from an index list (Section 3.2: the
// samples a member has not used yet): row r of the shared batch is sample idx[r] of a dataset
// resident on the device.  One block copies V * 256 bytes of one row.  An index outside the dataset
// yields a row of zeros with label -1 (which the loss kernel ignores) and sets bit 1 of the flag.
template <int V>
__global__ __launch_bounds__(256) void gather_rows_kernel(const char* __restrict__ data, const int32_t* __restrict__ labels_all,
                                                         const long long* __restrict__ idx, long long n_samples,
                                                         long long row_bytes, char* __restrict__ x_out,
                                                         int32_t* __restrict__ labels_out, int* __restrict__ err_flag) {
    typedef typename std::conditional<V == 16, u32x4_t, typename std::conditional<V == 4, unsigned, unsigned short>::type>::type vec_t;
    const long long r = blockIdx.x;
    const long long i = idx[r];
    const bool ok = i >= 0 && i < n_samples;
    const long long off = ((long long)blockIdx.y * 256 + threadIdx.x) * V;
    if (off < row_bytes) {
        vec_t v = vec_t{};
        if (ok) v = __builtin_nontemporal_load(reinterpret_cast<const vec_t*>(data + i * row_bytes + off));
        *reinterpret_cast<vec_t*>(x_out + r * row_bytes + off) = v;
    }
    if (blockIdx.y == 0 && threadIdx.x == 0) {
        labels_out[r] = ok ? labels_all[i] : -1;
        if (!ok) atomicOr(err_flag, 2);
    }
}

hipError_t launch_gather_rows(const void* data, const int32_t* labels_all, const long long* idx, long long n_samples,
                              int rows, long long row_bytes, void* x_out, int32_t* labels_out, int* err_flag, hipStream_t st) {
    if (rows <= 0) return hipSuccess;
    const uintptr_t align = (uintptr_t)data | (uintptr_t)x_out | (uintptr_t)row_bytes;
    const int V = (align % 16 == 0) ? 16 : (align % 4 == 0) ? 4 : 2;
    const dim3 grid((unsigned)rows, (unsigned)((row_bytes + (long long)V * 256 - 1) / ((long long)V * 256)));
    if (V == 16)
        hipLaunchKernelGGL(gather_rows_kernel<16>, grid, dim3(256), 0, st, (const char*)data, labels_all, idx, n_samples, row_bytes, (char*)x_out, labels_out, err_flag);
    else if (V == 4)
        hipLaunchKernelGGL(gather_rows_kernel<4>, grid, dim3(256), 0, st, (const char*)data, labels_all, idx, n_samples, row_bytes, (char*)x_out, labels_out, err_flag);
    else
        hipLaunchKernelGGL(gather_rows_kernel<2>, grid, dim3(256), 0, st, (const char*)data, labels_all, idx, n_samples, row_bytes, (char*)x_out, labels_out, err_flag);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4_t* __restrict__ dst, long long n16) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) dst[i] = u32x4_t{0u, 0u, 0u, 0u};
}

hipError_t launch_fill_zero(void* dst, long long bytes, hipStream_t st) {
    if (bytes <= 0) return hipSuccess;
    const long long n16 = bytes / 16;   // buffers are allocated in multiples of 256 bytes
    const int blocks = (int)((n16 + 255) / 256);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, st, (u32x4_t*)dst, n16);
    return hipGetLastError();
}

// ---- scratch memory the library owns without allocating it ---------------------------------------
// For callers that may not allocate device memory (pack_step_static): the partial sums of split weight
// gradients go here instead of into the pack's own workspace.  Every GPU the library runs on holds its
// own copy of the array, at its own address, until the process ends; host code never uses the array's
// name as an address, only what hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

hipError_t static_scratch(char** ptr) {
    void* dev = nullptr;
    const hipError_t e = hipGetSymbolAddress(&dev, HIP_SYMBOL(scratch));
    *ptr = (e == hipSuccess) ? (char*)dev : nullptr;
    return e;
}

// ---- measured ceilings --------------------------------------------------------------------------
// Two measuring aids, so that a kernel's rate can be set beside what this chip delivers on the
// simplest possible code as well as beside the published peak: a streaming copy (every byte read
// once and written once, 64 bytes in flight per thread) and a loop of matrix instructions on
// operands that never leave the registers (four independent accumulator tiles per wave, so that
// no instruction waits for the one before it).
__global__ __launch_bounds__(256) void ceiling_copy_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst, long long n16) {
    const long long base = (long long)blockIdx.x * 1024 + threadIdx.x;
    u32x4_t v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (base + j * 256 < n16) v[j] = __builtin_nontemporal_load(src + base + j * 256);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (base + j * 256 < n16) __builtin_nontemporal_store(v[j], dst + base + j * 256);
}

template <bool BF16>
__global__ __launch_bounds__(256) void ceiling_mfma_kernel(float* __restrict__ out, int iters) {
    f32x16_t acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.0f;
    // operands near 1.0 that depend on the lane, so that nothing can be folded at compile time
    const unsigned lane_bit = threadIdx.x & 1u;
    const u32x4_t a = u32x4_t{0x3f803f80u + lane_bit, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    const u32x4_t b = u32x4_t{0x3f803f80u, 0x3f803f80u + lane_bit, 0x3f803f80u, 0x3f803f80u};
    const float af = 1.0f + 0.5f * (float)lane_bit, bf = 1.0f - 0.25f * (float)lane_bit;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (BF16)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), acc[j], 0, 0, 0);
            else
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af, bf, acc[j], 0, 0, 0);
        }
    }
    float sum = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) sum += acc[j][e];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = sum;
}

hipError_t launch_ceiling_copy(const void* src, void* dst, long long bytes, hipStream_t st) {
    const long long n16 = bytes / 16;
    if (n16 <= 0) return hipSuccess;
    hipLaunchKernelGGL(ceiling_copy_kernel, dim3((unsigned)((n16 + 1023) / 1024)), dim3(256), 0, st, (const u32x4_t*)src, (u32x4_t*)dst, n16);
    return hipGetLastError();
}

// `out` holds blocks * 256 floats; returns the flops of the launch in *flops
hipError_t launch_ceiling_mfma(bool bf16, float* out, int blocks, int iters, double* flops, hipStream_t st) {
    if (bf16) hipLaunchKernelGGL(ceiling_mfma_kernel<true>, dim3(blocks), dim3(256), 0, st, out, iters);
    else hipLaunchKernelGGL(ceiling_mfma_kernel<false>, dim3(blocks), dim3(256), 0, st, out, iters);
    const double per = bf16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
    *flops = (double)blocks * 4.0 * (double)iters * 4.0 * per;
    return hipGetLastError();
}

}  // namespace packk
