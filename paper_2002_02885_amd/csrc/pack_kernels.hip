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
// 16-byte access.  Everything else (softmax cross-entropy, pooling, bias gradients, the SGD
// update) is bandwidth work written as coalesced streaming kernels.  All reductions have a
// fixed order: results are bit-reproducible and a member's result does not depend on which
// other members share the pack (the isolation guarantee of Section 2.2).
#include "pack_internal.h"

namespace packk {

typedef unsigned short bf16_t;   // bfloat16 = upper half of an IEEE binary32
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

// round to nearest, ties to even; NaN stays NaN (quiet)
__device__ __forceinline__ bf16_t f2bf(float f) {
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((unsigned int)h) << 16); }

template <typename T> struct ET;
template <> struct ET<float> {
    static constexpr int V = 4;    // elements per 16-byte vector
    static constexpr int BK = 32;  // reduction indices per LDS tile
    static __device__ __forceinline__ float to_f(float v) { return v; }
    static __device__ __forceinline__ float from_f(float v) { return v; }
};
template <> struct ET<bf16_t> {
    static constexpr int V = 8;
    static constexpr int BK = 64;
    static __device__ __forceinline__ float to_f(bf16_t v) { return bf2f(v); }
    static __device__ __forceinline__ bf16_t from_f(float v) { return f2bf(v); }
};

// ------------------------------------------------------------------------------------------------
// operand address rules: element (row, k) of operand A / B for each mode, or null for "zero"
// ------------------------------------------------------------------------------------------------
template <int MODE, typename T>
__device__ __forceinline__ const T* addr_a(const GemmProb& p, int r, int k) {
    if (r >= p.R || k >= p.Kd) return nullptr;
    const T* A = (const T*)p.A;
    if constexpr (MODE == LIN_FWD || MODE == LIN_DX) {
        return A + (size_t)r * p.lda + k;
    } else if constexpr (MODE == LIN_DW || MODE == CONV_DW) {
        return A + (size_t)k * p.lda + r;
    } else if constexpr (MODE == CONV_FWD) {
        const int hw = p.Ho * p.Wo;
        const int b = r / hw, rem = r - b * hw;
        const int i = rem / p.Wo, j = rem - i * p.Wo;
        const int tap = k / p.Cin, c = k - tap * p.Cin;
        const int u = tap / 3, v = tap - 3 * u;
        const int y = p.stride * i + u - 1, x = p.stride * j + v - 1;
        if ((unsigned)y >= (unsigned)p.H || (unsigned)x >= (unsigned)p.W) return nullptr;
        return A + ((size_t)(b * p.H + y) * p.W + x) * p.Cin + c;
    } else {  // CONV_DX: row = input pixel (b, y, x), k = (tap, o)
        const int hw = p.H * p.W;
        const int b = r / hw, rem = r - b * hw;
        const int y = rem / p.W, x = rem - y * p.W;
        const int tap = k / p.Cout, o = k - tap * p.Cout;
        const int u = tap / 3, v = tap - 3 * u;
        int ty = y + 1 - u, tx = x + 1 - v;
        if (ty < 0 || tx < 0) return nullptr;
        if (p.stride == 2) {
            if ((ty | tx) & 1) return nullptr;
            ty >>= 1;
            tx >>= 1;
        }
        if (ty >= p.Ho || tx >= p.Wo) return nullptr;
        return A + ((size_t)(b * p.Ho + ty) * p.Wo + tx) * p.Cout + o;
    }
}

template <int MODE, typename T>
__device__ __forceinline__ const T* addr_b(const GemmProb& p, int q, int k) {
    if (q >= p.Q || k >= p.Kd) return nullptr;
    const T* B = (const T*)p.B;
    if constexpr (MODE == LIN_FWD || MODE == CONV_FWD) {
        return B + (size_t)q * p.ldb + k;
    } else if constexpr (MODE == LIN_DX || MODE == LIN_DW) {
        return B + (size_t)k * p.ldb + q;
    } else if constexpr (MODE == CONV_DX) {   // q = input channel c, k = (tap, o); W is [Cout][9][Cin]
        const int tap = k / p.Cout, o = k - tap * p.Cout;
        return B + ((size_t)o * 9 + tap) * p.Cin + q;
    } else {  // CONV_DW: q = (tap, c), k = output pixel (b, i, j)
        const int tap = q / p.Cin, c = q - tap * p.Cin;
        const int u = tap / 3, v = tap - 3 * u;
        const int hw = p.Ho * p.Wo;
        const int b = k / hw, rem = k - b * hw;
        const int i = rem / p.Wo, j = rem - i * p.Wo;
        const int y = p.stride * i + u - 1, x = p.stride * j + v - 1;
        if ((unsigned)y >= (unsigned)p.H || (unsigned)x >= (unsigned)p.W) return nullptr;
        return B + ((size_t)(b * p.H + y) * p.W + x) * p.Cin + c;
    }
}

// Which operands are contiguous along the reduction (KC) and which along their row index (RC).
template <int MODE> struct OperandLayout {
    static constexpr bool A_KC = (MODE == LIN_FWD || MODE == LIN_DX || MODE == CONV_FWD || MODE == CONV_DX);
    static constexpr bool B_KC = (MODE == LIN_FWD || MODE == CONV_FWD);
};

// ------------------------------------------------------------------------------------------------
// grouped MFMA GEMM
// ------------------------------------------------------------------------------------------------
// LDS tile of one operand: BR rows x BK reduction indices, each row padded by 16 bytes so that
// the 16-byte fragment reads of 16 consecutive rows fall into 64 different banks.
template <typename T, int BR>
struct TileGeom {
    static constexpr int V = ET<T>::V;
    static constexpr int BK = ET<T>::BK;
    static constexpr int LDS_LD = BK + V;
    static constexpr int VPR = BK / V;                 // KC: 16-byte vectors per row
    static constexpr int KC_SLOTS = BR * BK / V / 256; // KC: vectors per thread
    static constexpr int RPV = BR / V;                 // RC scalar fallback: row-vectors per reduction index
    static constexpr int KQ = BK / 4;                  // RC: groups of 4 reduction indices
    static constexpr int RC_BLOCKS = KQ * (BR / V);    // RC: (4 x V) blocks per tile, one per thread
    static constexpr int SLOTS = 4;                    // registers reserved per operand (u32x4 each)
    static_assert(KC_SLOTS <= SLOTS && RC_BLOCKS <= 256 && BR * BK / V / 256 >= 1, "tile too large or too small");
};

template <int MODE, typename T, bool IS_A>
__device__ __forceinline__ const T* operand_addr(const GemmProb& p, int r, int k) {
    if constexpr (IS_A) return addr_a<MODE, T>(p, r, k);
    else return addr_b<MODE, T>(p, r, k);
}

// gathers V scalars into one 16-byte register group (slow path for unaligned shapes)
template <int MODE, typename T, bool IS_A, bool KC>
__device__ __forceinline__ u32x4_t fetch_scalars(const GemmProb& p, int r, int k, int kend) {
    constexpr int V = ET<T>::V;
    T tmp[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
        const int rr = KC ? r : r + e;
        const int kk = KC ? k + e : k;
        const T* ptr = (kk < kend) ? operand_addr<MODE, T, IS_A>(p, rr, kk) : nullptr;
        tmp[e] = ptr ? *ptr : (T)0;
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
// RC operands (contiguous along the row index): with `vec`, each thread takes a block of 4
// reduction indices x V rows as four 16-byte vectors, thread index varying fastest along the
// reduction so that the transposed LDS stores of a wave fall into distinct banks.
template <int MODE, typename T, bool IS_A, int BR>
__device__ __forceinline__ void fetch_tile(const GemmProb& p, int row0, int k0, int kend, bool vec,
                                           u32x4_t (&regs)[4]) {
    typedef TileGeom<T, BR> G;
    constexpr bool KC = IS_A ? OperandLayout<MODE>::A_KC : OperandLayout<MODE>::B_KC;
    const int tid = threadIdx.x;
    if constexpr (KC) {
#pragma unroll
        for (int s = 0; s < G::KC_SLOTS; ++s) {
            const int vid = tid + 256 * s;
            const int r = row0 + vid / G::VPR;
            const int k = k0 + (vid % G::VPR) * G::V;
            if (vec) {
                const T* ptr = (k < kend) ? operand_addr<MODE, T, IS_A>(p, r, k) : nullptr;
                regs[s] = ptr ? *reinterpret_cast<const u32x4_t*>(ptr) : u32x4_t{0u, 0u, 0u, 0u};
            } else {
                regs[s] = fetch_scalars<MODE, T, IS_A, true>(p, r, k, kend);
            }
        }
    } else {
        if (vec) {
            if (tid < G::RC_BLOCKS) {
                const int kq = tid % G::KQ, rv = tid / G::KQ;
                const int r = row0 + rv * G::V;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k = k0 + kq * 4 + e;
                    const T* ptr = (k < kend) ? operand_addr<MODE, T, IS_A>(p, r, k) : nullptr;
                    regs[e] = ptr ? *reinterpret_cast<const u32x4_t*>(ptr) : u32x4_t{0u, 0u, 0u, 0u};
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < G::KC_SLOTS; ++s) {
                const int vid = tid + 256 * s;
                const int k = k0 + vid / G::RPV;
                const int r = row0 + (vid % G::RPV) * G::V;
                regs[s] = fetch_scalars<MODE, T, IS_A, false>(p, r, k, kend);
            }
        }
    }
}

// Registers -> LDS, always as rows with the reduction index contiguous.
template <int MODE, typename T, bool IS_A, int BR>
__device__ __forceinline__ void stash_tile(T* __restrict__ Sbase, bool vec, const u32x4_t (&regs)[4]) {
    typedef TileGeom<T, BR> G;
    constexpr bool KC = IS_A ? OperandLayout<MODE>::A_KC : OperandLayout<MODE>::B_KC;
    T(*S)[G::LDS_LD] = reinterpret_cast<T(*)[G::LDS_LD]>(Sbase);
    const int tid = threadIdx.x;
    if constexpr (KC) {
#pragma unroll
        for (int s = 0; s < G::KC_SLOTS; ++s) {
            const int vid = tid + 256 * s;
            *reinterpret_cast<u32x4_t*>(&S[vid / G::VPR][(vid % G::VPR) * G::V]) = regs[s];
        }
    } else if (vec) {
        if (tid < G::RC_BLOCKS) {
            const int kq = tid % G::KQ, rv = tid / G::KQ;
            if constexpr (sizeof(T) == 4) {
                // 4x4 transpose is a renaming of registers: row j gets component j of each vector
                const u32x4_t c0 = {regs[0].x, regs[1].x, regs[2].x, regs[3].x};
                const u32x4_t c1 = {regs[0].y, regs[1].y, regs[2].y, regs[3].y};
                const u32x4_t c2 = {regs[0].z, regs[1].z, regs[2].z, regs[3].z};
                const u32x4_t c3 = {regs[0].w, regs[1].w, regs[2].w, regs[3].w};
                *reinterpret_cast<u32x4_t*>(&S[rv * 4 + 0][kq * 4]) = c0;
                *reinterpret_cast<u32x4_t*>(&S[rv * 4 + 1][kq * 4]) = c1;
                *reinterpret_cast<u32x4_t*>(&S[rv * 4 + 2][kq * 4]) = c2;
                *reinterpret_cast<u32x4_t*>(&S[rv * 4 + 3][kq * 4]) = c3;
            } else {
                // 4 (reduction) x 8 (rows) block of 16-bit values: row j collects element j of
                // each of the four vectors into 8 bytes
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const unsigned a0 = regs[0][d], a1 = regs[1][d], a2 = regs[2][d], a3 = regs[3][d];
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
// the sum over the reduction in ascending chunks of BK, whatever BM and BN are, so the choice of
// tile shape never changes a result bit.
template <int MODE, typename T, int BM, int BN>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmProb* __restrict__ probs,
                                                   const TileRef* __restrict__ tiles,
                                                   const void* __restrict__ x) {
    typedef TileGeom<T, BM> GA;
    typedef TileGeom<T, BN> GB;
    constexpr int V = ET<T>::V, BK = ET<T>::BK;
    constexpr int TM = BM / 64, TN = BN / 64;   // 32x32 MFMA blocks per wave in each direction
    constexpr bool IS_DW = (MODE == LIN_DW || MODE == CONV_DW);

    const TileRef tr = tiles[blockIdx.x];
    if (tr.prob < 0) return;
    GemmProb p = probs[tr.prob];
    // the shared input batch (Section 3.4) arrives per step; every member's first layer reads it
    if (p.flags & F_A_INPUT) p.A = x;
    if (p.flags & F_B_INPUT) p.B = x;
    if (p.flags & F_AUX_INPUT) p.aux = x;

    __shared__ __attribute__((aligned(16))) T As[BM][GA::LDS_LD];
    __shared__ __attribute__((aligned(16))) T Bs[BN][GB::LDS_LD];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int row0 = tr.tm * BM, col0 = tr.tn * BN;
    const int kbeg = tr.ks * p.ksplit;
    const int kend = min(p.Kd, kbeg + p.ksplit);
    const bool vecA = (p.flags & F_VEC_A) != 0, vecB = (p.flags & F_VEC_B) != 0;
    const bool do_bias_grad = IS_DW && tr.tn == 0 && p.dbias != nullptr;

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;
    float bias_grad = 0.f;

    u32x4_t ra[4], rb[4];
    if (kbeg < kend) {
        fetch_tile<MODE, T, true, BM>(p, row0, kbeg, kend, vecA, ra);
        fetch_tile<MODE, T, false, BN>(p, col0, kbeg, kend, vecB, rb);
    }
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads();   // all waves are done reading the previous tile
        stash_tile<MODE, T, true, BM>(&As[0][0], vecA, ra);
        stash_tile<MODE, T, false, BN>(&Bs[0][0], vecB, rb);
        __syncthreads();
        if (k0 + BK < kend) {   // next tile's global loads fly while this tile is multiplied
            fetch_tile<MODE, T, true, BM>(p, row0, k0 + BK, kend, vecA, ra);
            fetch_tile<MODE, T, false, BN>(p, col0, k0 + BK, kend, vecB, rb);
        }
        if constexpr (IS_DW) {
            // bias gradient = sum of dz over the reduction: rows of the A tile, summed in order
            if (do_bias_grad && threadIdx.x < BM) {
#pragma unroll
                for (int kk = 0; kk < BK; kk += V) {
                    const u32x4_t v = *reinterpret_cast<const u32x4_t*>(&As[threadIdx.x][kk]);
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
                fa[a] = *reinterpret_cast<const u32x4_t*>(&As[wm * (BM / 2) + a * 32 + (lane & 31)][kk + (lane >> 5) * V]);
#pragma unroll
            for (int b = 0; b < TN; ++b)
                fb[b] = *reinterpret_cast<const u32x4_t*>(&Bs[wn * (BN / 2) + b * 32 + (lane & 31)][kk + (lane >> 5) * V]);
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
        }
    }

    if constexpr (IS_DW) {
        if (do_bias_grad && threadIdx.x < BM && row0 + (int)threadIdx.x < p.R)
            p.dbias[(size_t)tr.ks * p.R + row0 + threadIdx.x] = bias_grad;
    }

    // epilogue: accumulator register e of a 32x32 block holds row 8*(e/4) + 4*(lane/32) + e%4,
    // column lane%32
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = row0 + wm * (BM / 2) + a * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                const int col = col0 + wn * (BN / 2) + b * 32 + (lane & 31);
                if (row >= p.R || col >= p.Q) continue;
                float v = acc[a][b][e];
                const size_t off = (size_t)row * p.ldc + col;
                if constexpr (MODE == LIN_FWD || MODE == CONV_FWD) {
                    v += p.bias[col];
                    if (p.flags & F_RES_ID) v += ET<T>::to_f(((const T*)p.aux)[off]);
                    if (p.flags & F_RES_DOWN) {
                        if (col < p.resC) {
                            const int hw = p.Ho * p.Wo;
                            const int bb = row / hw, rem = row - bb * hw;
                            const int i = rem / p.Wo, j = rem - i * p.Wo;
                            v += ET<T>::to_f(((const T*)p.aux)[((size_t)(bb * p.resH + 2 * i) * p.resW + 2 * j) * p.resC + col]);
                        }
                    }
                    if (p.flags & F_RELU) v = fmaxf(v, 0.f);
                    if (p.flags & F_OUT_F32) ((float*)p.C)[off] = v;
                    else ((T*)p.C)[off] = ET<T>::from_f(v);
                } else if constexpr (MODE == LIN_DX || MODE == CONV_DX) {
                    if (p.flags & F_MASK) {
                        if (!(ET<T>::to_f(((const T*)p.aux)[off]) > 0.f)) v = 0.f;
                    }
                    if (p.flags & F_ACCUM) v += ET<T>::to_f(((const T*)p.C)[off]);
                    ((T*)p.C)[off] = ET<T>::from_f(v);
                } else {
                    ((float*)p.C)[(size_t)tr.ks * p.split_stride + off] = v;
                }
            }
}

template <int MODE, typename T>
static void launch_gemm_tile(int tile_cfg, const GemmProb* probs, const TileRef* tiles, int n, const void* x, hipStream_t st) {
    switch (tile_cfg) {
        case 0: hipLaunchKernelGGL((gemm_kernel<MODE, T, 128, 128>), dim3(n), dim3(256), 0, st, probs, tiles, x); break;
        case 1: hipLaunchKernelGGL((gemm_kernel<MODE, T, 128, 64>), dim3(n), dim3(256), 0, st, probs, tiles, x); break;
        default: hipLaunchKernelGGL((gemm_kernel<MODE, T, 64, 64>), dim3(n), dim3(256), 0, st, probs, tiles, x); break;
    }
}

template <int MODE>
static hipError_t launch_gemm_mode(bool bf16, int tile_cfg, const GemmProb* probs, const TileRef* tiles, int n, const void* x, hipStream_t st) {
    if (bf16) launch_gemm_tile<MODE, bf16_t>(tile_cfg, probs, tiles, n, x, st);
    else launch_gemm_tile<MODE, float>(tile_cfg, probs, tiles, n, x, st);
    return hipGetLastError();
}

hipError_t launch_gemm(int mode, bool bf16, int tile_cfg, const GemmProb* probs, const TileRef* tiles, int n, const void* x, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    switch (mode) {
        case LIN_FWD: return launch_gemm_mode<LIN_FWD>(bf16, tile_cfg, probs, tiles, n, x, st);
        case LIN_DX: return launch_gemm_mode<LIN_DX>(bf16, tile_cfg, probs, tiles, n, x, st);
        case LIN_DW: return launch_gemm_mode<LIN_DW>(bf16, tile_cfg, probs, tiles, n, x, st);
        case CONV_FWD: return launch_gemm_mode<CONV_FWD>(bf16, tile_cfg, probs, tiles, n, x, st);
        case CONV_DX: return launch_gemm_mode<CONV_DX>(bf16, tile_cfg, probs, tiles, n, x, st);
        case CONV_DW: return launch_gemm_mode<CONV_DW>(bf16, tile_cfg, probs, tiles, n, x, st);
        default: return hipErrorInvalidValue;
    }
}

// out[e] = sum over S partials, in order
__global__ __launch_bounds__(256) void reduce_kernel(const ReduceProb* __restrict__ probs, const int2* __restrict__ map) {
    const int2 m = map[blockIdx.x];
    const ReduceProb p = probs[m.x];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = m.y * 1024 + i * 256 + threadIdx.x;
        if (e < p.n) {
            float s = 0.f;
            for (int k = 0; k < p.S; ++k) s += p.in[(size_t)k * p.stride + e];
            p.out[e] = s;
        }
    }
}

hipError_t launch_reduce(const ReduceProb* probs, const int2* map, int n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(reduce_kernel, dim3(n), dim3(256), 0, st, probs, map);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// softmax cross-entropy, its gradient, and the argmax: one workgroup per member
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ce_kernel(const CeProb* __restrict__ probs, const int32_t* __restrict__ labels,
                                                 int* __restrict__ err_flag) {
    const CeProb p = probs[blockIdx.x];
    const float inv_rows = 1.f / (float)p.rows;
    float local = 0.f;
    for (int row = threadIdx.x; row < p.rows; row += 256) {
        const float* z = p.logits + (size_t)row * p.ld;
        float mx = z[0];
        int arg = 0;
        for (int c = 1; c < p.C; ++c) {
            const float v = z[c];
            if (v > mx) { mx = v; arg = c; }   // strict: the lowest index wins ties
        }
        float s = 0.f;
        for (int c = 0; c < p.C; ++c) s += expf(z[c] - mx);
        const int y = labels[row];
        const bool ok = (y >= 0 && y < p.C);
        if (!ok) atomicOr(err_flag, 1);
        const float lse = mx + logf(s);
        if (ok) local += lse - z[y];
        const float inv_s = 1.f / s;
        T* d = (T*)p.dlogits + (size_t)row * p.ldd;
        for (int c = 0; c < p.C; ++c) {
            float g = 0.f;
            if (ok) g = (expf(z[c] - mx) * inv_s - (c == y ? 1.f : 0.f)) * inv_rows;
            d[c] = ET<T>::from_f(g);
        }
        p.pred[row] = arg;
    }
    __shared__ float red[256];
    red[threadIdx.x] = local;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) *p.loss = red[0] * inv_rows;
}

hipError_t launch_ce(bool bf16, const CeProb* probs, int K, const int32_t* labels, int* err_flag, hipStream_t st) {
    if (bf16) hipLaunchKernelGGL(ce_kernel<bf16_t>, dim3(K), dim3(256), 0, st, probs, labels, err_flag);
    else hipLaunchKernelGGL(ce_kernel<float>, dim3(K), dim3(256), 0, st, probs, labels, err_flag);
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
    float s = 0.f;
    for (int i = 0; i < p.hw; ++i) s += ET<T>::to_f(in[(size_t)i * p.c]);
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
        if (p.mask && !(ET<T>::to_f(((const T*)p.in)[e]) > 0.f)) g = 0.f;
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
        if (p.mask && !(ET<T>::to_f(((const T*)p.src)[e]) > 0.f)) g = 0.f;
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
            o.x = wv[i].x - r * gv[i].x;
            o.y = wv[i].y - r * gv[i].y;
            o.z = wv[i].z - r * gv[i].z;
            o.w = wv[i].w - r * gv[i].w;
            *reinterpret_cast<f32x4_t*>(w + idx[i]) = o;
            if constexpr (SHADOW) {
                uint2 pk;
                pk.x = (unsigned)f2bf(o.x) | ((unsigned)f2bf(o.y) << 16);
                pk.y = (unsigned)f2bf(o.z) | ((unsigned)f2bf(o.w) << 16);
                *reinterpret_cast<uint2*>(shadow + idx[i]) = pk;
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

__global__ __launch_bounds__(256) void cast_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst, long long n) {
    const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= n) return;
    const f32x4_t v = *reinterpret_cast<const f32x4_t*>(src + i);
    uint2 pk;
    pk.x = (unsigned)f2bf(v.x) | ((unsigned)f2bf(v.y) << 16);
    pk.y = (unsigned)f2bf(v.z) | ((unsigned)f2bf(v.w) << 16);
    *reinterpret_cast<uint2*>(dst + i) = pk;
}

hipError_t launch_cast_bf16(const float* src, void* dst, long long n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    const int blocks = (int)((n / 4 + 255) / 256);
    hipLaunchKernelGGL(cast_bf16_kernel, dim3(blocks), dim3(256), 0, st, src, (bf16_t*)dst, n);
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

}  // namespace packk
