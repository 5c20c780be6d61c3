// Halo form of the convolution weight gradient for gfx950 (see conv_dw_halo.h for the address rules).
//
// The staged-tile form in pack_kernels.hip treats the weight gradient as a product with a gathered
// operand: every 128 x 128 output tile gathers its input pixels again for each tap it covers, and the
// output-gradient rows again for every column tile, so a layer's activations cross the L2 -> LDS path
// about seven times more often than they exist.  Here a workgroup keeps ALL NINE taps of a 64 x 64 block
// of (output channel, input channel) pairs in its accumulators (nine 32 x 32 blocks per wave, 144
// registers), so per chunk of output pixels it needs the output gradient once and the input rows the
// chunk can reach once; both lie in LDS exactly as they lie in memory (pixel-major, channels contiguous)
// and the matrix-instruction operands, which want the reduction index (the pixel) contiguous per lane, are
// formed by CDNA4's transposing LDS reads (bfloat16) or plain 4-byte reads (float, one pixel per lane).
//
// The reduction order is that of the staged-tile form: ascending chunks, inside a chunk ascending steps of
// sixteen pixels (two for float), every pixel in the same slot of the matrix instruction, splits with the
// same boundaries summed in split order by reduce_kernel.  The two forms therefore give the same bits.
#include "conv_dw_halo.h"
#include "pack_device.h"

#include <utility>

namespace packk {

typedef short v4s_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4s_t* lds_v4s_ptr;

template <int... Is, typename F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, Is...>, F&& f) {
    (f(std::integral_constant<int, Is>{}), ...);
}

// The work of one wave; TGI: its tap group (compile-time, so that every accumulator index is static).
template <typename T, int WM, int WN, int STRIDE, int TG, int TGI>
__device__ __forceinline__ void conv_dw_halo_body(const GemmProb& p, const TileRef& tr, char* __restrict__ lds, const float lrk) {
    constexpr int ESZ = (int)sizeof(T);
    typedef HaloCfg<ESZ, WM, WN, STRIDE, TG> Cfg;
    constexpr int NT = Cfg::NT, CH = Cfg::CH, NLD = Cfg::NLD, NLA = Cfg::NLA, LOADS = NLD + NLA;
    constexpr int PIXB_A = Cfg::PIXB_A, PIXB_B = Cfg::PIXB_B;
    constexpr int TAP0 = tap_first<TG>(TGI), NTAP = tap_count<TG>(TGI);
    const HaloGeom g = halo_geom<ESZ, CH>(p);
    const int tid = threadIdx.x, lane = tid & 63, wave = (tid >> 6) % (WM * WN);
    const int wm = wave / WN, wn = wave % WN;
    const int o0 = tr.tm * Cfg::CO_T, c0 = tr.tn * Cfg::CI_T;
    const int kbeg = tr.ks * p.ksplit;
    const int kend = min(p.Kd, kbeg + p.ksplit);
    const int nk = (kend - kbeg) / CH;
    const bool do_bias_grad = tr.tn == 0 && p.dbias != nullptr;

    // what a thread loads per chunk, relative to the chunk's origin (fixed for the whole tile)
    unsigned hv[NLD], av[NLA];
#pragma unroll
    for (int i = 0; i < NLD; ++i) hv[i] = halo_vec_offset<Cfg, ESZ>(g, c0, tid + NT * i);
#pragma unroll
    for (int j = 0; j < NLA; ++j) av[j] = dz_vec_offset<Cfg, ESZ>(g, o0, tid + NT * j);

    // Chunk t: the output gradient through a descriptor over the whole tensor, the chunk's position in
    // the scalar offset; the input through a descriptor over the ONE image the chunk lies in, so that a
    // halo row above or below the image is out of the descriptor's range and reads as zeros.  A chunk
    // beyond the reduction (the pipeline always prefetches ahead) gets empty descriptors.
    // (called for t = 0, 1, 2, ... in turn: the cursor steps from chunk to chunk)
    HaloCursor cur = halo_cursor(g, kbeg);
    auto issue = [&](int t, u32x4_t(&rh)[NLD], u32x4_t(&ra)[NLA]) {
        const int k0 = kbeg + t * CH;
        const bool live = t < nk;
        const int img = live ? cur.img : 0;
        const int i0 = live ? (cur.pix >> g.lgWo) : 0;
        halo_cursor_advance(g, CH, cur);
        const unsigned long long ib = (unsigned long long)p.B + (unsigned long long)img * (unsigned long long)g.img_bytes;
        i32x4_t rs;
        rs.x = __builtin_amdgcn_readfirstlane((int)(unsigned)ib);
        rs.y = __builtin_amdgcn_readfirstlane((int)(unsigned)(ib >> 32));
        rs.z = __builtin_amdgcn_readfirstlane(live ? (int)g.img_bytes : 0);
        rs.w = 0x00020000;
        const unsigned roff = (unsigned)halo_row_offset(g, i0);
#pragma unroll
        for (int i = 0; i < NLD; ++i) rh[i] = buf_load16(rs, hv[i] + roff, 0u);
        const unsigned long long ab = (unsigned long long)p.A;
        i32x4_t rz;
        rz.x = __builtin_amdgcn_readfirstlane((int)(unsigned)ab);
        rz.y = __builtin_amdgcn_readfirstlane((int)(unsigned)(ab >> 32));
        rz.z = __builtin_amdgcn_readfirstlane(live ? (int)BUF_RECORDS : 0);
        rz.w = 0x00020000;
        const unsigned soff = live ? (unsigned)k0 * (unsigned)(g.Cout * ESZ) : 0u;
#pragma unroll
        for (int j = 0; j < NLA; ++j) ra[j] = buf_load16(rz, av[j], soff);
    };
    auto stash = [&](int buf, const u32x4_t(&rh)[NLD], const u32x4_t(&ra)[NLA]) {
        char* const hb = lds + buf * (Cfg::HALO_BYTES + Cfg::DZ_BYTES);
        char* const db = hb + Cfg::HALO_BYTES;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            // (load slots beyond the halo hold zeros and go to pixel slots beyond it, which nothing reads)
            *reinterpret_cast<u32x4_t*>(hb + halo_lds_offset<Cfg>(tid + NT * i)) = rh[i];
        }
#pragma unroll
        for (int j = 0; j < NLA; ++j)
            if (Cfg::CH * Cfg::VPP_A % NT == 0 || tid + NT * j < Cfg::CH * Cfg::VPP_A)
                *reinterpret_cast<u32x4_t*>(db + dz_lds_offset<Cfg>(tid + NT * j)) = ra[j];
    };

    f32x16_t acc[NTAP];
#pragma unroll
    for (int t = 0; t < NTAP; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
    // Bias gradient = sum of dZ over the pixels, in pixel order.  The waves of the first column of the wave
    // grid hold it: lane l < 32 of wave (wm, 0) owns output channel o0 + 32 * wm + l, and the values to add
    // are the ones the wave holds anyway as its dZ operand (see bias_step).
    float bias_grad = 0.f;
    const bool bias_wave = do_bias_grad && wn == 0 && TGI == 0;

    // lane constants of the fragment reads
    int a_lane, b_lane;          // byte offset of the lane's channels inside a pixel of the dZ / halo block
    int b_slot[4];               // bf16: halo pixel slot of the lane's first pixel in each of the four steps of a chunk
    if constexpr (ESZ == 2) {
        a_lane = (wm * 32 + frag_channel_bf16(lane)) * 2;
        b_lane = (wn * 32 + frag_channel_bf16(lane)) * 2;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) b_slot[kk] = halo_slot(g, frag_pixel_bf16(lane, kk, 0));
    } else {
        a_lane = (wm * 32 + (lane & 31)) * 4;
        b_lane = (wn * 32 + (lane & 31)) * 4;
    }
    const int row_step = g.HWD * PIXB_B;   // bytes from a tap row to the next

    // One step of the reduction = sixteen pixels (bfloat16: one matrix instruction per tap) or eight (float:
    // four instructions per tap, instruction j pairing pixel j with pixel j + 4).  A chunk is a fixed
    // sequence of NI matrix instructions, instruction idx = (step, j, tap of this wave's tap group).  With one wave per SIMD nothing
    // but the wave's own matrix instructions can hide the latency of its LDS reads, so the operands of
    // instruction idx + AHEAD are requested before instruction idx is issued (a ring of AHEAD + 1 operand
    // registers), and scheduling barriers keep the compiler from undoing that order.
    constexpr int SUB = (ESZ == 2) ? 1 : 4, PER_STEP = SUB * NTAP, NI = 4 * PER_STEP;
    constexpr int AHEAD = (TG >= 3) ? 4 : 6, RING = AHEAD + 1;
    static_assert(CH == ((ESZ == 2) ? 64 : 32), "four steps per chunk");
    typedef short v8s_t __attribute__((ext_vector_type(8)));
    // (the dZ operand of a step is shared by the step's taps and is requested with the first of them, up to
    // AHEAD instructions early, i.e. possibly two steps ahead of the one being multiplied: a ring of three)
    static_assert(AHEAD < 2 * PER_STEP, "the dZ operand ring holds three steps");
    v8s_t a16[3], b16[RING];       // bfloat16 operands: eight pixels per lane
    float a32[3][4], b32[RING];    // float operands: one pixel per lane and instruction
    const char* bp = nullptr;      // LDS address of the lane's tap (0, 0) operand of the (step, j) being read
    auto read_operands = [&](int buf, auto IDX) {
        constexpr int idx = decltype(IDX)::value;
        constexpr int kk = idx / PER_STEP, j = (idx / NTAP) % SUB, t = idx % NTAP, tap = TAP0 + t, u = tap / 3, v = tap % 3;
        const char* const hb = lds + buf * (Cfg::HALO_BYTES + Cfg::DZ_BYTES);
        const char* const db = hb + Cfg::HALO_BYTES;
        if constexpr (ESZ == 2) {
            if constexpr (t == 0) {
                const char* ap = db + frag_pixel_bf16(lane, kk, 0) * PIXB_A + a_lane;
                const v4s_t a_lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)ap);
                const v4s_t a_hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(ap + 4 * PIXB_A));
                a16[kk % 3] = __builtin_shufflevector(a_lo, a_hi, 0, 1, 2, 3, 4, 5, 6, 7);
                bp = hb + b_slot[kk] * PIXB_B + b_lane;
            }
            const char* tp = bp + u * row_step + v * PIXB_B;
            const v4s_t b_lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)tp);
            const v4s_t b_hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(tp + 4 * STRIDE * PIXB_B));
            b16[idx % RING] = __builtin_shufflevector(b_lo, b_hi, 0, 1, 2, 3, 4, 5, 6, 7);
        } else {
            if constexpr (t == 0) {
                const int q = frag_pixel_f32(lane, kk, j);
                a32[kk % 3][j] = *reinterpret_cast<const float*>(db + q * PIXB_A + a_lane);
                bp = hb + halo_slot(g, q) * PIXB_B + b_lane;
            }
            b32[idx % RING] = *reinterpret_cast<const float*>(bp + u * row_step + v * PIXB_B);
        }
    };
    auto multiply = [&](auto IDX) {
        constexpr int idx = decltype(IDX)::value;
        constexpr int kk = idx / PER_STEP, j = (idx / NTAP) % SUB, t = idx % NTAP;
        if constexpr (ESZ == 2)
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a16[kk % 3]), __builtin_bit_cast(bf16x8_t, b16[idx % RING]),
                                                             acc[t], 0, 0, 0);
        else
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a32[kk % 3][j], b32[idx % RING], acc[t], 0, 0, 0);
    };
    // The pixels of a step in ascending order: lanes 0-31 hold the first half of them (eight, or four) for
    // their channel, lanes 32-63 the second half.  The running sum sits in the lower lanes, is carried to
    // the upper lanes for their half and back, so every channel's pixels are added one by one in order.
    // lanes 32-63 receive what lanes 0-31 hold (v_permlane32_swap: a vector-ALU exchange of the two halves,
    // unlike a shuffle through the LDS crossbar it does not wait for the operand reads in flight)
    auto lower_to_upper = [](float v) {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        return __uint_as_float(r[0]);
    };
    auto upper_to_lower = [](float v) {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        return __uint_as_float(r[1]);
    };
    auto bias_step = [&](auto KK) {
        constexpr int kk = decltype(KK)::value;
        if (!bias_wave) return;
        float s0 = bias_grad;
        if constexpr (ESZ == 2) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s0 += bf2f((bf16_t)a16[kk % 3][e]);
            float s1 = lower_to_upper(s0);
#pragma unroll
            for (int e = 0; e < 8; ++e) s1 += bf2f((bf16_t)a16[kk % 3][e]);
            bias_grad = upper_to_lower(s1);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) s0 += a32[kk % 3][j];
            float s1 = lower_to_upper(s0);
#pragma unroll
            for (int j = 0; j < 4; ++j) s1 += a32[kk % 3][j];
            bias_grad = upper_to_lower(s1);
        }
    };

    // ST register stages and two LDS buffers, one barrier per chunk.  After the barrier of chunk `it`
    // (complete in its buffer; nobody reads the other buffer any more): the first matrix instructions of chunk
    // `it` are issued, behind them the stage emptied by the previous chunk is refilled with the loads of chunk
    // it + ST, the rest of the first step is multiplied, chunk
    // it + 1 (whose loads were requested ST - 1 chunks ago: a chunk's worth of matrix instructions is shorter
    // than the slowest of a chunk's loads takes to come back, which is what two stages ran into) is stored
    // to the other buffer under those matrix instructions, then the remaining steps.
    constexpr int ST = (TG >= 2 && STRIDE == 1) ? 3 : 2;   // (three stages of the larger stride-2 halo do not fit the register file)
    u32x4_t rh[ST][NLD], ra[ST][NLA];
#pragma unroll
    for (int s = 0; s < ST; ++s) {
        issue(s, rh[s], ra[s]);
        __builtin_amdgcn_sched_barrier(0);
    }
    wait_loads<(ST - 1) * LOADS>();
    pin_regs(rh[0]);
    pin_regs(ra[0]);
    stash(0, rh[0], ra[0]);
    using std::integral_constant;
    auto chunk = [&](auto STG, auto PAR, const int it) {
        constexpr int stg = decltype(STG)::value, par = decltype(PAR)::value, nxt = (stg + 1) % ST;
        __syncthreads();
        static_for(std::make_integer_sequence<int, AHEAD>{}, [&](auto I) { read_operands(par, I); });
        __builtin_amdgcn_sched_barrier(0);
        static_for(std::make_integer_sequence<int, NI>{}, [&](auto I) {
            constexpr int idx = decltype(I)::value;
            if constexpr (idx + AHEAD < NI) read_operands(par, integral_constant<int, idx + AHEAD>{});
            __builtin_amdgcn_sched_barrier(0);
            multiply(I);
            // (the requests of chunk it + ST go out behind the chunk's first matrix instructions, under which
            // their address arithmetic runs, instead of between the barrier and the first of them)
            if constexpr (idx == 1) issue(it + ST, rh[stg], ra[stg]);
            if constexpr (idx % PER_STEP == PER_STEP - 1) bias_step(integral_constant<int, idx / PER_STEP>{});
            if constexpr (idx == PER_STEP - 1) {
                wait_loads<(ST - 1) * LOADS>();
                pin_regs(rh[nxt]);
                pin_regs(ra[nxt]);
                stash(par ^ 1, rh[nxt], ra[nxt]);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // chunks run in groups of G (a multiple of the stage count and of the two buffers), so that stage and
    // buffer of every chunk in the unrolled body are compile-time constants
    constexpr int G = (ST % 2 == 0) ? ST : 2 * ST;
    int it = 0;
    for (; it + G <= nk; it += G)
        static_for(std::make_integer_sequence<int, G>{}, [&](auto J) {
            constexpr int j = decltype(J)::value;
            chunk(integral_constant<int, j % ST>{}, integral_constant<int, j & 1>{}, it + j);
        });
    // (the remaining chunks as nested conditions: chunk j + 1 only after chunk j, so that no path through
    // the code skips a chunk and runs a later one with the stages out of step)
    auto rest = [&](auto self, auto J) -> void {
        constexpr int j = decltype(J)::value;
        if constexpr (j < G - 1) {
            if (it + j < nk) {
                chunk(integral_constant<int, j % ST>{}, integral_constant<int, j & 1>{}, it + j);
                self(self, integral_constant<int, j + 1>{});
            }
        }
    };
    rest(rest, integral_constant<int, 0>{});
    // the last chunks requested loads beyond the reduction (empty descriptors): they still target the
    // stage registers, which must not count as free before they have landed
    wait_loads<0>();
#pragma unroll
    for (int s = 0; s < ST; ++s) {
        pin_regs(rh[s]);
        pin_regs(ra[s]);
    }

    // ---- epilogue ----
    // Accumulator register e of a wave's 32 x 32 block: output channel 8*(e/4) + 4*(lane/32) + e%4, input
    // channel lane%32; the 32 lanes of a half-wave cover 128 contiguous bytes of one (output channel, tap) row.
    const bool upd = (p.flags & F_UPDATE) != 0;
    const bool keep_g = !upd || (p.flags & F_KEEP_G);
    if (bias_wave && lane < 32) {
        const int o = o0 + wm * 32 + lane;
        if (keep_g) p.dbias[(size_t)tr.ks * p.R + o] = bias_grad;
        if (upd) p.upd_b[o] = sgd_apply(p.upd_b[o], bias_grad, lrk);
    }
    float* const gf = (float*)p.C + (size_t)tr.ks * p.split_stride;
    const int c = c0 + wn * 32 + (lane & 31);
#pragma unroll
    for (int t = 0; t < NTAP; ++t) {
        float wv[16];
        size_t off[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int o = o0 + wm * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            off[e] = (size_t)o * p.ldc + (size_t)(TAP0 + t) * g.Cin + c;
            if (upd) wv[e] = p.upd_w[off[e]];
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float gr = acc[t][e];
            if (upd) {
                const float w = sgd_apply(wv[e], gr, lrk);
                p.upd_w[off[e]] = w;
                if (p.upd_shadow) ((bf16_t*)p.upd_shadow)[off[e]] = f2bf(w);
            }
            if (keep_g) gf[off[e]] = gr;
        }
    }
}

template <typename T, int WM, int WN, int STRIDE, int TG>
__global__ __launch_bounds__(64 * WM * WN * TG) void conv_dw_halo_kernel(const GemmProb* __restrict__ probs,
                                                                         const TileRef* __restrict__ tiles,
                                                                         const void* __restrict__ x, char* __restrict__ ws, LrTable lr) {
    typedef HaloCfg<(int)sizeof(T), WM, WN, STRIDE, TG> Cfg;
    __shared__ __attribute__((aligned(16))) char lds[Cfg::LDS_BYTES];
    const TileRef tr = tiles[blockIdx.x];
    if (tr.prob < 0) return;
    GemmProb p = probs[tr.prob];
    if (p.flags & F_B_INPUT) p.B = (const char*)x + p.x_off;
    if (p.flags & F_WS) {   // partial sums of a split reduction go to the workspace this launch was given
        p.C = ws + (size_t)p.C;
        p.dbias = (float*)(ws + (size_t)p.dbias);
    }
    const float lrk = lr.lr[p.member];
    // the waves of a tap group run the same instruction sequence (same number of barriers in both groups)
    const int tg = (int)(threadIdx.x >> 6) / (WM * WN);
    if (TG == 1 || tg == 0) conv_dw_halo_body<T, WM, WN, STRIDE, TG, 0>(p, tr, lds, lrk);
    else if (TG == 2 || tg == 1) conv_dw_halo_body<T, WM, WN, STRIDE, TG, (TG > 1 ? 1 : 0)>(p, tr, lds, lrk);
    else conv_dw_halo_body<T, WM, WN, STRIDE, TG, (TG > 2 ? 2 : 0)>(p, tr, lds, lrk);
}

template <typename T, int WM, int WN, int STRIDE, int TG>
static hipError_t launch_halo(const GemmProb* probs, const TileRef* tiles, int n, const void* x, char* ws, const LrTable& lr, hipStream_t st) {
    hipLaunchKernelGGL((conv_dw_halo_kernel<T, WM, WN, STRIDE, TG>), dim3(n), dim3(64 * WM * WN * TG), 0, st, probs, tiles, x, ws, lr);
    return hipGetLastError();
}

hipError_t launch_conv_dw_halo(bool bf16, int tile_cfg, const GemmProb* probs, const TileRef* tiles, int n, const void* x,
                               char* ws, const LrTable& lr, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    switch (tile_cfg) {
        case GEMM_CFG_HALO_S1:
            return bf16 ? launch_halo<bf16_t, 2, 2, 1, 2>(probs, tiles, n, x, ws, lr, st) : launch_halo<float, 2, 2, 1, 1>(probs, tiles, n, x, ws, lr, st);
        case GEMM_CFG_HALO_S2:
            return bf16 ? launch_halo<bf16_t, 2, 2, 2, 2>(probs, tiles, n, x, ws, lr, st) : launch_halo<float, 2, 2, 2, 1>(probs, tiles, n, x, ws, lr, st);
        case GEMM_CFG_HALO32_S1:
            return bf16 ? launch_halo<bf16_t, 2, 1, 1, 1>(probs, tiles, n, x, ws, lr, st) : launch_halo<float, 2, 1, 1, 1>(probs, tiles, n, x, ws, lr, st);
        default: return hipErrorInvalidValue;   // (no 32-channel form at stride 2: its load stages do not fit the register file)
    }
}

int conv_dw_halo_cfg(bool bf16, const GemmProb& p) {
    if (p.stride != 1 && p.stride != 2) return -1;
    const bool s1 = p.stride == 1;
    bool wide, narrow;
    if (bf16) {
        wide = s1 ? halo_supported<HaloCfg<2, 2, 2, 1, 2>, 2>(p) : halo_supported<HaloCfg<2, 2, 2, 2, 2>, 2>(p);
        narrow = s1 && halo_supported<HaloCfg<2, 2, 1, 1>, 2>(p);
    } else {
        wide = s1 ? halo_supported<HaloCfg<4, 2, 2, 1>, 4>(p) : halo_supported<HaloCfg<4, 2, 2, 2>, 4>(p);
        narrow = s1 && halo_supported<HaloCfg<4, 2, 1, 1>, 4>(p);
    }
    if (wide) return s1 ? GEMM_CFG_HALO_S1 : GEMM_CFG_HALO_S2;
    if (narrow) return GEMM_CFG_HALO32_S1;
    return -1;
}

}  // namespace packk
