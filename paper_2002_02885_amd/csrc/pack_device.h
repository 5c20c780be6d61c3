// Device-side helpers shared by the kernel source files of the packed training step: element types,
// bfloat16 conversion, activations, the SGD expression, raw buffer loads issued as assembly statements
// and the hand-placed waits that go with them.  Nothing here is part of the public ABI.
#pragma once
#include "pack_internal.h"

#include <type_traits>

namespace packk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

// float -> bfloat16, round to nearest with ties to even, NaN stays NaN: the hardware conversion
// (one instruction per pair of values)
__device__ __forceinline__ unsigned pack2bf(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bf16_t f2bf(float f) { return (bf16_t)(pack2bf(f, 0.f) & 0xffffu); }
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((unsigned int)h) << 16); }

// activations of the paper's search space (Table 3) and their derivatives written in terms of the
// stored output (what the backward pass has at hand); leaky ReLU slope 0.2
constexpr float LEAKY_SLOPE = 0.2f;
__device__ __forceinline__ float act_apply(int kind, float z) {
    switch (kind) {
        case ACT_RELU: return fmaxf(z, 0.f);
        case ACT_LEAKY: return z > 0.f ? z : LEAKY_SLOPE * z;
        case ACT_SIGMOID: return 1.f / (1.f + expf(-z));
        case ACT_TANH: return tanhf(z);
        default: return z;
    }
}
__device__ __forceinline__ float act_deriv(int kind, float out) {
    switch (kind) {
        case ACT_RELU: return out > 0.f ? 1.f : 0.f;
        case ACT_LEAKY: return out > 0.f ? 1.f : LEAKY_SLOPE;
        case ACT_SIGMOID: return out * (1.f - out);
        case ACT_TANH: return 1.f - out * out;
        default: return 1.f;
    }
}

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

__device__ __forceinline__ u32x4_t buf_load16(const i32x4_t rsrc, unsigned voff, unsigned soff) {
    u32x4_t v;
    // the scalar operands are wave-uniform by construction; say so, since values that went through
    // vector arithmetic (an integer division) would otherwise be handed over in vector registers
    const unsigned so = __builtin_amdgcn_readfirstlane(soff);
    asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen" : "=v"(v) : "v"(voff), "s"(rsrc), "s"(so) : "memory");
    return v;
}

// Blocks until at most NEWER asm loads issued after the given registers' loads are outstanding.
// The registers are in-out operands so that nothing that reads them can move above the wait.
template <int NEWER, int N>
__device__ __forceinline__ void wait_stage(u32x4_t (&regs)[N]) {
    static_assert(NEWER >= 0 && NEWER < 64, "vmcnt is a 6-bit counter");
    if constexpr (N == 1) asm volatile("s_waitcnt vmcnt(%1)" : "+v"(regs[0]) : "n"(NEWER));
    else if constexpr (N == 2) asm volatile("s_waitcnt vmcnt(%2)" : "+v"(regs[0]), "+v"(regs[1]) : "n"(NEWER));
    else if constexpr (N == 4)
        asm volatile("s_waitcnt vmcnt(%4)" : "+v"(regs[0]), "+v"(regs[1]), "+v"(regs[2]), "+v"(regs[3]) : "n"(NEWER));
    else if constexpr (N == 8)
        asm volatile("s_waitcnt vmcnt(%8)"
                     : "+v"(regs[0]), "+v"(regs[1]), "+v"(regs[2]), "+v"(regs[3]), "+v"(regs[4]), "+v"(regs[5]),
                       "+v"(regs[6]), "+v"(regs[7])
                     : "n"(NEWER));
    else static_assert(N == 1 || N == 2 || N == 4 || N == 8, "unsupported register count");
}

template <int N>
__device__ __forceinline__ void pin_regs(u32x4_t (&r)[N]) {
    // makes every register of a load stage an operand of a statement that sits after the wait, so that
    // nothing that reads them can be moved above it (the loads themselves are assembly statements whose
    // completion the compiler does not track)
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(r[i]));
}
template <int NEWER>
__device__ __forceinline__ void wait_loads() {
    static_assert(NEWER >= 0 && NEWER < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NEWER) : "memory");
}

// the SGD update of one parameter; every path that applies it (update kernels, fused epilogues)
// uses this one expression so that a member's bits do not depend on which path its pack takes
__device__ __forceinline__ float sgd_apply(float w, float g, float lr) { return __builtin_fmaf(-lr, g, w); }

}  // namespace packk
