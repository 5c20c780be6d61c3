// Driver of the host-side walk of the aligned staged-tile kernels' fetchers (csrc/gemm_fetch_check.cpp) for
// one hand-made convolution forward problem: tests/test_plan_check_host.py compiles it once as it is (the
// walk must pass) and once per planted mistake (-DPACK_HALO_PLANT=n: the walk must fail).  No GPU code is
// compiled or run.
#include "pack_internal.h"

#include <cstdio>
#include <cstdlib>
#include <string>

namespace packk {
std::string gemm_fetch_walk(bool bf16, int mode, int bm, int bn, const GemmProb& p, const TileRef& tr, unsigned long long* a_lo,
                            unsigned long long* a_hi, unsigned long long* b_lo, unsigned long long* b_hi, long long* loads);
}

int main(int argc, char** argv) {
    // usage: driver bf16(0|1) stride B H W Cin Cout   (3x3 convolution forward, padding 1)
    if (argc != 8) return 2;
    using namespace packk;
    const bool bf16 = std::atoi(argv[1]) != 0;
    GemmProb p{};
    p.stride = std::atoi(argv[2]);
    const int B = std::atoi(argv[3]);
    p.H = std::atoi(argv[4]); p.W = std::atoi(argv[5]); p.Cin = std::atoi(argv[6]); p.Cout = std::atoi(argv[7]);
    p.Ho = (p.H - 1) / p.stride + 1; p.Wo = (p.W - 1) / p.stride + 1;
    p.R = B * p.Ho * p.Wo; p.Q = p.Cout; p.Kd = 9 * p.Cin; p.ksplit = p.Kd;
    p.lda = p.Cin; p.ldb = p.Kd; p.ldc = p.Cout;
    p.row_w = p.Wo; p.row_hw = p.Ho * p.Wo;
    auto lg = [](int v) { int l = 0; while ((1 << l) < v) ++l; return ((1 << l) == v) ? l : -1; };
    p.lg_row_w = lg(p.row_w); p.lg_row_hw = lg(p.row_hw);
    if (p.lg_row_w < 0 || p.lg_row_hw < 0) p.lg_row_w = p.lg_row_hw = -1;
    p.flags = F_VEC_A | F_VEC_B;
    // made-up operand addresses, far apart
    const unsigned long long esz = bf16 ? 2 : 4;
    const unsigned long long a_base = 0x100000000ull, b_base = 0x300000000ull;
    const unsigned long long a_bytes = (unsigned long long)B * p.H * p.W * p.Cin * esz, b_bytes = (unsigned long long)p.Q * p.ldb * esz;
    p.A = (const void*)a_base; p.B = (const void*)b_base;
    long long loads = 0;
    for (int tm = 0; tm < (p.R + 127) / 128; ++tm)
        for (int tn = 0; tn < (p.Q + 63) / 64; ++tn) {
            const TileRef tr{0, tm, tn, 0};
            unsigned long long alo, ahi, blo, bhi;
            std::string err = gemm_fetch_walk(bf16, CONV_FWD, 128, 64, p, tr, &alo, &ahi, &blo, &bhi, &loads);
            if (err.empty() && alo < ahi && (alo < a_base || ahi > a_base + a_bytes)) err = "loads of operand A leave it";
            if (err.empty() && blo < bhi && (blo < b_base || bhi > b_base + b_bytes)) err = "loads of operand B leave it";
            if (!err.empty()) {
                std::printf("FAIL tile (%d, %d): %s\n", tm, tn, err.c_str());
                return 1;
            }
        }
    std::printf("OK %lld loads\n", loads);
    return 0;
}
