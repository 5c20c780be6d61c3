// Driver of the host-side walk of the halo weight-gradient kernel (csrc/conv_dw_halo_check.cpp) for one
// hand-made problem: tests/test_plan_check_host.py compiles it once as it is (the walk must pass) and once
// per planted mistake (-DPACK_HALO_PLANT=n: the walk must fail).  No GPU code is compiled or run.
#include "conv_dw_halo.h"

#include <cstdio>
#include <cstdlib>
#include <string>

namespace packk {
std::string conv_dw_halo_walk(bool bf16, bool wide, const GemmProb& p, const TileRef& tr, long long a_bytes, long long b_bytes,
                              bool every_chunk, long long* loads, long long* frag_reads);
}

int main(int argc, char** argv) {
    // usage: driver bf16(0|1) stride B H W Cin Cout
    if (argc != 8) return 2;
    const bool bf16 = std::atoi(argv[1]) != 0;
    packk::GemmProb p{};
    p.stride = std::atoi(argv[2]);
    const int B = std::atoi(argv[3]);
    p.H = std::atoi(argv[4]); p.W = std::atoi(argv[5]); p.Cin = std::atoi(argv[6]); p.Cout = std::atoi(argv[7]);
    p.Ho = (p.H - 1) / p.stride + 1; p.Wo = (p.W - 1) / p.stride + 1;
    p.R = p.Cout; p.Q = 9 * p.Cin; p.Kd = B * p.Ho * p.Wo; p.ksplit = p.Kd; p.ldc = 9 * p.Cin;
    const long long esz = bf16 ? 2 : 4;
    const long long a_bytes = (long long)p.Kd * p.Cout * esz, b_bytes = (long long)B * p.H * p.W * p.Cin * esz;
    long long loads = 0, frags = 0;
    const bool wide = p.Cin % 64 == 0;               // 64 input channels per tile, else 32
    for (int tm = 0; tm < p.Cout / 64; ++tm)
        for (int tn = 0; tn < p.Cin / (wide ? 64 : 32); ++tn) {
            const packk::TileRef tr{0, tm, tn, 0};
            const std::string err = packk::conv_dw_halo_walk(bf16, wide, p, tr, a_bytes, b_bytes, true, &loads, &frags);
            if (!err.empty()) {
                std::printf("FAIL tile (%d, %d): %s\n", tm, tn, err.c_str());
                return 1;
            }
        }
    std::printf("OK %lld loads %lld operand reads\n", loads, frags);
    return 0;
}
