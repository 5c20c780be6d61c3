// Driver of the host-side walk of the stride-1 forward / input-gradient halo kernel
// (csrc/conv_rows_halo_check.cpp) for one hand-made problem: tests/test_plan_check_host.py compiles it once
// as it is (the walk must pass) and once per planted mistake (-DPACK_HALO_PLANT=n: the walk must fail).
// No GPU code is compiled or run.
#include "conv_rows_halo.h"

#include <cstdio>
#include <cstdlib>
#include <string>

namespace packk {
std::string conv_rows_halo_walk(bool bf16, bool narrow, bool dx, const GemmProb& p, const TileRef& tr, long long a_bytes,
                                long long* loads, long long* frag_reads);
}

int main(int argc, char** argv) {
    // usage: driver bf16(0|1) dx(0|1) B H W Cin Cout
    if (argc != 8) return 2;
    const bool bf16 = std::atoi(argv[1]) != 0, dx = std::atoi(argv[2]) != 0;
    packk::GemmProb p{};
    p.stride = 1;
    const int B = std::atoi(argv[3]);
    p.H = p.Ho = std::atoi(argv[4]); p.W = p.Wo = std::atoi(argv[5]); p.Cin = std::atoi(argv[6]); p.Cout = std::atoi(argv[7]);
    p.R = B * p.H * p.W;
    p.Q = dx ? p.Cin : p.Cout;
    p.Kd = 9 * (dx ? p.Cout : p.Cin);
    p.ksplit = p.Kd;
    const long long esz = bf16 ? 2 : 4;
    const long long a_bytes = (long long)p.R * (dx ? p.Cout : p.Cin) * esz;
    const bool narrow = p.Q <= 32;
    long long loads = 0, frags = 0;
    for (int tm = 0; tm < p.R / 256; ++tm) {
        const packk::TileRef tr{0, tm, 0, 0};
        const std::string err = packk::conv_rows_halo_walk(bf16, narrow, dx, p, tr, a_bytes, &loads, &frags);
        if (!err.empty()) {
            std::printf("FAIL tile %d: %s\n", tm, err.c_str());
            return 1;
        }
    }
    std::printf("OK %lld loads %lld operand reads\n", loads, frags);
    return 0;
}
