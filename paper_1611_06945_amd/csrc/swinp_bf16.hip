// bf16-storage instantiations of the first-layer kernel that pools its own output (3x3 stride-2 max-pool fused).
#include "swinp16_kernel.h"

namespace convfwd {

//                                                              DT   C  R  S  ST TMB NBW PTH PTW PITCH
#define SWP(C, R, S, ST, TMB, NBW, PTH, PTW, PITCH) SwinP16Cfg<CONV_BF16, C, R, S, ST, TMB, NBW, PTH, PTW, PITCH>

void register_swinp_bf16(std::vector<Variant>& out)
{
    // 11x11 stride 4 over 3 channels: 9x9 pooled outputs from 19x19 convolution outputs (12 blocks), 83 input rows x 84
    // columns.  One block per wave: with 3 blocks per wave (4 waves) the multiply loop would be bound by the matrix units
    // instead of LDS reads, but one wave per SIMD hides neither the LDS latency nor the staging arithmetic (measured:
    // 18.2 us against 12.7 us for the stack's first layer at batch 20).
    swinp16_register<SWP(3, 11, 11, 4, 3, 1, 9, 9, 92)>(out);  // M96
    swinp16_register<SWP(3, 11, 11, 4, 2, 1, 9, 9, 92)>(out);  // M64
    swinp16_register<SWP(3, 11, 11, 4, 1, 1, 9, 9, 92)>(out);  // M32
    // 7x7 stride 2 over 3 channels: 43 input rows x 44 columns
    swinp16_register<SWP(3, 7, 7, 2, 2, 1, 9, 9, 44)>(out);    // M64
    swinp16_register<SWP(3, 7, 7, 2, 1, 1, 9, 9, 44)>(out);    // M32
}

}  // namespace convfwd
