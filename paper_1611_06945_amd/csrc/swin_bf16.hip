// bf16-storage instantiations of the strided window kernel for first layers (few input channels, large strided filters).
#include "swin16_kernel.h"

namespace convfwd {

//                               DT        C  R   S   ST TMB IRMAX PITCH
#define SW(C, R, S, ST, TMB, IRMAX, PITCH) Swin16Cfg<CONV_BF16, C, R, S, ST, TMB, IRMAX, PITCH>

void register_swin_bf16(std::vector<Variant>& out)
{
    // 11x11 stride 4 over 3 channels (rows of 43..62 outputs: a tile spans 4 output rows, 23 input rows)
    swin16_register<SW(3, 11, 11, 4, 3, 23, 256)>(out);  // M96
    swin16_register<SW(3, 11, 11, 4, 2, 23, 256)>(out);  // M64
    swin16_register<SW(3, 11, 11, 4, 1, 23, 256)>(out);  // M32
    // 7x7 stride 2 over 3 channels (rows of 64..125 outputs: a tile spans 3 output rows, 11 input rows)
    swin16_register<SW(3, 7, 7, 2, 2, 11, 256)>(out);    // M64
    swin16_register<SW(3, 7, 7, 2, 1, 11, 256)>(out);    // M32
}

}  // namespace convfwd
