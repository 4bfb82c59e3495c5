// Instantiations of the fp32 pointwise kernel whose waves split the channels of one output tile.
#include "pwk_kernel.h"

namespace convfwd {

void register_pwk_f32(std::vector<Variant>& out)
{
    //                             KW TMB NBW GD
    pwk_register<PwkCfg<CONV_F32, 8, 2, 1, 4>>(out);   // M64 N32, 8 waves
    pwk_register<PwkCfg<CONV_F32, 4, 2, 1, 4>>(out);   // M64 N32, 4 waves
    pwk_register<PwkCfg<CONV_F32, 8, 1, 1, 4>>(out);   // M32 N32, 8 waves
    pwk_register<PwkCfg<CONV_F32, 16, 1, 1, 4>>(out);  // M32 N32, 16 waves
    pwk_register<PwkCfg<CONV_F32, 16, 2, 1, 2>>(out);  // M64 N32, 16 waves
    pwk_register<PwkCfg<CONV_F32, 4, 2, 2, 4>>(out);   // M64 N64, 4 waves
    pwk_register<PwkCfg<CONV_F32, 8, 2, 2, 2>>(out);   // M64 N64, 8 waves
    pwk_register<PwkCfg<CONV_F32, 4, 1, 2, 4>>(out);   // M32 N64, 4 waves
}

}  // namespace convfwd
