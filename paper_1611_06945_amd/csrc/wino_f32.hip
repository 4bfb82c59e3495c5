// Instantiations of the Winograd F(2x2, 3x3) kernel (fp32, 3x3 stride-1 layers).
#include "wino_kernel.h"

namespace convfwd {

void register_wino_f32(std::vector<Variant>& out)
{
    //                    MBLK NBLK XW LBE CB     TM x TT tiles, planes per wave, staging slots per thread, channels per step
    wino_register<WinoCfg<2, 3, 2, 1, 8>>(out);
    wino_register<WinoCfg<2, 3, 2, 2, 8>>(out);
    wino_register<WinoCfg<3, 2, 2, 1, 8>>(out);
    wino_register<WinoCfg<3, 2, 2, 2, 8>>(out);
    wino_register<WinoCfg<2, 2, 2, 1, 8>>(out);
    wino_register<WinoCfg<2, 2, 2, 2, 8>>(out);
    wino_register<WinoCfg<2, 2, 2, 1, 16>>(out);
    wino_register<WinoCfg<1, 2, 2, 1, 16>>(out);
    wino_register<WinoCfg<1, 3, 2, 1, 8>>(out);
    wino_register<WinoCfg<4, 2, 2, 1, 8>>(out);
    wino_register<WinoCfg<2, 4, 2, 2, 8>>(out);
    // filter transform inside the product kernel: no filter kernel, no workspace
    wino_register<WinoCfg<2, 3, 2, 1, 8, 1>>(out);
    wino_register<WinoCfg<3, 2, 2, 1, 8, 1>>(out);
    wino_register<WinoCfg<2, 2, 2, 1, 8, 1>>(out);
}

hipError_t launch_wino_filter_transform(const float* filt, float* out, int K, int C, hipStream_t s)
{
    hipLaunchKernelGGL(wino_filter_kernel<8>, dim3((unsigned)((K + 31) / 32), (unsigned)(C / 8)), dim3(256), 0, s, filt, out, K, C);
    return hipGetLastError();
}

size_t wino_transformed_filter_bytes(int K, int C) { return (size_t)16 * wino_kpitch(K) * C * sizeof(float); }

}  // namespace convfwd
