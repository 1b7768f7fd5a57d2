// K2 kernels, one max-abs scale per 256-coordinate block.
#include "agc_quantize.h"

namespace agc {

hipError_t launch_quantize_band1(const float* G, const CodeDev& code, const Workspace& ws, const QuantArgs& a,
                                 hipStream_t stream)
{
    return launch_quantize_band<1>(G, code, ws, a, stream);
}

}  // namespace agc
