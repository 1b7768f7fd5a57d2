// K2 kernels, one Euclidean scale per 256-coordinate block.
#include "agc_quantize.h"

namespace agc {

hipError_t launch_quantize_band2(const float* G, const CodeDev& code, const Workspace& ws, const QuantArgs& a,
                                 hipStream_t stream)
{
    return launch_quantize_band<2>(G, code, ws, a, stream);
}

}  // namespace agc
