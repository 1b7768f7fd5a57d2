// K2 kernels, multiplier from the per-worker table (one scale per coded vector).
#include "agc_quantize.h"

namespace agc {

hipError_t launch_quantize_band0(const float* G, const CodeDev& code, const Workspace& ws, const QuantArgs& a,
                                 hipStream_t stream)
{
    return launch_quantize_band<0>(G, code, ws, a, stream);
}

}  // namespace agc
