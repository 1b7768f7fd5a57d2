// K2 kernels, one Euclidean scale per 256-coordinate block, found in the pass; all workers fit one fill of the staging area.
#include "agc_quantize.h"

namespace agc {

AGC_QUANT_UNIT(launch_quantize_band2s)
{
    return launch_quantize_band<2, false>(G, code, ws, a, stream);
}

}  // namespace agc
