// K2 kernels, one Euclidean scale per 256-coordinate block, found in the pass; several fills of the staging area.
#include "agc_quantize.h"

namespace agc {

AGC_QUANT_UNIT(launch_quantize_band2m)
{
    return launch_quantize_band<2, true>(G, code, ws, a, stream);
}

}  // namespace agc
