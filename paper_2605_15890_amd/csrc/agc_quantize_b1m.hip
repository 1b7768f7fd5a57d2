// K2 kernels, one max-abs scale per 256-coordinate block, found in the pass; several fills of the staging area.
#include "agc_quantize.h"

namespace agc {

AGC_QUANT_UNIT(launch_quantize_band1m)
{
    return launch_quantize_band<1, true>(G, code, ws, a, stream);
}

}  // namespace agc
