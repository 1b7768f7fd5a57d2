// K2 kernels, multiplier from the per-worker table (one scale per coded vector); all workers fit one fill of the staging area.
#include "agc_quantize.h"

namespace agc {

AGC_QUANT_UNIT(launch_quantize_band0s)
{
    return launch_quantize_band<0, false>(G, code, ws, a, stream);
}

}  // namespace agc
