// K2 kernels, multiplier from the per-worker table (one scale per coded vector); several fills of the staging area.
#include "agc_quantize.h"

namespace agc {

AGC_QUANT_UNIT(launch_quantize_band0m)
{
    return launch_quantize_band<0, true>(G, code, ws, a, stream);
}

}  // namespace agc
