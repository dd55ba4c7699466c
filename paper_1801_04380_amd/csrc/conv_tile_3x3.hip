// Instantiations of the tile convolution kernel (conv_tile.h) for one group of filters.
#include "conv_tile.h"

namespace sn {

hipError_t launch_tile_3x3(const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, bool staged, hipStream_t st)
{
    return launch_rs<3, 3, true>(in, w, out, pl, staged, st);
}

}  // namespace sn
