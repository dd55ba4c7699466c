// Instantiations of the tile convolution kernel (conv_tile.h) for one group of filters.
#include "conv_tile.h"

namespace sn {

hipError_t launch_tile_other(int R, int S, const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, bool staged,
                             hipStream_t st)
{
    if (R == 2 && S == 2) return launch_rs<2, 2, false>(in, w, out, pl, staged, st);
    if (R == 5 && S == 5) return launch_rs<5, 5, true>(in, w, out, pl, staged, st);
    if (R == 1 && S == 7) return launch_rs<1, 7, false>(in, w, out, pl, staged, st);
    if (R == 7 && S == 1) return launch_rs<7, 1, false>(in, w, out, pl, staged, st);
    return hipErrorInvalidValue;
}

}  // namespace sn
