// Instantiations of the second-generation tile convolution kernel (conv_tile2.h) for 3x3 filters.
#include "conv_tile2.h"

namespace sn {

hipError_t launch_tile2_3x3(const bf16_t *in, const bf16_t *w, void *out, const Plan &pl, hipStream_t st)
{
    if (pl.KT == 64) {
        if (pl.NF != 2 || !pl.wide || pl.dw != 16 || pl.ks != 1) return hipErrorInvalidValue;
        return launch2_one<3, 3, 2, true, 16, 1, 4>(in, w, out, pl, st);
    }
    const int sel = (pl.ks == 2 ? 8 : 0) | (pl.NF == 4 ? 4 : 0) | (pl.wide ? 2 : 0) | (pl.dw == 16 ? 1 : 0);
    switch (sel) {
    case 9: return launch2_one<3, 3, 2, false, 16, 2>(in, w, out, pl, st);
    case 8: return launch2_one<3, 3, 2, false, 4, 2>(in, w, out, pl, st);
    case 7: return launch2_one<3, 3, 4, true, 16>(in, w, out, pl, st);
    case 5: return launch2_one<3, 3, 4, false, 16>(in, w, out, pl, st);
    case 4: return launch2_one<3, 3, 4, false, 4>(in, w, out, pl, st);
    case 3: return launch2_one<3, 3, 2, true, 16>(in, w, out, pl, st);
    case 1: return launch2_one<3, 3, 2, false, 16>(in, w, out, pl, st);
    case 0: return launch2_one<3, 3, 2, false, 4>(in, w, out, pl, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace sn
