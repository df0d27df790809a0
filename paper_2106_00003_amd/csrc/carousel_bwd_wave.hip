// Reverse-sweep carousel kernels for workgroups of one wavefront with the exchange inside the wavefront (see
// carousel_fwd_wave.hip): 4 or 2 slots per lane (n up to 512), strips of 1, 2 or 4 columns.
#include "carousel_kernels.hpp"

namespace givens {

int carousel_backward_wave(const CarouselBwdArgs &a, int M, int W)
{
    switch (M) {
    case 4: return carousel_backward_wave_slots<4>(a, W);
    case 2: return carousel_backward_wave_slots<2>(a, W);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

} // namespace givens
