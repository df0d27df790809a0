// Forward carousel kernels for workgroups of one wavefront that exchange slots with DPP wavefront shifts instead
// of LDS (n = 2 M L with L <= 64: up to 1024 with 8 slots per lane, 512 with 4, 256 with 2), strips of 1 to 8
// columns: the shapes of small problems, whose sweeps are bound by the block-to-block chain when the batch is small
// and whose LDS-exchange shapes would leave lanes idle when it is large.
#include "carousel_kernels.hpp"

namespace givens {

int carousel_forward_wave(const CarouselFwdArgs &a, int M, int W)
{
    switch (M) {
    case 8: return carousel_forward_wave_slots<8>(a, W);
    case 4: return carousel_forward_wave_slots<4>(a, W);
    case 2: return carousel_forward_wave_slots<2>(a, W);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

} // namespace givens
