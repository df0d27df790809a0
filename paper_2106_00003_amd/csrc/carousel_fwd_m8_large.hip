// Forward carousel kernels with 8 slots per lane, workgroups of 5 to 8 wavefronts (n = 4112 .. 8192).
#include "carousel_kernels.hpp"

namespace givens {
int carousel_forward_m8_large(const CarouselFwdArgs &a, int waves, int W)
{
    return carousel_forward_slots_5to8<8>(a, waves, W);
}
} // namespace givens
