// Unitary carousel kernels: the reverse sweep with 2 slots per lane (n up to 2048; strips of 8 floats).
#include "unitary_carousel_kernels.hpp"

namespace givens {

int unitary_carousel_backward_m2(const UnitaryCarouselBwdArgs &a, int waves, int W)
{
    return unitary_carousel_backward_slots<2>(a, waves, W);
}

} // namespace givens
