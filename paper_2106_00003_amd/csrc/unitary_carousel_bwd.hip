// Unitary carousel kernels: the reverse sweep (4 slots per lane).
#include "unitary_carousel_kernels.hpp"

namespace givens {

int unitary_carousel_backward_m4(const UnitaryCarouselBwdArgs &a, int waves, int W)
{
    return unitary_carousel_backward_slots<4>(a, waves, W);
}

} // namespace givens
