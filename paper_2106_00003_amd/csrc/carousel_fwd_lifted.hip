// Forward carousel kernels of the lifted rotation form, all shapes and strip widths.
#include "carousel_kernels.hpp"

namespace givens {
int carousel_forward_lifted(const CarouselFwdArgs &a, CarouselShape s, int W)
{
    return carousel_forward_form<2>(a, s, W);
}
} // namespace givens
