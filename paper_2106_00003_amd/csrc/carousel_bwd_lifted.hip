// Reverse-sweep carousel kernels of the lifted rotation form, all shapes and strip widths.
#include "carousel_kernels.hpp"

namespace givens {
int carousel_backward_lifted(const CarouselBwdArgs &a, CarouselShape s, int W)
{
    return carousel_backward_form<2>(a, s, W);
}
} // namespace givens
