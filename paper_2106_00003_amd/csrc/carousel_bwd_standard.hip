// Reverse-sweep carousel kernels of the standard rotation form, all shapes and strip widths.
#include "carousel_kernels.hpp"

namespace givens {
int carousel_backward_standard(const CarouselBwdArgs &a, CarouselShape s, int W)
{
    return carousel_backward_form<0>(a, s, W);
}
} // namespace givens
