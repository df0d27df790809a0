// Reverse-sweep carousel kernels of the scaled rotation form, all shapes and strip widths.
#include "carousel_kernels.hpp"

namespace givens {
int carousel_backward_scaled(const CarouselBwdArgs &a, CarouselShape s, int W)
{
    return carousel_backward_form<1>(a, s, W);
}
} // namespace givens
