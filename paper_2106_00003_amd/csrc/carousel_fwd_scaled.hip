// Forward carousel kernels of the scaled rotation form, all shapes and strip widths.
#include "carousel_kernels.hpp"

namespace givens {
int carousel_forward_scaled(const CarouselFwdArgs &a, CarouselShape s, int W)
{
    return carousel_forward_form<1>(a, s, W);
}
} // namespace givens
