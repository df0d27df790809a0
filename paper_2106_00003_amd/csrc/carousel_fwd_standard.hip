// Forward carousel kernels of the standard rotation form, all shapes and strip widths.
#include "carousel_kernels.hpp"

namespace givens {
int carousel_forward_standard(const CarouselFwdArgs &a, CarouselShape s, int W)
{
    return carousel_forward_form<0>(a, s, W);
}
} // namespace givens
