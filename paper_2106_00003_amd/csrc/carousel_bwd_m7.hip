// Reverse-sweep carousel kernels with 7 slots per lane (n = 14 L, up to 1024 lanes), standard rotation form,
// strips of at most 4 columns.
#include "carousel_kernels.hpp"

namespace givens {
int carousel_backward_m7(const CarouselBwdArgs &a, int waves, int W) { return carousel_backward_odd_slots<7>(a, waves, W); }
} // namespace givens
