// Reverse-sweep carousel kernels with 3 slots per lane (n = 6 L, up to 1024 lanes), standard rotation form,
// strips of at most 4 columns.
#include "carousel_kernels.hpp"

namespace givens {
int carousel_backward_m3(const CarouselBwdArgs &a, int waves, int W) { return carousel_backward_odd_slots<3>(a, waves, W); }
} // namespace givens
