// Forward carousel kernels with 3 slots per lane (n = 6 L, up to 1024 lanes): sizes whose half has no factor
// 2 to spare, e.g. the padded size of an odd n.  Standard rotation form only.
#include "carousel_kernels.hpp"

namespace givens {
int carousel_forward_m3(const CarouselFwdArgs &a, int waves, int W) { return carousel_forward_odd_slots<3>(a, waves, W); }
} // namespace givens
