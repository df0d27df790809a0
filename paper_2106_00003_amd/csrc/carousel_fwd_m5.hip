// Forward carousel kernels with 5 slots per lane (n = 10 L, up to 1024 lanes): sizes whose half has no factor
// 2 to spare, e.g. the padded size of an odd n.  Standard rotation form only.
#include "carousel_kernels.hpp"

namespace givens {
int carousel_forward_m5(const CarouselFwdArgs &a, int waves, int W) { return carousel_forward_odd_slots<5>(a, waves, W); }
} // namespace givens
