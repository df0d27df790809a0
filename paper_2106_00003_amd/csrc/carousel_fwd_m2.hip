// Forward carousel kernels with 2 slots per lane: all workgroup sizes and strip widths, the three rotation
// forms inside each kernel.
#include "carousel_kernels.hpp"

namespace givens {
int carousel_forward_m2(const CarouselFwdArgs &a, int waves, int W) { return carousel_forward_slots<2>(a, waves, W); }
} // namespace givens
