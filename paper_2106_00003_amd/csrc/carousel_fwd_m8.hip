// Forward carousel kernels with 8 slots per lane, workgroups of 1 to 4 wavefronts (5 to 8: carousel_fwd_m8_large.hip):
// all strip widths, the three rotation forms inside each kernel.
#include "carousel_kernels.hpp"

namespace givens {
int carousel_forward_m8_large(const CarouselFwdArgs &a, int waves, int W);
int carousel_forward_m8(const CarouselFwdArgs &a, int waves, int W)
{
    return waves <= 4 ? carousel_forward_slots_1to4<8>(a, waves, W) : carousel_forward_m8_large(a, waves, W);
}
} // namespace givens
