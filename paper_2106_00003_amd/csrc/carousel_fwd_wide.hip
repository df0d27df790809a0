// Forward carousel kernels for 513 to 1024 lanes (10, 12, 14 or 16 wavefronts, one workgroup per compute unit):
// the multiples of 8 beyond 4096 that are not multiples of 16 (4 slots per lane) and the multiples of 4 beyond 2048
// that are not multiples of 8 (2 slots per lane).
#include "carousel_kernels.hpp"

namespace givens {

template <int M>
static int fwd_wide_slots(const CarouselFwdArgs &a, int waves, int W)
{
    switch (waves) {
    case 10: return carousel_fwd_widths<M, 10>(W, a);
    case 12: return carousel_fwd_widths<M, 12>(W, a);
    case 14: return carousel_fwd_widths<M, 14>(W, a);
    case 16: return carousel_fwd_widths<M, 16>(W, a);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

int carousel_forward_wide(const CarouselFwdArgs &a, int M, int waves, int W)
{
    switch (M) {
    case 4: return fwd_wide_slots<4>(a, waves, W);
    case 2: return fwd_wide_slots<2>(a, waves, W);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

} // namespace givens
