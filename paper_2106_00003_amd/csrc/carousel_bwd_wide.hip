// Reverse-sweep carousel kernels for 513 to 1024 lanes (10, 12, 14 or 16 wavefronts, one workgroup per compute
// unit, strips of at most 4 columns: registers and LDS): the same shapes as carousel_fwd_wide.hip.
#include "carousel_kernels.hpp"

namespace givens {

template <int M, int WAVES>
static int bwd_wide_widths(int W, const CarouselBwdArgs &a)
{
    switch (W) {
    case 4: carousel_launch_bwd<M, 4, WAVES>(a); return GIVENS_OK;
    case 2: carousel_launch_bwd<M, 2, WAVES>(a); return GIVENS_OK;
    case 1: carousel_launch_bwd<M, 1, WAVES>(a); return GIVENS_OK;
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}
template <int M>
static int bwd_wide_slots(const CarouselBwdArgs &a, int waves, int W)
{
    switch (waves) {
    case 10: return bwd_wide_widths<M, 10>(W, a);
    case 12: return bwd_wide_widths<M, 12>(W, a);
    case 14: return bwd_wide_widths<M, 14>(W, a);
    case 16: return bwd_wide_widths<M, 16>(W, a);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

int carousel_backward_wide(const CarouselBwdArgs &a, int M, int waves, int W)
{
    switch (M) {
    case 4: return bwd_wide_slots<4>(a, waves, W);
    case 2: return bwd_wide_slots<2>(a, waves, W);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

} // namespace givens
