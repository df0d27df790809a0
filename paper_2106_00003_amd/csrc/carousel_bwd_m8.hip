// Reverse-sweep carousel kernels with 8 slots per lane: the shapes beyond n = 4096 (multiples of 16 up to 8192,
// 257 to 512 lanes, i.e. 5 to 8 wavefronts), strips of at most 4 columns (two strips of 8 rows x 4 columns per lane
// are the 128 data registers the 4-slot kernels hold as 4 rows x 8 columns).
#include "carousel_kernels.hpp"

namespace givens {

template <int WAVES>
static int bwd_m8_widths(int W, const CarouselBwdArgs &a)
{
    switch (W) {
    case 4: carousel_launch_bwd<8, 4, WAVES>(a); return GIVENS_OK;
    case 2: carousel_launch_bwd<8, 2, WAVES>(a); return GIVENS_OK;
    case 1: carousel_launch_bwd<8, 1, WAVES>(a); return GIVENS_OK;
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

int carousel_backward_m8(const CarouselBwdArgs &a, int waves, int W)
{
    switch (waves) {
    case 5: return bwd_m8_widths<5>(W, a);
    case 6: return bwd_m8_widths<6>(W, a);
    case 7: return bwd_m8_widths<7>(W, a);
    case 8: return bwd_m8_widths<8>(W, a);
    default: return GIVENS_ERR_UNSUPPORTED;
    }
}

} // namespace givens
