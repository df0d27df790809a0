// Reverse-sweep carousel kernels whose persistent workgroups are linked into chains that share rows of partial
// sums (4 slots per lane, 5 to 8 wavefronts, strips of 8 or 4 columns): the large reverse sweeps.
#include "carousel_kernels.hpp"

namespace givens {

int carousel_backward_chain(const CarouselBwdArgs &a, const CarouselChainArgs &c, int M, int waves, int W)
{
    if (M != 4) return GIVENS_ERR_UNSUPPORTED;
    return carousel_backward_chain_slots<4>(a, c, waves, W);
}

} // namespace givens
