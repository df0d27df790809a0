// Unitary carousel kernels: the phase pass, the coefficient tables and the forward sweep (8 slots per lane).
#include "unitary_carousel_kernels.hpp"
#include "unitary_phase_kernels.hpp"

namespace givens {

template <bool REVERSE>
static void launch_phase_scan(int n, const uint2 *q, unsigned *turn, float2 *fin, hipStream_t stream)
{
    // one thread per pair up to 1024 threads, then two pairs per thread (more pairs per thread measured slower: the pass is bound by the
    // latency of its LDS round trip per pair, not by the barrier)
    const int H = n / 2;
    if (H <= kPhaseScanThreads)
        hipLaunchKernelGGL((unitary_phase_scan_kernel<REVERSE, 1>), dim3(1), dim3((H + 63) / 64 * 64), 0, stream, n, q,
                           turn, fin);
    else
        hipLaunchKernelGGL((unitary_phase_scan_kernel<REVERSE, 2>), dim3(1), dim3(kPhaseScanThreads), 0, stream, n, q,
                           turn, fin);
}

int unitary_carousel_coefficients(int n, const float *theta, const float *phi, int reverse, uint2 *q, unsigned *turn,
                                  float *sgn, float2 *rot, float2 *phs, float *orient, float2 *fin, hipStream_t stream)
{
    if (!unitary_carousel_supported(n) || n / 2 > 2 * kPhaseScanThreads) return GIVENS_ERR_UNSUPPORTED;
    const long long N = (long long)n * (n - 1) / 2;
    const int threads = 256;
    const unsigned blocks = (unsigned)((N + threads - 1) / threads < 8192 ? (N + threads - 1) / threads : 8192);
    if (reverse) {
        hipLaunchKernelGGL(unitary_phase_input_kernel<true>, dim3(blocks), dim3(threads), 0, stream, n, theta, phi, q);
        launch_phase_scan<true>(n, q, turn, fin, stream);
        hipLaunchKernelGGL(unitary_carousel_table_kernel<true>, dim3(blocks), dim3(threads), 0, stream, n, theta, turn,
                           sgn, rot, phs, orient);
    } else {
        hipLaunchKernelGGL(unitary_phase_input_kernel<false>, dim3(blocks), dim3(threads), 0, stream, n, theta, phi, q);
        launch_phase_scan<false>(n, q, turn, fin, stream);
        hipLaunchKernelGGL(unitary_carousel_table_kernel<false>, dim3(blocks), dim3(threads), 0, stream, n, theta, turn,
                           sgn, rot, phs, orient);
    }
    return GIVENS_OK;
}

int unitary_carousel_forward_m8(const UnitaryCarouselFwdArgs &a, int waves, int W)
{
    return unitary_carousel_forward_slots<8>(a, waves, W);
}

} // namespace givens
