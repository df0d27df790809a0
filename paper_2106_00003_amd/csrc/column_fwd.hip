// Column forward kernels (small n): one instance per even n up to kColumnMaxN.
#include "carousel_host.hpp"
#include "column_kernels.hpp"

namespace givens {
namespace {
template <int N>
int column_dispatch(int n, int rows, long long B, const float2 *table, const float *X, float *Y, int identity,
                    int mirror, hipStream_t stream)
{
    if constexpr (N > kColumnMaxN) {
        return GIVENS_ERR_UNSUPPORTED;
    } else {
        if (n != N) return column_dispatch<N + 2>(n, rows, B, table, X, Y, identity, mirror, stream);
        const long long groups = (B + kColumnThreads - 1) / kColumnThreads;
        hipLaunchKernelGGL(column_forward_kernel<N>, dim3((unsigned)groups), dim3(kColumnThreads), 0, stream, rows, B,
                           table, X, Y, identity, mirror);
        return GIVENS_OK;
    }
}
} // namespace

int column_forward(int n, int rows, long long B, const float2 *table, const float *X, float *Y, int identity,
                   int mirror, hipStream_t stream)
{
    if (n < 2 || (n & 1) || n > kColumnMaxN) return GIVENS_ERR_UNSUPPORTED;
    return column_dispatch<2>(n, rows, B, table, X, Y, identity, mirror, stream);
}
} // namespace givens
